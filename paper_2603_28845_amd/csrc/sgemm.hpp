// fp32 GEMM on v_mfma_f32_32x32x2_f32 shared by the kernels that need fp32 products (QEP target, JointQ gradient).
#pragma once
#include "common.hpp"

namespace onecomp {

enum : int { S_BTRANS = 1, S_BUPPER_T = 2, S_BUPPER = 4 };

struct SgemmArgs {
    const float* A; int64_t lda;     // m x k, k contiguous
    const float* B; int64_t ldb;     // S_BTRANS: n x k (k contiguous), else k x n
    float* C; int64_t ldc;           // m x n out (plain store), or nullptr when the fused epilogue is used
    int m, n, k;
    int flags;                       // S_BUPPER_T: B given transposed is upper triangular as n x k (zero for k < n)
                                     // S_BUPPER:   B (k x n) is upper triangular (zero for k > n)
    // fused epilogue (C == nullptr): out[r][colmap ? colmap[c] : c] = base[r][c] + alpha * acc
    const float* base; int64_t ldbase;
    const int32_t* colmap;
    float* out; int64_t ldout;
    float alpha;
};

onecomp_status sgemm(const SgemmArgs& g, hipStream_t stream);

}  // namespace onecomp
