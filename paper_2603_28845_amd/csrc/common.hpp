// Shared host/device helpers of the gfx950 library (no arithmetic of the method lives here).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/onecomp.h"

namespace onecomp {

typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef double double4v __attribute__((ext_vector_type(4)));

#define ONECOMP_LDS __attribute__((address_space(3)))

// Returns ONECOMP_ERR_HIP from the enclosing function if the last launch failed.
#define ONECOMP_CHECK_LAUNCH()                                   \
    do {                                                         \
        if (hipGetLastError() != hipSuccess) return ONECOMP_ERR_HIP; \
    } while (0)

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---- entry points implemented in the kernel files -------------------------------------------
onecomp_status gram_accumulate_bf16(const void* X, int64_t n_tokens, int64_t d_in, int64_t ldx,
                                    float* H, hipStream_t stream);
onecomp_status gram_accumulate_f32(const void* X, int64_t n_tokens, int64_t d_in, int64_t ldx,
                                   float* H, hipStream_t stream);

size_t factor_workspace_bytes(int64_t d_in);
onecomp_status factor_run(const float* H, int64_t d_in, float damp, int act_order, int32_t* perm_out,
                          float* U, int32_t* info, void* workspace, hipStream_t stream);

size_t sweep_workspace_bytes(int64_t d_out, int64_t d_in, int block);
onecomp_status sweep_run(const void* W, onecomp_dtype w_dtype, int64_t d_out, int64_t d_in,
                         const float* U, const int32_t* perm, int bits, int group_size, int block,
                         uint8_t* Q, float* scales, float* zeros, float* W_hat, float* loss,
                         void* workspace, hipStream_t stream);

}  // namespace onecomp
