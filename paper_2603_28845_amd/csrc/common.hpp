// Shared host/device helpers of the gfx950 library (no arithmetic of the method lives here).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <atomic>
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

// Raises a kernel's limit of dynamic LDS once per device (the attribute belongs to the device's copy of the code).
// `done` is that kernel's bit mask of devices already prepared; the only host-side state the library keeps is such
// caches of device properties, safe to use from several host threads and with several devices.
static inline onecomp_status allow_dynamic_lds(const void* fn, int bytes, std::atomic<uint64_t>& done) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return ONECOMP_ERR_HIP;
    const uint64_t bit = uint64_t(1) << (dev & 63);
    if (dev < 64 && (done.load(std::memory_order_acquire) & bit)) return ONECOMP_OK;
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) return ONECOMP_ERR_HIP;
    if (dev < 64) done.fetch_or(bit, std::memory_order_release);
    return ONECOMP_OK;
}

// compute units of the current device (0 on failure); looked up once per device
static inline int device_cus() {
    static std::atomic<int> cus[64];
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (dev >= 0 && dev < 64 && (v = cus[dev].load(std::memory_order_relaxed)) > 0) return v;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) return 0;
    if (dev >= 0 && dev < 64) cus[dev].store(v, std::memory_order_relaxed);
    return v;
}

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---- direct global -> LDS loads ---------------------------------------------------------------
// One wave-wide 16-byte load: lane l's 16 bytes, read at buffer offset voffset, land at LDS byte address
// lds_byte_addr + 16 l.  Lanes whose offset is outside the descriptor's range deposit zeros.  Inline assembly, so
// the compiler neither counts the load nor orders LDS reads behind it: the caller waits with
// __builtin_amdgcn_s_waitcnt(wait_vmcnt(n)) and a workgroup barrier before reading the data.
__device__ __forceinline__ void lds_load16(uint32_t lds_byte_addr, uint32_t voffset, __amdgpu_buffer_rsrc_t rsrc) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :: "s"(lds_byte_addr), "v"(voffset), "s"(rsrc) : "memory", "m0");
}
// a buffer offset that is out of range for every descriptor used here
constexpr uint32_t LDS_DMA_OOB = 0xFFFFFFF0u;
// s_waitcnt immediate that waits until at most n (< 64) vector memory loads are outstanding and for nothing else
// (expcnt and lgkmcnt fields at their no-wait maximum; vmcnt is split over bits 3:0 and 15:14)
constexpr int wait_vmcnt(int n) { return 0x0F70 | (n & 15) | ((n >> 4) << 14); }

// Device scalars of a split-fp16 product: maxima (as the bit patterns of non-negative floats, which order like
// unsigned integers, so an integer atomic max is exact and order independent) and the power-of-two scales derived
// from them.
struct Scalars {
    uint32_t max_w_bits;   // max |left operand| (the sweep: max |W|)
    uint32_t max_u_bits;   // max |right operand| (the sweep: max |U_jk / U_jj| over the strict upper triangle)
    float f_d;             // the left operand is stored as fp16 hi + lo of  x * f_d
    float f_u;             // the right operand as fp16 hi + lo of  y * f_u
    float f_all;           // f_d * f_u
    float f_inv;           // 1 / (f_d * f_u)
};

// C[:, c0 .. c1) += f_inv * D^T B over k = 0 .. K-1 with fp32 accuracy from fp16 MFMAs (operands split hi + lo, three
// products): C fp32 d_out x d_in row-major; D k-major, row ek + k holds the d_out left-operand values of k
// (hi in Dh, lo in Dl, row length ldD = split_update_ld(d_out), the padding may hold anything finite);
// B row-major with d_in columns, row u0 + k (hi in Bh, lo in Bl); sc->f_all and sc->f_inv are read on the device.
// K % 32 == 0, c0 % 8 == 0, c1 % 8 == 0.
onecomp_status split_update(float* C, int64_t d_out, int64_t d_in, const uint16_t* Dh, const uint16_t* Dl, int64_t ldD,
                            const uint16_t* Bh, const uint16_t* Bl, const Scalars* sc, int ek, int K, int u0, int c0,
                            int c1, hipStream_t stream);
int64_t split_update_ld(int64_t d_out);
// Left operand of split_update from a row-major fp32 matrix: rows [0, k_count rounded up to 32) of Dh / Dl receive
// (src[:, k] d[k] f_d)^T as fp16 hi + lo (d == nullptr: 1; zero behind k_count), with f_d the power of two that puts
// the maximum found in sc->max_w_bits (left there by the producer of src: max |src d|) into [2^12, 2^13).  Expects
// sc->f_u (power of two, the right operand's scale); leaves f_d, f_all, f_inv in sc; clears other->max_w_bits if
// other is given.
onecomp_status split_left_operand(const float* src, int64_t ld_src, int64_t d_out, int k_count, const float* d,
                                  Scalars* sc, Scalars* other, uint16_t* Dh, uint16_t* Dl, hipStream_t stream);

// ---- small device helpers shared by the kernel files -------------------------------------------
__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
    return x;
}

// Workgroup maximum of non-negative values into *dst (bit patterns of non-negative floats order like the values);
// s_max is one word of LDS.  One atomic per workgroup at most: atomics on one address are serialized, and the
// maximum only grows, so a workgroup that does not exceed what is already there (even a stale copy of it) has
// nothing to add.  Every thread of the workgroup must call it.
__device__ __forceinline__ void block_max_bits(uint32_t* dst, float v, uint32_t* s_max) {
    if (threadIdx.x == 0) *s_max = 0u;
    __syncthreads();
    v = wave_max(v);
    if ((threadIdx.x & 63) == 0) atomicMax(s_max, __float_as_uint(v));
    __syncthreads();
    if (threadIdx.x == 0 && *s_max > __hip_atomic_load(dst, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(dst, *s_max);
}

// p[0 .. 4 n4) = 0 with a kernel (callers may be under graph capture, where memset nodes are avoided)
onecomp_status fill_zero(float* p, int64_t n4, hipStream_t stream);

// ---- entry points implemented in the kernel files -------------------------------------------
size_t gram_workspace_bytes(int64_t d_in);
// schedule of an accumulate call: tile shape of its main kernel and how many times that kernel is launched
struct GramPlanInfo {
    int tile_rows, tile_cols, launches;
};
// info != nullptr: describe the call (ws_bytes is the size a workspace would have), launch nothing
onecomp_status gram_accumulate_bf16(const void* X, int64_t n_tokens, int64_t d_in, int64_t ldx,
                                    float* H, void* ws, size_t ws_bytes, hipStream_t stream,
                                    GramPlanInfo* info = nullptr);
onecomp_status gram_accumulate_f32(const void* X, int64_t n_tokens, int64_t d_in, int64_t ldx,
                                   float* H, hipStream_t stream);

onecomp_status gram_cross_accumulate_bf16(const void* Xh, const void* X, int64_t n_tokens, int64_t d_in, int64_t ldxh,
                                          int64_t ldx, float* G, hipStream_t stream);

size_t factor_workspace_bytes(int64_t d_in);
onecomp_status factor_run(const float* H, int64_t d_in, float damp, int act_order, int form, int32_t* perm_out,
                          float* U, int32_t* info, void* workspace, hipStream_t stream);

size_t sweep_workspace_bytes(int64_t d_out, int64_t d_in, int block);
onecomp_status sweep_run(const void* W, onecomp_dtype w_dtype, int64_t d_out, int64_t d_in,
                         const float* U, int form, const int32_t* perm, int bits, int group_size, int block, int grid,
                         uint8_t* Q, float* scales, float* zeros, float* W_hat, float* loss,
                         void* workspace, hipStream_t stream);

size_t qep_workspace_bytes(int64_t d_out, int64_t d_in);
onecomp_status qep_target_run(const void* W, onecomp_dtype w_dtype, int64_t d_out, int64_t d_in, const float* G,
                              const float* H, const float* U, const int32_t* perm, float alpha, float* W_star,
                              void* workspace, hipStream_t stream);

size_t sensitivity_workspace_bytes();
onecomp_status sensitivity_run(const void* W, onecomp_dtype w_dtype, int64_t d_out, int64_t d_in, const float* a_diag,
                               const float* b_diag, int bits, int group_size, int grid, float* err, void* workspace,
                               hipStream_t stream);

onecomp_status sensitivity_run_static(const void* W, onecomp_dtype w_dtype, int64_t d_out, int64_t d_in,
                                      const float* a_diag, const float* b_diag, int bits, int group_size, int grid,
                                      float* err, hipStream_t stream);

// register-only MFMA loop (kind 0: bf16 32x32x16, 1: fp64 16x16x4) on every CU with waves_per_simd waves per SIMD,
// operands constant (random == 0) or pseudo-random; *flops (host) receives the flop count of the launch
onecomp_status mfma_rate_probe(int kind, int waves_per_simd, int random, int64_t iters, float* sink, double* flops,
                               hipStream_t stream);

size_t jointq_workspace_bytes(int64_t d_out, int64_t d_in, int group_size);
onecomp_status jointq_run(const void* W, onecomp_dtype w_dtype, int64_t d_out, int64_t d_in, const float* A,
                          const int32_t* perm, float lam, int bits, int group_size, int grid, int n_pass, int max_scans, uint8_t* Q, float* scales,
                          const float* zeros, float* W_hat, float* objective, int32_t* n_moves, void* workspace,
                          hipStream_t stream);

}  // namespace onecomp
