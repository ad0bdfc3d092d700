// Measurement aid: the rate the matrix pipes of this device sustain on a register-only loop of independent MFMAs
// (no LDS, no memory traffic), for the two instructions the hot path is priced on: v_mfma_f32_32x32x16_bf16 (Gram)
// and v_mfma_f64_16x16x4_f64 (factor).  The published peaks assume the 2.4 GHz boost clock; what a kernel can reach is
// bounded by what these loops reach.  The operands are either the same small constant in every lane or pseudo-random
// per lane and per MFMA: the pipes draw more power on data that toggles, and the clock follows.  Nothing of the
// method's arithmetic lives here.
#include "common.hpp"

namespace onecomp {
namespace {

constexpr int PROBE_THREADS = 256;   // 4 waves: one per SIMD; waves per SIMD = workgroups per CU
constexpr int PROBE_ACC = 8;         // independent accumulator tiles per wave

// uniform in [-1, 1) from a counter (integer hash, top 24 bits)
__device__ __forceinline__ float probe_uniform(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return float(x >> 8) * (1.0f / 8388608.0f) - 1.0f;
}

__global__ __launch_bounds__(PROBE_THREADS, 2) void mfma_rate_bf16_kernel(float* __restrict__ sink, int64_t iters,
                                                                          int random) {
    const uint32_t id = (blockIdx.x * PROBE_THREADS + threadIdx.x) * 64u;
    bf16x8 a[PROBE_ACC], b[PROBE_ACC];
#pragma unroll
    for (int t = 0; t < PROBE_ACC; ++t)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            a[t][e] = __bf16(random ? probe_uniform(id + t * 8 + e) : 1.0f / 1024.0f);
            b[t][e] = __bf16(random ? probe_uniform(id + 0x9e3779b9u + t * 8 + e) : 1.0f / 2048.0f);
        }
    float16v acc[PROBE_ACC];
#pragma unroll
    for (int t = 0; t < PROBE_ACC; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
#pragma unroll 1
    for (int64_t i = 0; i < iters; ++i) {
#pragma unroll
        for (int t = 0; t < PROBE_ACC; ++t)
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[t], b[(t + 3) % PROBE_ACC], acc[t], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int t = 0; t < PROBE_ACC; ++t) s += acc[t][0] + acc[t][15];
    if (s == 123456.789f) sink[0] = s;   // practically never true: keeps the loop alive
}

__global__ __launch_bounds__(PROBE_THREADS, 2) void mfma_rate_f64_kernel(float* __restrict__ sink, int64_t iters,
                                                                         int random) {
    const uint32_t id = (blockIdx.x * PROBE_THREADS + threadIdx.x) * 64u;
    double a[PROBE_ACC], b[PROBE_ACC];
#pragma unroll
    for (int t = 0; t < PROBE_ACC; ++t) {
        // random: 53 significant bits from two draws, so that the low mantissa bits toggle as well
        a[t] = random ? double(probe_uniform(id + t)) + double(probe_uniform(id + 32 + t)) * 0x1p-24 : 1.0 / 1024.0;
        b[t] = random ? double(probe_uniform(id + 0x9e3779b9u + t)) + double(probe_uniform(id + 77 + t)) * 0x1p-24
                      : 1.0 / 2048.0;
    }
    double4v acc[PROBE_ACC];
#pragma unroll
    for (int t = 0; t < PROBE_ACC; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[t][r] = 0.0;
#pragma unroll 1
    for (int64_t i = 0; i < iters; ++i) {
#pragma unroll
        for (int t = 0; t < PROBE_ACC; ++t)
            acc[t] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[t], b[(t + 3) % PROBE_ACC], acc[t], 0, 0, 0);
    }
    double s = 0.0;
#pragma unroll
    for (int t = 0; t < PROBE_ACC; ++t) s += acc[t][0] + acc[t][3];
    if (s == 123456.789) sink[0] = float(s);
}

}  // namespace

onecomp_status mfma_rate_probe(int kind, int waves_per_simd, int random, int64_t iters, float* sink, double* flops,
                               hipStream_t stream) {
    const int n_cus = device_cus();
    if (n_cus <= 0) return ONECOMP_ERR_HIP;
    const unsigned grid = unsigned(n_cus) * unsigned(waves_per_simd);
    // flop per MFMA: 2 * M * N * K
    const double per_mfma = (kind == 0) ? 2.0 * 32 * 32 * 16 : 2.0 * 16 * 16 * 4;
    *flops = double(grid) * (PROBE_THREADS / 64) * double(iters) * PROBE_ACC * per_mfma;
    if (kind == 0) hipLaunchKernelGGL(mfma_rate_bf16_kernel, dim3(grid), dim3(PROBE_THREADS), 0, stream, sink, iters, random);
    else hipLaunchKernelGGL(mfma_rate_f64_kernel, dim3(grid), dim3(PROBE_THREADS), 0, stream, sink, iters, random);
    ONECOMP_CHECK_LAUNCH();
    return ONECOMP_OK;
}

}  // namespace onecomp
