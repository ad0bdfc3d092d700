// Activation-aware sensitivity of one layer under a candidate quantization configuration (Sec. 4.1 of the
// paper, "AutoBit"): the weight perturbation dW = W^ - W of a fast round-to-nearest (RTN) proxy, weighted by the
// diagonals of the Kronecker-factored curvature,
//     err = 1/2 tr(B dW A dW^T)  ->  1/2 sum_r sum_c b_r a_c dW_rc^2      (A, B diagonal, as the paper uses them)
// in this library's d_out x d_in storage (a over input channels, b over output rows).  The RTN proxy rounds
// every group of G consecutive input channels of a row to its own grid (Eq. (1), (2) or (3), (4)), no feedback.
//
// gfx950: memory bound (W is read once from HBM, a second time from cache).  A team of TS <= 64 lanes of one
// wave owns a group at a time, 16 bytes per lane and load: pass for min / max (shuffle reduction inside the team),
// second pass to round and accumulate.  Per-workgroup partial sums are combined in a fixed order: bit-wise reproducible.
#include "common.hpp"

namespace onecomp {
namespace {

// V consecutive elements (16 bytes) as floats
template <typename T>
struct Vec;
template <>
struct Vec<float> {
    static constexpr int V = 4;
    static __device__ inline void load(const float* p, float (&v)[4]) {
        const float4v x = *reinterpret_cast<const float4v*>(p);
        v[0] = x[0]; v[1] = x[1]; v[2] = x[2]; v[3] = x[3];
    }
};
template <>
struct Vec<uint16_t> {
    static constexpr int V = 8;
    static __device__ inline void load(const uint16_t* p, float (&v)[8]) {
        const uint4v x = *reinterpret_cast<const uint4v*>(p);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            v[2 * e] = __uint_as_float(x[e] << 16);
            v[2 * e + 1] = __uint_as_float(x[e] & 0xFFFF0000u);
        }
    }
};

struct SensArgs {
    const void* W;
    const float* a;      // [d_in]
    const float* b;      // [d_out] or nullptr (ones)
    float* partial;      // [gridDim.x]
    int64_t n_groups;    // d_out * d_in / G
    int d_in, G, n_g, ts;
    float qmax, qs;      // highest code; qs > 0: symmetric grid with zero-point qs
};

template <typename T>
__global__ __launch_bounds__(256) void sens_kernel(SensArgs g) {
    constexpr int V = Vec<T>::V;
    __shared__ float team_sum[128];
    const T* W = static_cast<const T*>(g.W);
    const int tid = threadIdx.x;
    const int ts = g.ts;                         // lanes per team, a power of two in 2 .. 64; a lane takes V elements
    const int team = tid / ts, tl = tid % ts, teams = 256 / ts;
    float acc = 0.f;
    for (int64_t gi = int64_t(blockIdx.x) * teams + team; gi < g.n_groups; gi += int64_t(gridDim.x) * teams) {
        const int64_t row = gi / g.n_g;
        const int c0 = int(gi % g.n_g) * g.G;
        const T* wp = W + row * g.d_in + c0;
        float mn = 3.0e38f, mx = -3.0e38f;
        for (int c = tl * V; c < g.G; c += ts * V) {
            float v[V];
            Vec<T>::load(wp + c, v);
#pragma unroll
            for (int e = 0; e < V; ++e) { mn = fminf(mn, v[e]); mx = fmaxf(mx, v[e]); }
        }
        for (int off = ts >> 1; off > 0; off >>= 1) {
            mn = fminf(mn, __shfl_xor(mn, off, 64));
            mx = fmaxf(mx, __shfl_xor(mx, off, 64));
        }
        float s, z;
        if (g.qs > 0.f) {
            s = fmaxf(fabsf(mn), fabsf(mx)) / g.qs;
            if (s == 0.f) s = 1.f;
            z = g.qs;
        } else {
            s = (mx - mn) / g.qmax;
            if (s == 0.f) s = 1.f;
            z = fminf(fmaxf(rintf(-mn / s), 0.f), g.qmax);
        }
        const float rs = 1.0f / s;
        const float br = g.b ? g.b[row] : 1.0f;
        float part = 0.f;
        for (int c = tl * V; c < g.G; c += ts * V) {     // second pass: the group is in cache
            float v[V], av[V];
            Vec<T>::load(wp + c, v);
#pragma unroll
            for (int e = 0; e < V; e += 4) {
                const float4v x = *reinterpret_cast<const float4v*>(g.a + c0 + c + e);
                av[e] = x[0]; av[e + 1] = x[1]; av[e + 2] = x[2]; av[e + 3] = x[3];
            }
#pragma unroll
            for (int e = 0; e < V; ++e) {
                const float q = fminf(fmaxf(rintf(v[e] * rs) + z, 0.f), g.qmax);
                const float d = v[e] - s * (q - z);
                part = __builtin_fmaf(av[e] * d, d, part);
            }
        }
        acc = __builtin_fmaf(br, part, acc);
    }
    // team sum (fixed butterfly), then teams and workgroups in index order
    for (int off = ts >> 1; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (tl == 0) team_sum[team] = acc;
    __syncthreads();
    if (tid == 0) {
        float t = 0.f;
        for (int i = 0; i < teams; ++i) t += team_sum[i];
        g.partial[blockIdx.x] = t;
    }
}

__global__ __launch_bounds__(256) void sens_final_kernel(const float* __restrict__ partial, int n, float* __restrict__ err) {
    __shared__ double part[256];
    double s = 0.0;
    for (int i = threadIdx.x; i < n; i += 256) s += double(partial[i]);
    part[threadIdx.x] = s;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if (int(threadIdx.x) < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) *err = float(0.5 * part[0]);
}

constexpr int SENS_WGS = 2048;

// Scratch of the entry point that takes no workspace: the per-workgroup partial sums, SENS_WGS floats (8 KB), in
// device memory that belongs to the loaded code object (one copy per GPU, held until the process ends).  In host
// code the array's name is only a handle: the device address is looked up once per device and used from then on.
static __device__ __align__(256) float scratch[SENS_WGS];

// device address of `scratch` on the current device (nullptr on failure); looked up on the first call per device
float* scratch_address() {
    static std::atomic<float*> cache[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return nullptr;
    const bool cached = dev >= 0 && dev < 64;
    float* p = cached ? cache[dev].load(std::memory_order_acquire) : nullptr;
    if (p) return p;
    if (hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
    if (cached) cache[dev].store(p, std::memory_order_release);
    return p;
}

}  // namespace

size_t sensitivity_workspace_bytes() { return size_t(SENS_WGS) * sizeof(float); }

onecomp_status sensitivity_run_static(const void* W, onecomp_dtype w_dtype, int64_t d_out, int64_t d_in,
                                      const float* a_diag, const float* b_diag, int bits, int group_size, int grid,
                                      float* err, hipStream_t stream) {
    float* ws = scratch_address();
    if (!ws) return ONECOMP_ERR_HIP;
    return sensitivity_run(W, w_dtype, d_out, d_in, a_diag, b_diag, bits, group_size, grid, err, ws, stream);
}

onecomp_status sensitivity_run(const void* W, onecomp_dtype w_dtype, int64_t d_out, int64_t d_in, const float* a_diag,
                               const float* b_diag, int bits, int group_size, int grid, float* err, void* workspace,
                               hipStream_t stream) {
    SensArgs g;
    g.W = W; g.a = a_diag; g.b = b_diag; g.partial = static_cast<float*>(workspace);
    g.d_in = int(d_in); g.G = group_size; g.n_g = int(d_in / group_size);
    g.n_groups = d_out * int64_t(g.n_g);
    const int vec = w_dtype == ONECOMP_BF16 ? 8 : 4;          // elements per 16-byte lane load
    int ts = 2;
    while (ts < 64 && ts * 2 * vec <= group_size) ts *= 2;    // one pass over the group if it fits 64 lanes
    g.ts = ts;
    g.qs = grid == ONECOMP_GRID_SYMMETRIC ? float((1 << (bits - 1)) - 1) : 0.f;
    g.qmax = grid == ONECOMP_GRID_SYMMETRIC ? 2.f * g.qs : float((1 << bits) - 1);
    const int64_t teams = 256 / ts;
    const int wgs = int(ceil_div(g.n_groups, teams) < SENS_WGS ? ceil_div(g.n_groups, teams) : SENS_WGS);
    if (w_dtype == ONECOMP_BF16) hipLaunchKernelGGL(sens_kernel<uint16_t>, dim3(wgs), dim3(256), 0, stream, g);
    else hipLaunchKernelGGL(sens_kernel<float>, dim3(wgs), dim3(256), 0, stream, g);
    ONECOMP_CHECK_LAUNCH();
    hipLaunchKernelGGL(sens_final_kernel, dim3(1), dim3(256), 0, stream, g.partial, wgs, err);
    ONECOMP_CHECK_LAUNCH();
    return ONECOMP_OK;
}

}  // namespace onecomp
