// Corrected quantization target of error propagation (QEP, Sec. 4.2.1 of the paper, Eq. (qep)):
//     W* = (I + alpha (H^ + lambda I)^-1 C) W        (paper: W is d_in x d_out, C = X^^T (X - X^))
// In this library's d_out x d_in storage, with H = 2 X^^T X^ and G = 2 X^^T X (so 2 C = G - H) and the factor
// U of onecomp_hessian_factor, U^T U = (H + lambda I)^-1 in sweep order:
//     W*_p = W_p + alpha ((W_p Cp^T) U^T) U,     Cp = (G - H)[perm][:, perm],  W_p = W[:, perm],
// and W* is W*_p with its columns put back into the original order.
//
// gfx950: three fp32 GEMMs on v_mfma_f32_32x32x2_f32 (fp32 products and sums: the correction is a difference of
// nearly equal Gram matrices times an inverse, bf16 operands would lose it).  128 x 128 tile per workgroup,
// 4 waves in 2 x 2 (64 x 64 each), operands staged through registers into double-buffered LDS, K step 16.
// The triangular structure of U halves the second and third product (k ranges cut per column tile).
#include "common.hpp"
#include "sgemm.hpp"

namespace onecomp {
namespace {

constexpr int ST = 128;    // tile side
constexpr int SK = 16;     // K per LDS stage
constexpr int SPA = SK + 1;      // pitch of a k-contiguous tile (rows x SK)
constexpr int SPB = ST + 4;      // pitch of a k-major tile (SK x cols)
constexpr int SSB = ST * SPA;    // >= SK * SPB

template <bool bt>
__global__ __launch_bounds__(256, 2) void sgemm_kernel(SgemmArgs g) {
    __shared__ float sA[2][ST * SPA];
    __shared__ float sB[2][SSB];
    const int tm = blockIdx.y, tn = blockIdx.x;
    const int m0 = tm * ST, n0 = tn * ST;
    int k_lo = 0, k_hi = g.k;
    if (g.flags & S_BUPPER_T) k_lo = n0;                       // B^T[n][k] = 0 for k < n
    if (g.flags & S_BUPPER) k_hi = min(g.k, n0 + ST);          // B[k][n] = 0 for k > n
    k_lo = (k_lo / SK) * SK;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1;
    // loaders: k-contiguous tile (rows x SK): row = tid / 2, 8 floats at k = (tid % 2) * 8
    //          k-major B tile (SK x cols): krow = tid / 16, 8 floats at col (tid % 16) * 8
    const int a_row = tid >> 1, a_k = (tid & 1) * 8;
    const int b_kr = tid >> 4, b_c = (tid & 15) * 8;
    float4v ra[2], rb[2];
    const float4v zero = {0.f, 0.f, 0.f, 0.f};
    auto gload = [&](int k0) __attribute__((always_inline)) {
        {
            const int r = m0 + a_row, kk = k0 + a_k;
            const bool ok = (r < g.m) && (kk < k_hi);
            const float4v* p = reinterpret_cast<const float4v*>(g.A + int64_t(r) * g.lda + kk);
            ra[0] = ok ? p[0] : zero;
            ra[1] = ok ? p[1] : zero;
        }
        if (bt) {
            const int r = n0 + a_row, kk = k0 + a_k;
            const bool ok = (r < g.n) && (kk < k_hi);
            const float4v* p = reinterpret_cast<const float4v*>(g.B + int64_t(r) * g.ldb + kk);
            rb[0] = ok ? p[0] : zero;
            rb[1] = ok ? p[1] : zero;
        } else {
            const int kk = k0 + b_kr, c = n0 + b_c;
            const bool ok = (kk < k_hi) && (c < g.n);
            const float4v* p = reinterpret_cast<const float4v*>(g.B + int64_t(kk) * g.ldb + c);
            rb[0] = ok ? p[0] : zero;
            rb[1] = ok ? p[1] : zero;
        }
    };
    auto lstore = [&](int st) __attribute__((always_inline)) {
#pragma unroll
        for (int e = 0; e < 8; ++e) sA[st][a_row * SPA + a_k + e] = ra[e / 4][e % 4];
        if (bt) {
#pragma unroll
            for (int e = 0; e < 8; ++e) sB[st][a_row * SPA + a_k + e] = rb[e / 4][e % 4];
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) sB[st][b_kr * SPB + b_c + e] = rb[e / 4][e % 4];
        }
    };

    float16v acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // MFMA operand layouts (lane l): A[i][k]: i = l % 32, k = l / 32;  B[k][j]: k = l / 32, j = l % 32
    const int l32 = lane & 31, lk = lane >> 5;
    if (k_lo < k_hi) {
        gload(k_lo);
        lstore(0);
    }
    __syncthreads();
    int st = 0;
    for (int k0 = k_lo; k0 < k_hi; k0 += SK) {
        const bool more = (k0 + SK < k_hi);
        if (more) gload(k0 + SK);
#pragma unroll
        for (int k2 = 0; k2 < SK; k2 += 2) {
            float a[2], b[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) a[i] = sA[st][(wr * 64 + i * 32 + l32) * SPA + k2 + lk];
#pragma unroll
            for (int j = 0; j < 2; ++j)
                b[j] = bt ? sB[st][(wc * 64 + j * 32 + l32) * SPA + k2 + lk]
                          : sB[st][(k2 + lk) * SPB + wc * 64 + j * 32 + l32];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        if (more) lstore(st ^ 1);
        __syncthreads();
        st ^= 1;
    }

    // accumulator register r of lane l: row (r/4)*8 + (l/32)*4 + r%4, column l%32 of its 32 x 32 tile
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wr * 64 + i * 32 + (r / 4) * 8 + lk * 4 + (r % 4);
                const int col = n0 + wc * 64 + j * 32 + l32;
                if (row >= g.m || col >= g.n) continue;
                if (g.C) {
                    g.C[int64_t(row) * g.ldc + col] = acc[i][j][r];
                } else {
                    const int oc = g.colmap ? g.colmap[col] : col;
                    g.out[int64_t(row) * g.ldout + oc] = g.base[int64_t(row) * g.ldbase + col] + g.alpha * acc[i][j][r];
                }
            }
}

}  // namespace

onecomp_status sgemm(const SgemmArgs& g, hipStream_t stream) {
    if (g.m <= 0 || g.n <= 0) return ONECOMP_OK;
    dim3 grid(unsigned(ceil_div(g.n, ST)), unsigned(ceil_div(g.m, ST)));
    if (g.flags & S_BTRANS) hipLaunchKernelGGL(sgemm_kernel<true>, grid, dim3(256), 0, stream, g);
    else hipLaunchKernelGGL(sgemm_kernel<false>, grid, dim3(256), 0, stream, g);
    ONECOMP_CHECK_LAUNCH();
    return ONECOMP_OK;
}

namespace {

// Cp[a][b] = G[p(a)][p(b)] - H[p(a)][p(b)]   (p = perm, or the identity)
__global__ __launch_bounds__(256) void cp_kernel(const float* __restrict__ G, const float* __restrict__ H, int n,
                                                const int32_t* __restrict__ perm, float* __restrict__ Cp) {
    const int a = blockIdx.y;
    const int b = blockIdx.x * 256 + threadIdx.x;
    if (b >= n) return;
    const int64_t src = int64_t(perm ? perm[a] : a) * n + (perm ? perm[b] : b);
    Cp[int64_t(a) * n + b] = G[src] - H[src];
}

// Wp[r][a] = float(W[r][p(a)])
template <typename T>
__global__ __launch_bounds__(256) void wp_kernel(const T* __restrict__ W, int64_t d_in, const int32_t* __restrict__ perm,
                                                float* __restrict__ Wp) {
    const int64_t r = blockIdx.y;
    const int a = blockIdx.x * 256 + threadIdx.x;
    if (a >= d_in) return;
    const int c = perm ? perm[a] : a;
    float v;
    if constexpr (sizeof(T) == 2) v = __uint_as_float(uint32_t(W[r * d_in + c]) << 16);
    else v = W[r * d_in + c];
    Wp[r * d_in + a] = v;
}

struct QepWs {
    float* Cp;   // [d_in x d_in]
    float* Wp;   // [d_out x d_in]
    float* M1;   // [d_out x d_in]
    float* M2;   // [d_out x d_in]
};

QepWs carve_qep(void* ws, int64_t d_out, int64_t d_in) {
    char* p = static_cast<char*>(ws);
    QepWs w;
    w.Cp = reinterpret_cast<float*>(p); p += align_up(size_t(d_in) * d_in * 4, 256);
    w.Wp = reinterpret_cast<float*>(p); p += align_up(size_t(d_out) * d_in * 4, 256);
    w.M1 = reinterpret_cast<float*>(p); p += align_up(size_t(d_out) * d_in * 4, 256);
    w.M2 = reinterpret_cast<float*>(p);
    return w;
}

}  // namespace

size_t qep_workspace_bytes(int64_t d_out, int64_t d_in) {
    return align_up(size_t(d_in) * d_in * 4, 256) + 3 * align_up(size_t(d_out) * d_in * 4, 256);
}

onecomp_status qep_target_run(const void* W, onecomp_dtype w_dtype, int64_t d_out, int64_t d_in, const float* G,
                              const float* H, const float* U, const int32_t* perm, float alpha, float* W_star,
                              void* workspace, hipStream_t stream) {
    QepWs w = carve_qep(workspace, d_out, d_in);
    const int n = int(d_in);
    hipLaunchKernelGGL(cp_kernel, dim3(unsigned(ceil_div(n, 256)), unsigned(n)), dim3(256), 0, stream, G, H, n, perm,
                       w.Cp);
    ONECOMP_CHECK_LAUNCH();
    dim3 wgrid(unsigned(ceil_div(n, 256)), unsigned(d_out));
    if (w_dtype == ONECOMP_BF16)
        hipLaunchKernelGGL(wp_kernel<uint16_t>, wgrid, dim3(256), 0, stream, static_cast<const uint16_t*>(W), d_in, perm,
                           w.Wp);
    else
        hipLaunchKernelGGL(wp_kernel<float>, wgrid, dim3(256), 0, stream, static_cast<const float*>(W), d_in, perm, w.Wp);
    ONECOMP_CHECK_LAUNCH();

    onecomp_status st;
    SgemmArgs g{};
    g.m = int(d_out); g.n = n; g.k = n;
    // M1 = Wp Cp^T
    g.A = w.Wp; g.lda = d_in; g.B = w.Cp; g.ldb = d_in; g.C = w.M1; g.ldc = d_in; g.flags = S_BTRANS;
    if ((st = sgemm(g, stream)) != ONECOMP_OK) return st;
    // M2 = M1 U^T
    g.A = w.M1; g.B = U; g.C = w.M2; g.flags = S_BTRANS | S_BUPPER_T;
    if ((st = sgemm(g, stream)) != ONECOMP_OK) return st;
    // W*[:, p(c)] = Wp[:, c] + alpha (M2 U)[:, c]
    g.A = w.M2; g.B = U; g.C = nullptr; g.flags = S_BUPPER;
    g.base = w.Wp; g.ldbase = d_in; g.colmap = perm; g.out = W_star; g.ldout = d_in; g.alpha = alpha;
    return sgemm(g, stream);
}

}  // namespace onecomp
