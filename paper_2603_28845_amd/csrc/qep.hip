// Corrected quantization target of error propagation (QEP, Sec. 4.3.1 of the paper, Eq. (qep)):
//     W* = (I + alpha (H^ + lambda I)^-1 C) W        (paper: W is d_in x d_out, C = X^^T (X - X^))
// In this library's d_out x d_in storage, with H = 2 X^^T X^ and G = 2 X^^T X (so 2 C = G - H) and the factor
// U of onecomp_hessian_factor, U^T U = (H + lambda I)^-1 in sweep order:
//     W*_p = W_p + alpha ((W_p Cp^T) U^T) U,     Cp = (G - H)[perm][:, perm],  W_p = W[:, perm],
// and W* is W*_p with its columns put back into the original order.
//
// gfx950: the three products run on the fp16 MFMAs with fp32 accuracy (operands split hi + lo, three products each,
// fp32 accumulation: split_update); see qep_target_run for the scaling that makes fp16's range suffice.
#include "common.hpp"

namespace onecomp {
namespace {

// Cp[a][b] = G[p(a)][p(b)] - H[p(a)][p(b)]   (p = perm, or the identity); max |Cp[a][b] rd[a] rd[b]| into
// sc->max_u_bits (the scale of the first product's right operand)
__global__ __launch_bounds__(256) void cp_kernel(const float* __restrict__ G, const float* __restrict__ H, int n,
                                                const int32_t* __restrict__ perm, const float* __restrict__ rd,
                                                float* __restrict__ Cp, Scalars* sc) {
    __shared__ uint32_t s_max;
    const int b = blockIdx.x * 256 + threadIdx.x;
    float mx = 0.f;
    if (b < n) {
        const int ob = perm ? perm[b] : b;
        const float rb = rd[b];
        for (int a = blockIdx.y; a < n; a += gridDim.y) {
            const int64_t src = int64_t(perm ? perm[a] : a) * n + ob;
            const float c = G[src] - H[src];
            Cp[int64_t(a) * n + b] = c;
            mx = fmaxf(mx, fabsf(c) * rd[a] * rb);
        }
    }
    block_max_bits(&sc->max_u_bits, mx, &s_max);
}

__global__ void qep_copy_max_kernel(const Scalars* from, Scalars* to) { to->max_u_bits = from->max_u_bits; }

__global__ void qep_scalars_init_kernel(Scalars* sc, int n) {
    for (int i = threadIdx.x; i < n; i += blockDim.x) {
        sc[i].max_w_bits = 0u; sc[i].max_u_bits = 0u;
        sc[i].f_d = 1.f; sc[i].f_u = 1.f; sc[i].f_all = 1.f; sc[i].f_inv = 1.f;
    }
}

// d[k] = sqrt(H[p(k)][p(k)]) (1 for a dead channel), rd = 1 / d
__global__ __launch_bounds__(256) void qep_diag_kernel(const float* __restrict__ H, int n, const int32_t* __restrict__ perm,
                                                       float* __restrict__ d, float* __restrict__ rd) {
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k >= n) return;
    const int o = perm ? perm[k] : k;
    const float x = H[int64_t(o) * n + o];
    const float v = x > 0.f ? sqrtf(x) : 1.f;
    d[k] = v;
    rd[k] = 1.0f / v;
}

// Wp[r][a] = float(W[r][p(a)]); max |Wp d| into sc->max_w_bits
template <typename T>
__global__ __launch_bounds__(256) void wp_kernel(const T* __restrict__ W, int64_t d_out, int64_t d_in,
                                                const int32_t* __restrict__ perm, const float* __restrict__ d,
                                                float* __restrict__ Wp, Scalars* sc) {
    __shared__ uint32_t s_max;
    const int a = blockIdx.x * 256 + threadIdx.x;
    float mx = 0.f;
    if (a < d_in) {
        const int c = perm ? perm[a] : a;
        const float da = d[a];
        for (int64_t r = blockIdx.y; r < d_out; r += gridDim.y) {   // few workgroups: one atomic each at the end
            float v;
            if constexpr (sizeof(T) == 2) v = __uint_as_float(uint32_t(W[r * d_in + c]) << 16);
            else v = W[r * d_in + c];
            Wp[r * d_in + a] = v;
            mx = fmaxf(mx, fabsf(v) * da);
        }
    }
    block_max_bits(&sc->max_w_bits, mx, &s_max);
}

// max |M| of a row-major matrix into sc->max_w_bits
__global__ __launch_bounds__(256) void qep_max_kernel(const float* __restrict__ M, int64_t n4, Scalars* sc) {
    __shared__ uint32_t s_max;
    float mx = 0.f;
    for (int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x; i < n4; i += int64_t(gridDim.x) * 256) {
        const float4v v = reinterpret_cast<const float4v*>(M)[i];
        mx = fmaxf(fmaxf(fmaxf(mx, fabsf(v[0])), fmaxf(fabsf(v[1]), fabsf(v[2]))), fabsf(v[3]));
    }
    block_max_bits(&sc->max_w_bits, mx, &s_max);
}

// Right operand of a split product, B[k][n] (n contiguous, n_rows rows of which those behind n - 1 are zero), from a
// square fp32 matrix S:  TRANS: B[k][n] = S[n][k] rs[k] cs[n],  else B[k][n] = S[k][n] rs[k] cs[n]  (rs / cs == nullptr:
// 1);  upper: entries of S below its diagonal count as zero.  WRITE = false collects max |B| into sc->max_u_bits;
// WRITE = true stores B f_u as fp16 hi + lo with f_u = 2^(14 - exponent of that maximum), which thread 0 of the grid
// leaves in sc->f_u.  64 x 64 tiles, transposed through LDS where needed, so that reads and writes are coalesced.
template <bool WRITE, bool TRANS>
__global__ __launch_bounds__(256) void qep_right_kernel(const float* __restrict__ S, int n, int n_rows, int upper,
                                                        const float* __restrict__ rs, const float* __restrict__ cs,
                                                        Scalars* sc, uint16_t* __restrict__ Bh, uint16_t* __restrict__ Bl) {
    __shared__ float tile[64][65];
    __shared__ uint32_t s_max;
    const int k0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    float f_u = 1.f;
    if (WRITE) {
        const float mx = __uint_as_float(sc->max_u_bits);
        int e = 0;
        if (mx > 0.f) (void)frexpf(mx, &e);
        f_u = ldexpf(1.f, max(-60, min(60, 14 - e)));
        if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) sc->f_u = f_u;
    }
    // tile[kk][nn] = B[k0 + kk][n0 + nn]
    for (int i = ty; i < 64; i += 4) {
        if (TRANS) {   // read S[n0 + i][k0 + tx]
            const int sr = n0 + i, scn = k0 + tx;
            float v = 0.f;
            if (sr < n && scn < n && !(upper && scn < sr)) v = S[int64_t(sr) * n + scn] * (rs ? rs[scn] : 1.f) * (cs ? cs[sr] : 1.f);
            tile[tx][i] = v;
        } else {       // read S[k0 + i][n0 + tx]
            const int sr = k0 + i, scn = n0 + tx;
            float v = 0.f;
            if (sr < n && scn < n && !(upper && scn < sr)) v = S[int64_t(sr) * n + scn] * (rs ? rs[sr] : 1.f) * (cs ? cs[scn] : 1.f);
            tile[i][tx] = v;
        }
    }
    __syncthreads();
    float mx = 0.f;
    for (int kk = ty; kk < 64; kk += 4) {
        const int k = k0 + kk, c = n0 + tx;
        if (k >= n_rows || c >= n) continue;
        const float v = tile[kk][tx];
        if (WRITE) {
            const float x = fminf(fmaxf(v * f_u, -60000.f), 60000.f);
            const _Float16 h = (_Float16)x;
            const _Float16 lo = (_Float16)(x - (float)h);
            Bh[int64_t(k) * n + c] = __builtin_bit_cast(uint16_t, h);
            Bl[int64_t(k) * n + c] = __builtin_bit_cast(uint16_t, lo);
        } else {
            mx = fmaxf(mx, fabsf(v));
        }
    }
    if (!WRITE) block_max_bits(&sc->max_u_bits, mx, &s_max);
}

// W*[r][p(c)] = Wp[r][c] + alpha M[r][c] rd[c]
__global__ __launch_bounds__(256) void qep_final_kernel(const float* __restrict__ Wp, const float* __restrict__ M,
                                                        const float* __restrict__ rd, const int32_t* __restrict__ perm,
                                                        int64_t d_in, float alpha, float* __restrict__ W_star) {
    const int64_t r = blockIdx.y;
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= d_in) return;
    const int oc = perm ? perm[c] : c;
    W_star[r * d_in + oc] = Wp[r * d_in + c] + alpha * M[r * d_in + c] * rd[c];
}

struct QepWs {
    float* Cp;   // [d_in x d_in]
    float* Wp;   // [d_out x d_in]
    float* M1;   // [d_out x d_in]
    float* M2;   // [d_out x d_in]
    uint16_t *Bh, *Bl;   // [(d_in + 32) x d_in]: right operand of the current product
    uint16_t *Dh, *Dl;   // [pad32(d_in) x ldD]: left operand of the current product
    float *d, *rd;       // [d_in]
    Scalars* sc;         // one per product
};

inline int64_t pad32(int64_t k) { return (k + 31) / 32 * 32; }

QepWs carve_qep(void* ws, int64_t d_out, int64_t d_in) {
    char* p = static_cast<char*>(ws);
    const int64_t ldD = split_update_ld(d_out);
    QepWs w;
    w.Cp = reinterpret_cast<float*>(p); p += align_up(size_t(d_in) * d_in * 4, 256);
    w.Wp = reinterpret_cast<float*>(p); p += align_up(size_t(d_out) * d_in * 4, 256);
    w.M1 = reinterpret_cast<float*>(p); p += align_up(size_t(d_out) * d_in * 4, 256);
    w.M2 = reinterpret_cast<float*>(p); p += align_up(size_t(d_out) * d_in * 4, 256);
    w.Bh = reinterpret_cast<uint16_t*>(p); p += align_up(size_t(d_in + 32) * d_in * 2, 256);
    w.Bl = reinterpret_cast<uint16_t*>(p); p += align_up(size_t(d_in + 32) * d_in * 2, 256);
    w.Dh = reinterpret_cast<uint16_t*>(p); p += align_up(size_t(pad32(d_in)) * ldD * 2, 256);
    w.Dl = reinterpret_cast<uint16_t*>(p); p += align_up(size_t(pad32(d_in)) * ldD * 2, 256);
    w.d = reinterpret_cast<float*>(p); p += align_up(size_t(d_in) * 4, 256);
    w.rd = reinterpret_cast<float*>(p); p += align_up(size_t(d_in) * 4, 256);
    w.sc = reinterpret_cast<Scalars*>(p);
    return w;
}

}  // namespace

size_t qep_workspace_bytes(int64_t d_out, int64_t d_in) {
    const int64_t ldD = split_update_ld(d_out);
    return align_up(size_t(d_in) * d_in * 4, 256) + 3 * align_up(size_t(d_out) * d_in * 4, 256) +
           2 * align_up(size_t(d_in + 32) * d_in * 2, 256) + 2 * align_up(size_t(pad32(d_in)) * ldD * 2, 256) +
           2 * align_up(size_t(d_in) * 4, 256) + 256;
}

// The correction alpha Wp Cp^T U^T U as three products on the fp16 MFMAs with fp32 accuracy (split_update: operands
// hi + lo, three products each).  fp16 leaves no range to spare, so every factor is used in the scaling of the
// correlation matrix: with D = diag(sqrt(H_jj)) in sweep order, Cp = D C~ D and U = U~ D^-1, hence
//     Wp Cp^T U^T U = (Wp D) C~^T U~^T U~ D^-1,
// each right operand (C~^T, U~^T, U~) scaled by a power of two from its own maximum, each left operand (Wp D, then
// the two intermediate products) likewise; D^-1 goes into the last step together with alpha and the column order.
// U is upper triangular: the second product needs k >= n, the third k <= n, taken in column chunks of 1024.
onecomp_status qep_target_run(const void* W, onecomp_dtype w_dtype, int64_t d_out, int64_t d_in, const float* G,
                              const float* H, const float* U, const int32_t* perm, float alpha, float* W_star,
                              void* workspace, hipStream_t stream) {
    QepWs w = carve_qep(workspace, d_out, d_in);
    const int n = int(d_in);
    const int64_t ldD = split_update_ld(d_out);
    const int kp = int(pad32(d_in));
    onecomp_status st;
    hipLaunchKernelGGL(qep_scalars_init_kernel, dim3(1), dim3(64), 0, stream, w.sc, 3);
    ONECOMP_CHECK_LAUNCH();
    hipLaunchKernelGGL(qep_diag_kernel, dim3(unsigned(ceil_div(n, 256))), dim3(256), 0, stream, H, n, perm, w.d, w.rd);
    ONECOMP_CHECK_LAUNCH();
    hipLaunchKernelGGL(cp_kernel, dim3(unsigned(ceil_div(n, 256)), unsigned(n < 128 ? n : 128)), dim3(256), 0, stream, G,
                       H, n, perm, w.rd, w.Cp, w.sc);
    ONECOMP_CHECK_LAUNCH();
    dim3 wgrid(unsigned(ceil_div(n, 256)), unsigned(d_out));
    dim3 pgrid(unsigned(ceil_div(n, 256)), unsigned(d_out < 64 ? d_out : 64));
    if (w_dtype == ONECOMP_BF16)
        hipLaunchKernelGGL(wp_kernel<uint16_t>, pgrid, dim3(256), 0, stream, static_cast<const uint16_t*>(W), d_out, d_in,
                           perm, w.d, w.Wp, w.sc);
    else
        hipLaunchKernelGGL(wp_kernel<float>, pgrid, dim3(256), 0, stream, static_cast<const float*>(W), d_out, d_in, perm,
                           w.d, w.Wp, w.sc);
    ONECOMP_CHECK_LAUNCH();

    const dim3 bgrid(unsigned(ceil_div(n, 64)), unsigned(ceil_div(n + 32, 64)));
    const dim3 fgrid{2048};
    // right operand of product i from S (products 0 and 1: transposed; product 2: as stored; the maximum that sets
    // its scale comes from cp_kernel, from a pass of its own, from product 1), then the left operand from `left` (its
    // maximum is in sc[i])
    auto operands = [&](int i, const float* S, int upper, const float* rs, const float* cs, const float* left,
                        const float* dl) -> onecomp_status {
        Scalars* sc = w.sc + i;
        if (i == 2) {   // the entries of U~ are those of U~^T: the maximum of product 1 serves
            hipLaunchKernelGGL(qep_copy_max_kernel, dim3(1), dim3(1), 0, stream, w.sc + 1, sc);
            ONECOMP_CHECK_LAUNCH();
            hipLaunchKernelGGL((qep_right_kernel<true, false>), bgrid, dim3(256), 0, stream, S, n, n + 32, upper, rs, cs, sc,
                               w.Bh, w.Bl);
        } else if (i == 0) {   // cp_kernel has left the maximum of C~ in sc[0]
            hipLaunchKernelGGL((qep_right_kernel<true, true>), bgrid, dim3(256), 0, stream, S, n, n + 32, upper, rs, cs, sc,
                               w.Bh, w.Bl);
        } else {
            hipLaunchKernelGGL((qep_right_kernel<false, true>), bgrid, dim3(256), 0, stream, S, n, n + 32, upper, rs, cs, sc,
                               w.Bh, w.Bl);
            ONECOMP_CHECK_LAUNCH();
            hipLaunchKernelGGL((qep_right_kernel<true, true>), bgrid, dim3(256), 0, stream, S, n, n + 32, upper, rs, cs, sc,
                               w.Bh, w.Bl);
        }
        ONECOMP_CHECK_LAUNCH();
        return split_left_operand(left, d_in, d_out, n, dl, sc, nullptr, w.Dh, w.Dl, stream);
    };
    auto matmax = [&](const float* M, Scalars* sc) -> onecomp_status {
        hipLaunchKernelGGL(qep_max_kernel, fgrid, dim3(256), 0, stream, M, d_out * d_in / 4, sc);
        ONECOMP_CHECK_LAUNCH();
        return ONECOMP_OK;
    };
    auto zero = [&](float* M) -> onecomp_status { return fill_zero(M, d_out * d_in / 4, stream); };
    // M1 = (Wp D) C~^T:  B[k][n] = Cp[n][k] / (d_n d_k)
    if ((st = operands(0, w.Cp, 0, w.rd, w.rd, w.Wp, w.d)) != ONECOMP_OK) return st;
    if ((st = zero(w.M1)) != ONECOMP_OK) return st;
    if ((st = split_update(w.M1, d_out, d_in, w.Dh, w.Dl, ldD, w.Bh, w.Bl, w.sc, 0, kp, 0, 0, n, stream)) != ONECOMP_OK)
        return st;
    // M2 = M1 U~^T:  B[k][n] = U[n][k] d_k, zero for k < n
    if ((st = matmax(w.M1, w.sc + 1)) != ONECOMP_OK) return st;
    if ((st = operands(1, U, 1, w.d, nullptr, w.M1, nullptr)) != ONECOMP_OK) return st;
    if ((st = zero(w.M2)) != ONECOMP_OK) return st;
    constexpr int CH = 1024;
    for (int c0 = 0; c0 < n; c0 += CH) {
        const int c1 = c0 + CH < n ? c0 + CH : n;
        const int k0 = c0 / 32 * 32;
        if ((st = split_update(w.M2, d_out, d_in, w.Dh, w.Dl, ldD, w.Bh, w.Bl, w.sc + 1, k0, kp - k0, k0, c0, c1,
                               stream)) != ONECOMP_OK)
            return st;
    }
    // M3 = M2 U~ (into M1's place):  B[k][n] = U[k][n] d_n, zero for k > n
    if ((st = matmax(w.M2, w.sc + 2)) != ONECOMP_OK) return st;
    if ((st = operands(2, U, 1, nullptr, w.d, w.M2, nullptr)) != ONECOMP_OK) return st;
    if ((st = zero(w.M1)) != ONECOMP_OK) return st;
    for (int c0 = 0; c0 < n; c0 += CH) {
        const int c1 = c0 + CH < n ? c0 + CH : n;
        if ((st = split_update(w.M1, d_out, d_in, w.Dh, w.Dl, ldD, w.Bh, w.Bl, w.sc + 2, 0, int(pad32(c1)), 0, c0, c1,
                               stream)) != ONECOMP_OK)
            return st;
    }
    hipLaunchKernelGGL(qep_final_kernel, wgrid, dim3(256), 0, stream, w.Wp, w.M1, w.rd, perm, d_in, alpha, W_star);
    ONECOMP_CHECK_LAUNCH();
    return ONECOMP_OK;
}

}  // namespace onecomp
