// JointQ (Sec. 4.2.2 of the paper, Eq. (jointq)): local search over the integer codes of a solution in the per-group
// format of Eq. (4), the scale of the touched group refit in the same move.  Per output row the objective is
// f = r A r^T with r = w - w^ and A = H + lam I (Eq. (jointq_reg): the regularizer is an augmented input).
//
// Reading of what the paper leaves open (moves, order, stopping): a move changes one code by +-1 inside the codebook;
// zero-points stay; groups are visited in order, n_pass times; inside a visit the group's columns are scanned in
// order, +1 is tried before -1 and the first improving one is taken at once (at most one per column and scan); a visit
// ends with the first scan that takes nothing or after max_scans scans; on entering a visit the scale is refit to the
// current codes; a group whose codes all equal the zero-point is left alone.
//
// One visit of group t for one row (u = q - z, a = A_tt u, p = (A r)_t + s_old a, b = u.p, c = u.a, s* = b / c):
// the move u + d e_j changes b^2 / c by N / c' with
//     g = p_j - s* a_j,   N = 2 d b g + g^2 + 2 s* g a_j - s*^2 (c A_jj - a_j^2),   c' = c + 2 d a_j + A_jj,
// and is taken iff N > 0 and c' > 0.
//
// gfx950 mapping.  The rows are independent and a visit only needs the row's gradient restricted to the group,
// (A r)_t, so the whole layer moves through the groups together:
//   * Gm = R A (d_out x d_in, fp32) is built once (fp32 MFMA GEMM) and kept current;
//   * visit kernel: one wave per row, the group's columns spread over the lanes (two per lane at G = 128), A_tt in
//     LDS (shared by the 16 rows of a workgroup); the lanes evaluate their columns' moves together, a ballot picks
//     the first improving one in scan order, a taken move updates a with one LDS row;
//   * the change of the residual, dR = r_new - r_old on the group's columns, is fed back as Gm += dR A[t, :] (fp32
//     MFMA GEMM, 2 d_out d_in^2 flops per pass: where the time goes).  Only the columns of the groups visited next
//     need it at once: groups are bundled into super-blocks of up to 512 columns; after a visit the update goes to
//     the super-block's own columns (k = G, n <= 512), and once the super-block is done all other columns receive
//     its groups' updates in one product with k <= 512, so Gm is read and written d_in / 512 times per pass
//     instead of d_in / G times.
#include "common.hpp"
#include "sgemm.hpp"

namespace onecomp {
namespace {

constexpr int JQ_SBW = 512;   // columns of a super-block (at most)
constexpr int JQ_ROWS = 16;   // rows (waves) per workgroup of the visit kernel

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}

__device__ __forceinline__ float readlane_f(float x, int l) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), l));
}

__device__ __forceinline__ float load_w(const void* W, int bf16, int64_t i) {
    if (bf16) return __uint_as_float(uint32_t(static_cast<const uint16_t*>(W)[i]) << 16);
    return static_cast<const float*>(W)[i];
}

// R = W - s (q - z) over the whole layer
__global__ __launch_bounds__(256) void jq_residual_kernel(const void* __restrict__ W, int bf16, int d_out, int d_in,
                                                          const uint8_t* __restrict__ Q, const float* __restrict__ scales,
                                                          const float* __restrict__ zeros, int G, int n_g,
                                                          float* __restrict__ R) {
    for (int64_t r = blockIdx.x; r < d_out; r += gridDim.x)
        for (int c = threadIdx.x; c < d_in; c += 256) {
            const int64_t i = r * d_in + c;
            const int g = c / G;
            R[i] = load_w(W, bf16, i) - scales[r * n_g + g] * (float(Q[i]) - zeros[r * n_g + g]);
        }
}

// rowf[r] = sum_j r_j (Gm_rj + lam r_j) with r recomputed from the codes; optional W^ output
__global__ __launch_bounds__(256) void jq_objective_kernel(const void* __restrict__ W, int bf16, int d_out, int d_in,
                                                           const uint8_t* __restrict__ Q, const float* __restrict__ scales,
                                                           const float* __restrict__ zeros, int G, int n_g,
                                                           const float* __restrict__ Gm, float lam,
                                                           float* __restrict__ rowf, float* __restrict__ W_hat) {
    __shared__ float red[256];
    for (int64_t r = blockIdx.x; r < d_out; r += gridDim.x) {
        float acc = 0.f;
        for (int c = threadIdx.x; c < d_in; c += 256) {
            const int64_t i = r * d_in + c;
            const int g = c / G;
            const float wh = scales[r * n_g + g] * (float(Q[i]) - zeros[r * n_g + g]);
            const float rr = load_w(W, bf16, i) - wh;
            acc += rr * (Gm[i] + lam * rr);
            if (W_hat) W_hat[i] = wh;
        }
        red[threadIdx.x] = acc;
        __syncthreads();
        for (int w = 128; w > 0; w >>= 1) {
            if (int(threadIdx.x) < w) red[threadIdx.x] += red[threadIdx.x + w];
            __syncthreads();
        }
        if (threadIdx.x == 0) rowf[r] = red[0];
        __syncthreads();
    }
}

// out[0] = sum of rowf in a fixed order (one workgroup)
__global__ __launch_bounds__(1024) void jq_total_kernel(const float* __restrict__ rowf, int n, float* __restrict__ out) {
    __shared__ float red[1024];
    float acc = 0.f;
    for (int i = threadIdx.x; i < n; i += 1024) acc += rowf[i];
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int w = 512; w > 0; w >>= 1) {
        if (int(threadIdx.x) < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[0] = red[0];
}

__global__ void jq_zero_kernel(int32_t* p) { p[0] = 0; }

struct VisitArgs {
    const void* W; int w_bf16;
    int d_out, d_in, G, n_g, t;
    const float* A; float lam;
    float qtop;
    uint8_t* Q; float* scales; const float* zeros;
    const float* Gm;
    float* dR; int ldr;        // the group's dR: row r at dR + r * ldr
    int max_scans;
    int32_t* moves;
};

// NC = columns per lane (1: G <= 64, 2: G <= 128).  The scan "columns in order, first improving move wins" is run as:
// every lane evaluates the gain of its own columns under the current state, a ballot finds the first improving
// column behind the last one taken, that move is applied, and the evaluation is repeated.  The columns between two
// taken moves are rejected under the same state the sequential scan would see, so the sequence of moves is the same,
// at one wave-wide evaluation per taken move instead of one per column.
template <int NC>
__global__ __launch_bounds__(64 * JQ_ROWS) void jq_visit_kernel(VisitArgs v) {
    extern __shared__ float sA[];   // G x G: A_tt + lam I
    const int G = v.G;
    const int c0 = v.t * G;
    for (int e = threadIdx.x * 4; e < G * G; e += 64 * JQ_ROWS * 4) {
        const int k = e / G, c = e - k * G;
        float4v x = *reinterpret_cast<const float4v*>(v.A + int64_t(c0 + k) * v.d_in + c0 + c);
        if (k >= c && k < c + 4) x[k - c] += v.lam;
        *reinterpret_cast<float4v*>(sA + e) = x;
    }
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * JQ_ROWS + (threadIdx.x >> 6);
    if (row >= v.d_out) return;

    const float z = v.zeros[int64_t(row) * v.n_g + v.t];
    const float s_old = v.scales[int64_t(row) * v.n_g + v.t];
    float u[NC], u0[NC], a[NC], p[NC], q[NC], ad[NC];
    bool has[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const int col = lane + 64 * c;
        has[c] = col < G;
        const int64_t i = int64_t(row) * v.d_in + c0 + (has[c] ? col : 0);
        q[c] = has[c] ? float(v.Q[i]) : z;
        u[c] = q[c] - z;
        u0[c] = u[c];
        a[c] = 0.f;
        ad[c] = has[c] ? sA[col * G + col] : 1.f;
        // (A r)_t + lam r_t + s_old (A_tt + lam I) u  =  Gm + lam w + s_old A_tt u; the lam u part comes with a below
        p[c] = has[c] ? v.Gm[i] + v.lam * (load_w(v.W, v.w_bf16, i) - s_old * u[c]) : 0.f;
    }
    // a = (A_tt + lam I) u
#pragma unroll
    for (int cu = 0; cu < NC; ++cu) {
        const int kn = G - 64 * cu < 64 ? G - 64 * cu : 64;
        for (int k = 0; k < kn; ++k) {
            const float uk = readlane_f(u[cu], k);
            const float* rowk = sA + (64 * cu + k) * G + lane;
#pragma unroll
            for (int c = 0; c < NC; ++c)
                if (has[c]) a[c] += rowk[64 * c] * uk;
        }
    }
    float b = 0.f, cc = 0.f;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        p[c] += s_old * a[c];
        b += u[c] * p[c];
        cc += u[c] * a[c];
    }
    b = wave_sum(b);
    cc = wave_sum(cc);
    const bool live = cc > 0.f;
    int n_moves = 0;
    if (live) {
        float ss = b / cc;
        int scan = 0, j0 = -1;   // j0: the column of the last move taken in this scan
        bool took = false;
        for (;;) {
            bool imp[NC];
            float dd[NC];
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const float gs = p[c] - ss * a[c];
                const float base = gs * gs + 2.0f * ss * gs * a[c] - ss * ss * (cc * ad[c] - a[c] * a[c]);
                const float t1 = 2.0f * b * gs;
                const bool up = q[c] + 1.0f <= v.qtop && base + t1 > 0.f && cc + 2.0f * a[c] + ad[c] > 0.f;
                const bool dn = q[c] - 1.0f >= 0.f && base - t1 > 0.f && cc - 2.0f * a[c] + ad[c] > 0.f;
                imp[c] = has[c] && (up || dn);
                dd[c] = up ? 1.0f : -1.0f;
            }
            int j = -1;
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                if (j >= 0) continue;
                uint64_t m = __ballot(imp[c]);
                const int lo = j0 - 64 * c;          // columns up to lo (local numbering) are behind
                if (lo >= 63) m = 0;
                else if (lo >= 0) m &= ~((uint64_t(2) << lo) - 1);
                if (m) j = 64 * c + __builtin_ctzll(m);
            }
            if (j < 0) {   // the scan is over
                if (!took || ++scan >= v.max_scans) break;
                took = false;
                j0 = -1;
                continue;
            }
            float d, pj, aj, adj;
            if (NC == 1 || j < 64) {
                d = readlane_f(dd[0], j); pj = readlane_f(p[0], j); aj = readlane_f(a[0], j); adj = readlane_f(ad[0], j);
                if (lane == j) { u[0] += d; q[0] += d; }
            } else {
                d = readlane_f(dd[NC - 1], j - 64); pj = readlane_f(p[NC - 1], j - 64);
                aj = readlane_f(a[NC - 1], j - 64); adj = readlane_f(ad[NC - 1], j - 64);
                if (lane == j - 64) { u[NC - 1] += d; q[NC - 1] += d; }
            }
            b += d * pj;
            cc += 2.0f * d * aj + adj;
            ss = b / cc;
            const float* rowj = sA + j * G + lane;
#pragma unroll
            for (int c = 0; c < NC; ++c)
                if (has[c]) a[c] += d * rowj[64 * c];
            took = true;
            j0 = j;
            ++n_moves;
        }
    }
    const float s_new = live ? b / cc : s_old;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        if (!has[c]) continue;
        const int col = lane + 64 * c;
        const int64_t i = int64_t(row) * v.d_in + c0 + col;
        v.Q[i] = uint8_t(q[c]);
        v.dR[int64_t(row) * v.ldr + col] = s_old * u0[c] - s_new * u[c];   // change of the residual w - w^
    }
    if (lane == 0) {
        v.scales[int64_t(row) * v.n_g + v.t] = s_new;
        if (n_moves > 0) atomicAdd(v.moves, n_moves);
    }
}

struct JqWs {
    float* R;      // d_out x d_in: residual at the start (operand of the first GEMM)
    float* Gm;     // d_out x d_in: R A, kept current
    float* dR;     // d_out x JQ_SBW: dR of the groups of the current super-block side by side
    float* rowf;   // d_out
};

JqWs carve(void* ws, int64_t d_out, int64_t d_in, int G) {
    char* p = static_cast<char*>(ws);
    JqWs w;
    w.R = reinterpret_cast<float*>(p); p += align_up(size_t(d_out) * d_in * 4, 256);
    w.Gm = reinterpret_cast<float*>(p); p += align_up(size_t(d_out) * d_in * 4, 256);
    w.dR = reinterpret_cast<float*>(p); p += align_up(size_t(d_out) * JQ_SBW * 4, 256);
    w.rowf = reinterpret_cast<float*>(p);
    return w;
}

}  // namespace

size_t jointq_workspace_bytes(int64_t d_out, int64_t d_in, int group_size) {
    (void)group_size;
    return 2 * align_up(size_t(d_out) * d_in * 4, 256) + align_up(size_t(d_out) * JQ_SBW * 4, 256) +
           align_up(size_t(d_out) * 4, 256);
}

onecomp_status jointq_run(const void* W, onecomp_dtype w_dtype, int64_t d_out, int64_t d_in, const float* A, float lam,
                          int bits, int group_size, int grid, int n_pass, int max_scans, uint8_t* Q, float* scales,
                          const float* zeros, float* W_hat, float* objective, int32_t* n_moves, void* workspace,
                          hipStream_t stream) {
    const int G = group_size;
    const int n_g = int(d_in / G);
    const bool symmetric = grid == ONECOMP_GRID_SYMMETRIC || grid == ONECOMP_GRID_SYMMETRIC_MSE;
    const float qtop = symmetric ? float(2 * ((1 << (bits - 1)) - 1)) : float((1 << bits) - 1);
    const int bf16 = w_dtype == ONECOMP_BF16;
    JqWs w = carve(workspace, d_out, d_in, G);
    const dim3 rgrid{unsigned(d_out < 4096 ? d_out : 4096)};

    hipLaunchKernelGGL(jq_zero_kernel, dim3(1), dim3(1), 0, stream, n_moves);
    ONECOMP_CHECK_LAUNCH();
    hipLaunchKernelGGL(jq_residual_kernel, rgrid, dim3(256), 0, stream, W, bf16, int(d_out), int(d_in), Q, scales, zeros,
                       G, n_g, w.R);
    ONECOMP_CHECK_LAUNCH();
    SgemmArgs g{};
    g.A = w.R; g.lda = d_in; g.B = A; g.ldb = d_in; g.C = w.Gm; g.ldc = d_in;
    g.m = int(d_out); g.n = int(d_in); g.k = int(d_in); g.flags = 0;
    onecomp_status st = sgemm(g, stream);
    if (st != ONECOMP_OK) return st;
    hipLaunchKernelGGL(jq_objective_kernel, rgrid, dim3(256), 0, stream, W, bf16, int(d_out), int(d_in), Q, scales, zeros,
                       G, n_g, w.Gm, lam, w.rowf, static_cast<float*>(nullptr));
    ONECOMP_CHECK_LAUNCH();
    hipLaunchKernelGGL(jq_total_kernel, dim3(1), dim3(1024), 0, stream, w.rowf, int(d_out), objective);
    ONECOMP_CHECK_LAUNCH();

    static std::atomic<uint64_t> lds1{0}, lds2{0};
    const int lds_bytes = G * G * 4;
    if (G <= 64) {
        if (allow_dynamic_lds(reinterpret_cast<const void*>(&jq_visit_kernel<1>), 64 * 64 * 4, lds1) != ONECOMP_OK)
            return ONECOMP_ERR_HIP;
    } else {
        if (allow_dynamic_lds(reinterpret_cast<const void*>(&jq_visit_kernel<2>), 128 * 128 * 4, lds2) != ONECOMP_OK)
            return ONECOMP_ERR_HIP;
    }
    VisitArgs v;
    v.W = W; v.w_bf16 = bf16; v.d_out = int(d_out); v.d_in = int(d_in); v.G = G; v.n_g = n_g; v.t = 0;
    v.A = A; v.lam = lam; v.qtop = qtop; v.Q = Q; v.scales = scales; v.zeros = zeros; v.Gm = w.Gm; v.dR = w.dR;
    v.max_scans = max_scans; v.moves = n_moves;
    const dim3 vgrid{unsigned(ceil_div(d_out, JQ_ROWS))};
    const int sbg = JQ_SBW / G > 0 ? JQ_SBW / G : 1;   // groups per super-block
    v.ldr = sbg * G;
    SgemmArgs up{};
    up.lda = v.ldr; up.ldb = d_in; up.C = nullptr; up.ldc = 0;
    up.m = int(d_out); up.flags = 0;
    up.ldbase = d_in; up.colmap = nullptr; up.ldout = d_in; up.alpha = 1.0f;
    // Gm[:, c_lo .. c_hi) += dR[:, k_lo .. k_hi) A[t0 G + k_lo .. t0 G + k_hi, c_lo .. c_hi)
    auto update = [&](int t0, int k_lo, int k_hi, int c_lo, int c_hi) -> onecomp_status {
        if (c_hi <= c_lo || k_hi <= k_lo) return ONECOMP_OK;
        up.A = w.dR + k_lo; up.k = k_hi - k_lo;
        up.B = A + (int64_t(t0) * G + k_lo) * d_in + c_lo;
        up.n = c_hi - c_lo;
        up.base = w.Gm + c_lo; up.out = w.Gm + c_lo;
        return sgemm(up, stream);
    };
    for (int ps = 0; ps < n_pass; ++ps)
        for (int t0 = 0; t0 < n_g; t0 += sbg) {
            const int t1 = t0 + sbg < n_g ? t0 + sbg : n_g;
            for (int t = t0; t < t1; ++t) {
                v.t = t;
                v.dR = w.dR + (t - t0) * G;
                if (G <= 64) hipLaunchKernelGGL(jq_visit_kernel<1>, vgrid, dim3(64 * JQ_ROWS), lds_bytes, stream, v);
                else hipLaunchKernelGGL(jq_visit_kernel<2>, vgrid, dim3(64 * JQ_ROWS), lds_bytes, stream, v);
                ONECOMP_CHECK_LAUNCH();
                if ((st = update(t0, (t - t0) * G, (t - t0 + 1) * G, t0 * G, t1 * G)) != ONECOMP_OK) return st;
            }
            if ((st = update(t0, 0, (t1 - t0) * G, 0, t0 * G)) != ONECOMP_OK) return st;
            if ((st = update(t0, 0, (t1 - t0) * G, t1 * G, int(d_in))) != ONECOMP_OK) return st;
        }
    hipLaunchKernelGGL(jq_objective_kernel, rgrid, dim3(256), 0, stream, W, bf16, int(d_out), int(d_in), Q, scales, zeros,
                       G, n_g, w.Gm, lam, w.rowf, W_hat);
    ONECOMP_CHECK_LAUNCH();
    hipLaunchKernelGGL(jq_total_kernel, dim3(1), dim3(1024), 0, stream, w.rowf, int(d_out), objective + 1);
    ONECOMP_CHECK_LAUNCH();
    return ONECOMP_OK;
}

}  // namespace onecomp
