// JointQ (Sec. 4.3.2 of the paper, Eq. (jointq)): local search over the integer codes of a solution in the per-group
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
// and is taken iff N > 0 and c' > 0; a move that would leave every code of the group at its zero-point (c' = 0, the
// scale undefined) is no candidate, which the kernel decides on the codes.  (The last three terms of N equal
// p_j^2 - s*^2 c A_jj, which is how the kernel forms them; what matters for fp32 is that the small g is computed
// first and multiplied by the large b.)
//
// gfx950 mapping.  The rows are independent and a visit only needs the row's gradient restricted to the group,
// (A r)_t, so the whole layer moves through the groups together:
//   * the gradient Gm = R A (d_out x d_in, fp32) is built once and kept current, stored column-normalized,
//     Gm~_j = Gm_j / d_j with d_j = sqrt(A_jj);
//   * visit kernel: one wave per row, the group's columns spread over the lanes (two per lane at G = 128), A_tt in
//     LDS (shared by the 16 rows of a workgroup); the lanes evaluate their columns' moves together, a ballot picks
//     the first improving one in scan order, a taken move updates a with one LDS row;
//   * the change of the residual, dR = r_new - r_old on the group's columns, is fed back as Gm += dR A[t, :]
//     (2 d_out d_in^2 flops per pass: where the time goes).  Only the columns of the groups visited next need it at
//     once: groups are bundled into super-blocks of up to 512 columns; after a visit the update goes to the
//     super-block's own columns (k = G), and once the super-block is done all other columns receive its groups'
//     updates in one product with k <= 512, so Gm is read and written d_in / 512 times per pass.
//   * the products run on the fp16 MFMAs with fp32 accuracy, the split_update of the sweep (operands hi + lo, three
//     products).  fp16 has no range to spare, and A's diagonal spans decades on activations with outlier channels,
//     so A is used as the correlation matrix A~_kj = A_kj / (d_k d_j) (entries within [-1, 1], scaled by 2^14) and
//     the left operands as (R d) resp. (dR d) scaled by a power of two taken from their own maximum on the device:
//     Gm~ += (dR d) A~.  Each operand keeps 22 significant bits relative to itself.
#include "common.hpp"

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

// original column of sweep position c (perm == nullptr: natural order)
__device__ __forceinline__ int pcol(const int32_t* perm, int c) { return perm ? perm[c] : c; }

__device__ __forceinline__ float load_w(const void* W, int bf16, int64_t i) {
    if (bf16) return __uint_as_float(uint32_t(static_cast<const uint16_t*>(W)[i]) << 16);
    return static_cast<const float*>(W)[i];
}

constexpr float JQ_FU = 16384.f;   // scale of A~ (|A~| <= 1) in fp16

__global__ void jq_scalars_init_kernel(Scalars* sc, int n) {
    for (int i = threadIdx.x; i < n; i += blockDim.x) {
        sc[i].max_w_bits = 0u; sc[i].max_u_bits = 0u;
        sc[i].f_d = 1.f; sc[i].f_u = JQ_FU; sc[i].f_all = JQ_FU; sc[i].f_inv = 1.f / JQ_FU;
    }
}

// d_j = sqrt(A_jj + lam); 1 for a dead channel without regularizer (its row and column of A are zero)
__global__ __launch_bounds__(256) void jq_diag_kernel(const float* __restrict__ A, int n, float lam,
                                                      const int32_t* __restrict__ perm, float* __restrict__ d) {
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= n) return;
    const int oj = pcol(perm, j);
    const float x = A[int64_t(oj) * n + oj] + lam;
    d[j] = x > 0.f ? sqrtf(x) : 1.f;
}

// A~ = (A + lam I)_kj / (d_k d_j) * 2^14 as fp16 hi + lo; the rows of the grid behind row n - 1 (padding of the k
// range) are zero
__global__ __launch_bounds__(256) void jq_asplit_kernel(const float* __restrict__ A, int n, float lam,
                                                        const int32_t* __restrict__ perm,
                                                        const float* __restrict__ d, uint16_t* __restrict__ Bh,
                                                        uint16_t* __restrict__ Bl) {
    const int k = blockIdx.y;
    const int j4 = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (j4 >= n) return;
    short4v h4 = {0, 0, 0, 0}, l4 = {0, 0, 0, 0};
    if (k < n) {
        float4v v;
        if (perm) {
            const float* rowp = A + int64_t(perm[k]) * n;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = rowp[perm[j4 + e]];
        } else {
            v = *reinterpret_cast<const float4v*>(A + int64_t(k) * n + j4);
        }
        const float rk = 1.0f / d[k];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float x = (v[e] + (j4 + e == k ? lam : 0.f)) * rk / d[j4 + e] * JQ_FU;
            x = fminf(fmaxf(x, -60000.f), 60000.f);
            const _Float16 h = (_Float16)x;
            const _Float16 lo = (_Float16)(x - (float)h);
            h4[e] = __builtin_bit_cast(short, h);
            l4[e] = __builtin_bit_cast(short, lo);
        }
    }
    *reinterpret_cast<short4v*>(Bh + int64_t(k) * n + j4) = h4;
    *reinterpret_cast<short4v*>(Bl + int64_t(k) * n + j4) = l4;
}

// R = W - s (q - z) over the whole layer; max |R d| into sc->max_w_bits
__global__ __launch_bounds__(256) void jq_residual_kernel(const void* __restrict__ W, int bf16, int d_out, int d_in,
                                                          const uint8_t* __restrict__ Q, const float* __restrict__ scales,
                                                          const float* __restrict__ zeros, int G, int n_g,
                                                          const int32_t* __restrict__ perm,
                                                          const float* __restrict__ d, float* __restrict__ R,
                                                          Scalars* sc) {
    __shared__ uint32_t s_max;
    float mx = 0.f;
    for (int64_t r = blockIdx.x; r < d_out; r += gridDim.x)
        for (int c = threadIdx.x; c < d_in; c += 256) {
            const int64_t i = r * d_in + pcol(perm, c);
            const int g = c / G;
            const float x = load_w(W, bf16, i) - scales[r * n_g + g] * (float(Q[i]) - zeros[r * n_g + g]);
            R[r * d_in + c] = x;
            mx = fmaxf(mx, fabsf(x) * d[c]);
        }
    block_max_bits(&sc->max_w_bits, mx, &s_max);
}

// Left operand of a split product: Dt[k][row] = src[row][k] * d[k] * f_d (d == nullptr: 1) as fp16 hi + lo for
// k < k_count, zero for k_count <= k < k_pad and for the padding rows up to ldD.  f_d = 2^(13 - exponent of the
// maximum in sc), so that the largest value lands in [2^12, 2^13); thread 0 of the grid leaves f_d, f_all = f_d f_u
// and f_inv in sc for the product (f_u, a power of two, is already there) and clears the maximum of `other` (the
// slot the next producer accumulates into).  64 x 64 tiles through LDS.
__global__ __launch_bounds__(256) void jq_dsplit_kernel(const float* __restrict__ src, int64_t ld_src, int d_out,
                                                        int k_count, int k_pad, const float* __restrict__ d,
                                                        Scalars* sc, Scalars* other, uint16_t* __restrict__ Dh,
                                                        uint16_t* __restrict__ Dl, int64_t ldD) {
    __shared__ float tile[64][65];
    const float mx = __uint_as_float(sc->max_w_bits);
    int e = 0;
    if (mx > 0.f) (void)frexpf(mx, &e);
    const int sd = max(-60, min(60, 13 - e));
    const float f_d = ldexpf(1.f, sd);
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) {
        const float f_u = sc->f_u;
        sc->f_d = f_d;
        sc->f_all = f_d * f_u;
        sc->f_inv = 1.0f / (f_d * f_u);
        if (other) other->max_w_bits = 0u;
    }
    const int k0 = blockIdx.x * 64, r0 = blockIdx.y * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int rr = ty; rr < 64; rr += 4) {
        const int r = r0 + rr, k = k0 + tx;
        tile[rr][tx] = (r < d_out && k < k_count) ? src[int64_t(r) * ld_src + k] * (d ? d[k] : 1.0f) * f_d : 0.f;
    }
    __syncthreads();
    for (int kk = ty; kk < 64; kk += 4) {
        const int k = k0 + kk, r = r0 + tx;
        if (k >= k_pad || r >= ldD) continue;
        float x = tile[tx][kk];
        x = fminf(fmaxf(x, -60000.f), 60000.f);
        const _Float16 h = (_Float16)x;
        const _Float16 lo = (_Float16)(x - (float)h);
        Dh[int64_t(k) * ldD + r] = __builtin_bit_cast(uint16_t, h);
        Dl[int64_t(k) * ldD + r] = __builtin_bit_cast(uint16_t, lo);
    }
}

__global__ __launch_bounds__(256) void jq_fill0_kernel(float* __restrict__ p, int64_t n4) {
    const float4v z = {0.f, 0.f, 0.f, 0.f};
    for (int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x; i < n4; i += int64_t(gridDim.x) * 256)
        reinterpret_cast<float4v*>(p)[i] = z;
}

// rowf[r] = sum_j r_j Gm~_rj d_j with r recomputed from the codes; optional W^ output
__global__ __launch_bounds__(256) void jq_objective_kernel(const void* __restrict__ W, int bf16, int d_out, int d_in,
                                                           const uint8_t* __restrict__ Q, const float* __restrict__ scales,
                                                           const float* __restrict__ zeros, int G, int n_g,
                                                           const int32_t* __restrict__ perm,
                                                           const float* __restrict__ Gm, const float* __restrict__ d,
                                                           float* __restrict__ rowf, float* __restrict__ W_hat) {
    __shared__ float red[256];
    for (int64_t r = blockIdx.x; r < d_out; r += gridDim.x) {
        float acc = 0.f;
        for (int c = threadIdx.x; c < d_in; c += 256) {
            const int64_t i = r * d_in + pcol(perm, c);
            const int g = c / G;
            const float wh = scales[r * n_g + g] * (float(Q[i]) - zeros[r * n_g + g]);
            const float rr = load_w(W, bf16, i) - wh;
            acc += rr * Gm[r * d_in + c] * d[c];
            if (W_hat) W_hat[i] = wh;   // i: the caller's column order
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
    int d_out, d_in, G, n_g, t;
    const float* A; float lam;
    const int32_t* perm;       // sweep position -> original column of A, W and Q (nullptr: natural order)
    float qtop;
    uint8_t* Q; float* scales; const float* zeros;
    const float* Gm;           // column-normalized gradient of the whole objective (lam included)
    const float* d;            // d_j = sqrt(A_jj + lam)
    float* dR; int ldr;        // the group's dR: row r at dR + r * ldr
    Scalars* sc_near;          // max |dR d| of this visit
    Scalars* sc_far;           // max |dR d| of the super-block
    // groups wider than a block (WIDE): the launch covers the block of v.G = 128 columns starting at col0
    int col0;                  // first column of the block (groups up to 128 columns: t * G)
    const float* Am;           // column-normalized a = (A_gg + lam I) u of the group, kept current
    const float* P;            // p of the group's columns, fixed during the visit
    float* bc;                 // per row b, c of the visited group
    int32_t* flags;            // per row (4 slots): [0] still scanning this visit, [1] took a move in this scan,
                               // [2] codes of the visited group that differ from its zero-point
    int max_scans;
    int32_t* moves;
};

// NC = columns per lane (1: G <= 64, 2: G <= 128).  The scan "columns in order, first improving move wins" is run as:
// every lane evaluates the gain of its own columns under the current state, a ballot finds the first improving
// column behind the last one taken, that move is applied, and the evaluation is repeated.  The columns between two
// taken moves are rejected under the same state the sequential scan would see, so the sequence of moves is the same,
// at one wave-wide evaluation per taken move instead of one per column.
//
// WIDE (groups of several 128-column blocks): one launch is one block's share of one scan of the visit.  b and c
// live in memory across the launches, a = (A_gg + lam I) u comes from Am (updated between the launches with the
// same split products as the gradient, for every column of the group), p from P; the launch scans its columns once,
// writes the code changes dU = u_new - u_old (the update's left operand) and marks the row when it took a move.
template <int NC, bool WIDE>
__global__ __launch_bounds__(64 * JQ_ROWS) void jq_visit_kernel(VisitArgs v) {
    extern __shared__ float sA[];   // G x G: A_tt + lam I
    __shared__ uint32_t s_max;
    __shared__ int s_moves;
    const int G = v.G;
    const int c0 = v.col0;
    for (int e = threadIdx.x * 4; e < G * G; e += 64 * JQ_ROWS * 4) {
        const int k = e / G, c = e - k * G;
        float4v x;
        if (v.perm) {
            const float* rowp = v.A + int64_t(v.perm[c0 + k]) * v.d_in;
#pragma unroll
            for (int i = 0; i < 4; ++i) x[i] = rowp[v.perm[c0 + c + i]];
        } else {
            x = *reinterpret_cast<const float4v*>(v.A + int64_t(c0 + k) * v.d_in + c0 + c);
        }
        if (k >= c && k < c + 4) x[k - c] += v.lam;
        *reinterpret_cast<float4v*>(sA + e) = x;
    }
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * JQ_ROWS + (threadIdx.x >> 6);
    float dr_max = 0.f;
    int wave_moves = 0;
    bool run = row < v.d_out;
    if (WIDE && run && v.flags[4 * row] == 0) {   // the row's visit is over: no change from this block
        run = false;
#pragma unroll
        for (int c = 0; c < NC; ++c)
            if (lane + 64 * c < G) v.dR[int64_t(row) * v.ldr + lane + 64 * c] = 0.f;
    }
    if (run) {
    const float z = v.zeros[int64_t(row) * v.n_g + v.t];
    const float s_old = v.scales[int64_t(row) * v.n_g + v.t];
    float u[NC], u0[NC], a[NC], p[NC], q[NC], ad[NC], dj[NC];
    bool has[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const int col = lane + 64 * c;
        has[c] = col < G;
        const int64_t i = int64_t(row) * v.d_in + c0 + (has[c] ? col : 0);     // sweep order: Gm, Am, P
        const int64_t iq = int64_t(row) * v.d_in + pcol(v.perm, c0 + (has[c] ? col : 0));   // caller's order: Q
        q[c] = has[c] ? float(v.Q[iq]) : z;
        u[c] = q[c] - z;
        u0[c] = u[c];
        a[c] = 0.f;
        ad[c] = has[c] ? sA[col * G + col] : 1.f;
        dj[c] = has[c] ? v.d[c0 + col] : 0.f;
        if (WIDE) {
            p[c] = has[c] ? v.P[i] : 0.f;
            a[c] = has[c] ? v.Am[i] * dj[c] : 0.f;
        } else {
            p[c] = has[c] ? v.Gm[i] * dj[c] : 0.f;   // ((A + lam I) r)_t; s_old (A_tt + lam I) u is added below
        }
    }
    // a = (A_tt + lam I) u
#pragma unroll
    for (int cu = 0; cu < (WIDE ? 0 : NC); ++cu) {
        const int kn = G - 64 * cu < 64 ? G - 64 * cu : 64;
        for (int k = 0; k < kn; k += 8) {   // kn is a multiple of 16; eight rows' LDS reads in flight at a time
            float x[8][NC];
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int c = 0; c < NC; ++c) x[i][c] = has[c] ? sA[(64 * cu + k + i) * G + lane + 64 * c] : 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float uk = readlane_f(u[cu], k + i);
#pragma unroll
                for (int c = 0; c < NC; ++c) a[c] = fmaf(x[i][c], uk, a[c]);
            }
        }
    }
    float b = 0.f, cc = 0.f;
    if (WIDE) {
        b = v.bc[2 * row];
        cc = v.bc[2 * row + 1];
    } else {
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            p[c] += s_old * a[c];
            b += u[c] * p[c];
            cc += u[c] * a[c];
        }
        b = wave_sum(b);
        cc = wave_sum(cc);
    }
    const bool live = cc > 0.f;
    // Codes of the group that differ from its zero-point.  The move that would take the last of them there has
    // c' = 0 exactly and N = 0 from below, so it is never taken; in fp32, with c carried through earlier moves, both
    // come out as rounding noise of either sign, and once taken the scale b / c is noise over noise.  The count
    // settles it on the integers: ballots of u != 0 plus, for a group wider than a block, the count in its other
    // blocks.  A move changes the count by at most one, so after a count of n the next n - 2 moves cannot meet the
    // case and run without the check (the kernel is bound by its instruction count, and groups with one or two such
    // codes are rare).
    auto count_here = [&]() __attribute__((always_inline)) {
        int n = 0;
#pragma unroll
        for (int c = 0; c < NC; ++c) n += __builtin_popcountll(__ballot(has[c] && u[c] != 0.f));
        return n;
    };
    const int nnz_other = WIDE ? v.flags[4 * row + 2] - count_here() : 0;
    int n_moves = 0;
    if (live) {
        // b / cc to within rounding, in fewer dependent steps than the correctly rounded division
        auto ratio = [](float x, float y) __attribute__((always_inline)) {
            float r = __builtin_amdgcn_rcpf(y);
            r = fmaf(fmaf(-y, r, 1.0f), r, r);
            return x * r;
        };
        float ss = ratio(b, cc);
        int scan = 0, j0 = -1;   // j0: the column of the last move taken in this scan
        int unchecked = 0;       // moves that may still be taken before the codes are counted again
        float qup[NC], qdn[NC];  // a lane may go up from codes <= qup, down from codes >= qdn
        bool took = false;
        for (;;) {
            // N = 2 d b g + (p^2 - s*^2 c A_jj): the bracket is the expanded form's g^2 + 2 s* g a - s*^2 (c A_jj - a^2)
            const float twob = 2.0f * b, bss = b * ss, hcc = 0.5f * cc, qtop1 = v.qtop - 1.0f;
            if (unchecked <= 0) {
                // the guard lives in the per-lane code bounds of the two directions, which the step compares
                // anyway: with one code left, its lane may not move towards the zero-point
                const int n = nnz_other + count_here();
                const bool last = n == 1;
                unchecked = n - 2;
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    qup[c] = (last && u[c] == -1.0f) ? -1.0f : qtop1;
                    qdn[c] = (last && u[c] == 1.0f) ? 3.0e38f : 1.0f;
                }
            }
            uint64_t m[NC];
            float dd[NC];
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const float gs = fmaf(-ss, a[c], p[c]);
                const float base = fmaf(p[c], p[c], -bss * ad[c]);
                const float t1 = twob * gs;
                const float hc = fmaf(0.5f, ad[c], hcc);    // (c + A_jj) / 2: c' > 0  <=>  hc + d a > 0
                const bool up = q[c] <= qup[c] && base > -t1 && hc > -a[c];
                const bool dn = q[c] >= qdn[c] && base > t1 && hc > a[c];
                dd[c] = up ? 1.0f : -1.0f;
                m[c] = __ballot(has[c] && (up || dn));
                const int lo = j0 - 64 * c;          // columns up to lo (local numbering) are behind
                if (lo >= 63) m[c] = 0;
                else if (lo >= 0) m[c] &= ~((uint64_t(2) << lo) - 1);
            }
            int j = -1;
            if (m[0]) j = __builtin_ctzll(m[0]);
            else if (NC > 1 && m[NC - 1]) j = 64 + __builtin_ctzll(m[NC - 1]);
            if (j < 0) {   // the scan is over
                if (WIDE || !took || ++scan >= v.max_scans) break;
                took = false;
                j0 = -1;
                continue;
            }
            const float* rowj = sA + j * G + lane;
            float arow[NC];
#pragma unroll
            for (int c = 0; c < NC; ++c) arow[c] = has[c] ? rowj[64 * c] : 0.f;
            float d, pj, aj, adj;
            if (NC == 1 || j < 64) {
                d = readlane_f(dd[0], j); pj = readlane_f(p[0], j); aj = readlane_f(a[0], j); adj = readlane_f(ad[0], j);
                if (lane == j) { u[0] += d; q[0] += d; }
            } else {
                d = readlane_f(dd[NC - 1], j - 64); pj = readlane_f(p[NC - 1], j - 64);
                aj = readlane_f(a[NC - 1], j - 64); adj = readlane_f(ad[NC - 1], j - 64);
                if (lane == j - 64) { u[NC - 1] += d; q[NC - 1] += d; }
            }
            b = fmaf(d, pj, b);
            cc += fmaf(2.0f * d, aj, adj);
            ss = ratio(b, cc);
#pragma unroll
            for (int c = 0; c < NC; ++c) a[c] = fmaf(d, arow[c], a[c]);
            took = true;
            j0 = j;
            ++n_moves;
            --unchecked;
        }
    }
    const float s_new = live ? b / cc : s_old;
    const int nnz_here = WIDE ? count_here() : 0;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        if (!has[c]) continue;
        const int col = lane + 64 * c;
        v.Q[int64_t(row) * v.d_in + pcol(v.perm, c0 + col)] = uint8_t(q[c]);
        // groups up to a block: change of the residual w - w^;  wider: change of the codes
        const float dr = WIDE ? u[c] - u0[c] : s_old * u0[c] - s_new * u[c];
        v.dR[int64_t(row) * v.ldr + col] = dr;
        dr_max = fmaxf(dr_max, fabsf(dr) * dj[c]);
    }
    if (lane == 0) {
        if (WIDE) {
            v.bc[2 * row] = b;
            v.bc[2 * row + 1] = cc;
            v.flags[4 * row + 2] = nnz_other + nnz_here;
            if (n_moves > 0) v.flags[4 * row + 1] = 1;
        } else {
            v.scales[int64_t(row) * v.n_g + v.t] = s_new;
        }
    }
    wave_moves = n_moves;
    }
    // one atomic per workgroup and target: atomics on one address are serialized
    if (threadIdx.x == 0) { s_max = 0u; s_moves = 0; }
    __syncthreads();
    dr_max = wave_max(dr_max);
    if (lane == 0) {
        atomicMax(&s_max, __float_as_uint(dr_max));
        if (wave_moves > 0) atomicAdd(&s_moves, wave_moves);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        if (s_max > __hip_atomic_load(&v.sc_near->max_w_bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
            atomicMax(&v.sc_near->max_w_bits, s_max);
        if (s_max > __hip_atomic_load(&v.sc_far->max_w_bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
            atomicMax(&v.sc_far->max_w_bits, s_max);
        if (s_moves > 0) atomicAdd(v.moves, s_moves);
    }
}

// ---- groups wider than a block -----------------------------------------------------------------------------------
// start of a visit: U[row][c] = q - z over the group's columns (left operand of a = (A_gg + lam I) u); max |u d|
__global__ __launch_bounds__(256) void jq_wide_begin_kernel(int d_out, int d_in, const uint8_t* __restrict__ Q,
                                                            const float* __restrict__ zeros, int n_g, int g, int G,
                                                            const int32_t* __restrict__ perm,
                                                            const float* __restrict__ d, float* __restrict__ U,
                                                            Scalars* sc) {
    __shared__ uint32_t s_max;
    float mx = 0.f;
    const int g0 = g * G;
    for (int64_t r = blockIdx.x; r < d_out; r += gridDim.x) {
        const float z = zeros[r * n_g + g];
        for (int c = threadIdx.x; c < G; c += 256) {
            const int64_t i = r * d_in + g0 + c;
            const float u = float(Q[r * d_in + pcol(perm, g0 + c)]) - z;
            U[i] = u;
            mx = fmaxf(mx, fabsf(u) * d[g0 + c]);
        }
    }
    block_max_bits(&sc->max_w_bits, mx, &s_max);
}

// P = ((A + lam I) r)_g + s_old a,  b = u.P,  c = u.a  with a = Am d (one workgroup per row at a time)
__global__ __launch_bounds__(256) void jq_wide_p_kernel(int d_out, int d_in, const float* __restrict__ scales, int n_g,
                                                        int g, int G, const float* __restrict__ d,
                                                        const float* __restrict__ U, const float* __restrict__ Gm,
                                                        const float* __restrict__ Am, float* __restrict__ P,
                                                        float* __restrict__ bc, int32_t* __restrict__ flags) {
    __shared__ float rb[256], rc[256];
    __shared__ int rn[256];
    const int g0 = g * G;
    for (int64_t r = blockIdx.x; r < d_out; r += gridDim.x) {
        const float s_old = scales[r * n_g + g];
        float b = 0.f, c = 0.f;
        int nz = 0;
        for (int k = threadIdx.x; k < G; k += 256) {
            const int64_t i = r * d_in + g0 + k;
            const float dj = d[g0 + k], a = Am[i] * dj, u = U[i];
            const float p = Gm[i] * dj + s_old * a;
            P[i] = p;
            b += u * p;
            c += u * a;
            nz += u != 0.f ? 1 : 0;
        }
        rb[threadIdx.x] = b; rc[threadIdx.x] = c; rn[threadIdx.x] = nz;
        __syncthreads();
        for (int w = 128; w > 0; w >>= 1) {
            if (int(threadIdx.x) < w) {
                rb[threadIdx.x] += rb[threadIdx.x + w]; rc[threadIdx.x] += rc[threadIdx.x + w];
                rn[threadIdx.x] += rn[threadIdx.x + w];
            }
            __syncthreads();
        }
        if (threadIdx.x == 0) {
            bc[2 * r] = rb[0]; bc[2 * r + 1] = rc[0];
            flags[4 * r] = rc[0] > 0.f ? 1 : 0;
            flags[4 * r + 1] = 0;
            flags[4 * r + 2] = rn[0];
        }
        __syncthreads();
    }
}

// end of a scan: a row whose scan took nothing has finished its visit
__global__ __launch_bounds__(256) void jq_scan_end_kernel(int d_out, int32_t* __restrict__ flags) {
    const int r = blockIdx.x * 256 + threadIdx.x;
    if (r >= d_out) return;
    if (flags[4 * r + 1] == 0) flags[4 * r] = 0;
    flags[4 * r + 1] = 0;
}

// end of a visit: s = b / c; U <- change of the residual s_old u_old - s_new u_new; max |dR d|
__global__ __launch_bounds__(256) void jq_wide_end_kernel(int d_out, int d_in, const uint8_t* __restrict__ Q,
                                                          float* __restrict__ scales, const float* __restrict__ zeros,
                                                          int n_g, int g, int G, const int32_t* __restrict__ perm,
                                                          const float* __restrict__ d,
                                                          const float* __restrict__ bc, float* __restrict__ U,
                                                          Scalars* sc) {
    __shared__ uint32_t s_max;
    float mx = 0.f;
    const int g0 = g * G;
    for (int64_t r = blockIdx.x; r < d_out; r += gridDim.x) {
        const float z = zeros[r * n_g + g], s_old = scales[r * n_g + g];
        const float b = bc[2 * r], c = bc[2 * r + 1];
        const float s_new = c > 0.f ? b / c : s_old;
        for (int k = threadIdx.x; k < G; k += 256) {
            const int64_t i = r * d_in + g0 + k;
            const float dr = s_old * U[i] - s_new * (float(Q[r * d_in + pcol(perm, g0 + k)]) - z);
            U[i] = dr;
            mx = fmaxf(mx, fabsf(dr) * d[g0 + k]);
        }
        __syncthreads();   // every thread has read the old scale
        if (threadIdx.x == 0) scales[r * n_g + g] = s_new;
    }
    block_max_bits(&sc->max_w_bits, mx, &s_max);
}

constexpr int JQ_NEAR0 = 608;   // first row of the staging area of the per-visit left operand (the far one uses 0 ..)

struct JqWs {
    float* Gm;        // d_out x d_in: column-normalized gradient, kept current
    float* R;         // d_out x d_in: residual at the start (left operand of the first product)
    uint16_t *Bh, *Bl;   // (d_in + 32) x d_in: A~ hi / lo, zero rows behind the matrix
    uint16_t *Dh, *Dl;   // rows_d x ldD: left operands, k-major
    float* dR;        // d_out x JQ_SBW: dR of the groups of the current super-block side by side
    float* d;         // d_in
    float* rowf;      // d_out
    Scalars* sc;      // [0] first product, [1], [2] visits (alternating), [3], [4] super-blocks (alternating),
                      // [5] start, [6] end of a wide group's visit
    // groups wider than a block only
    float* Am;        // d_out x d_in: column-normalized a of the visited group
    float* P;         // d_out x d_in: p of the visited group
    float* bc;        // d_out x 2
    int32_t* flags;   // d_out x 4
};

int64_t rows_d(int64_t d_in) { return d_in + 32 > JQ_NEAR0 + 160 ? d_in + 32 : JQ_NEAR0 + 160; }

JqWs carve(void* ws, int64_t d_out, int64_t d_in, bool wide) {
    char* p = static_cast<char*>(ws);
    const int64_t ldD = split_update_ld(d_out);
    JqWs w;
    w.Gm = reinterpret_cast<float*>(p); p += align_up(size_t(d_out) * d_in * 4, 256);
    w.R = reinterpret_cast<float*>(p); p += align_up(size_t(d_out) * d_in * 4, 256);
    w.Bh = reinterpret_cast<uint16_t*>(p); p += align_up(size_t(d_in + 32) * d_in * 2, 256);
    w.Bl = reinterpret_cast<uint16_t*>(p); p += align_up(size_t(d_in + 32) * d_in * 2, 256);
    w.Dh = reinterpret_cast<uint16_t*>(p); p += align_up(size_t(rows_d(d_in)) * ldD * 2, 256);
    w.Dl = reinterpret_cast<uint16_t*>(p); p += align_up(size_t(rows_d(d_in)) * ldD * 2, 256);
    w.dR = reinterpret_cast<float*>(p); p += align_up(size_t(d_out) * JQ_SBW * 4, 256);
    w.d = reinterpret_cast<float*>(p); p += align_up(size_t(d_in) * 4, 256);
    w.rowf = reinterpret_cast<float*>(p); p += align_up(size_t(d_out) * 4, 256);
    w.sc = reinterpret_cast<Scalars*>(p); p += 256;
    w.Am = w.P = w.bc = nullptr; w.flags = nullptr;
    if (wide) {
        w.Am = reinterpret_cast<float*>(p); p += align_up(size_t(d_out) * d_in * 4, 256);
        w.P = reinterpret_cast<float*>(p); p += align_up(size_t(d_out) * d_in * 4, 256);
        w.bc = reinterpret_cast<float*>(p); p += align_up(size_t(d_out) * 8, 256);
        w.flags = reinterpret_cast<int32_t*>(p);
    }
    return w;
}

}  // namespace

onecomp_status fill_zero(float* p, int64_t n4, hipStream_t stream) {
    if (n4 <= 0) return ONECOMP_OK;
    hipLaunchKernelGGL(jq_fill0_kernel, dim3(2048), dim3(256), 0, stream, p, n4);
    ONECOMP_CHECK_LAUNCH();
    return ONECOMP_OK;
}

onecomp_status split_left_operand(const float* src, int64_t ld_src, int64_t d_out, int k_count, const float* d,
                                  Scalars* sc, Scalars* other, uint16_t* Dh, uint16_t* Dl, hipStream_t stream) {
    const int64_t ldD = split_update_ld(d_out);
    const int k_pad = (k_count + 31) / 32 * 32;
    hipLaunchKernelGGL(jq_dsplit_kernel, dim3(unsigned(ceil_div(k_pad, 64)), unsigned(ceil_div(ldD, 64))), dim3(256), 0,
                       stream, src, ld_src, int(d_out), k_count, k_pad, d, sc, other, Dh, Dl, ldD);
    ONECOMP_CHECK_LAUNCH();
    return ONECOMP_OK;
}

size_t jointq_workspace_bytes(int64_t d_out, int64_t d_in, int group_size) {
    const int64_t ldD = split_update_ld(d_out);
    const size_t wide = group_size > 128 ? 2 * align_up(size_t(d_out) * d_in * 4, 256) + align_up(size_t(d_out) * 8, 256) +
                                               align_up(size_t(d_out) * 16, 256)
                                         : 0;
    return 2 * align_up(size_t(d_out) * d_in * 4, 256) + 2 * align_up(size_t(d_in + 32) * d_in * 2, 256) +
           2 * align_up(size_t(rows_d(d_in)) * ldD * 2, 256) + align_up(size_t(d_out) * JQ_SBW * 4, 256) +
           align_up(size_t(d_in) * 4, 256) + align_up(size_t(d_out) * 4, 256) + 256 + wide;
}

onecomp_status jointq_run(const void* W, onecomp_dtype w_dtype, int64_t d_out, int64_t d_in, const float* A,
                          const int32_t* perm, float lam, int bits, int group_size, int grid, int n_pass, int max_scans, uint8_t* Q, float* scales,
                          const float* zeros, float* W_hat, float* objective, int32_t* n_moves, void* workspace,
                          hipStream_t stream) {
    const int G = group_size;
    const int n_g = int(d_in / G);
    const bool symmetric = grid == ONECOMP_GRID_SYMMETRIC || grid == ONECOMP_GRID_SYMMETRIC_MSE;
    const float qtop = symmetric ? float(2 * ((1 << (bits - 1)) - 1)) : float((1 << bits) - 1);
    const int bf16 = w_dtype == ONECOMP_BF16;
    const bool wide = G > 128;
    JqWs w = carve(workspace, d_out, d_in, wide);
    const int64_t ldD = split_update_ld(d_out);
    const dim3 rgrid{unsigned(d_out < 4096 ? d_out : 4096)};
    auto pad32 = [](int k) { return (k + 31) / 32 * 32; };
    onecomp_status st;

    hipLaunchKernelGGL(jq_zero_kernel, dim3(1), dim3(1), 0, stream, n_moves);
    ONECOMP_CHECK_LAUNCH();
    hipLaunchKernelGGL(jq_scalars_init_kernel, dim3(1), dim3(64), 0, stream, w.sc, 7);
    ONECOMP_CHECK_LAUNCH();
    hipLaunchKernelGGL(jq_diag_kernel, dim3(unsigned(ceil_div(d_in, 256))), dim3(256), 0, stream, A, int(d_in), lam, perm,
                       w.d);
    ONECOMP_CHECK_LAUNCH();
    hipLaunchKernelGGL(jq_asplit_kernel, dim3(unsigned(ceil_div(d_in, 1024)), unsigned(d_in + 32)), dim3(256), 0, stream,
                       A, int(d_in), lam, perm, w.d, w.Bh, w.Bl);
    ONECOMP_CHECK_LAUNCH();
    hipLaunchKernelGGL(jq_residual_kernel, rgrid, dim3(256), 0, stream, W, bf16, int(d_out), int(d_in), Q, scales, zeros,
                       G, n_g, perm, w.d, w.R, w.sc);
    ONECOMP_CHECK_LAUNCH();
    // left operand rows [row0, row0 + pad32(k_count)) of the D buffers from src[:, 0 .. k_count), columns c_first ..
    auto dsplit = [&](const float* src, int64_t ld_src, int k_count, int c_first, int row0, Scalars* sc,
                      Scalars* other) -> onecomp_status {
        const int k_pad = pad32(k_count);
        hipLaunchKernelGGL(jq_dsplit_kernel, dim3(unsigned(ceil_div(k_pad, 64)), unsigned(ceil_div(ldD, 64))), dim3(256), 0,
                           stream, src, ld_src, int(d_out), k_count, k_pad, w.d + c_first, sc, other,
                           w.Dh + int64_t(row0) * ldD, w.Dl + int64_t(row0) * ldD, ldD);
        ONECOMP_CHECK_LAUNCH();
        return ONECOMP_OK;
    };
    // Gm~[:, c_lo .. c_hi) += (rows row0 .. of D)^T A~[u0 .. u0 + pad32(k_count), c_lo .. c_hi)
    auto update_to = [&](float* C, int row0, int k_count, int u0, int c_lo, int c_hi,
                         const Scalars* sc) -> onecomp_status {
        return split_update(C, d_out, d_in, w.Dh, w.Dl, ldD, w.Bh, w.Bl, sc, row0, pad32(k_count), u0, c_lo, c_hi, stream);
    };
    auto update = [&](int row0, int k_count, int u0, int c_lo, int c_hi, const Scalars* sc) -> onecomp_status {
        return update_to(w.Gm, row0, k_count, u0, c_lo, c_hi, sc);
    };
    if ((st = dsplit(w.R, d_in, int(d_in), 0, 0, w.sc, nullptr)) != ONECOMP_OK) return st;
    if ((st = fill_zero(w.Gm, d_out * d_in / 4, stream)) != ONECOMP_OK) return st;
    if ((st = update(0, int(d_in), 0, 0, int(d_in), w.sc)) != ONECOMP_OK) return st;
    hipLaunchKernelGGL(jq_objective_kernel, rgrid, dim3(256), 0, stream, W, bf16, int(d_out), int(d_in), Q, scales, zeros,
                       G, n_g, perm, w.Gm, w.d, w.rowf, static_cast<float*>(nullptr));
    ONECOMP_CHECK_LAUNCH();
    hipLaunchKernelGGL(jq_total_kernel, dim3(1), dim3(1024), 0, stream, w.rowf, int(d_out), objective);
    ONECOMP_CHECK_LAUNCH();

    static std::atomic<uint64_t> lds1{0}, lds2{0}, lds3{0};
    const int GB = wide ? 128 : G;   // columns of one launch of the visit kernel
    const int lds_bytes = GB * GB * 4;
    if (wide) {
        if (allow_dynamic_lds(reinterpret_cast<const void*>(&jq_visit_kernel<2, true>), 128 * 128 * 4, lds3) != ONECOMP_OK)
            return ONECOMP_ERR_HIP;
    } else if (G <= 64) {
        if (allow_dynamic_lds(reinterpret_cast<const void*>(&jq_visit_kernel<1, false>), 64 * 64 * 4, lds1) != ONECOMP_OK)
            return ONECOMP_ERR_HIP;
    } else {
        if (allow_dynamic_lds(reinterpret_cast<const void*>(&jq_visit_kernel<2, false>), 128 * 128 * 4, lds2) != ONECOMP_OK)
            return ONECOMP_ERR_HIP;
    }
    VisitArgs v;
    v.d_out = int(d_out); v.d_in = int(d_in); v.G = GB; v.n_g = n_g; v.t = 0;
    v.A = A; v.lam = lam; v.perm = perm; v.qtop = qtop; v.Q = Q; v.scales = scales; v.zeros = zeros; v.Gm = w.Gm; v.d = w.d;
    v.dR = w.dR; v.max_scans = max_scans; v.moves = n_moves;
    v.col0 = 0; v.Am = w.Am; v.P = w.P; v.bc = w.bc; v.flags = w.flags;
    const dim3 vgrid{unsigned(ceil_div(d_out, JQ_ROWS))};
    const int sbg = JQ_SBW / GB > 0 ? JQ_SBW / GB : 1;   // launches of the visit kernel per super-block
    v.ldr = sbg * GB;
    int n_visit = 0, n_sb = 0;
    if (!wide) {
        for (int ps = 0; ps < n_pass; ++ps)
            for (int t0 = 0; t0 < n_g; t0 += sbg, ++n_sb) {
                const int t1 = t0 + sbg < n_g ? t0 + sbg : n_g;
                Scalars* sc_far = w.sc + 3 + (n_sb & 1);
                for (int t = t0; t < t1; ++t, ++n_visit) {
                    Scalars* sc_near = w.sc + 1 + (n_visit & 1);
                    v.t = t;
                    v.col0 = t * G;
                    v.dR = w.dR + (t - t0) * G;
                    v.sc_near = sc_near; v.sc_far = sc_far;
                    if (G <= 64)
                        hipLaunchKernelGGL((jq_visit_kernel<1, false>), vgrid, dim3(64 * JQ_ROWS), lds_bytes, stream, v);
                    else
                        hipLaunchKernelGGL((jq_visit_kernel<2, false>), vgrid, dim3(64 * JQ_ROWS), lds_bytes, stream, v);
                    ONECOMP_CHECK_LAUNCH();
                    // the super-block's own columns at once
                    if ((st = dsplit(v.dR, v.ldr, G, t * G, JQ_NEAR0, sc_near, w.sc + 1 + ((n_visit + 1) & 1))) != ONECOMP_OK)
                        return st;
                    if ((st = update(JQ_NEAR0, G, t * G, t0 * G, t1 * G, sc_near)) != ONECOMP_OK) return st;
                }
                // all other columns once per super-block
                if ((st = dsplit(w.dR, v.ldr, (t1 - t0) * G, t0 * G, 0, sc_far, w.sc + 3 + ((n_sb + 1) & 1))) != ONECOMP_OK)
                    return st;
                if ((st = update(0, (t1 - t0) * G, t0 * G, 0, t0 * G, sc_far)) != ONECOMP_OK) return st;
                if ((st = update(0, (t1 - t0) * G, t0 * G, t1 * G, int(d_in), sc_far)) != ONECOMP_OK) return st;
            }
    } else {
        // A group spans n_b blocks of 128 columns.  Visit of group g: a = (A_gg + lam I) u for the whole group by one
        // product (Am), p, b, c from it; then up to max_scans scans, each one launch per block in column order with
        // Am brought up to date between the launches (the super-block's columns at once, the group's other columns
        // once per super-block); at the end the scale, and the gradient of all columns from the group's dR.
        const int n_b = G / 128;
        for (int ps = 0; ps < n_pass; ++ps)
            for (int g = 0; g < n_g; ++g) {
                const int g0 = g * G;
                v.t = g;
                hipLaunchKernelGGL(jq_wide_begin_kernel, rgrid, dim3(256), 0, stream, int(d_out), int(d_in), Q, zeros, n_g, g,
                                   G, perm, w.d, w.R, w.sc + 5);
                ONECOMP_CHECK_LAUNCH();
                if ((st = dsplit(w.R + g0, d_in, G, g0, 0, w.sc + 5, w.sc + 6)) != ONECOMP_OK) return st;
                if ((st = fill_zero(w.Am, d_out * d_in / 4, stream)) != ONECOMP_OK) return st;
                if ((st = update_to(w.Am, 0, G, g0, g0, g0 + G, w.sc + 5)) != ONECOMP_OK) return st;
                hipLaunchKernelGGL(jq_wide_p_kernel, rgrid, dim3(256), 0, stream, int(d_out), int(d_in), scales, n_g, g, G,
                                   w.d, w.R, w.Gm, w.Am, w.P, w.bc, w.flags);
                ONECOMP_CHECK_LAUNCH();
                for (int scan = 0; scan < max_scans; ++scan) {
                    for (int i0 = 0; i0 < n_b; i0 += sbg, ++n_sb) {
                        const int i1 = i0 + sbg < n_b ? i0 + sbg : n_b;
                        const int sb0 = g0 + i0 * 128, sb1 = g0 + i1 * 128;
                        Scalars* sc_far = w.sc + 3 + (n_sb & 1);
                        for (int i = i0; i < i1; ++i, ++n_visit) {
                            Scalars* sc_near = w.sc + 1 + (n_visit & 1);
                            v.col0 = g0 + i * 128;
                            v.dR = w.dR + (i - i0) * 128;
                            v.sc_near = sc_near; v.sc_far = sc_far;
                            hipLaunchKernelGGL((jq_visit_kernel<2, true>), vgrid, dim3(64 * JQ_ROWS), lds_bytes, stream, v);
                            ONECOMP_CHECK_LAUNCH();
                            if ((st = dsplit(v.dR, v.ldr, 128, v.col0, JQ_NEAR0, sc_near,
                                             w.sc + 1 + ((n_visit + 1) & 1))) != ONECOMP_OK)
                                return st;
                            if ((st = update_to(w.Am, JQ_NEAR0, 128, v.col0, sb0, sb1, sc_near)) != ONECOMP_OK) return st;
                        }
                        if ((st = dsplit(w.dR, v.ldr, sb1 - sb0, sb0, 0, sc_far, w.sc + 3 + ((n_sb + 1) & 1))) != ONECOMP_OK)
                            return st;
                        if ((st = update_to(w.Am, 0, sb1 - sb0, sb0, g0, sb0, sc_far)) != ONECOMP_OK) return st;
                        if ((st = update_to(w.Am, 0, sb1 - sb0, sb0, sb1, g0 + G, sc_far)) != ONECOMP_OK) return st;
                    }
                    hipLaunchKernelGGL(jq_scan_end_kernel, dim3(unsigned(ceil_div(d_out, 256))), dim3(256), 0, stream,
                                       int(d_out), w.flags);
                    ONECOMP_CHECK_LAUNCH();
                }
                hipLaunchKernelGGL(jq_wide_end_kernel, rgrid, dim3(256), 0, stream, int(d_out), int(d_in), Q, scales, zeros,
                                   n_g, g, G, perm, w.d, w.bc, w.R, w.sc + 6);
                ONECOMP_CHECK_LAUNCH();
                if ((st = dsplit(w.R + g0, d_in, G, g0, 0, w.sc + 6, w.sc + 5)) != ONECOMP_OK) return st;
                if ((st = update(0, G, g0, 0, int(d_in), w.sc + 6)) != ONECOMP_OK) return st;
            }
    }
    hipLaunchKernelGGL(jq_objective_kernel, rgrid, dim3(256), 0, stream, W, bf16, int(d_out), int(d_in), Q, scales, zeros,
                       G, n_g, perm, w.Gm, w.d, w.rowf, W_hat);
    ONECOMP_CHECK_LAUNCH();
    hipLaunchKernelGGL(jq_total_kernel, dim3(1), dim3(1024), 0, stream, w.rowf, int(d_out), objective + 1);
    ONECOMP_CHECK_LAUNCH();
    return ONECOMP_OK;
}

}  // namespace onecomp
