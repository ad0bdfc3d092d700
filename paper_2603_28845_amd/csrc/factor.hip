// Damping, activation ordering and the Cholesky-based inverse factor (Sec. 4.2.1 of the paper:
// lambda = eta * mean(diag H), Cholesky of H + lambda I; Sec. 4.2: optional "actorder").
//
// Wanted: upper-triangular U, positive diagonal, U^T U = Hd^-1 for the damped (permuted) matrix Hd.
// Route: let R be Hd with both index orders reversed, R = L L^T its lower Cholesky factor and
// V = L^-1.  Reversing a lower-triangular matrix gives an upper-triangular one, so
// Hd = M M^T with M = rev(L) upper, and U = M^-1 = rev(V):  U[i][k] = V[n-1-i][n-1-k].
// One Cholesky plus one triangular inverse (2 n^3 / 3 flops), all in fp64; U is rounded once to fp32.
//
// gfx950 design
//   * blocked right-looking Cholesky, block 128: diagonal block factored (and inverted) inside one
//     workgroup's LDS; panel solve and trailing update are fp64 MFMA GEMMs (v_mfma_f64_16x16x4_f64),
//     128 x 128 tile per workgroup, LDS double-buffered.
//   * triangular inverse by recursive doubling over aligned block pairs: for block size s = 128 * 2^l,
//     V[C,A] = -V[C,C] (L[C,A] V[A,A]); every level is two batched GEMMs, so the whole inverse is
//     ~2 log2(n/128) large launches instead of n/128 skinny ones.
//   * ordering by rank counting (stable, deterministic), no floating-point atomics anywhere.
#include "common.hpp"

namespace onecomp {
namespace {

constexpr int NB = 128;  // block size of the factorization (= GEMM tile side)

// ------------------------------------------------------------------------------------------
// small preparation kernels
// ------------------------------------------------------------------------------------------
// diag -> keys (original diagonal), dfix (dead channels -> 1), lambda = damp * mean(dfix).  One workgroup.
__global__ __launch_bounds__(1024) void prep_diag_kernel(const float* __restrict__ H, int n, double damp,
                                                        float* __restrict__ keys, double* __restrict__ dfix,
                                                        double* __restrict__ lam, int32_t* __restrict__ info) {
    __shared__ double part[1024];
    double s = 0.0;
    for (int i = threadIdx.x; i < n; i += 1024) {
        float h = H[int64_t(i) * n + i];
        keys[i] = h;
        double d = (h == 0.0f) ? 1.0 : double(h);
        dfix[i] = d;
        s += d;  // fixed order per thread
    }
    part[threadIdx.x] = s;
    __syncthreads();
    for (int w = 512; w > 0; w >>= 1) {
        if (threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        *lam = damp * (part[0] / double(n));
        *info = 0;
    }
}

// perm: act_order ? stable descending order of keys : identity.  rank by counting.
__global__ __launch_bounds__(256) void order_kernel(const float* __restrict__ keys, int n, int act_order,
                                                   int32_t* __restrict__ perm, int32_t* __restrict__ perm_out) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    int pos = i;
    if (act_order) {
        const float ki = keys[i];
        int rank = 0;
        for (int k = 0; k < n; ++k) {
            const float kk = keys[k];
            rank += (kk > ki) || (kk == ki && k < i);
        }
        pos = rank;
    }
    perm[pos] = i;
    if (perm_out) perm_out[pos] = i;
}

// A[r][c] = Hd[p[n-1-r]][p[n-1-c]] in fp64 (reversed, permuted, damped); upper triangle of H is read.
__global__ __launch_bounds__(256) void build_kernel(const float* __restrict__ H, int n,
                                                   const int32_t* __restrict__ perm,
                                                   const double* __restrict__ dfix, const double* __restrict__ lam,
                                                   double* __restrict__ A) {
    const int c = blockIdx.x * 256 + threadIdx.x;
    const int r = blockIdx.y;
    if (c >= n) return;
    const int i = perm[n - 1 - r], k = perm[n - 1 - c];
    double v;
    if (i == k) v = dfix[i] + *lam;
    else v = double(H[int64_t(min(i, k)) * n + max(i, k)]);
    A[int64_t(r) * n + c] = v;
}

// U[i][k] = float(V[n-1-i][n-1-k]) for k >= i, 0 below the diagonal.
__global__ __launch_bounds__(256) void output_kernel(const double* __restrict__ V, int n, float* __restrict__ U) {
    const int k = blockIdx.x * 256 + threadIdx.x;
    const int i = blockIdx.y;
    if (k >= n) return;
    float u = 0.f;
    if (k >= i) u = float(V[int64_t(n - 1 - i) * n + (n - 1 - k)]);
    U[int64_t(i) * n + k] = u;
}

// ------------------------------------------------------------------------------------------
// diagonal block: Cholesky in LDS, then in-place triangular inverse.  One workgroup of 256 threads.
// A block (bs x bs, bs <= 128) at A + off*(n+1); L written back to A (lower part), L^-1 to V (full block,
// zeros above the diagonal).  A non-positive pivot sets *info (first one wins) and is replaced by 1.
//
// Both halves work on 16-wide sub-blocks so that the number of workgroup barriers is ~60 instead of one or
// more per column: the 16 x 16 diagonal sub-block is factored by a single wave (in-order LDS traffic, no
// workgroup barrier), rows below it are solved one thread per row in registers, the trailing part gets a
// rank-16 update.  Square roots and reciprocals come from v_rsq_f64 plus two Newton steps.
// ------------------------------------------------------------------------------------------
constexpr int SBW = 16;      // sub-block width
// LDS layout of the block: only the sub-blocks on and below the diagonal are stored, 16 x 16 each with a row
// pitch of 17 doubles, block row after block row (36 sub-blocks, 78 KB): small enough for two workgroups per CU,
// so the factorization can share a launch with GEMM tiles.
constexpr int SBP = SBW + 1;
constexpr int SBS = SBW * SBP;
constexpr int POTRF_LDS_DOUBLES = (NB / SBW) * (NB / SBW + 1) / 2 * SBS + NB;   // + NB reciprocal diagonal entries
__device__ __forceinline__ int tri(int r, int c) {   // element (r, c), c / 16 <= r / 16
    const int rb = r >> 4, cb = c >> 4;
    return ((rb * (rb + 1)) / 2 + cb) * SBS + (r & 15) * SBP + (c & 15);
}

__device__ inline double rsqrt_refined(double p) {
    double y = __builtin_amdgcn_rsq(p);
    const double h = 0.5 * p;
    y = y * __builtin_fma(-h * y, y, 1.5);
    y = y * __builtin_fma(-h * y, y, 1.5);
    return y;
}

// S: POTRF_LDS_DOUBLES doubles of LDS.  preloaded: the block (lower sub-blocks, identity padding beyond bs) is
// already in S and a barrier has been passed.
__device__ __forceinline__ void potrf_body(double* __restrict__ A, double* __restrict__ V, int n, int off, int bs,
                                           int32_t* __restrict__ info, double* S, bool preloaded) {
    double* dinv = S + POTRF_LDS_DOUBLES - NB;
    const int tid = threadIdx.x;
    if (!preloaded) {
        for (int e = tid; e < NB * NB; e += 256) {
            const int r = e / NB, c = e % NB;
            if ((c >> 4) > (r >> 4)) continue;
            double v = (r == c) ? 1.0 : 0.0;   // identity padding for a short last block
            if (r < bs && c < bs) v = A[int64_t(off + r) * n + off + c];
            S[tri(r, c)] = v;
        }
        __syncthreads();
    }

    // ---------------- Cholesky, 8 panels of 16 columns ----------------
    for (int c0 = 0; c0 < NB; c0 += SBW) {
        // (a1) diagonal 16 x 16 sub-block: wave 0, lane i (mod 16) = row c0 + i, row segment in registers;
        // lanes exchange finished entries with wave shuffles, so no LDS traffic or barrier is needed inside.
        // (Lanes 16..63 shadow lanes 0..15 so that every shuffle source is active; they store nothing.)
        if (tid < 64) {
            const int i = tid & 15;
            double r[SBW];
            double my_dinv = 1.0;
#pragma unroll
            for (int c = 0; c < SBW; ++c) r[c] = S[tri(c0 + i, c0 + c)];
#pragma unroll
            for (int j = 0; j < SBW; ++j) {
                double p = r[j];                       // meaningful in lane j only
                const bool bad = !(p > 0.0);
                if (bad) p = 1.0;
                const double ri = rsqrt_refined(p);
                double sq = p * ri;
                sq = __builtin_fma(0.5 * ri, __builtin_fma(-sq, sq, p), sq);
                const double ri_j = __shfl(ri, j, 16);
                if (i == j) {
                    if (bad && tid == j && *info == 0) *info = off + c0 + j + 1;
                    r[j] = sq;
                    my_dinv = ri;
                }
                const double lij = r[j] * ri_j;        // l_ij for rows below the pivot
                if (i > j) r[j] = lij;
#pragma unroll
                for (int c = j + 1; c < SBW; ++c) {
                    const double lcj = __shfl(lij, c, 16);
                    if (i >= c) r[c] = __builtin_fma(-lij, lcj, r[c]);
                }
            }
            if (tid < SBW) {
                dinv[c0 + i] = my_dinv;
#pragma unroll
                for (int c = 0; c < SBW; ++c)
                    if (c <= i) S[tri(c0 + i, c0 + c)] = r[c];
            }
        }
        __syncthreads();
        // (a2) rows below the sub-block: x_j = (a_ij - sum_{m<j} x_m L[j][m]) / L[j][j], one thread per row
        {
            const int i = c0 + SBW + tid;
            if (i < NB) {
                double x[SBW];
#pragma unroll
                for (int c = 0; c < SBW; ++c) x[c] = S[tri(i, c0 + c)];
#pragma unroll
                for (int j = 0; j < SBW; ++j) {
                    double acc = x[j];
#pragma unroll
                    for (int m = 0; m < j; ++m) acc = __builtin_fma(-x[m], S[tri(c0 + j, c0 + m)], acc);
                    x[j] = acc * dinv[c0 + j];
                }
#pragma unroll
                for (int c = 0; c < SBW; ++c) S[tri(i, c0 + c)] = x[c];
            }
        }
        __syncthreads();
        // (b) rank-16 update of the trailing lower triangle: S[i][c] -= sum_m L[i][c0+m] L[c][c0+m]
        {
            const int t0 = c0 + SBW;
            for (int i = t0 + (tid >> 4); i < NB; i += 16) {
                double li[SBW];
#pragma unroll
                for (int m = 0; m < SBW; ++m) li[m] = S[tri(i, c0 + m)];
                for (int c = t0 + (tid & 15); c <= i; c += 16) {
                    double acc = S[tri(i, c)];
#pragma unroll
                    for (int m = 0; m < SBW; ++m) acc = __builtin_fma(-li[m], S[tri(c, c0 + m)], acc);
                    S[tri(i, c)] = acc;
                }
            }
        }
        __syncthreads();
    }
    for (int e = tid; e < bs * NB; e += 256) {
        const int r = e / NB, c = e % NB;
        if (c <= r) A[int64_t(off + r) * n + off + c] = S[tri(r, c)];
    }
    __syncthreads();

    // ---------------- X = L^-1 in place, 16 x 16 sub-blocks ----------------
    // diagonal sub-blocks: thread t < 128 solves column t of its sub-block by forward substitution
    {
        double x[SBW];
        const int b0 = (tid >> 4) * SBW, c = tid & 15;
        if (tid < NB) {
#pragma unroll
            for (int i = 0; i < SBW; ++i) {
                double acc = (i == c) ? 1.0 : 0.0;
#pragma unroll
                for (int m = 0; m < i; ++m)
                    if (m >= c) acc = __builtin_fma(-S[tri(b0 + i, b0 + m)], x[m], acc);
                x[i] = (i >= c) ? acc * dinv[b0 + i] : 0.0;
            }
        }
        __syncthreads();
        if (tid < NB) {
#pragma unroll
            for (int i = 0; i < SBW; ++i)
                if (i >= c) S[tri(b0 + i, b0 + c)] = x[i];
        }
        __syncthreads();
    }
    // block rows top to bottom: X_ij = -X_ii * sum_{m=j}^{i-1} L_im X_mj  (j < i).  Row i of S still holds L_im.
    for (int ib = 1; ib < NB / SBW; ++ib) {
        const int i0 = ib * SBW;
        const int n_out = SBW * i0;            // outputs of this block row: 16 rows x i0 columns
        double t[7];                           // <= 7 outputs per thread (16 * 112 / 256)
#pragma unroll
        for (int q = 0; q < 7; ++q) {
            const int e = tid + 256 * q;
            t[q] = 0.0;
            if (e < n_out) {
                const int r = e / i0, c = e % i0;          // row i0 + r, column c
                double acc = 0.0;                          // X[m][c] is zero for m < c
                for (int m = c; m < i0; ++m) acc = __builtin_fma(S[tri(i0 + r, m)], S[tri(m, c)], acc);
                t[q] = acc;
            }
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < 7; ++q) {
            const int e = tid + 256 * q;
            if (e < n_out) S[tri(i0 + e / i0, e % i0)] = t[q];
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < 7; ++q) {
            const int e = tid + 256 * q;
            t[q] = 0.0;
            if (e < n_out) {
                const int r = e / i0, c = e % i0;
                double acc = 0.0;
#pragma unroll
                for (int m = 0; m < SBW; ++m)
                    if (m <= r) acc = __builtin_fma(S[tri(i0 + r, i0 + m)], S[tri(i0 + m, c)], acc);
                t[q] = -acc;
            }
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < 7; ++q) {
            const int e = tid + 256 * q;
            if (e < n_out) S[tri(i0 + e / i0, e % i0)] = t[q];
        }
        __syncthreads();
    }
    for (int e = tid; e < bs * bs; e += 256) {
        const int r = e / bs, c = e % bs;
        V[int64_t(off + r) * n + off + c] = (c <= r) ? S[tri(r, c)] : 0.0;
    }
}

// ------------------------------------------------------------------------------------------
// fp64 MFMA GEMM:  C = alpha * A * op(B) + beta * C   (batched, optional triangular structure)
// ------------------------------------------------------------------------------------------
constexpr int GT = 128;  // tile side
constexpr int GK = 16;   // K per LDS stage
constexpr int GPA = GK + 1;
constexpr int GPB = GT + 4;
constexpr int GSB = GT * GPA;  // >= GK * GPB

enum : int { G_BTRANS = 1, G_ALOWER = 2, G_BLOWER = 4, G_CLOWER = 8 };

struct GemmArgs {
    const double* A; int64_t lda, sa;
    const double* B; int64_t ldb, sb;
    double* C; int64_t ldc, sc;
    int m, n, k;   // sizes of every batch entry but the last
    int m_last;    // rows of the last batch entry (<= m)
    int k_last;    // inner size of the last batch entry (<= k)
    int batch;
    double alpha, beta;
    int flags;
};

constexpr int GEMM_LDS_DOUBLES = 2 * GT * GPA + 2 * GSB;
constexpr int LDS_DOUBLES = GEMM_LDS_DOUBLES > POTRF_LDS_DOUBLES ? GEMM_LDS_DOUBLES : POTRF_LDS_DOUBLES;

// The workgroup's LDS: one static array per kernel, shared by the GEMM tile code and the factorization code.
__device__ __forceinline__ double* wg_lds() {
    __shared__ double lds[LDS_DOUBLES];
    return lds;
}

// One 128 x 128 tile (tm, tn) of batch entry z.  tri_out: the finished tile is also left in LDS (from its start,
// over the dead operand tiles) in the layout of potrf_body (lower sub-blocks, identity beyond the matrix edge),
// for a diagonal tile that the same workgroup factors next.
template <bool bt>   // B is given transposed (n x k, k contiguous)
__device__ __forceinline__ void dgemm_tile(const GemmArgs& g, const int tn, const int tm, const int z,
                                           const bool tri_out) {
    double* lds = wg_lds();
    double(*sA)[GT * GPA] = reinterpret_cast<double(*)[GT * GPA]>(lds);
    double(*sB)[GSB] = reinterpret_cast<double(*)[GSB]>(lds + 2 * GT * GPA);
    const bool last = (z == g.batch - 1);
    const int m = last ? g.m_last : g.m;
    const int kdim = last ? g.k_last : g.k;
    if (tm * GT >= m) return;
    if ((g.flags & G_CLOWER) && tn > tm) return;
    const double* __restrict__ A = g.A + z * g.sa;
    const double* __restrict__ B = g.B + z * g.sb;
    double* __restrict__ C = g.C + z * g.sc;
    int k_lo = 0, k_hi = kdim;
    if (g.flags & G_BLOWER) k_lo = tn * GT;
    if (g.flags & G_ALOWER) k_hi = min(kdim, (tm + 1) * GT);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1;
    const int m0 = tm * GT, n0 = tn * GT;

    // loaders: A-form tile (rows x GK, k contiguous): row = tid/2, 8 doubles at k = (tid%2)*8
    //          NN B tile (GK x cols): krow = tid/16, 8 doubles at col (tid%16)*8
    const int a_row = tid >> 1, a_k = (tid & 1) * 8;
    const int b_kr = tid >> 4, b_c = (tid & 15) * 8;
    double ra[8], rb[8];
    auto gload = [&](int k0) {
        {
            const int r = m0 + a_row, kk = k0 + a_k;
            const bool ok = (r < m) && (kk < k_hi);
            const double2* p = reinterpret_cast<const double2*>(A + int64_t(r) * g.lda + kk);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                double2 v = ok ? p[e] : make_double2(0.0, 0.0);
                ra[2 * e] = v.x; ra[2 * e + 1] = v.y;
            }
        }
        if (bt) {
            const int r = n0 + a_row, kk = k0 + a_k;
            const bool ok = (r < g.n) && (kk < k_hi);
            const double2* p = reinterpret_cast<const double2*>(B + int64_t(r) * g.ldb + kk);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                double2 v = ok ? p[e] : make_double2(0.0, 0.0);
                rb[2 * e] = v.x; rb[2 * e + 1] = v.y;
            }
        } else {
            const int kk = k0 + b_kr, c = n0 + b_c;
            const bool ok = (kk < k_hi) && (c < g.n);
            const double2* p = reinterpret_cast<const double2*>(B + int64_t(kk) * g.ldb + c);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                double2 v = ok ? p[e] : make_double2(0.0, 0.0);
                rb[2 * e] = v.x; rb[2 * e + 1] = v.y;
            }
        }
    };
    auto lstore = [&](int st) {
#pragma unroll
        for (int e = 0; e < 8; ++e) sA[st][a_row * GPA + a_k + e] = g.alpha * ra[e];   // alpha folded into A
        if (bt) {
#pragma unroll
            for (int e = 0; e < 8; ++e) sB[st][a_row * GPA + a_k + e] = rb[e];
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) sB[st][b_kr * GPB + b_c + e] = rb[e];
        }
    };

    const int l16 = lane & 15, lk = lane >> 4;
    if (k_lo < k_hi) gload(k_lo);
    // accumulators start as beta * C (register r of lane l: row 4 r + l / 16, column l % 16 of its 16 x 16 tile),
    // so the C tile is in flight together with the first operand tiles
    double4v acc[4][4];
    const bool full = (m0 + GT <= m) && (n0 + GT <= g.n);   // uniform: interior tiles need no per-element masks
    double* __restrict__ ct = C + int64_t(m0 + wr * 64 + lk) * g.ldc + n0 + wc * 64 + l16;
    if (g.beta == 0.0) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.0;
    } else if (full) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[i][j][r] = g.beta * ct[int64_t(i * 16 + 4 * r) * g.ldc + j * 16];
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = m0 + wr * 64 + i * 16 + 4 * r + lk;
                    const int col = n0 + wc * 64 + j * 16 + l16;
                    double c = 0.0;
                    if (row < m && col < g.n) c = g.beta * C[int64_t(row) * g.ldc + col];
                    acc[i][j][r] = c;
                }
    }

    if (k_lo < k_hi) lstore(0);
    __syncthreads();
    int st = 0;
    for (int k0 = k_lo; k0 < k_hi; k0 += GK) {
        const bool more = (k0 + GK < k_hi);
        if (more) gload(k0 + GK);
#pragma unroll
        for (int k4 = 0; k4 < GK; k4 += 4) {
            double a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = sA[st][(wr * 64 + i * 16 + l16) * GPA + k4 + lk];
#pragma unroll
            for (int j = 0; j < 4; ++j)
                b[j] = bt ? sB[st][(wc * 64 + j * 16 + l16) * GPA + k4 + lk]
                          : sB[st][(k4 + lk) * GPB + wc * 64 + j * 16 + l16];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        if (more) lstore(st ^ 1);
        __syncthreads();
        st ^= 1;
    }

    // accumulator register r of lane l: row 4 r + l / 16, column l % 16 of its 16 x 16 tile
    if (full) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) ct[int64_t(i * 16 + 4 * r) * g.ldc + j * 16] = acc[i][j][r];
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = m0 + wr * 64 + i * 16 + 4 * r + lk;
                    const int col = n0 + wc * 64 + j * 16 + l16;
                    if (row < m && col < g.n) C[int64_t(row) * g.ldc + col] = acc[i][j][r];
                }
    }
    if (tri_out) {   // uniform; the K loop ended with a barrier, so the operand tiles are dead
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int lrow = wr * 64 + i * 16 + 4 * r + lk, lcol = wc * 64 + j * 16 + l16;
                    if ((lcol >> 4) > (lrow >> 4)) continue;
                    const bool inside = (m0 + lrow < m) && (n0 + lcol < g.n);
                    lds[tri(lrow, lcol)] = inside ? acc[i][j][r] : (lrow == lcol ? 1.0 : 0.0);
                }
    }
}

template <bool bt>
__global__ __launch_bounds__(256, 2) void dgemm_kernel(GemmArgs g) {
    dgemm_tile<bt>(g, blockIdx.x, blockIdx.y, blockIdx.z, false);
}

__global__ __launch_bounds__(256) void potrf_diag_kernel(double* __restrict__ A, double* __restrict__ V, int n,
                                                        int off, int bs, int32_t* __restrict__ info) {
    potrf_body(A, V, n, off, bs, info, wg_lds(), false);
}

// Trailing update of one step of the blocked Cholesky together with the factorization of the next diagonal block:
// workgroup (0, 0), the first of the grid and therefore resident from the start, computes the updated diagonal
// tile, keeps it in LDS and factors / inverts it while the other workgroups update the rest of the trailing
// matrix.  Takes the single-workgroup factorization off the critical path of every step whose update is longer.
__global__ __launch_bounds__(256, 2) void syrk_potrf_kernel(GemmArgs g, double* __restrict__ A, double* __restrict__ V,
                                                           int n, int off, int bs, int32_t* __restrict__ info) {
    const bool first = (blockIdx.x == 0 && blockIdx.y == 0);
    dgemm_tile<true>(g, blockIdx.x, blockIdx.y, 0, first);
    if (first) {
        __syncthreads();
        potrf_body(A, V, n, off, bs, info, wg_lds(), true);
    }
}

onecomp_status dgemm(const GemmArgs& g, hipStream_t stream) {
    if (g.m <= 0 || g.n <= 0 || g.batch <= 0) return ONECOMP_OK;
    dim3 grid(unsigned(ceil_div(g.n, GT)), unsigned(ceil_div(g.m, GT)), unsigned(g.batch));
    if (g.flags & G_BTRANS) hipLaunchKernelGGL(dgemm_kernel<true>, grid, dim3(256), 0, stream, g);
    else hipLaunchKernelGGL(dgemm_kernel<false>, grid, dim3(256), 0, stream, g);
    ONECOMP_CHECK_LAUNCH();
    return ONECOMP_OK;
}

struct Workspace {
    double* A;      // n x n: reversed damped matrix, then L in its lower triangle
    double* V;      // n x n: L^-1 (lower)
    double* T;      // n x n: temporaries of the inverse
    double* dfix;   // n
    double* lam;    // 1
    float* keys;    // n
    int32_t* perm;  // n
};

Workspace carve(void* ws, int64_t n) {
    char* p = static_cast<char*>(ws);
    const size_t mat = align_up(size_t(n) * n * sizeof(double), 256);
    Workspace w;
    w.A = reinterpret_cast<double*>(p); p += mat;
    w.V = reinterpret_cast<double*>(p); p += mat;
    w.T = reinterpret_cast<double*>(p); p += mat;
    w.dfix = reinterpret_cast<double*>(p); p += align_up(size_t(n) * sizeof(double), 256);
    w.lam = reinterpret_cast<double*>(p); p += 256;
    w.keys = reinterpret_cast<float*>(p); p += align_up(size_t(n) * sizeof(float), 256);
    w.perm = reinterpret_cast<int32_t*>(p);
    return w;
}

}  // namespace

size_t factor_workspace_bytes(int64_t n) {
    return 3 * align_up(size_t(n) * n * sizeof(double), 256) + align_up(size_t(n) * sizeof(double), 256) + 256 +
           2 * align_up(size_t(n) * sizeof(float), 256);
}

onecomp_status factor_run(const float* H, int64_t d_in, float damp, int act_order, int32_t* perm_out, float* U,
                          int32_t* info, void* workspace, hipStream_t stream) {
    const int n = int(d_in);
    Workspace w = carve(workspace, n);
    onecomp_status st;

    hipLaunchKernelGGL(prep_diag_kernel, dim3(1), dim3(1024), 0, stream, H, n, double(damp), w.keys, w.dfix, w.lam,
                       info);
    ONECOMP_CHECK_LAUNCH();
    hipLaunchKernelGGL(order_kernel, dim3(unsigned(ceil_div(n, 256))), dim3(256), 0, stream, w.keys, n, act_order,
                       w.perm, perm_out);
    ONECOMP_CHECK_LAUNCH();
    hipLaunchKernelGGL(build_kernel, dim3(unsigned(ceil_div(n, 256)), unsigned(n)), dim3(256), 0, stream, H, n,
                       w.perm, w.dfix, w.lam, w.A);
    ONECOMP_CHECK_LAUNCH();

    // ---- blocked right-looking Cholesky of A (lower) ----
    // diagonal block 0 on its own; every later one inside the launch that updates the trailing matrix before it
    const int nblk = int(ceil_div(n, NB));
    hipLaunchKernelGGL(potrf_diag_kernel, dim3(1), dim3(256), 0, stream, w.A, w.V, n, 0, min(NB, n), info);
    ONECOMP_CHECK_LAUNCH();
    for (int kb = 0; kb < nblk; ++kb) {
        const int off = kb * NB;
        const int bs = min(NB, n - off);
        const int rest = n - off - bs;
        if (rest <= 0) break;
        // panel: A[off+bs:, off:off+bs] <- A[off+bs:, off:off+bs] * Linv_kk^T   (in place, one column tile)
        GemmArgs p{};
        p.A = w.A + int64_t(off + bs) * n + off; p.lda = n; p.sa = 0;
        p.B = w.V + int64_t(off) * n + off; p.ldb = n; p.sb = 0;
        p.C = w.A + int64_t(off + bs) * n + off; p.ldc = n; p.sc = 0;
        p.m = rest; p.m_last = rest; p.n = bs; p.k = bs; p.k_last = bs; p.batch = 1;
        p.alpha = 1.0; p.beta = 0.0; p.flags = G_BTRANS;
        if ((st = dgemm(p, stream)) != ONECOMP_OK) return st;
        // trailing: A[i][j] -= P[i] P[j]^T on the lower tiles
        GemmArgs s{};
        s.A = p.C; s.lda = n; s.sa = 0;
        s.B = p.C; s.ldb = n; s.sb = 0;
        s.C = w.A + int64_t(off + bs) * n + (off + bs); s.ldc = n; s.sc = 0;
        s.m = rest; s.m_last = rest; s.n = rest; s.k = bs; s.k_last = bs; s.batch = 1;
        s.alpha = -1.0; s.beta = 1.0; s.flags = G_BTRANS | G_CLOWER;
        {
            const int off1 = off + bs;
            dim3 grid(unsigned(ceil_div(rest, GT)), unsigned(ceil_div(rest, GT)), 1);
            hipLaunchKernelGGL(syrk_potrf_kernel, grid, dim3(256), 0, stream, s, w.A, w.V, n, off1, min(NB, n - off1),
                               info);
            ONECOMP_CHECK_LAUNCH();
        }
    }

    // ---- V = L^-1 by recursive doubling over aligned block pairs ----
    for (int64_t s = NB; s < n; s *= 2) {
        const int64_t pairs = ceil_div(n, 2 * s);
        // last pair may have a short or empty C range
        int64_t m_last = n - ((pairs - 1) * 2 * s + s);
        int64_t batch = pairs;
        if (m_last <= 0) { batch = pairs - 1; m_last = s; }
        if (batch <= 0) continue;
        if (m_last > s) m_last = s;
        const int64_t stride = 2 * s * (int64_t(n) + 1);
        // T[C,A] = L[C,A] * V[A,A]        (V[A,A] lower triangular)
        GemmArgs a{};
        a.A = w.A + s * n; a.lda = n; a.sa = stride;
        a.B = w.V; a.ldb = n; a.sb = stride;
        a.C = w.T + s * n; a.ldc = n; a.sc = stride;
        a.m = int(s); a.m_last = int(m_last); a.n = int(s); a.k = int(s); a.k_last = int(s); a.batch = int(batch);
        a.alpha = 1.0; a.beta = 0.0; a.flags = G_BLOWER;
        if ((st = dgemm(a, stream)) != ONECOMP_OK) return st;
        // V[C,A] = -V[C,C] * T[C,A]       (V[C,C] lower triangular)
        GemmArgs b{};
        b.A = w.V + s * (int64_t(n) + 1); b.lda = n; b.sa = stride;
        b.B = w.T + s * n; b.ldb = n; b.sb = stride;
        b.C = w.V + s * n; b.ldc = n; b.sc = stride;
        b.m = int(s); b.m_last = int(m_last); b.n = int(s); b.k = int(s); b.k_last = int(m_last); b.batch = int(batch);
        b.alpha = -1.0; b.beta = 0.0; b.flags = G_ALOWER;
        if ((st = dgemm(b, stream)) != ONECOMP_OK) return st;
    }

    hipLaunchKernelGGL(output_kernel, dim3(unsigned(ceil_div(n, 256)), unsigned(n)), dim3(256), 0, stream, w.V, n, U);
    ONECOMP_CHECK_LAUNCH();
    return ONECOMP_OK;
}

}  // namespace onecomp
