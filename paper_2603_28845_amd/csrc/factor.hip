// Damping, activation ordering and the Cholesky-based inverse factor (Sec. 4.3.1 of the paper:
// lambda = eta * mean(diag H), Cholesky of H + lambda I; Sec. 4.3: optional "actorder").
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
//     128 x 128 tile per workgroup, operands streamed global -> LDS directly through a four-slot ring; a launch
//     has one workgroup per tile that has work, the longest tiles first.
//   * triangular inverse by recursive doubling over aligned block pairs: for block size s = 128 * 2^l,
//     V[C,A] = -V[C,C] (L[C,A] V[A,A]); every level is two batched GEMMs, so the whole inverse is
//     ~2 log2(n/128) large launches instead of n/128 skinny ones.
//   * ordering by rank counting (stable, deterministic), no floating-point atomics anywhere.
#include "common.hpp"
#include "planner.hpp"
#include <type_traits>

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

// A[r][c] = Hd[p[n-1-r]][p[n-1-c]] in fp64 (reversed, permuted, damped); upper triangle of H is read.  Only the
// 128 x 128 blocks on and below the diagonal are written: the factorization never reads the others, and in natural
// order those are the ones whose source rows are read along the row.
__global__ __launch_bounds__(256) void build_kernel(const float* __restrict__ H, int n,
                                                   const int32_t* __restrict__ perm,
                                                   const double* __restrict__ dfix, const double* __restrict__ lam,
                                                   double* __restrict__ A) {
    const int c = blockIdx.x * 256 + threadIdx.x;
    const int r = blockIdx.y;
    if (c >= n || c / NB > r / NB) return;
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

// Block form (no triangular inverse of the whole factor).  With R = U^-1, i.e. R[i][k] = L[n-1-i][n-1-k] and
// Hd = R R^T:  F = U on the NB x NB diagonal blocks (the index-reversed inverses of the diagonal blocks of L, which
// the factorization leaves in V);  F[i][k] = -U_ii R_ik / R_kk where i and k lie in different blocks.
// rdiag[r] = 1 / L[r][r] = V[r][r].
__global__ __launch_bounds__(256) void rdiag_kernel(const double* __restrict__ V, int n, double* __restrict__ rdiag) {
    const int r = blockIdx.x * 256 + threadIdx.x;
    if (r < n) rdiag[r] = V[int64_t(r) * n + r];
}

__global__ __launch_bounds__(256) void output_block_kernel(const double* __restrict__ L, const double* __restrict__ V,
                                                          const double* __restrict__ rdiag, int n,
                                                          float* __restrict__ F) {
    const int k = blockIdx.x * 256 + threadIdx.x;
    const int i = blockIdx.y;
    if (k >= n) return;
    float f = 0.f;
    if (k >= i) {
        const int ri = n - 1 - i, rk = n - 1 - k;   // ri >= rk
        if (ri / NB == rk / NB) f = float(V[int64_t(ri) * n + rk]);
        else f = float(-(rdiag[ri] * rdiag[rk]) * L[int64_t(ri) * n + rk]);
    }
    F[int64_t(i) * n + k] = f;
}

// ------------------------------------------------------------------------------------------
// diagonal block: Cholesky in LDS, then in-place triangular inverse.  One workgroup of 256 threads (4 waves).
// A block (bs x bs, bs <= 128) at A + off*(n+1); L^-1 is written to V (full block, zeros above the diagonal); the
// factor L_kk of the block itself stays in LDS (nothing downstream reads it).  A non-positive pivot sets *info (first one wins) and is replaced by 1.
//
// The block lives in LDS as 16 x 16 sub-blocks (only those on and below the diagonal, 36 of them, row pitch 17
// doubles, 76.5 KB: small enough for two workgroups per CU, so the factorization can share a launch with GEMM
// tiles).  Everything but the 16 x 16 leaves runs on v_mfma_f64_16x16x4_f64 with sub-blocks as operands:
//   Cholesky, block column J:  leaf factorization of (J,J) by wave 0 in registers (pivot and column broadcasts
//     by DPP row_newbcast, reciprocal square roots from v_rsq_f64 + a Newton step), which leaves T = L_JJ^-1 in the
//     sub-block's place;  L_IJ = A_IJ T^T for the sub-blocks below;  A_IK -= L_IJ L_KJ^T for J < K <= I, of which
//     wave 0 takes (J+1, J+1) alone and goes straight on to the next leaf while the other waves do the rest.
//   Inverse:  the diagonal sub-blocks hold their inverses already; recursive doubling over aligned pairs of
//     s = 16, 32, 64:  X[C,A] = -X[C,C] (L[C,A] X[A,A]), both products in place: the first by sub-block rows
//     (a wave holds its row of L[C,A] in registers while it overwrites it), the second by sub-block columns.
//     Every level has exactly four row / column tasks: one per wave.
// MFMA operand layouts (lane l): A[i][k]: i = l % 16, k = l / 16;  B[k][j]: k = l / 16, j = l % 16;
// C/D register r: row 4 r + l / 16, column l % 16.
// ------------------------------------------------------------------------------------------
constexpr int SBW = 16;      // sub-block width
constexpr int SBP = SBW + 1;
constexpr int SBS = SBW * SBP;
constexpr int NSB = NB / SBW;
constexpr int POTRF_LDS_DOUBLES = NSB * (NSB + 1) / 2 * SBS;   // the lower sub-blocks
__device__ __forceinline__ int tri(int r, int c) {   // element (r, c), c / 16 <= r / 16
    const int rb = r >> 4, cb = c >> 4;
    return ((rb * (rb + 1)) / 2 + cb) * SBS + (r & 15) * SBP + (c & 15);
}
__device__ __forceinline__ int sub(int I, int J) { return ((I * (I + 1)) / 2 + J) * SBS; }   // J <= I

// 1 / sqrt(p): v_rsq_f64 is good to 5e-8 relative (measured over 120 binades), one Newton step brings it to 4e-15.
// That is what scales a column of the factor; the diagonal entry itself gets a further correction step where it is
// computed.  The step sits on the dependency chain of every pivot, so there is exactly one.
__device__ inline double rsqrt_refined(double p) {
    double y = __builtin_amdgcn_rsq(p);
    const double h = 0.5 * p;
    y = y * __builtin_fma(-h * y, y, 1.5);
    return y;
}

// value of lane J of every 16-lane row, in all lanes of the row
template <int J>
__device__ __forceinline__ double bcast16(double v) {
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __builtin_amdgcn_update_dpp(0, lo, 0x150 + J, 0xF, 0xF, true);   // row_newbcast:J
    hi = __builtin_amdgcn_update_dpp(0, hi, 0x150 + J, 0xF, 0xF, true);
    return __hiloint2double(hi, lo);
}

template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// Inverse of a 16 x 16 lower-triangular block by one wave, all in registers.  Every 16-lane row of the wave holds
// the block (lane i of each row: row i of L in r[], entries above the diagonal arbitrary, 1 / L_ii in rdi); row q
// of lanes computes the columns c = 4 k + q of L^-1, so lane (q, i) returns X[i][4 k + q] in x[k], k = 0 .. 3.
// With L = Lh D (Lh = columns of L divided by their diagonal entries, unit diagonal) L^-1 = D^-1 Lh^-1: the rows of
// Z = Lh^-1 follow without divisions, z_m = e_m - sum_{k<m} Lh[m][k] z_k, row m being final once rows 0 .. m-1 have
// been eliminated from it and then broadcast inside each 16-lane row (DPP row_newbcast) to the lanes below; the
// scaling by 1 / L_ii at the end is local to the lane.  Entries of Lh on and above the diagonal are set to zero
// beforehand, so the elimination needs no per-step predicates: 40 broadcast + FMA pairs, no memory traffic.
__device__ __forceinline__ void tri_inverse16(const double (&r)[SBW], const double rdi, const int i, const int q,
                                              double (&x)[4]) {
    double lh[SBW];
    static_for<0, SBW>([&](auto mc) {
        constexpr int m = decltype(mc)::value;
        const double rdm = bcast16<m>(rdi);
        lh[m] = (i > m) ? r[m] * rdm : 0.0;
    });
#pragma unroll
    for (int k = 0; k < 4; ++k) x[k] = (4 * k + q == i) ? 1.0 : 0.0;
    static_for<0, SBW - 1>([&](auto mc) {
        constexpr int m = decltype(mc)::value;
        static_for<0, m / 4 + 1>([&](auto kc) {   // columns beyond m are still zero in row m: harmless
            constexpr int k = decltype(kc)::value;
            const double zm = bcast16<m>(x[k]);
            x[k] = __builtin_fma(-lh[m], zm, x[k]);
        });
        __builtin_amdgcn_sched_barrier(0);   // keeps the scheduler from issuing later rows' broadcasts early (registers)
    });
#pragma unroll
    for (int k = 0; k < 4; ++k) x[k] *= rdi;
}

// S: POTRF_LDS_DOUBLES doubles of LDS.  preloaded: the block (lower sub-blocks, identity padding beyond bs) is
// already in S and a barrier has been passed.
__device__ __forceinline__ void potrf_body(double* __restrict__ A, double* __restrict__ V, int n, int off, int bs,
                                           int32_t* __restrict__ info, double* S, bool preloaded) {
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, lk = lane >> 4;
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
    // operand fragments of a sub-block M (pointer to its first element), k-step q = 0..3
    auto frag_rowk = [&](const double* M, int q) __attribute__((always_inline)) {   // M[l%16][4q + l/16]
        return M[l16 * SBP + 4 * q + lk];
    };
    auto frag_krow = [&](const double* M, int q) __attribute__((always_inline)) {   // M[4q + l/16][l%16]
        return M[(4 * q + lk) * SBP + l16];
    };
    auto load_c = [&](const double* M) __attribute__((always_inline)) {
        double4v c;
#pragma unroll
        for (int r = 0; r < 4; ++r) c[r] = M[(4 * r + lk) * SBP + l16];
        return c;
    };
    auto store_c = [&](double* M, const double4v& c) __attribute__((always_inline)) {
#pragma unroll
        for (int r = 0; r < 4; ++r) M[(4 * r + lk) * SBP + l16] = c[r];
    };

    // ---------------- Cholesky, 8 block columns of 16 ----------------
    // Leaf of block column J: wave 0 factors the diagonal sub-block in registers (lane i (mod 16) = row i; lanes
    // 16..63 shadow lanes 0..15) and leaves its INVERSE in the sub-block's place: the panel solves below and the
    // inversion of the whole block need T = L_JJ^-1, nothing reads L_JJ itself.
    auto leaf = [&](int J) __attribute__((always_inline)) {
        double* DJ = S + sub(J, J);
        const int i = l16;
        // Entries above the diagonal (c > i) are carried along unmasked: they never reach a valid entry (a
        // broadcast of column j takes lane c >= j).  The first bad pivot is remembered in a register, so the 16
        // steps form one straight-line block.
        double r[SBW];
        double my_dinv = 1.0;
        int bad_at = -1;
#pragma unroll
        for (int c = 0; c < SBW; ++c) r[c] = DJ[i * SBP + c];
        static_for<0, SBW>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            double p = bcast16<j>(r[j]);           // pivot, the same in every lane
            const bool bad = !(p > 0.0);
            if (bad) p = 1.0;
            bad_at = (bad && bad_at < 0) ? j : bad_at;
            const double ri = rsqrt_refined(p);
            double sq = p * ri;
            sq = __builtin_fma(0.5 * ri, __builtin_fma(-sq, sq, p), sq);
            const double lij = (i == j) ? sq : r[j] * ri;   // column j on and below the pivot
            r[j] = lij;
            if (i == j) my_dinv = ri;
            static_for<j + 1, SBW>([&](auto cc) {
                constexpr int c = decltype(cc)::value;
                const double lcj = bcast16<c>(lij);
                r[c] = __builtin_fma(-lij, lcj, r[c]);
            });
        });
        if (bad_at >= 0 && tid == 0 && *info == 0) *info = off + J * SBW + bad_at + 1;
        // T = L_JJ^-1 from the rows still in registers (all four 16-lane rows hold them); every lane has read its
        // row before any lane overwrites the sub-block (one wave: program order); zeros above the diagonal
        double x[4];
        tri_inverse16(r, my_dinv, i, lk, x);
#pragma unroll
        for (int k = 0; k < 4; ++k) DJ[i * SBP + 4 * k + lk] = x[k];
    };
    // A_IK -= L_IJ L_KJ^T for the pair p of the sub-blocks below J (row-major over the triangle, kk <= ii)
    auto update_pair = [&](int J, int p) __attribute__((always_inline)) {
        int ii = 0;
        while ((ii + 1) * (ii + 2) / 2 <= p) ++ii;
        const int kk = p - ii * (ii + 1) / 2;
        const int I = J + 1 + ii, K = J + 1 + kk;
        double* M = S + sub(I, K);
        const double* LI = S + sub(I, J);
        const double* LK = S + sub(K, J);
        double4v c = load_c(M);
#pragma unroll
        for (int q = 0; q < 4; ++q)
            c = __builtin_amdgcn_mfma_f64_16x16x4f64(-frag_rowk(LI, q), frag_rowk(LK, q), c, 0, 0, 0);
        store_c(M, c);
    };
    // The leaves are a chain of latencies on one wave (16 dependent pivots each, then the 16 x 16 inverse), so the
    // next leaf runs beside the update it does not depend on: after the panel solve of column J, wave 0 updates the
    // next diagonal sub-block alone and factors it at once, while the other three waves update the rest.
    if (wave == 0) leaf(0);
    __syncthreads();
#pragma unroll 1
    for (int J = 0; J < NSB - 1; ++J) {
        const double* TJ = S + sub(J, J);
        // L_IJ = A_IJ T^T for I > J (in place: the wave holds A_IJ's fragments before it writes)
        for (int I = J + 1 + wave; I < NSB; I += 4) {
            double* M = S + sub(I, J);
            double a[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) a[q] = frag_rowk(M, q);
            double4v c = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
            for (int q = 0; q < 4; ++q) c = __builtin_amdgcn_mfma_f64_16x16x4f64(a[q], frag_rowk(TJ, q), c, 0, 0, 0);
            store_c(M, c);
        }
        __syncthreads();
        const int nr = NSB - 1 - J;                 // sub-block rows below J
        const int np = nr * (nr + 1) / 2;
        if (wave == 0) {
            update_pair(J, 0);                      // the next diagonal sub-block
            leaf(J + 1);
        } else {
            for (int p = wave; p < np; p += 3) update_pair(J, p);
        }
        __syncthreads();
    }
    // L_kk itself is not written back to A: nothing reads the diagonal blocks of L afterwards (the panel solve, the
    // triangular inverse and the block-form output take L_kk^-1 from V; the trailing updates and the off-diagonal
    // blocks of the inverse and of the block form read only blocks below the block diagonal).
    (void)A;

    // ---------------- X = L^-1 in place ----------------
    // the diagonal sub-blocks hold their inverses already
    // recursive doubling: ns = sub-blocks per side of a pair
    static_for<0, 3>([&](auto lc) {
        constexpr int ns = 1 << decltype(lc)::value;     // 1, 2, 4
        const int pr = wave / ns, t = wave % ns;         // pair and row / column task of this wave
        const int a0 = pr * 2 * ns, c0 = a0 + ns;        // first sub-block of A and of C
        {   // T = L[C,A] X[A,A], sub-block row I = c0 + t, in place
            const int I = c0 + t;
            double a[ns][4];
#pragma unroll
            for (int kb = 0; kb < ns; ++kb)
#pragma unroll
                for (int q = 0; q < 4; ++q) a[kb][q] = frag_rowk(S + sub(I, a0 + kb), q);
#pragma unroll
            for (int jb = 0; jb < ns; ++jb) {
                double4v c = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
                for (int kb = jb; kb < ns; ++kb)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        c = __builtin_amdgcn_mfma_f64_16x16x4f64(a[kb][q], frag_krow(S + sub(a0 + kb, a0 + jb), q), c, 0,
                                                                 0, 0);
                store_c(S + sub(I, a0 + jb), c);
            }
        }
        __syncthreads();
        {   // X[C,A] = -X[C,C] T, sub-block column a0 + t, in place
            const int Jc = a0 + t;
            double b[ns][4];
#pragma unroll
            for (int kb = 0; kb < ns; ++kb)
#pragma unroll
                for (int q = 0; q < 4; ++q) b[kb][q] = frag_krow(S + sub(c0 + kb, Jc), q);
#pragma unroll
            for (int ib = 0; ib < ns; ++ib) {
                double4v c = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
                for (int kb = 0; kb <= ib; ++kb)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        c = __builtin_amdgcn_mfma_f64_16x16x4f64(-frag_rowk(S + sub(c0 + ib, c0 + kb), q), b[kb][q], c, 0,
                                                                 0, 0);
                store_c(S + sub(c0 + ib, Jc), c);
            }
        }
        __syncthreads();
    });
    // L_kk^-1 to V (zeros above the diagonal), sub-block by sub-block: wave w takes the sub-block rows w and 7 - w
    // (eight sub-blocks each), a lane four rows of one column, so that addresses step by constants and a store
    // instruction writes four 128-byte row segments
    {
        const int rows2[2] = {wave, NSB - 1 - wave};
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int I = rows2[h];
#pragma unroll 2
            for (int J = 0; J < NSB; ++J) {
                double v[4] = {0.0, 0.0, 0.0, 0.0};
                if (J <= I) {   // uniform
                    const double* M = S + sub(I, J);
#pragma unroll
                    for (int r = 0; r < 4; ++r) v[r] = M[(4 * r + lk) * SBP + l16];
                }
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = I * SBW + 4 * r + lk, col = J * SBW + l16;
                    if (row < bs && col < bs) V[int64_t(off + row) * n + off + col] = v[r];
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// fp64 MFMA GEMM:  C = alpha * A * op(B) + beta * C   (batched, optional triangular structure)
// ------------------------------------------------------------------------------------------
constexpr int GT = 128;  // tile side

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

constexpr int RK = 8, RNS = 4;                      // inner steps per ring slot, ring slots of the GEMM tile
constexpr int R_PART_BYTES = GT * RK * 8;           // 8 KB: the A part or the B part of a stage
constexpr int R_STAGE_BYTES = 2 * R_PART_BYTES;
constexpr int GEMM_LDS_DOUBLES = RNS * R_STAGE_BYTES / 8;
constexpr int LDS_DOUBLES = GEMM_LDS_DOUBLES > POTRF_LDS_DOUBLES ? GEMM_LDS_DOUBLES : POTRF_LDS_DOUBLES;

// The workgroup's LDS: one static array per kernel, shared by the GEMM tile code and the factorization code.
__device__ __forceinline__ double* wg_lds() {
    __shared__ double lds[LDS_DOUBLES];
    return lds;
}

// ------------------------------------------------------------------------------------------
// One 128 x 128 tile (tm, tn) of batch entry z with NW waves: 4 (2 x 2 waves of 64 x 64) or 8 (2 x 4 waves of
// 64 x 32: half the accumulators per lane, so that four waves share a SIMD and cover each other's waits).
// tri_out: the finished tile is also left in LDS (from its start, over the dead operand slots) in the layout of
// potrf_body (lower sub-blocks, identity beyond the matrix edge), for a diagonal tile that the same workgroup
// factors next.
// The operands are streamed global -> LDS directly (buffer_load ... lds) through a ring of RNS slots
// of RK inner steps each, three stages ahead of the MFMAs: no staging registers, no LDS stores, no multiplication by
// alpha on the way (alpha = +-1 is folded into the accumulators: they start as (beta / alpha) C and the result is
// alpha acc, both exact), one barrier per stage.  A direct load deposits lane l at slot + 16 l, so rows cannot be
// padded; the 16-byte chunks (two doubles) are permuted instead, which costs nothing on the global side because
// every lane supplies its own address:
//   A-form part (128 rows x RK k, a row is 64 B = 4 chunks): chunk c of row r sits at position c ^ ((r >> 2) & 3);
//     the 16 rows x 2 k that one half-wave reads for an MFMA operand then fall into 64 different banks.
//   NN B part (RK k-rows x 128 columns, a k-row is 1 KB = 64 chunks): chunk c of k-row kr sits at c ^ ((kr & 1) << 3).
// ------------------------------------------------------------------------------------------

template <bool bt, int NW>
__device__ __forceinline__ void dgemm_tile_ring(const GemmArgs& g, const int tn, const int tm, const int z,
                                                const bool tri_out) {
    constexpr int NJ = 16 / NW;    // 16-column MFMA tiles per wave
    constexpr int LPW = 16 / NW;   // 1 KB loads per wave and stage: 8 for the A part, 8 for the B part
    double* lds = wg_lds();
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
    const int n_st = k_hi > k_lo ? (k_hi - k_lo) / RK : 0;   // inner ranges are multiples of 16

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave / (NW / 2), wc = wave % (NW / 2);
    const int m0 = tm * GT, n0 = tn * GT;
    const int cw = wc * (NJ * 16);
    const int l16 = lane & 15, lk = lane >> 4;
    const uint32_t lds0 = uint32_t(uintptr_t((ONECOMP_LDS char*)lds));

    // descriptor bases: the tile's first operand row / column at the start of the inner range; a stage's descriptor
    // starts RK inner steps further on (64-bit scalar arithmetic), so that the 32-bit offsets of the lanes stay
    // below 128 rows x ld
    const double* const abase = A + int64_t(m0) * g.lda + k_lo;
    const double* const bbase = bt ? B + int64_t(n0) * g.ldb + k_lo : B + int64_t(k_lo) * g.ldb + n0;
    const int64_t step_b = bt ? int64_t(RK) : int64_t(RK) * g.ldb;   // doubles along k per stage
    uint32_t voff[LPW], ldst[LPW];
#pragma unroll
    for (int q = 0; q < LPW; ++q) {
        const int j = wave + NW * q;            // load of the stage: 0 .. 7 A part, 8 .. 15 B part (uniform per q)
        const bool is_a = q * NW < 8;
        const int jj = is_a ? j : j - 8;
        if (is_a || bt) {
            const int row = 16 * jj + (lane >> 2);
            const int c = (lane & 3) ^ ((row >> 2) & 3);
            const bool ok = is_a ? (m0 + row < m) : (n0 + row < g.n);
            voff[q] = ok ? uint32_t((int64_t(row) * (is_a ? g.lda : g.ldb) + 2 * c) * 8) : LDS_DMA_OOB;
        } else {
            const int kr = jj;
            const int c = lane ^ ((kr & 1) << 3);
            voff[q] = (n0 + 2 * c < g.n) ? uint32_t((int64_t(kr) * g.ldb + 2 * c) * 8) : LDS_DMA_OOB;
        }
        ldst[q] = (is_a ? 0 : R_PART_BYTES) + jj * 1024;
    }
    auto issue = [&](int st) __attribute__((always_inline)) {   // loads of stage st into its slot; past the end: zeros
        const uint32_t slot = lds0 + uint32_t(st % RNS) * R_STAGE_BYTES;
        const bool live = st < n_st;
        const int64_t sk = live ? int64_t(st) : 0;
        const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<double*>(abase + sk * RK), 0, 0x7FFFFFFF, 0x00020000);
        const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<double*>(bbase + sk * step_b), 0, 0x7FFFFFFF, 0x00020000);
#pragma unroll
        for (int q = 0; q < LPW; ++q)
            lds_load16(slot + ldst[q], live ? voff[q] : LDS_DMA_OOB, (q * NW < 8) ? ra : rb);
    };
    for (int st = 0; st < RNS - 1; ++st) issue(st);

    // accumulators start as (beta / alpha) C (alpha = +-1: exact); register r of lane l: row 4 r + l / 16,
    // column l % 16 of its 16 x 16 tile
    const double binit = g.beta * g.alpha;   // beta / alpha for alpha = +-1
    double4v acc[4][NJ];
    const bool full = (m0 + GT <= m) && (n0 + GT <= g.n);
    double* __restrict__ ct = C + int64_t(m0 + wr * 64 + lk) * g.ldc + n0 + cw + l16;
    if (g.beta == 0.0) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.0;
    } else if (full) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[i][j][r] = binit * ct[int64_t(i * 16 + 4 * r) * g.ldc + j * 16];
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = m0 + wr * 64 + i * 16 + 4 * r + lk;
                    const int col = n0 + cw + j * 16 + l16;
                    double c = 0.0;
                    if (row < m && col < g.n) c = binit * C[int64_t(row) * g.ldc + col];
                    acc[i][j][r] = c;
                }
    }

    // fragment addresses inside a stage (bytes), inner steps 0 .. 3; steps 4 .. 7: A-form ^ 32, NN + 4 KB
    int fa[4], fb[NJ];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = wr * 64 + i * 16 + l16;
        fa[i] = row * 64 + (((lk >> 1) ^ ((row >> 2) & 3)) << 4) + (lk & 1) * 8;
    }
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const int col = cw + j * 16 + l16;
        if (bt) fb[j] = R_PART_BYTES + col * 64 + (((lk >> 1) ^ ((col >> 2) & 3)) << 4) + (lk & 1) * 8;
        else fb[j] = R_PART_BYTES + lk * 1024 + (((col >> 1) ^ ((lk & 1) << 3)) << 4) + (col & 1) * 8;
    }
    const char* ldsc = reinterpret_cast<const char*>(lds);

    for (int st = 0; st < n_st; ++st) {
        // the loads of stages st + 1 and st + 2 may still be in flight: wait for those of stage st, publish them,
        // and refill the slot every wave has finished reading (stage st - 1)
        __builtin_amdgcn_s_waitcnt(wait_vmcnt(LPW * (RNS - 2)));
        __syncthreads();
        issue(st + RNS - 1);
        const char* sp = ldsc + (st % RNS) * R_STAGE_BYTES;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            double a[4], b[NJ];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = *reinterpret_cast<const double*>(sp + (h ? fa[i] ^ 32 : fa[i]));
#pragma unroll
            for (int j = 0; j < NJ; ++j)
                b[j] = *reinterpret_cast<const double*>(sp + (bt ? (h ? fb[j] ^ 32 : fb[j]) : fb[j] + h * 4096));
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[i], b[j], acc[i][j], 0, 0, 0);
        }
    }
    __builtin_amdgcn_s_waitcnt(wait_vmcnt(0));   // no LDS write may be in flight when the slots are reused or the workgroup ends

    const double aout = g.alpha;
    if (full) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) ct[int64_t(i * 16 + 4 * r) * g.ldc + j * 16] = aout * acc[i][j][r];
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = m0 + wr * 64 + i * 16 + 4 * r + lk;
                    const int col = n0 + cw + j * 16 + l16;
                    if (row < m && col < g.n) C[int64_t(row) * g.ldc + col] = aout * acc[i][j][r];
                }
    }
    if (tri_out) {   // uniform; every wave must be done with the last stage before the operand slots are overwritten
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int lrow = wr * 64 + i * 16 + 4 * r + lk, lcol = cw + j * 16 + l16;
                    if ((lcol >> 4) > (lrow >> 4)) continue;
                    const bool inside = (m0 + lrow < m) && (n0 + lcol < g.n);
                    lds[tri(lrow, lcol)] = inside ? aout * acc[i][j][r] : (lrow == lcol ? 1.0 : 0.0);
                }
    }
}

// Tile (0, 0) of a trailing update C -= P P^T whose first tile lies on the diagonal: the tile the next diagonal block
// is waiting for.  Its workgroup is the first of the launch and what counts is how soon it is done, not throughput.
// A 128 x 128 x 128 tile is 512 fp64 MFMAs per wave, 64 cycles each: 17 us on a CU to itself, twice that next to a
// second workgroup.  Only the 36 sub-blocks of 16 x 16 on and below the diagonal are needed (potrf_body takes
// nothing else), so wave w computes the sub-block rows w and 7 - w: (w + 1) + (8 - w) = 9 sub-blocks each instead
// of 16.  Both operands are the same 128 rows, so a stage holds that one 8 KB part only and the same LDS takes a
// ring of eight slots.  Every sub-block sees the MFMAs of dgemm_tile_ring<true, 4> in the same order: bit-equal
// results.  The updated tile goes, as lower 16 x 16 sub-blocks (identity beyond the matrix edge), to the LDS layout
// of potrf_body and nowhere else: the block column it heads is finished with this step and nothing reads the tile
// from C again.
constexpr int DNS = 2 * RNS;   // slots of the diagonal tile's ring
static_assert(DNS * R_PART_BYTES <= LDS_DOUBLES * 8, "the diagonal tile's ring fits into the workgroup's LDS");
template <int W>
__device__ __forceinline__ void dgemm_diag_tile_wave(const GemmArgs& g, double* lds) {
    constexpr int NW = 4, LPW = 2;           // waves; 1 KB loads per wave and stage
    constexpr int RA = W, RB = 7 - W;        // this wave's sub-block rows; row R needs the sub-block columns 0 .. R
    constexpr int NB_COLS = RB + 1;          // operand fragments of the second kind: sub-block columns 0 .. RB
    const int m = g.m_last, nc = g.n;        // rows and columns of C that exist (the last block may be short)
    const int n_st = g.k_last / RK;
    const double* __restrict__ A = g.A;
    const double* __restrict__ C = g.C;
    const int lane = threadIdx.x & 63;
    const int l16 = lane & 15, lk = lane >> 4;
    const uint32_t lds0 = uint32_t(uintptr_t((ONECOMP_LDS char*)lds));
    uint32_t voff[LPW], ldst[LPW];
#pragma unroll
    for (int q = 0; q < LPW; ++q) {
        const int j = W + NW * q;               // load 0 .. 7 of the stage: rows 16 j .. 16 j + 15
        const int row = 16 * j + (lane >> 2);
        const int c = (lane & 3) ^ ((row >> 2) & 3);
        voff[q] = (row < m) ? uint32_t((int64_t(row) * g.lda + 2 * c) * 8) : LDS_DMA_OOB;
        ldst[q] = j * 1024;
    }
    auto issue = [&](int st) __attribute__((always_inline)) {   // loads of stage st into its slot; past the end: zeros
        const uint32_t slot = lds0 + uint32_t(st % DNS) * R_PART_BYTES;
        const bool live = st < n_st;
        const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<double*>(A + (live ? int64_t(st) : 0) * RK), 0, 0x7FFFFFFF, 0x00020000);
#pragma unroll
        for (int q = 0; q < LPW; ++q) lds_load16(slot + ldst[q], live ? voff[q] : LDS_DMA_OOB, ra);
    };
    for (int st = 0; st < DNS - 1; ++st) issue(st);

    // accumulators start as (beta / alpha) C (alpha = +-1: exact); register r of lane l: row 4 r + l / 16,
    // column l % 16 of its sub-block
    const double binit = g.beta * g.alpha;
    double4v accA[RA + 1], accB[RB + 1];
    const bool full = m >= GT && nc >= GT;
    auto init = [&](double4v& acc, int R, int c, auto whole) __attribute__((always_inline)) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = R * 16 + 4 * r + lk, col = c * 16 + l16;
            if constexpr (decltype(whole)::value) {   // unconditional loads: all in flight together
                acc[r] = binit * C[int64_t(row) * g.ldc + col];
            } else {
                double v = 0.0;
                if (row < m && col < nc) v = binit * C[int64_t(row) * g.ldc + col];
                acc[r] = v;
            }
        }
    };
    if (full) {
#pragma unroll
        for (int c = 0; c <= RA; ++c) init(accA[c], RA, c, std::true_type{});
#pragma unroll
        for (int c = 0; c <= RB; ++c) init(accB[c], RB, c, std::true_type{});
    } else {
#pragma unroll
        for (int c = 0; c <= RA; ++c) init(accA[c], RA, c, std::false_type{});
#pragma unroll
        for (int c = 0; c <= RB; ++c) init(accB[c], RB, c, std::false_type{});
    }

    // fragment addresses inside a stage (bytes), inner steps 0 .. 3; steps 4 .. 7: ^ 32
    auto frag = [&](int sb) __attribute__((always_inline)) {
        const int row = sb * 16 + l16;
        return row * 64 + (((lk >> 1) ^ ((row >> 2) & 3)) << 4) + (lk & 1) * 8;
    };
    int fr[NB_COLS];
#pragma unroll
    for (int c = 0; c < NB_COLS; ++c) fr[c] = frag(c);
    const int faA = frag(RA), faB = frag(RB);
    const char* ldsc = reinterpret_cast<const char*>(lds);
    for (int st = 0; st < n_st; ++st) {
        __builtin_amdgcn_s_waitcnt(wait_vmcnt(LPW * (DNS - 2)));   // stage st has landed
        __syncthreads();
        issue(st + DNS - 1);                                        // into the slot every wave has finished reading
        const char* sp = ldsc + (st % DNS) * R_PART_BYTES;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            double b[NB_COLS];
#pragma unroll
            for (int c = 0; c < NB_COLS; ++c) b[c] = *reinterpret_cast<const double*>(sp + (h ? fr[c] ^ 32 : fr[c]));
            const double aA = *reinterpret_cast<const double*>(sp + (h ? faA ^ 32 : faA));
            const double aB = *reinterpret_cast<const double*>(sp + (h ? faB ^ 32 : faB));
#pragma unroll
            for (int c = 0; c <= RB; ++c) {
                accB[c] = __builtin_amdgcn_mfma_f64_16x16x4f64(aB, b[c], accB[c], 0, 0, 0);
                if (c <= RA) accA[c] = __builtin_amdgcn_mfma_f64_16x16x4f64(aA, b[c], accA[c], 0, 0, 0);
            }
        }
    }
    __builtin_amdgcn_s_waitcnt(wait_vmcnt(0));   // no LDS write may be in flight when the slots are reused
    __syncthreads();   // every wave is done with the last stage before the operand slots are overwritten
    const double aout = g.alpha;
    auto put = [&](const double4v& acc, int R, int c) __attribute__((always_inline)) {
        double* M = lds + sub(R, c);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int lrow = R * 16 + 4 * r + lk, lcol = c * 16 + l16;
            const bool inside = full || ((lrow < m) && (lcol < nc));
            M[(4 * r + lk) * SBP + l16] = inside ? aout * acc[r] : (lrow == lcol ? 1.0 : 0.0);
        }
    };
#pragma unroll
    for (int c = 0; c <= RA; ++c) put(accA[c], RA, c);
#pragma unroll
    for (int c = 0; c <= RB; ++c) put(accB[c], RB, c);
}
__device__ __forceinline__ void dgemm_diag_tile(const GemmArgs& g) {
    double* lds = wg_lds();
    switch (__builtin_amdgcn_readfirstlane(threadIdx.x >> 6)) {
        case 0: dgemm_diag_tile_wave<0>(g, lds); break;
        case 1: dgemm_diag_tile_wave<1>(g, lds); break;
        case 2: dgemm_diag_tile_wave<2>(g, lds); break;
        default: dgemm_diag_tile_wave<3>(g, lds); break;
    }
}

// Tile (tm, tn), tn <= tm, of rank v in the row-major enumeration of a lower triangle of tiles.
__device__ __forceinline__ void lower_tile_from_rank(int v, int& tm, int& tn) {
    int r = int((__fsqrt_rn(8.0f * float(v) + 1.0f) - 1.0f) * 0.5f);
    while (r * (r + 1) / 2 > v) --r;
    while ((r + 1) * (r + 2) / 2 <= v) ++r;
    tm = r;
    tn = v - r * (r + 1) / 2;
}

// Work map of a GEMM launch: one workgroup per tile that has work, in a one-dimensional grid (workgroups that return
// at once are not free: each still waits for its turn at a CU, and a quarter of such workgroups in a launch cost a
// quarter of its time).  Workgroups are dispatched in rank order; with a triangular operand the tiles differ in
// length (B lower: the inner range starts at the tile's column, so tile columns get shorter to the right; A lower: it
// ends at the tile's row, so tile rows get longer downwards) and the longest tiles come first, so that no long tile
// starts when the rest of the launch is nearly done.  Order: the last batch entry (the only one that can be
// shorter), then the other entries interleaved tile by tile.
struct GemmGrid {
    int tn_cnt, tm_full, tm_last, per_full, per_last, total;
};
__host__ __device__ inline GemmGrid gemm_grid(const GemmArgs& g) {
    GemmGrid q;
    q.tn_cnt = (g.n + GT - 1) / GT;
    q.tm_full = (g.m + GT - 1) / GT;
    q.tm_last = (g.m_last + GT - 1) / GT;
    if (g.flags & G_CLOWER) {   // square C, lower tiles only
        q.per_full = q.tm_full * (q.tm_full + 1) / 2;
        q.per_last = q.tm_last * (q.tm_last + 1) / 2;
    } else {
        q.per_full = q.tm_full * q.tn_cnt;
        q.per_last = q.tm_last * q.tn_cnt;
    }
    q.total = q.per_last + (g.batch - 1) * q.per_full;
    return q;
}
__device__ __forceinline__ void gemm_tile_from_rank(const GemmArgs& g, int v, int& tm, int& tn, int& z) {
    const GemmGrid q = gemm_grid(g);
    int rem, tm_cnt;
    if (v < q.per_last) {
        z = g.batch - 1;
        rem = v;
        tm_cnt = q.tm_last;
    } else {
        v -= q.per_last;
        z = v % (g.batch - 1);
        rem = v / (g.batch - 1);
        tm_cnt = q.tm_full;
    }
    if (g.flags & G_CLOWER) {
        lower_tile_from_rank(rem, tm, tn);
    } else if (g.flags & G_BLOWER) {   // tile columns left to right, rows fastest
        tn = rem / tm_cnt;
        tm = rem % tm_cnt;
    } else if (g.flags & G_ALOWER) {   // tile rows from the bottom
        tm = tm_cnt - 1 - rem / q.tn_cnt;
        tn = rem % q.tn_cnt;
    } else {
        tm = rem / q.tn_cnt;
        tn = rem % q.tn_cnt;
    }
}

// Stand-alone GEMM launches run eight waves per workgroup (64 x 32 per wave, under 128 registers): four waves share a
// SIMD and cover each other's waits (k = 128 updates: 46 -> 51 TFLOP/s; large GEMMs 64 -> 66).
constexpr int GEMM_WAVES = 8;
template <bool bt>
__global__ __launch_bounds__(64 * GEMM_WAVES, 2) void dgemm_kernel(GemmArgs g) {
    int tm, tn, z;
    gemm_tile_from_rank(g, blockIdx.x, tm, tn, z);
    dgemm_tile_ring<bt, GEMM_WAVES>(g, tn, tm, z, false);
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
    const bool first = blockIdx.x == 0;
    int tm, tn;
    if (g.flags & G_CLOWER) {
        // Workgroup b runs on XCD b % 8; each XCD takes a run of consecutive ranks of the banded order (bands of eight
        // tile columns walked row by row), so that the 64 tiles resident on an XCD at one time form a patch of about
        // 8 x 8 and find the 16 operand panels they share in its L2 (in row-major order of the ranks the tiles of an XCD
        // were every eighth of five tile rows; 38.4 -> 38.0 ms at d_in 14336, 265 -> 261.5 at 28672).  Rank 0 is
        // tile (0, 0).
        const int nt = (g.m + GT - 1) / GT, total = nt * (nt + 1) / 2, chunk = (total + 7) >> 3;
        const int v = (int(blockIdx.x) & 7) * chunk + (int(blockIdx.x) >> 3);
        if (v >= total) return;
        plan::tile_from_rank_band<plan::SYRK_BAND>(v, nt, tn, tm);
    } else {   // one block column whose first tile lies on the diagonal: one workgroup per tile row
        tm = blockIdx.x;
        tn = 0;
    }
    if (first) {
        dgemm_diag_tile(g);
        __syncthreads();
        potrf_body(A, V, n, off, bs, info, wg_lds(), true);
    } else {
        dgemm_tile_ring<true, 4>(g, tn, tm, 0, false);
    }
}

// ------------------------------------------------------------------------------------------
// Panel solve of the blocked Cholesky:  P <- P Linv^T  for the m x 128 panel below a 128 x 128 diagonal block whose
// inverse Linv (lower triangular, zeros above the diagonal) is known.  A 128 x 128 GEMM tile per workgroup would
// occupy only m / 128 of the CUs for about 23 us (fp64 MFMA bound), on the critical path of every block step; here
// a workgroup takes 32 rows and only the non-zero half of Linv:  wave w computes the 16-column tiles 7 - w and w
// (k < 16 (c + 1) for tile c: 9 units of 16 k per wave).  The rows go through LDS (read once, written in place);
// the Linv operands, shared by all workgroups and resident in L2, are read from global memory straight in MFMA
// operand order.  Layouts as in potrf_body: A[i][k]: i = l % 16, k = l / 16; B[k][j]: k = l / 16, j = l % 16;
// D register r: row 4 r + l / 16, column l % 16.
// ------------------------------------------------------------------------------------------
constexpr int TR = 32;          // rows per workgroup
constexpr int TRP = NB + 1;     // LDS pitch in doubles

__global__ __launch_bounds__(256) void trsm_kernel(double* __restrict__ P, int64_t ldp, int m,
                                                  const double* __restrict__ Linv, int64_t ldl) {
    __shared__ double sA[TR * TRP];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m0 = blockIdx.x * TR;
    {
        const int r = tid >> 3, c0 = (tid & 7) * 16;
        const bool ok = m0 + r < m;
        const double2* src = reinterpret_cast<const double2*>(P + int64_t(ok ? m0 + r : 0) * ldp + c0);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const double2 v = ok ? src[e] : make_double2(0.0, 0.0);
            sA[r * TRP + c0 + 2 * e] = v.x;
            sA[r * TRP + c0 + 2 * e + 1] = v.y;
        }
    }
    const int li = lane & 15, lk = lane >> 4;
    // the Linv operands of both passes are requested before the rows arrive: one memory latency instead of three
    double bvs[2][32];
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int c = pass == 0 ? NB / 16 - 1 - wave : wave;
        const int nk = 4 * (c + 1);
        const double* bp = Linv + int64_t(c * 16 + li) * ldl + lk;
#pragma unroll
        for (int ks = 0; ks < 32; ++ks) bvs[pass][ks] = ks < nk ? bp[4 * ks] : 0.0;
    }
    __syncthreads();
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int c = pass == 0 ? NB / 16 - 1 - wave : wave;   // column tile
        const int nk = 4 * (c + 1);                             // MFMA steps of 4 k
        const double (&bv)[32] = bvs[pass];
        const double* ap0 = sA + li * TRP + lk;
        const double* ap1 = sA + (16 + li) * TRP + lk;
        double4v acc0 = {0.0, 0.0, 0.0, 0.0}, acc1 = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int ks = 0; ks < 32; ++ks) {
            if (ks < nk) {   // uniform per wave
                acc0 = __builtin_amdgcn_mfma_f64_16x16x4f64(ap0[4 * ks], bv[ks], acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f64_16x16x4f64(ap1[4 * ks], bv[ks], acc1, 0, 0, 0);
            }
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row0 = m0 + 4 * r + lk, row1 = row0 + 16;
            if (row0 < m) P[int64_t(row0) * ldp + c * 16 + li] = acc0[r];
            if (row1 < m) P[int64_t(row1) * ldp + c * 16 + li] = acc1[r];
        }
    }
}

onecomp_status dgemm(const GemmArgs& g, hipStream_t stream) {
    if (g.m <= 0 || g.n <= 0 || g.batch <= 0 || g.m_last <= 0) return ONECOMP_OK;
    const dim3 grid(unsigned(gemm_grid(g).total), 1, 1);
    if (g.flags & G_BTRANS) hipLaunchKernelGGL(dgemm_kernel<true>, grid, dim3(64 * GEMM_WAVES), 0, stream, g);
    else hipLaunchKernelGGL(dgemm_kernel<false>, grid, dim3(64 * GEMM_WAVES), 0, stream, g);
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

onecomp_status factor_run(const float* H, int64_t d_in, float damp, int act_order, int form, int32_t* perm_out,
                          float* U, int32_t* info, void* workspace, hipStream_t stream) {
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
    // One step: panel solve below diagonal block kb, then the trailing update fused with the factorization of the
    // next diagonal block.  While the trailing matrix is large the steps go in pairs: the first block's update is
    // applied to the next block column only (enough to factor and solve that one), and both blocks update everything
    // behind the pair in one pass with k = 256: the rank-128 update is bound by reading and writing the trailing
    // matrix (52 TFLOP/s at best, 60 with k = 256), and the additions happen in the same order, so the factor is
    // bit-equal.  The price is the second block's factorization, which now has only a short launch to hide behind
    // (about 70 us per pair): below PAIR_MIN_BLOCKS tile rows the saving no longer covers it.
    auto panel_solve = [&](int off, int rest) -> onecomp_status {
        // A[off+NB:, off:off+NB] <- A[off+NB:, off:off+NB] * Linv_kk^T   (in place)
        hipLaunchKernelGGL(trsm_kernel, dim3(unsigned(ceil_div(rest, TR))), dim3(256), 0, stream,
                           w.A + int64_t(off + NB) * n + off, int64_t(n), rest, w.V + int64_t(off) * n + off, int64_t(n));
        ONECOMP_CHECK_LAUNCH();
        return ONECOMP_OK;
    };
    // C[c_off:, c_off : c_off + cols) -= P P^T with P = A[c_off:, k_off : k_off + k), lower tiles when cols covers the
    // whole remainder; the first tile is the next diagonal block, factored by the same workgroup
    auto update = [&](int c_off, int cols, int k_off, int k, bool lower) -> onecomp_status {
        const int rows = n - c_off;
        GemmArgs s{};
        s.A = w.A + int64_t(c_off) * n + k_off; s.lda = n; s.sa = 0;
        s.B = s.A; s.ldb = n; s.sb = 0;
        s.C = w.A + int64_t(c_off) * n + c_off; s.ldc = n; s.sc = 0;
        s.m = rows; s.m_last = rows; s.n = cols; s.k = k; s.k_last = k; s.batch = 1;
        s.alpha = -1.0; s.beta = 1.0; s.flags = G_BTRANS | (lower ? G_CLOWER : 0);
        const unsigned nt = unsigned(ceil_div(rows, GT));
        const dim3 grid(lower ? 8 * ((nt * (nt + 1) / 2 + 7) / 8) : nt, 1, 1);   // tile (0, 0) first
        hipLaunchKernelGGL(syrk_potrf_kernel, grid, dim3(256), 0, stream, s, w.A, w.V, n, c_off, min(NB, n - c_off),
                           info);
        ONECOMP_CHECK_LAUNCH();
        return ONECOMP_OK;
    };
    constexpr int PAIR_MIN_BLOCKS = 60;
    for (int kb = 0; kb < nblk;) {
        const int off = kb * NB;
        const int rest = n - off - NB;     // rows below this block (only the last block can be shorter than NB,
        if (rest <= 0) break;              // and it has nothing below it)
        if ((st = panel_solve(off, rest)) != ONECOMP_OK) return st;
        const int rest2 = rest - NB;       // rows below the next block
        if (rest2 >= PAIR_MIN_BLOCKS * NB) {
            if ((st = update(off + NB, NB, off, NB, false)) != ONECOMP_OK) return st;       // next block column only
            if ((st = panel_solve(off + NB, rest2)) != ONECOMP_OK) return st;
            if ((st = update(off + 2 * NB, rest2, off, 2 * NB, true)) != ONECOMP_OK) return st;   // both blocks, k = 256
            kb += 2;
        } else {
            if ((st = update(off + NB, rest, off, NB, true)) != ONECOMP_OK) return st;
            kb += 1;
        }
    }

    if (form == ONECOMP_FACTOR_BLOCK) {   // diagonal blocks of L^-1 are in V already; the rest comes from L itself
        hipLaunchKernelGGL(rdiag_kernel, dim3(unsigned(ceil_div(n, 256))), dim3(256), 0, stream, w.V, n, w.dfix);
        ONECOMP_CHECK_LAUNCH();
        hipLaunchKernelGGL(output_block_kernel, dim3(unsigned(ceil_div(n, 256)), unsigned(n)), dim3(256), 0, stream, w.A,
                           w.V, w.dfix, n, U);
        ONECOMP_CHECK_LAUNCH();
        return ONECOMP_OK;
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
