// Gram / Hessian accumulation  H += 2 X^T X  (Sec. 2.5 and Sec. 4.3 of the paper: H_l = X_l^T X_l,
// rows of X are token activations; the factor 2 makes it the Hessian of the layer objective).
//
// gfx950 design
//   * Only tiles on or above the diagonal are computed; each result is stored to H[i][k] and to
//     its mirror H[k][i], so H stays bit-wise symmetric and one workgroup owns each tile
//     (no floating-point atomics, reproducible).
//   * bf16 path: X is token-major while the MFMA operands (v_mfma_f32_32x32x16_bf16) need 8 consecutive
//     TOKENS per lane, so the token-major LDS tile is read with ds_read_b64_tr_b16 (LDS transpose read) and no
//     register shuffles are needed.  Wide layers: ring kernel, tiles go global -> LDS directly (384 x 256 tile on
//     four waves with three quarters of the register file as accumulators; 256 x 256 tile, 8 waves; 128 x 256 tile,
//     two workgroups per CU; whichever the estimated cost favours).  Narrow layers (d_in < 1024): register-staged
//     128 x 128 kernel, double-buffered LDS.
//   * The workgroup -> tile map is XCD-aware: hardware deals consecutive workgroups round-robin to
//     the 8 XCDs, so workgroup b is given the tile with rank (b % 8) * chunk + b / 8 in an
//     order that walks bands of 4 tile rows column by column.  The 32 workgroups that share an
//     XCD's L2 at any time then cover a compact 4 x 8 patch of tiles (12 X panels, not 64).  A wide layer is
//     launched one round of tiles (one per CU) at a time, so that those 32 also stay together along the tokens.
//   * fp32 path (small layers): 128-wide tiles on v_mfma_f32_32x32x2_f32, products in fp32.
#include "common.hpp"
#include "planner.hpp"
#include <stdlib.h>
#include <string.h>
#include <type_traits>

namespace onecomp {
namespace {

constexpr int GRAM_THREADS = 256;
using plan::tile_from_rank;       // workgroup -> tile maps: planner.hpp
using plan::tile128_from_rank;
using plan::SplitPlan;
using plan::plan_split;
constexpr int BAND = plan::GRAM_BAND;

// -------------------------------------------------------------------------------------------
// Epilogue shared by the bf16 kernels: H[i][k] += 2 acc for this wave's MT x NT tiles of 32 x 32 and the
// mirrored entries H[k][i] (one owner per element, no atomics: bit-wise symmetric and reproducible).
// Accumulator register r of lane l holds row (r/4)*8 + (l/32)*4 + r%4, column l%32 of its tile; ibase / kbase are
// the wave's first row / column.  Tiles strictly above the diagonal and inside the matrix take a path without
// per-element masks whose loads are issued 32 at a time before the first use (left to itself the compiler
// waits for every load separately when the accumulators live in AGPRs).
// -------------------------------------------------------------------------------------------
// MIRROR = false: plain H[i][k] += 2 acc for every entry of the tile (cross-Gram of two different matrices).
template <int MT, int NT, bool MIRROR = true>
__device__ __forceinline__ void gram_store(float16v (&acc)[MT][NT], float* __restrict__ H, const int d_in,
                                           const int ibase, const int kbase, const bool diag, const int lane) {
    const int lr = (lane >> 5) * 4, lc = lane & 31;
    const bool interior = !diag && (ibase + 32 * MT <= d_in) && (kbase + 32 * NT <= d_in);
    if (interior) {
        constexpr int NBATCH = NT < 2 ? NT : 2;   // column tiles per batch of loads
#pragma unroll
        for (int m = 0; m < MT; ++m) {
#pragma unroll
            for (int n0 = 0; n0 < NT; n0 += NBATCH) {
                float* hp = H + int64_t(ibase + m * 32 + lr) * d_in + kbase + n0 * 32 + lc;
                float hv[NBATCH][16];
#pragma unroll
                for (int n = 0; n < NBATCH; ++n)
#pragma unroll
                    for (int r = 0; r < 16; ++r) hv[n][r] = hp[int64_t((r / 4) * 8 + (r % 4)) * d_in + n * 32];
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int n = 0; n < NBATCH; ++n) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        hv[n][r] = hv[n][r] + 2.0f * acc[m][n0 + n][r];
                        hp[int64_t((r / 4) * 8 + (r % 4)) * d_in + n * 32] = hv[n][r];
                    }
                    if constexpr (MIRROR) {
                        float* mp = H + int64_t(kbase + (n0 + n) * 32 + lc) * d_in + ibase + m * 32 + lr;
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const float4v o = {hv[n][q * 4], hv[n][q * 4 + 1], hv[n][q * 4 + 2], hv[n][q * 4 + 3]};
                            *reinterpret_cast<float4v*>(mp + q * 8) = o;
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        return;
    }
#pragma unroll
    for (int m = 0; m < MT; ++m) {
#pragma unroll
        for (int n = 0; n < NT; ++n) {
            const int k = kbase + n * 32 + lc;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int ib = ibase + m * 32 + q * 8 + lr;   // 4 consecutive rows ib..ib+3
                if (k >= d_in || ib >= d_in) continue;         // d_in % 16 == 0: the 4 rows are in or out together
                float nv[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int i = ib + e;
                    float* p = H + int64_t(i) * d_in + k;
                    nv[e] = *p + 2.0f * acc[m][n][q * 4 + e];
                    if (!diag || i <= k) *p = nv[e];
                }
                if constexpr (!MIRROR) continue;
                if (!diag) {
                    const float4v o = {nv[0], nv[1], nv[2], nv[3]};
                    *reinterpret_cast<float4v*>(H + int64_t(k) * d_in + ib) = o;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (ib + e < k) H[int64_t(k) * d_in + ib + e] = nv[e];
                }
            }
        }
    }
}

// -------------------------------------------------------------------------------------------
// bf16 kernel
// -------------------------------------------------------------------------------------------
template <int WT>
struct GramBf16Cfg {
    static constexpr int TS = 64 * WT;          // tile side in channels
    static constexpr int KT = 32;               // tokens per LDS stage
    static constexpr int PITCH = TS + 32;       // bf16 elements; +64 B per token row: the 4 rows x 2 lane groups of a transpose read hit 64 distinct banks
    static constexpr int PANEL = KT * PITCH;    // elements per panel
    static constexpr int CHUNKS = KT * TS / 8;  // 16-byte chunks per panel
    static constexpr int NLOAD = CHUNKS / GRAM_THREADS;
    static constexpr size_t LDS_BYTES = size_t(4) * PANEL * 2;  // 2 stages x (A, B)
};

template <int WT>
__global__ __launch_bounds__(GRAM_THREADS) void gram_bf16_kernel(const uint16_t* __restrict__ X,
                                                                int64_t n_tokens, int d_in, int64_t ldx,
                                                                float* __restrict__ H, int n_t,
                                                                int n_tiles, int chunk) {
    using C = GramBf16Cfg<WT>;
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];

    const int v = (blockIdx.x & 7) * chunk + (blockIdx.x >> 3);
    if (v >= n_tiles) return;
    int ti, tk;
    tile_from_rank(v, n_t, ti, tk);
    const bool diag = (ti == tk);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1;
    const int i0 = ti * C::TS, k0 = tk * C::TS;

    // global -> LDS assignment
    int ld_row[C::NLOAD], ld_col[C::NLOAD];
#pragma unroll
    for (int n = 0; n < C::NLOAD; ++n) {
        int id = tid + GRAM_THREADS * n;
        ld_row[n] = id / (C::TS / 8);
        ld_col[n] = (id % (C::TS / 8)) * 8;
    }
    uint4v ra[C::NLOAD], rb[C::NLOAD];
    auto gload = [&](int64_t t0) {
#pragma unroll
        for (int n = 0; n < C::NLOAD; ++n) {
            int64_t t = t0 + ld_row[n];
            int ca = i0 + ld_col[n], cb = k0 + ld_col[n];
            const uint4v z = {0u, 0u, 0u, 0u};
            ra[n] = (t < n_tokens && ca < d_in) ? *reinterpret_cast<const uint4v*>(X + t * ldx + ca) : z;
            if (!diag) rb[n] = (t < n_tokens && cb < d_in) ? *reinterpret_cast<const uint4v*>(X + t * ldx + cb) : z;
        }
    };
    auto lstore = [&](int stage) {
        uint16_t* pa = lds + stage * 2 * C::PANEL;
        uint16_t* pb = pa + C::PANEL;
#pragma unroll
        for (int n = 0; n < C::NLOAD; ++n) {
            *reinterpret_cast<uint4v*>(pa + ld_row[n] * C::PITCH + ld_col[n]) = ra[n];
            if (!diag) *reinterpret_cast<uint4v*>(pb + ld_row[n] * C::PITCH + ld_col[n]) = rb[n];
        }
    };

    // LDS transpose-read addressing: inside each 16-lane group, lane 4k+c points at 4 channels of token k;
    // the read returns, to lane i of the group, that group's channel i for tokens 0..3.
    const int i16 = lane & 15, g16 = (lane >> 4) & 1, kb8 = lane >> 5;
    const int frag_off = (kb8 * 8 + (i16 >> 2)) * C::PITCH + g16 * 16 + (i16 & 3) * 4;

    float16v acc[WT][WT];
#pragma unroll
    for (int m = 0; m < WT; ++m)
#pragma unroll
        for (int n = 0; n < WT; ++n)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[m][n][r] = 0.f;

    const int64_t n_stage = (n_tokens + C::KT - 1) / C::KT;
    gload(0);
    lstore(0);
    __syncthreads();
    for (int64_t s = 0; s < n_stage; ++s) {
        const int cur = int(s & 1);
        if (s + 1 < n_stage) gload((s + 1) * C::KT);
        const uint16_t* pa = lds + cur * 2 * C::PANEL;
        const uint16_t* pb = diag ? pa : pa + C::PANEL;
        const uint16_t* fa = pa + frag_off + wr * (32 * WT);
        const uint16_t* fb = pb + frag_off + wc * (32 * WT);
#pragma unroll
        for (int kb = 0; kb < C::KT / 16; ++kb) {
            bf16x8 a[WT], b[WT];
#pragma unroll
            for (int m = 0; m < WT; ++m) {
                const uint16_t* p = fa + kb * 16 * C::PITCH + m * 32;
                short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((ONECOMP_LDS short4v*)p);
                short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((ONECOMP_LDS short4v*)(p + 4 * C::PITCH));
                short8v w = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                a[m] = __builtin_bit_cast(bf16x8, w);
            }
#pragma unroll
            for (int n = 0; n < WT; ++n) {
                const uint16_t* p = fb + kb * 16 * C::PITCH + n * 32;
                short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((ONECOMP_LDS short4v*)p);
                short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((ONECOMP_LDS short4v*)(p + 4 * C::PITCH));
                short8v w = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                b[n] = __builtin_bit_cast(bf16x8, w);
            }
#pragma unroll
            for (int m = 0; m < WT; ++m)
#pragma unroll
                for (int n = 0; n < WT; ++n)
                    acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[m], b[n], acc[m][n], 0, 0, 0);
        }
        if (s + 1 < n_stage) lstore(cur ^ 1);
        __syncthreads();
    }

    gram_store<WT, WT>(acc, H, d_in, i0 + wr * (32 * WT), k0 + wc * (32 * WT), diag, lane);
}

// Epilogue of a tile whose tokens are split between two workgroups (see gram_bf16_ring_kernel): the tile lies
// strictly above the diagonal and inside the matrix.  The workgroup with the first half of the tokens adds its sum
// to H[i][k] and leaves the mirror alone; the one with the second half overwrites the mirror entries H[k][i] with
// its sum.  gram_merge_kernel then sets both to H[i][k] + H[k][i]: one fixed order of additions, bit-wise symmetric.
template <int MT, int NT>
__device__ __forceinline__ void gram_store_half(float16v (&acc)[MT][NT], float* __restrict__ H, const int d_in,
                                                const int ibase, const int kbase, const int half, const int lane) {
    const int lr = (lane >> 5) * 4, lc = lane & 31;
    if (half == 0) {
        constexpr int NBATCH = NT < 2 ? NT : 2;
#pragma unroll
        for (int m = 0; m < MT; ++m) {
#pragma unroll
            for (int n0 = 0; n0 < NT; n0 += NBATCH) {
                float* hp = H + int64_t(ibase + m * 32 + lr) * d_in + kbase + n0 * 32 + lc;
                float hv[NBATCH][16];
#pragma unroll
                for (int n = 0; n < NBATCH; ++n)
#pragma unroll
                    for (int r = 0; r < 16; ++r) hv[n][r] = hp[int64_t((r / 4) * 8 + (r % 4)) * d_in + n * 32];
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int n = 0; n < NBATCH; ++n)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        hp[int64_t((r / 4) * 8 + (r % 4)) * d_in + n * 32] = hv[n][r] + 2.0f * acc[m][n0 + n][r];
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    } else {
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int n = 0; n < NT; ++n) {
                float* mp = H + int64_t(kbase + n * 32 + lc) * d_in + ibase + m * 32 + lr;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4v o = {2.0f * acc[m][n][q * 4], 2.0f * acc[m][n][q * 4 + 1], 2.0f * acc[m][n][q * 4 + 2],
                                       2.0f * acc[m][n][q * 4 + 3]};
                    *reinterpret_cast<float4v*>(mp + q * 8) = o;
                }
            }
    }
}

// H[i][k] = H[k][i] = H[i][k] + H[k][i] on the 256 x 256 tiles with ranks split0 .. split0 + n_split - 1 of the
// first band (tile rows 0 .. 3, columns from 4 on: rank split0 + m is tile (m % 4, 4 + m / 4) when split0 is the
// size of the band's triangle).  One workgroup of 32 x 8 threads per 32 x 32 block, through LDS so that both
// matrices are read and written along rows.
__global__ __launch_bounds__(256) void gram_merge_kernel(float* __restrict__ H, int d_in, int n_split) {
    __shared__ float sa[32][33], sb[32][33];
    const int m = blockIdx.y;
    if (m >= n_split) return;
    const int ti = m % BAND, tk = BAND + m / BAND;
    const int bi = blockIdx.x / 8, bk = blockIdx.x % 8;            // 8 x 8 blocks of 32 x 32 per tile
    const int i0 = ti * 256 + bi * 32, k0 = tk * 256 + bk * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
#pragma unroll
    for (int y = ty; y < 32; y += 8) {
        sa[y][tx] = H[int64_t(i0 + y) * d_in + k0 + tx];
        sb[y][tx] = H[int64_t(k0 + y) * d_in + i0 + tx];
    }
    __syncthreads();
#pragma unroll
    for (int y = ty; y < 32; y += 8) {
        H[int64_t(i0 + y) * d_in + k0 + tx] = sa[y][tx] + sb[tx][y];
        H[int64_t(k0 + y) * d_in + i0 + tx] = sa[tx][y] + sb[y][tx];
    }
}

// -------------------------------------------------------------------------------------------
// bf16 ring kernel: global -> LDS without passing through registers (buffer_load_dwordx4 ... lds), in steps of
// 16 tokens through a ring of NBUF LDS slots.  Three shapes:
//   RingWide 384 x 256 tile, 4 waves (2 x 2, 192 x 128 each = 24 MFMA tiles = 384 accumulator registers per lane),
//            one wave per SIMD with the whole register file.  The fewest L2 and LDS bytes per flop (17 % less than
//            256 x 256, 10 fragments for 24 MFMAs per step instead of 6 for 8).  The compiler cannot place 384
//            accumulators by itself (it copies tiles between the VGPR and AGPR halves and spills), so for this shape
//            the MFMA is inline assembly whose operand constraints pin 16 tiles to AGPRs and 8 to VGPRs; being opaque
//            to the compiler's hazard handling, the last MFMAs are followed by explicit wait states before the
//            epilogue reads the accumulators.  Tile (i, k) = rows [384 i, +384) x columns [256 k, +256) is computed
//            when it reaches above the diagonal (k >= floor(3 i / 2)).
//   RingBig  256 x 256 tile, 8 waves (2 x 4, 128 x 64 each), i.e. two waves per SIMD: one wave's waits are covered
//            by the other's MFMAs.  Only tiles on or above the diagonal (banded, XCD-aware order of tile_from_rank).
//   RingMid  128 x 256 tile, 4 waves (2 x 2, 64 x 128 each), two workgroups per CU: for mid-size d_in, where
//            256 x 256 tiles are too few to fill the CUs.  Tile (i, k) = rows [128 i, +128) x columns [256 k, +256)
//            is computed when it reaches above the diagonal (k >= i / 2).
// Tiles that the diagonal crosses store only their entries on or above it (and the mirrors).
//   * One wave-wide 16-byte LDS load deposits lane l at M0 + 16 l, i.e. 1 KB contiguous = two (four) token rows
//     of a 256 (128)-channel panel.  Rows therefore cannot be padded against bank conflicts; instead the 16-byte
//     chunk c of token row r is stored at chunk position c ^ ((r & 3) << 2): the four token rows of one
//     transpose read then fall into four different 64-byte bank groups.  The swizzle costs nothing on the
//     global side because every lane supplies its own global address.
//   * The loads are inline assembly, so the compiler neither sees the LDS write (and does not serialize later
//     LDS reads behind it) nor counts them; the kernel waits explicitly with vmcnt(loads per step x steps still
//     allowed in flight) before the barrier that publishes a step.  Out-of-range lanes (token rows past the end,
//     channels past d_in) deposit zeros: that is the raw-buffer range check.
//   * An MFMA occupies the matrix pipe for 32 cycles but issues in 4: LDS reads and loads are placed one at a
//     time behind the MFMAs.  Half-iteration h: MT NT MFMAs on the fragments of step h (registers); LDS ->
//     fragments of step h+1; loads of step h+NBUF into the slot step h was read from; wait for step h+2 + barrier.
// -------------------------------------------------------------------------------------------
struct RingMid {
    static constexpr int TM = 128, TN = 256, WM = 2, WN = 2, NBUF = 6, MIN_WAVES = 2;
};
struct RingBig {
    static constexpr int TM = 256, TN = 256, WM = 2, WN = 4, NBUF = 8, MIN_WAVES = 2;
};
struct RingWide {
    static constexpr int TM = 384, TN = 256, WM = 2, WN = 2, NBUF = 7, MIN_WAVES = 1;
};
template <typename C>
struct Ring {
    static constexpr int KT = 16;
    static constexpr int WAVES = C::WM * C::WN, THREADS = 64 * WAVES;
    static constexpr int MT = C::TM / (32 * C::WM), NT = C::TN / (32 * C::WN);   // 32 x 32 tiles per wave
    static constexpr int A_ROWB = C::TM * 2, B_ROWB = C::TN * 2;
    static constexpr int A_PANELB = KT * A_ROWB, B_PANELB = KT * B_ROWB, STAGEB = A_PANELB + B_PANELB;
    static constexpr int NL_A = A_PANELB / 1024, NL_B = B_PANELB / 1024;          // 1 KB wave loads per panel
    static constexpr int LPW = (NL_A + NL_B) / WAVES;                            // loads per wave and step
    static constexpr size_t LDS_BYTES = size_t(C::NBUF) * STAGEB;
    static_assert((NL_A + NL_B) % WAVES == 0 && NL_A % WAVES == 0, "whole loads per wave, A loads first");
    static_assert(MT + NT <= MT * NT && LPW <= MT * NT, "fragment reads and loads are placed one behind each MFMA");
    static_assert((A_ROWB / 16) % 16 == 0 && (B_ROWB / 16) % 16 == 0, "the chunk swizzle stays inside groups of 16 chunks");
};
// CROSS = false: H += 2 X^T X, tiles on or above the diagonal, mirrored.  CROSS = true: H += 2 X^T Xb for two
// different matrices (A panels from X, B panels from Xb), every tile, no mirror.
// PACED: every wave sleeps 64 cycles at the start of each step.  In a launch of many thousand steps the workgroups of
// an XCD otherwise drift apart along the tokens until the panels they share no longer meet in its L2 (hit rate 55 %
// after 16384 steps against 79 % after 4096); with the pause they stay together (81 %, the ideal of the 4 x 8 patch is
// 82 %), 162 -> 69 GB come over the fabric per call at d_in 14336, and the clock the chip holds under this load rises
// from 1.65 to 1.76 GHz: 45.4 -> 44.6 ms per call.  The pause itself costs 0.5 - 2 % where there is no drift to cure
// (shorter launches), so the host asks for it only in long ones, and only for the symmetric product (the cross-Gram's
// launches gained 0.5 ms on one box and lost 1.3 on another).
template <typename C, bool CROSS, bool PACED = false>
__global__ __launch_bounds__(Ring<C>::THREADS, C::MIN_WAVES) void gram_bf16_ring_kernel(
    const uint16_t* __restrict__ X, const uint16_t* __restrict__ Xb, int64_t n_tokens, int d_in, int64_t ldx,
    int64_t ldxb, float* __restrict__ H, int n_rt, int n_ct, int n_tiles, int chunk, int split0, int n_split,
    int n_piece, float* __restrict__ ws, int bid0) {
    using R = Ring<C>;
    constexpr int KT = R::KT, NBUF = C::NBUF, MT = R::MT, NT = R::NT, LPW = R::LPW;
    constexpr int A_ROWB = R::A_ROWB, B_ROWB = R::B_ROWB, A_PANELB = R::A_PANELB, STAGEB = R::STAGEB;
    extern __shared__ __attribute__((aligned(1024))) char ldsb[];
    // Workgroups 0 .. 8 chunk - 1 take whole tiles: the ranks outside [split0, split0 + n_split), `chunk` of them
    // per XCD.  The workgroups after them take the n_split tiles of that range in n_piece pieces of the token axis
    // each, so that a short last round of whole tiles (or a matrix of fewer tiles than CUs) still fills the chip
    // (n_split = 0: no such tiles).  Without a workspace n_piece is 2 and the mirror positions hold the second
    // partial sum (gram_store_half); with one, every piece stores its sum there and gram_reduce_kernel adds them.
    // bid: rank of this workgroup in the whole schedule; a launch covers a run of ranks starting at bid0
    const int bid = int(blockIdx.x) + bid0;
    plan::RingWork rw;
    if (!plan::ring_work(bid, chunk, n_tiles, split0, n_split, rw)) return;
    const int v = rw.v, piece = rw.piece, m_split = rw.m_split;
    if (piece >= 0) {   // this workgroup's share of the tokens: whole steps of KT
        int64_t t_begin, count;
        plan::piece_tokens(n_tokens, n_piece, piece, KT, t_begin, count);
        X += t_begin * ldx;
        Xb += t_begin * ldxb;
        n_tokens = count;   // <= 0: nothing left, the sum is 0
    }
    int ti, tk;
    if constexpr (CROSS) plan::cross_tile_from_rank(v, n_rt, n_ct, ti, tk);
    else if constexpr (C::TM == C::TN) tile_from_rank(v, n_ct, ti, tk);
    else if constexpr (C::TM == 384) plan::tile_wide_from_rank(v, n_rt, n_ct, ti, tk);
    else tile128_from_rank(v, n_rt, n_ct, ti, tk);
    const int i0 = ti * C::TM, k0 = tk * C::TN;
    const bool diag = !CROSS && k0 < i0 + C::TM;   // some entry of the tile lies on or below the diagonal
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave / C::WN, wc = wave % C::WN;
    const uint32_t lds0 = uint32_t(uintptr_t((ONECOMP_LDS char*)ldsb));

    // this wave's LPW 1 KB loads per step: load j = wave + WAVES q; j < NL_A is a load of the A panel
    uint32_t voff[LPW], ldst[LPW];
#pragma unroll
    for (int q = 0; q < LPW; ++q) {
        const int j = wave + R::WAVES * q;
        const bool is_a = j < R::NL_A;
        const int jj = is_a ? j : j - R::NL_A;
        const int rowb = is_a ? A_ROWB : B_ROWB;
        const int cpr = rowb / 16;                         // 16-byte chunks per token row
        const int lin = jj * 64 + lane;                    // this lane's chunk of the panel as it lies in LDS
        const int row = lin / cpr;
        const int c = (lin % cpr) ^ ((row & 3) << 2);
        const int col = (is_a ? i0 : k0) + c * 8;
        voff[q] = (col < d_in) ? uint32_t((int64_t(row) * (is_a ? ldx : ldxb) + col) * 2) : LDS_DMA_OOB;
        ldst[q] = (is_a ? 0 : A_PANELB) + jj * 1024;
    }
    const int64_t n_st = (n_tokens + KT - 1) / KT;
    const int64_t n_st2 = (n_st + 1) & ~int64_t(1);   // the loop takes two steps at a time; an extra step is all zeros
    struct Desc {
        __amdgpu_buffer_rsrc_t a, b;   // A panels, B panels (the same matrix unless CROSS)
    };
    // descriptor of step st: base = its first token row, range = what is left of the matrix (none past the last
    // step).  The 64-bit products may be computed on the vector ALU: the wave-uniform results are brought back to
    // scalar registers, where a descriptor has to live.
    auto make_rsrc = [&](const uint16_t* base, int64_t ld, int64_t st) __attribute__((always_inline)) {
        const int64_t t0 = st * KT;
        const int64_t left = (n_tokens - t0) * ld * 2;
        const bool live = left > 0;
        const int range = __builtin_amdgcn_readfirstlane(!live ? 0 : (left > 0x7FFFFFFF ? 0x7FFFFFFF : int(left)));
        const int64_t boff = (live ? t0 : 0) * ld * 2;
        const uint32_t blo = __builtin_amdgcn_readfirstlane(uint32_t(boff));
        const uint32_t bhi = __builtin_amdgcn_readfirstlane(uint32_t(uint64_t(boff) >> 32));
        return __builtin_amdgcn_make_buffer_rsrc(
            const_cast<char*>(reinterpret_cast<const char*>(base) + int64_t((uint64_t(bhi) << 32) | blo)), 0, range,
            0x00020000);
    };
    auto make_desc = [&](int64_t st) __attribute__((always_inline)) {
        Desc d;
        d.a = make_rsrc(X, ldx, st);
        if constexpr (CROSS) d.b = make_rsrc(Xb, ldxb, st);
        else d.b = d.a;
        return d;
    };
    // load q of this wave (compile-time q): A panel loads come first
    auto gload = [&](const Desc& d, uint32_t dst, int q) __attribute__((always_inline)) {
        if (q * R::WAVES < R::NL_A) lds_load16(dst + ldst[q], voff[q], d.a);   // wave + WAVES q < NL_A for every wave
        else lds_load16(dst + ldst[q], voff[q], d.b);
    };

    const int i16 = lane & 15, g16 = (lane >> 4) & 1, kb8 = lane >> 5;
    const int kq = i16 >> 2;
    const int lo = (2 * g16 + ((i16 & 3) >> 1)) * 16 + (i16 & 1) * 8;
    int fa[MT], fb[NT];
#pragma unroll
    for (int m = 0; m < MT; ++m) fa[m] = (kb8 * 8 + kq) * A_ROWB + (((wr * MT + m) ^ kq) << 6) + lo;
#pragma unroll
    for (int n = 0; n < NT; ++n) fb[n] = A_PANELB + (kb8 * 8 + kq) * B_ROWB + (((wc * NT + n) ^ kq) << 6) + lo;

    struct Frags {
        bf16x8 a[MT], b[NT];
    };
    auto rd2 = [&](const char* p, int rowb) __attribute__((always_inline)) {
        short4v x0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((ONECOMP_LDS short4v*)(p));
        short4v x1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((ONECOMP_LDS short4v*)(p + 4 * rowb));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(x0, x1, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    // fragment r (0 .. MT+NT-1) of the slot at ldsb + sb: A fragments first
    auto rd = [&](Frags& f, int r, int sb) __attribute__((always_inline)) {
        const char* s = ldsb + sb;
        if (r < MT) f.a[r] = rd2(s + fa[r], A_ROWB);
        else f.b[r - MT] = rd2(s + fb[r - MT], B_ROWB);
    };

    for (int st = 0; st < NBUF; ++st) {
        const Desc d = make_desc(st);
#pragma unroll
        for (int q = 0; q < LPW; ++q) gload(d, lds0 + st * STAGEB, q);
    }
    float16v acc[MT][NT];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int n = 0; n < NT; ++n)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[m][n][r] = 0.f;
    __builtin_amdgcn_s_waitcnt(wait_vmcnt(0));
    __syncthreads();
    Frags Fc, FH;
#pragma unroll
    for (int r = 0; r < MT + NT; ++r) rd(Fc, r, 0);
    __syncthreads();   // slot 0 is overwritten by the loads of the first half-iteration

    // More than 256 accumulator registers per lane: the first 16 tiles are pinned to the AGPR half of the register
    // file and the rest to the VGPR half by the operand constraints of the instruction itself (left to choose, the
    // compiler copies tiles between the halves).
    constexpr int N_AGPR_TILES = (MT * NT > 16) ? 16 : MT * NT;
    // the tile of the last MFMA of an iteration (its statement carries the wait states) is one of the VGPR tiles
    constexpr bool BY_COLUMNS = MT * NT > 16;
    static_assert(!BY_COLUMNS || ((NT - 1) & 1), "the last column runs downwards and ends in tile (MT - 1, NT - 1), a VGPR tile");
    // These MFMAs are opaque to the compiler's hazard handling, which therefore puts no wait states between the last
    // of them and whatever reads an accumulator at the loop's exit (the epilogue, or a spill or a copy between the
    // register halves that the compiler places there).  The last MFMA of a loop iteration carries the wait states
    // itself; they pass while that MFMA executes, and the instructions that follow wait for the other waves anyway.
    auto mma = [&](const Frags& f, auto&& between, auto closes_iteration) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < MT * NT; ++i) {
            // Serpentine order over the wave's tiles: from one MFMA to the next only one of the two operands changes
            // (the pipes draw less on operands that stay, and the clock follows: 44.3 -> 44.1 ms per call at d_in
            // 14336, alternating in one process).  By rows, the columns of every second row backwards; the 6 x 4 tiles
            // of the 384 x 256 shape by columns instead (the B operand stays for six MFMAs: another 44.0 -> 43.8 ms),
            // odd columns downwards so that the last tile of a step is one of the VGPR tiles.
            const int tn_c = i / MT, tm_c = (tn_c & 1) ? i % MT : MT - 1 - i % MT;
            const int tm_r = i / NT, tn_r = (tm_r & 1) ? NT - 1 - i % NT : i % NT;
            const int tm = BY_COLUMNS ? tm_c : tm_r, tn = BY_COLUMNS ? tn_c : tn_r;
            if constexpr (MT * NT > 16) {
                if (decltype(closes_iteration)::value && i == MT * NT - 1)
                    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0\n\ts_nop 15\n\ts_nop 15"
                                 : "+v"(acc[tm][tn]) : "v"(f.a[tm]), "v"(f.b[tn]));
                else if (tm * NT + tn < N_AGPR_TILES)
                    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0"
                                 : "+a"(acc[tm][tn]) : "v"(f.a[tm]), "v"(f.b[tn]));
                else
                    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0"
                                 : "+v"(acc[tm][tn]) : "v"(f.a[tm]), "v"(f.b[tn]));
            } else {
                acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[tm], f.b[tn], acc[tm][tn], 0, 0, 0);
            }
            between(i);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    int s0 = 0;   // slot of step st
#pragma unroll 1
    for (int64_t st = 0; st < n_st2; st += 2) {
        const int s1 = (s0 == NBUF - 1) ? 0 : s0 + 1, s2 = (s1 == NBUF - 1) ? 0 : s1 + 1;
        // loads past the last step get an empty descriptor (zeros into a slot nobody reads again); fragment reads
        // past it fetch stale data nobody uses
        {
            if constexpr (PACED) __builtin_amdgcn_s_sleep(1);
            const Desc d = make_desc(st + NBUF);
            const uint32_t dst = lds0 + s0 * STAGEB;
            const int sb = s1 * STAGEB;
            mma(Fc, [&](int i) __attribute__((always_inline)) {
                if (i < MT + NT) rd(FH, i, sb);
                if (i < LPW) gload(d, dst, i);
            }, std::false_type{});
            __builtin_amdgcn_s_waitcnt(wait_vmcnt(LPW * (NBUF - 2)));   // step st+2 has landed
            __syncthreads();
        }
        {
            if constexpr (PACED) __builtin_amdgcn_s_sleep(1);
            const Desc d = make_desc(st + 1 + NBUF);
            const uint32_t dst = lds0 + s1 * STAGEB;
            const int sb = s2 * STAGEB;
            mma(FH, [&](int i) __attribute__((always_inline)) {
                if (i < MT + NT) rd(Fc, i, sb);
                if (i < LPW) gload(d, dst, i);
            }, std::true_type{});
            __builtin_amdgcn_s_waitcnt(wait_vmcnt(LPW * (NBUF - 2)));   // step st+3 has landed
            __syncthreads();
        }
        s0 = s2;
    }
    __builtin_amdgcn_s_waitcnt(wait_vmcnt(0));   // no LDS write may be in flight when the workgroup ends
    if (piece >= 0 && ws) {   // partial sum of the tile, in accumulator order: consecutive lanes, consecutive addresses
        float* slot = ws + (int64_t(m_split) * n_piece + piece) * (C::TM * C::TN) + wave * (MT * NT * 16 * 64) + lane;
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int n = 0; n < NT; ++n)
#pragma unroll
                for (int r = 0; r < 16; ++r) slot[((m * NT + n) * 16 + r) * 64] = acc[m][n][r];
    } else if (piece >= 0) {
        gram_store_half<MT, NT>(acc, H, d_in, i0 + wr * (32 * MT), k0 + wc * (32 * NT), piece, lane);
    } else {
        gram_store<MT, NT, !CROSS>(acc, H, d_in, i0 + wr * (32 * MT), k0 + wc * (32 * NT), diag, lane);
    }
}

// Sum of the n_piece partial sums of each split tile (fixed order), then the usual epilogue: H += 2 sum, mirrored.
// One single-wave workgroup per part of a tile: the share of one wave of the main kernel, cut into RS parts along its
// rows and NS along its columns when that share is more than 128 registers per lane.
template <typename C>
struct ReduceCfg {
    static constexpr int RS = (Ring<C>::MT * Ring<C>::NT > 8) ? 2 : 1;
    static constexpr int NS = RS;
    static constexpr int PARTS = Ring<C>::WAVES * RS * NS;   // workgroups per tile
    static_assert(Ring<C>::MT % RS == 0 && Ring<C>::NT % NS == 0, "whole 32 x 32 tiles per part");
};
template <typename C>
__global__ __launch_bounds__(64) void gram_reduce_kernel(const float* __restrict__ ws, float* __restrict__ H, int d_in,
                                                         int n_rt, int n_ct, int split0, int n_split, int n_piece) {
    using R = Ring<C>;
    using RC = ReduceCfg<C>;
    constexpr int MT = R::MT, NT = R::NT, MTS = MT / RC::RS, NTS = NT / RC::NS;
    const int m_split = blockIdx.x / RC::PARTS, sub = blockIdx.x % RC::PARTS;
    if (m_split >= n_split) return;
    int ti, tk;
    if constexpr (C::TM == C::TN) tile_from_rank(split0 + m_split, n_ct, ti, tk);
    else plan::tile_wide_from_rank(split0 + m_split, n_rt, n_ct, ti, tk);
    const int i0 = ti * C::TM, k0 = tk * C::TN;
    const int lane = threadIdx.x;
    const int wave = sub / (RC::RS * RC::NS), part = (sub / RC::NS) % RC::RS, nh = sub % RC::NS;
    const int wr = wave / C::WN, wc = wave % C::WN;
    float16v acc[MTS][NTS];
#pragma unroll
    for (int m = 0; m < MTS; ++m)
#pragma unroll
        for (int n = 0; n < NTS; ++n)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[m][n][r] = 0.f;
    for (int p = 0; p < n_piece; ++p) {
        const float* slot = ws + (int64_t(m_split) * n_piece + p) * (C::TM * C::TN) + wave * (MT * NT * 16 * 64) + lane;
#pragma unroll
        for (int m = 0; m < MTS; ++m)
#pragma unroll
            for (int n = 0; n < NTS; ++n)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    acc[m][n][r] += slot[(((part * MTS + m) * NT + nh * NTS + n) * 16 + r) * 64];
    }
    gram_store<MTS, NTS, true>(acc, H, d_in, i0 + wr * (32 * MT) + part * (32 * MTS),
                               k0 + wc * (32 * NT) + nh * (32 * NTS), k0 < i0 + C::TM, lane);
}

// -------------------------------------------------------------------------------------------
// fp32 kernel: 128 x 128 tile, 4 waves in 2x2, each 2x2 tiles of v_mfma_f32_32x32x2_f32
// -------------------------------------------------------------------------------------------
constexpr int F32_TS = 128, F32_KT = 16, F32_PITCH = F32_TS + 4, F32_PANEL = F32_KT * F32_PITCH;

__global__ __launch_bounds__(GRAM_THREADS) void gram_f32_kernel(const float* __restrict__ X, int64_t n_tokens,
                                                               int d_in, int64_t ldx, float* __restrict__ H,
                                                               int n_t, int n_tiles, int chunk) {
    __shared__ __attribute__((aligned(16))) float lds[4 * F32_PANEL];
    const int v = (blockIdx.x & 7) * chunk + (blockIdx.x >> 3);
    if (v >= n_tiles) return;
    int ti, tk;
    tile_from_rank(v, n_t, ti, tk);
    const bool diag = (ti == tk);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1;
    const int i0 = ti * F32_TS, k0 = tk * F32_TS;

    constexpr int NLOAD = F32_KT * F32_TS / 4 / GRAM_THREADS;  // 2
    int ld_row[NLOAD], ld_col[NLOAD];
#pragma unroll
    for (int n = 0; n < NLOAD; ++n) {
        int id = tid + GRAM_THREADS * n;
        ld_row[n] = id / (F32_TS / 4);
        ld_col[n] = (id % (F32_TS / 4)) * 4;
    }
    float4v ra[NLOAD], rb[NLOAD];
    auto gload = [&](int64_t t0) {
#pragma unroll
        for (int n = 0; n < NLOAD; ++n) {
            int64_t t = t0 + ld_row[n];
            int ca = i0 + ld_col[n], cb = k0 + ld_col[n];
            const float4v z = {0.f, 0.f, 0.f, 0.f};
            ra[n] = (t < n_tokens && ca < d_in) ? *reinterpret_cast<const float4v*>(X + t * ldx + ca) : z;
            if (!diag) rb[n] = (t < n_tokens && cb < d_in) ? *reinterpret_cast<const float4v*>(X + t * ldx + cb) : z;
        }
    };
    auto lstore = [&](int stage) {
        float* pa = lds + stage * 2 * F32_PANEL;
        float* pb = pa + F32_PANEL;
#pragma unroll
        for (int n = 0; n < NLOAD; ++n) {
            *reinterpret_cast<float4v*>(pa + ld_row[n] * F32_PITCH + ld_col[n]) = ra[n];
            if (!diag) *reinterpret_cast<float4v*>(pb + ld_row[n] * F32_PITCH + ld_col[n]) = rb[n];
        }
    };

    float16v acc[2][2];
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int n = 0; n < 2; ++n)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[m][n][r] = 0.f;

    const int64_t n_stage = (n_tokens + F32_KT - 1) / F32_KT;
    gload(0);
    lstore(0);
    __syncthreads();
    const int kl = lane >> 5, cl = lane & 31;  // operand: channel = lane % 32, token = lane / 32
    for (int64_t s = 0; s < n_stage; ++s) {
        const int cur = int(s & 1);
        if (s + 1 < n_stage) gload((s + 1) * F32_KT);
        const float* pa = lds + cur * 2 * F32_PANEL;
        const float* pb = diag ? pa : pa + F32_PANEL;
#pragma unroll
        for (int k2 = 0; k2 < F32_KT; k2 += 2) {
            float a[2], b[2];
#pragma unroll
            for (int m = 0; m < 2; ++m) a[m] = pa[(k2 + kl) * F32_PITCH + wr * 64 + m * 32 + cl];
#pragma unroll
            for (int n = 0; n < 2; ++n) b[n] = pb[(k2 + kl) * F32_PITCH + wc * 64 + n * 32 + cl];
#pragma unroll
            for (int m = 0; m < 2; ++m)
#pragma unroll
                for (int n = 0; n < 2; ++n)
                    acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[m], b[n], acc[m][n], 0, 0, 0);
        }
        if (s + 1 < n_stage) lstore(cur ^ 1);
        __syncthreads();
    }

    const int lr = (lane >> 5) * 4, lc = lane & 31;
#pragma unroll
    for (int m = 0; m < 2; ++m) {
#pragma unroll
        for (int n = 0; n < 2; ++n) {
            const int k = k0 + wc * 64 + n * 32 + lc;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int ib = i0 + wr * 64 + m * 32 + q * 8 + lr;
                if (k >= d_in || ib >= d_in) continue;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int i = ib + e;
                    if (diag && i > k) continue;
                    float* p = H + int64_t(i) * d_in + k;
                    float nv = *p + 2.0f * acc[m][n][q * 4 + e];
                    *p = nv;
                    if (i != k) H[int64_t(k) * d_in + i] = nv;
                }
            }
        }
    }
}

template <int WT>
onecomp_status launch_bf16(const void* X, int64_t n_tokens, int64_t d_in, int64_t ldx, float* H,
                           hipStream_t stream) {
    using C = GramBf16Cfg<WT>;
    const int n_t = int(ceil_div(d_in, C::TS));
    const int n_tiles = n_t * (n_t + 1) / 2;
    const int chunk = int(ceil_div(n_tiles, 8));
    static std::atomic<uint64_t> lds_ok{0};
    if (allow_dynamic_lds(reinterpret_cast<const void*>(&gram_bf16_kernel<WT>), int(C::LDS_BYTES), lds_ok) != ONECOMP_OK)
        return ONECOMP_ERR_HIP;
    hipLaunchKernelGGL(gram_bf16_kernel<WT>, dim3(chunk * 8), dim3(GRAM_THREADS), C::LDS_BYTES, stream,
                       static_cast<const uint16_t*>(X), n_tokens, int(d_in), ldx, H, n_t, n_tiles, chunk);
    ONECOMP_CHECK_LAUNCH();
    return ONECOMP_OK;
}



constexpr size_t GRAM_SLOT_BYTES = size_t(256) * 256 * sizeof(float);   // one partial sum of a 256 x 256 tile

// Whether a call of n_tokens launches its rounds of whole tiles one by one (see launch_bf16_ring).
// ONECOMP_GRAM_ROUND_LAUNCHES=0|1 in the environment forces the answer (tuning).
constexpr int64_t ROUND_LAUNCH_MIN_TOKENS = 49152;
// From this many tokens per call on, the launches of the 384 x 256 shape are paced (measured: a gain at 262144 tokens
// per launch, a small loss at 131072).
constexpr int64_t PACED_MIN_TOKENS = 196608;
bool launch_by_rounds(int64_t n_tokens) {
    const char* e = getenv("ONECOMP_GRAM_ROUND_LAUNCHES");
    if (e && (e[0] == '0' || e[0] == '1') && e[1] == 0) return e[0] == '1';
    return n_tokens >= ROUND_LAUNCH_MIN_TOKENS;
}

template <typename C, bool CROSS>
onecomp_status launch_bf16_ring(const void* X, const void* Xb, int64_t n_tokens, int64_t d_in, int64_t ldx,
                                int64_t ldxb, float* H, float* ws, size_t ws_bytes, hipStream_t stream,
                                GramPlanInfo* info = nullptr) {
    using R = Ring<C>;
    const int n_rt = int(ceil_div(d_in, C::TM)), n_ct = int(ceil_div(d_in, C::TN));
    int n_tiles = 0;
    if (CROSS) n_tiles = n_rt * n_ct;
    else if (C::TM == C::TN) n_tiles = n_ct * (n_ct + 1) / 2;
    else if (C::TM == 384) n_tiles = plan::n_tiles_wide(n_rt, n_ct);
    else n_tiles = plan::n_tiles128(n_rt, n_ct);
    // tiles computed in pieces of the token axis, dispatched after the whole tiles (see plan_split)
    SplitPlan sp;
    if (!CROSS && C::TM >= 256 && C::TN == 256) {
        const int n_cus = device_cus();
        if (n_cus <= 0) return ONECOMP_ERR_HIP;
        constexpr size_t slot_bytes = size_t(C::TM) * C::TN * sizeof(float);
        sp = plan_split(n_tiles, n_ct, d_in, n_tokens, n_cus, ws ? int64_t(ws_bytes / slot_bytes) : 0, C::TM == 256);
    }
    const int n_split = sp.n_split, split0 = sp.split0;
    const int chunk = int(ceil_div(n_tiles - n_split, 8));
    static std::atomic<uint64_t> lds_ok{0};
    if (!info && allow_dynamic_lds(reinterpret_cast<const void*>(&gram_bf16_ring_kernel<C, CROSS>), int(R::LDS_BYTES),
                                   lds_ok) != ONECOMP_OK)
        return ONECOMP_ERR_HIP;
    // One launch per round of whole tiles (one tile per CU), then one for the pieces.  Workgroups of one launch start
    // together, so the tiles an XCD works on walk through the tokens side by side and share their column panels in
    // its L2; in a single launch of many rounds the workgroups of later rounds start whenever a CU falls free and
    // drift apart (L2 hit rate 59 % against 78 % for a round on its own; 46.2 -> 44.7 ms at d_in 14336, 262144 tokens).
    // A call of few tokens is one launch instead: its time is the read-modify-write of H as much as the products, and
    // in one launch the epilogue of one tile runs beside the products of the tiles on other CUs (262144 tokens at
    // d_in 14336 in calls of 2048 / 8192 / 32768 tokens: 121 -> 80, 75 -> 60 (52 with 256 x 256 tiles), 48 -> 47 ms;
    // from 65536 tokens per call on, the launches by rounds win).
    const int total = plan::ring_total_blocks(chunk, n_split, sp.n_piece);
    const int n_cus_r = device_cus();
    const int per_launch = (C::TM >= 256 && C::TN == 256 && n_cus_r > 0 && n_cus_r % 8 == 0 && chunk * 8 >= 2 * n_cus_r &&
                            launch_by_rounds(n_tokens))
                               ? n_cus_r : total;
    // long launches of the 384 x 256 shape run paced (see the kernel)
    const bool paced = C::TM == 384 && !CROSS && per_launch < total && n_tokens >= PACED_MIN_TOKENS;
    if constexpr (C::TM == 384 && !CROSS) {
        static std::atomic<uint64_t> lds_ok_paced{0};
        if (!info && paced &&
            allow_dynamic_lds(reinterpret_cast<const void*>(&gram_bf16_ring_kernel<C, CROSS, true>), int(R::LDS_BYTES),
                              lds_ok_paced) != ONECOMP_OK)
            return ONECOMP_ERR_HIP;
    }
    for (int b0 = 0; b0 < total;) {
        int nb = total - b0;
        if (per_launch < total && b0 < chunk * 8) nb = (chunk * 8 - b0 < per_launch) ? chunk * 8 - b0 : per_launch;
        if (info) {   // describe the schedule, launch nothing
            ++info->launches;
            b0 += nb;
            continue;
        }
        if (paced) {
            if constexpr (C::TM == 384 && !CROSS)
                hipLaunchKernelGGL((gram_bf16_ring_kernel<C, CROSS, true>), dim3(unsigned(nb)), dim3(R::THREADS),
                                   R::LDS_BYTES, stream, static_cast<const uint16_t*>(X), static_cast<const uint16_t*>(Xb),
                                   n_tokens, int(d_in), ldx, ldxb, H, n_rt, n_ct, n_tiles, chunk, split0, n_split,
                                   sp.n_piece, sp.use_ws ? ws : nullptr, b0);
        } else {
            hipLaunchKernelGGL((gram_bf16_ring_kernel<C, CROSS>), dim3(unsigned(nb)), dim3(R::THREADS), R::LDS_BYTES,
                               stream, static_cast<const uint16_t*>(X), static_cast<const uint16_t*>(Xb), n_tokens,
                               int(d_in), ldx, ldxb, H, n_rt, n_ct, n_tiles, chunk, split0, n_split, sp.n_piece,
                               sp.use_ws ? ws : nullptr, b0);
        }
        ONECOMP_CHECK_LAUNCH();
        b0 += nb;
    }
    if (info) {
        info->tile_rows = C::TM;
        info->tile_cols = C::TN;
        return ONECOMP_OK;
    }
    if (n_split > 0 && sp.use_ws) {
        if constexpr (!CROSS && C::TM >= 256 && C::TN == 256) {
            hipLaunchKernelGGL(gram_reduce_kernel<C>, dim3(unsigned(n_split) * ReduceCfg<C>::PARTS), dim3(64), 0, stream,
                               ws, H, int(d_in), n_rt, n_ct, split0, n_split, sp.n_piece);
            ONECOMP_CHECK_LAUNCH();
        }
    } else if (n_split > 0) {   // 256 x 256 tiles only (plan_split: other shapes split with a workspace or not at all)
        hipLaunchKernelGGL(gram_merge_kernel, dim3(64, unsigned(n_split)), dim3(256), 0, stream, H, int(d_in), n_split);
        ONECOMP_CHECK_LAUNCH();
    }
    return ONECOMP_OK;
}

// Which ring kernel a symmetric call takes.  The estimated number of rounds decides: a 256 x 256 tile runs one per CU
// and costs two units; a 128 x 256 tile runs two per CU (a CU with two of them takes twice as long) and costs one unit
// plus 15 % for its higher L2 traffic per flop; a 384 x 256 tile runs one per CU, is 1.5 times the work and moves 17 %
// fewer L2 and LDS bytes per flop, which makes a round of them about 10 % shorter than its work (2.7 units).  The
// 384-row shape needs the workspace for a last round that is not full.
// ONECOMP_GRAM_SHAPE=big|mid|wide in the environment forces a shape (testing and tuning).
enum class GramShape { Big, Mid, Wide };
constexpr double WIDE_UNITS = 2.7;
// The 384-row shape pays for its size when a call has few tokens: its four waves read, add and write 1.2 MB of H per
// tile, a latency chain of 0.66 ms per call at d_in 14336 against 0.28 ms with 256 x 256 tiles on eight waves (close to
// what reading half of H and writing all of it costs).  Measured over 262144 tokens in calls of 4096 / 16384 / 32768
// tokens: 82 / 50.8 / 46.9 ms with 384 x 256 tiles, 60.5 / 48.9 / 47.9 ms with 256 x 256.
constexpr int64_t WIDE_MIN_TOKENS = 24576;
constexpr size_t GRAM_WIDE_SLOT_BYTES = size_t(384) * 256 * sizeof(float);
int forced_shape() {
    const char* e = getenv("ONECOMP_GRAM_SHAPE");
    if (!e) return -1;
    if (!strcmp(e, "big")) return int(GramShape::Big);
    if (!strcmp(e, "mid")) return int(GramShape::Mid);
    if (!strcmp(e, "wide")) return int(GramShape::Wide);
    return -1;
}
GramShape choose_shape(int64_t d_in, int64_t n_tokens, int n_cus, size_t ws_bytes) {
    const int64_t n256 = ceil_div(d_in, 256), n128 = ceil_div(d_in, 128), n384 = ceil_div(d_in, 384);
    const int64_t big = n256 * (n256 + 1) / 2;
    const int64_t mid = plan::n_tiles128(int(n128), int(n256)), wide = plan::n_tiles_wide(int(n384), int(n256));
    const double cost_big = 2.0 * plan_split(big, n256, d_in, n_tokens, n_cus, int64_t(ws_bytes / GRAM_SLOT_BYTES)).rounds;
    const double cost_mid = 1.15 * double(ceil_div(mid, n_cus));
    const double cost_wide =
        WIDE_UNITS * plan_split(wide, n256, d_in, n_tokens, n_cus, int64_t(ws_bytes / GRAM_WIDE_SLOT_BYTES), false).rounds;
    const int f = forced_shape();
    if (f >= 0) return GramShape(f);
    if (n_tokens >= WIDE_MIN_TOKENS && cost_wide < cost_big && cost_wide < cost_mid) return GramShape::Wide;
    return cost_big <= cost_mid ? GramShape::Big : GramShape::Mid;
}

}  // namespace

// bytes of workspace that let gram_accumulate_bf16 cut tiles into pieces (0: this width never does): the larger of
// what the 256 x 256 and the 384 x 256 schedule can use
size_t gram_workspace_bytes(int64_t d_in) {
    if (d_in < 1024) return 0;
    const int n_cus = device_cus();
    if (n_cus <= 0) return 0;
    const int64_t n256 = ceil_div(d_in, 256), big = n256 * (n256 + 1) / 2;
    const int64_t wide = plan::n_tiles_wide(int(ceil_div(d_in, 384)), int(n256));
    const SplitPlan sp = plan_split(big, n256, d_in, int64_t(1) << 40, n_cus, int64_t(1) << 40);
    const SplitPlan sw = plan_split(wide, n256, d_in, int64_t(1) << 40, n_cus, int64_t(1) << 40, false);
    const size_t b = sp.use_ws ? size_t(sp.n_split) * sp.n_piece * GRAM_SLOT_BYTES : 0;
    const size_t w = sw.use_ws ? size_t(sw.n_split) * sw.n_piece * GRAM_WIDE_SLOT_BYTES : 0;
    return b > w ? b : w;
}

onecomp_status gram_accumulate_bf16(const void* X, int64_t n_tokens, int64_t d_in, int64_t ldx, float* H, void* wsv,
                                    size_t ws_bytes, hipStream_t stream, GramPlanInfo* info) {
    float* ws = static_cast<float*>(wsv);
    if (info) *info = GramPlanInfo{128, 128, 0};
    // The direct-to-LDS kernels need 32-bit byte offsets inside a step of tokens; narrow layers take the
    // register-staged 128 x 128 kernel.
    if (ldx * 64 >= (int64_t(1) << 31) || d_in < 1024) {
        if (info) {
            info->launches = 1;
            return ONECOMP_OK;
        }
        return launch_bf16<2>(X, n_tokens, d_in, ldx, H, stream);
    }
    const int n_cus = device_cus();
    if (n_cus <= 0) return ONECOMP_ERR_HIP;
    // describing a call: the workspace is only a size
    float* wsp = info ? reinterpret_cast<float*>(uintptr_t(ws_bytes ? 256 : 0)) : ws;
    switch (choose_shape(d_in, n_tokens, n_cus, wsp ? ws_bytes : 0)) {
        case GramShape::Wide:
            return launch_bf16_ring<RingWide, false>(X, X, n_tokens, d_in, ldx, ldx, H, wsp, ws_bytes, stream, info);
        case GramShape::Big:
            return launch_bf16_ring<RingBig, false>(X, X, n_tokens, d_in, ldx, ldx, H, wsp, ws_bytes, stream, info);
        default:
            return launch_bf16_ring<RingMid, false>(X, X, n_tokens, d_in, ldx, ldx, H, nullptr, 0, stream, info);
    }
}

// G += 2 Xh^T X for two bf16 matrices of the same shape (every tile, no symmetry to use)
onecomp_status gram_cross_accumulate_bf16(const void* Xh, const void* X, int64_t n_tokens, int64_t d_in, int64_t ldxh,
                                          int64_t ldx, float* G, hipStream_t stream) {
    const int n_cus = device_cus();
    if (n_cus <= 0) return ONECOMP_ERR_HIP;
    const int64_t n256 = ceil_div(d_in, 256), n128 = ceil_div(d_in, 128), n384 = ceil_div(d_in, 384);
    const double cost_big = 2.0 * double(ceil_div(n256 * n256, n_cus)), cost_mid = 1.15 * double(ceil_div(n128 * n256, n_cus));
    const double cost_wide = WIDE_UNITS * double(ceil_div(n384 * n256, n_cus));
    int shape = forced_shape();
    if (shape < 0)
        shape = int((n_tokens >= WIDE_MIN_TOKENS && cost_wide < cost_big && cost_wide < cost_mid) ? GramShape::Wide
                    : cost_big <= cost_mid                         ? GramShape::Big
                                                                   : GramShape::Mid);
    if (shape == int(GramShape::Wide))
        return launch_bf16_ring<RingWide, true>(Xh, X, n_tokens, d_in, ldxh, ldx, G, nullptr, 0, stream);
    if (shape == int(GramShape::Big))
        return launch_bf16_ring<RingBig, true>(Xh, X, n_tokens, d_in, ldxh, ldx, G, nullptr, 0, stream);
    return launch_bf16_ring<RingMid, true>(Xh, X, n_tokens, d_in, ldxh, ldx, G, nullptr, 0, stream);
}

onecomp_status gram_accumulate_f32(const void* X, int64_t n_tokens, int64_t d_in, int64_t ldx, float* H,
                                   hipStream_t stream) {
    const int n_t = int(ceil_div(d_in, F32_TS));
    const int n_tiles = n_t * (n_t + 1) / 2;
    const int chunk = int(ceil_div(n_tiles, 8));
    hipLaunchKernelGGL(gram_f32_kernel, dim3(chunk * 8), dim3(GRAM_THREADS), 0, stream,
                       static_cast<const float*>(X), n_tokens, int(d_in), ldx, H, n_t, n_tiles, chunk);
    ONECOMP_CHECK_LAUNCH();
    return ONECOMP_OK;
}

}  // namespace onecomp
