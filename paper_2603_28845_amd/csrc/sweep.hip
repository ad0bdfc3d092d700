// Column sweep of the layer-wise quantizer (Sec. 4.3 of the paper: quantize one column, propagate its
// residual to the columns not yet quantized) on the per-group asymmetric min-max grid (Eq. (1), (2), (4)).
//
// Per output row, for sweep positions j = 0 .. d_in-1:
//   group start:  s = (max - min) / (2^b - 1) of the current values of the group (1 if max == min),
//                 z = clamp(rne(-min / s), 0, 2^b - 1)
//   q = clamp(rne(w_j / s) + z, 0, 2^b - 1),  w^ = s (q - z),  e = (w_j - w^) / U_jj
//   (w_j / s and the division by U_jj are multiplications by correctly rounded fp64 reciprocals),
//   w_k -= e U_jk for k > j.
//
// Precision.  A code is rne(w_j / s); one wrong rounding at a near-tie changes the rest of its row, so the value
// that is rounded has to agree with exact arithmetic to about 1e-7 of a grid step over thousands of columns.  The
// library therefore never stores the compensated weight w_j itself in fp32.  It keeps the ORIGINAL weight (exact)
// and, apart from it, the feedback sum  c_j = -sum_{i<j} e_i U_ij  (a fraction of a grid step, so its fp32 rounding
// is ~1e-8 of a step): the working copy in memory holds c, every MFMA accumulation starts from zero and is added
// to c once, and inside a 32-column inner block the values w = w0 + c, the scale, the decision and the feedback
// run in fp64 registers.
//
// gfx950 schedule (lazy batch of B = 128 columns inside super-blocks of up to 512 columns):
//   panel kernel    64 rows per workgroup carried through the blocks of a super-block: the feedback between the
//                   super-block's blocks is applied inside the kernel (split-fp16 MFMAs on operands stored in
//                   fragment order), the sequential part runs four lanes per row with DPP broadcasts, the rest of
//                   a block is updated with fp32 MFMAs on tiles in LDS.  See panel_body.
//   far update      W[:, cols] += D Un[rows, cols] for the columns beyond a super-block, once per super-block
//                   (K = its width), as a split-fp16 MFMA GEMM (three v_mfma_f32_32x32x16_f16 products per term,
//                   fp32 accuracy), 128 x 256 tile per workgroup, the W tile loaded straight into the accumulators;
//                   the part beyond the next super-block shares a launch with the next panel.  See trailing_tile.
//   Groups wider than a block are runs of whole super-blocks (width 512, 384, 256 or 128, whichever divides the
//   group; one group per row: 512): their scale and zero-point are fixed by group_params_kernel when the sweep
//   reaches them, after the far update has brought every later column up to date.
//   The loss is the sum of e^2 (equal to tr((W-W^) Hd (W-W^)^T) because U Hd U^T = I), kept per row and
//   reduced in a fixed order.
#include "common.hpp"
#include "planner.hpp"
#include <type_traits>

#pragma clang fp contract(off)

namespace onecomp {
namespace {

template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

constexpr int SB = 128;        // lazy-batch block
constexpr int SBIG = 512;      // super-block: columns beyond it are updated once per 512 columns
constexpr int ROWS = 64;       // rows per workgroup of the panel kernel
constexpr int SP = SB + 1;     // LDS pitch (floats) of row tiles: lane l reading column c hits bank (l + c) % 32

// ------------------------------------------------------------------------------------------
// working copy: Wf[r][p] = float(W[r][perm[p]])
// ------------------------------------------------------------------------------------------
template <typename T>
__device__ inline float to_f32(T v);
template <>
__device__ inline float to_f32<float>(float v) { return v; }
template <>
__device__ inline float to_f32<uint16_t>(uint16_t v) { return __uint_as_float(uint32_t(v) << 16); }

// the sweep's scalars live in a 256-byte slot: the Scalars of its split products, then (offset 64) the flag that
// a residual was saturated
__device__ __host__ inline uint32_t* sat_flag(Scalars* sc) { return reinterpret_cast<uint32_t*>(sc) + 16; }

__global__ void init_scalars_kernel(Scalars* sc) {
    sc->max_w_bits = 0u;
    sc->max_u_bits = 0u;
    *sat_flag(sc) = 0u;
}

__device__ inline void block_max_to(uint32_t* dst, float v) {
    // Atomics on one address are serialized in L2 (~10 ns each), so a launch issues few of them: wave maximum by
    // butterfly shuffles, workgroup maximum through LDS, one atomic per workgroup of up to 4 waves.
    __shared__ float wave_max[4];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        const int nw = (blockDim.x + 63) >> 6;
        for (int i = 1; i < nw; ++i) v = fmaxf(v, wave_max[i]);
        atomicMax(dst, __float_as_uint(v));
    }
}

template <typename T>
__global__ __launch_bounds__(256) void load_kernel(const T* __restrict__ W, int64_t d_out, int64_t d_in,
                                                  const int32_t* __restrict__ perm, float* __restrict__ Wf,
                                                  float* __restrict__ rowloss, Scalars* __restrict__ sc,
                                                  float* __restrict__ W0p) {
    // The working copy Wf starts as zeros: it holds only the accumulated feedback; the weights themselves are read
    // from W or, under a column order, from the gathered copy W0p written here.  Also max |W|.
    float m = 0.f;
    for (int64_t r = blockIdx.x; r < d_out; r += gridDim.x) {   // a workgroup per row, rows strided over the grid
    if (threadIdx.x == 0) rowloss[r] = 0.f;
    if (perm) {
        for (int p = threadIdx.x; p < d_in; p += 256) {
            const float v = to_f32<T>(W[r * d_in + perm[p]]);
            Wf[r * d_in + p] = 0.f;
            if (W0p) W0p[r * d_in + p] = v;
            m = fmaxf(m, fabsf(v));
        }
    } else {   // rows are 16-byte aligned: d_in is a multiple of 128
        constexpr int V = 16 / sizeof(T);
        for (int p = threadIdx.x * V; p < d_in; p += 256 * V) {
            const uint4v raw = *reinterpret_cast<const uint4v*>(W + r * d_in + p);
            float v[V];
            if constexpr (sizeof(T) == 2) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    v[2 * e] = __uint_as_float(raw[e] << 16);
                    v[2 * e + 1] = __uint_as_float(raw[e] & 0xFFFF0000u);
                }
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = __uint_as_float(raw[e]);
            }
#pragma unroll
            for (int e = 0; e < V; e += 4) {
                *reinterpret_cast<float4v*>(Wf + r * d_in + p + e) = float4v{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int e = 0; e < V; ++e) m = fmaxf(m, fabsf(v[e]));
        }
    }
    }
    block_max_to(&sc->max_w_bits, m);
}

constexpr int IB = 32;          // columns swept in registers at a time

// ------------------------------------------------------------------------------------------
// panel kernel: one launch sweeps a whole super-block of up to four
// 128-column blocks for 64 rows per workgroup.  Rows never interact, so the workgroup carries its rows through
// the blocks without any grid-wide step in between:
//   near update   (left-looking) before block b is swept, its columns receive the feedback of blocks 0 .. b-1 of
//                 the super-block: W_b += D_b' Un[b', b] as split-fp16 MFMAs (see the trailing kernel) whose
//                 operands are loaded from global memory already in MFMA fragment order, 16 bytes per lane:
//                 the residual fragments were written by this workgroup after block b', the fragments of the
//                 normalized U blocks by nearfrag_kernel.  Wave w owns the block's column tile w (64 x 32).
//   sequential    four lanes per row (a quad), each holding 8 of the 32 columns of the inner block; the current
//                 column is broadcast inside the quad by DPP, the grid arithmetic is replicated, the feedback is
//                 8 FMAs per lane.  All four waves work (16 rows each).
//   inner update  the inner block's 32 errors reach the remaining columns of the block through fp32 MFMAs
//                 (v_mfma_f32_32x32x2_f32) on the tiles in LDS.
// LDS tile sW holds current values; a finished column holds its code (as a float).
// ------------------------------------------------------------------------------------------
struct PanelArgs {
    const float* Wf;            // [d_out x d_in] accumulated feedback c of the earlier super-blocks (block form: the
                                // sums c_k = sum_i (w_i - w^_i) R_ik / R_kk)
    const void* W0;             // the layer's weights in sweep order (the caller's matrix, or the gathered fp32 copy
                                // under a column order)
    int w0_bf16;
    const double* s64;          // [d_out] wide groups: the current group's scale in fp64 (group_params_kernel)
    uint32_t* sat;              // set to 1 if a residual had to be saturated when it was split into fp16 halves
    const float* U;
    uint8_t* Q;                 // sweep order (the caller's array, or the staging copy under a column order)
    float* scales;
    float* zeros;
    float* W_hat;               // sweep order, or nullptr
    uint16_t *Dh, *Dl;          // [SBIG x ldD] transposed residual panels for the far update
    uint16_t *Fh, *Fl;          // [workgroup][3][8 k-steps][2 row tiles][64 lanes][8] residual fragments (own use)
    const uint16_t *Bh, *Bl;    // [6 block pairs][8 k-steps][4 column tiles][64 lanes][8] of this super-block
    const Scalars* sc;
    float* rowloss;
    int d_out, d_in, s0, nb, lgG, n_g, ldD;
    int wide_g;             // >= 0: the whole super-block lies in group wide_g, whose scale and zero-point are already
                            // in scales / zeros (groups of whole super-blocks, or one group per row); lgG is then 7
    float qmax;             // highest code of the grid
    float qs;               // 0: min-max grid of Eq. (2); > 0: symmetric grid of Eq. (3) with zero-point qs
    int mse;                // scale search: the group's range is shrunk by 1 - i / 100, i < 80; least squared error wins
};

// Scale and zero-point of a group from the smallest and largest of its current values, in fp64, operation by
// operation as the definition reads: Eq. (2), or Eq. (3) when qs > 0 (symmetric grid, zero-point qs); cand > 0: from
// the range shrunk by 1 - cand / 100 (scale search).
__device__ __forceinline__ void grid_params(double mn, double mx, const int cand, const double qmax, const double qs,
                                            double& s, double& z) {
    if (cand > 0) {
        const double p = 1.0 - double(cand) * 0.01;
        mn *= p; mx *= p;
    }
    if (qs > 0.0) {
        s = fmax(fabs(mn), fabs(mx)) / qs;
        if (s == 0.0) s = 1.0;
        z = qs;
    } else {
        s = (mx - mn) / qmax;
        if (s == 0.0) s = 1.0;
        z = fmin(fmax(rint(-mn / s), 0.0), qmax);
    }
}

// Scale search of one group ("mse" option of Sec. 4.3).  partial(z, 1 / s) returns the sum of ((w - w^) / s)^2 over
// this lane's values of the group on the grid (s, z) (mse_term per value); reduce(x) sums x over the lanes that share
// the group.  Candidate i takes (s, z) by the grid's rule from the range shrunk by p_i = 1 - i / 100 (grid_params,
// fp64: a zero-point at an exact rounding tie, e.g. a group with min = -max, then falls the same way for every
// candidate and for the final parameters); the errors are summed and compared in fp32; the first smallest error
// wins, candidate 0 is the plain rule.  All lanes of the group return the same index.
constexpr int MSE_CANDIDATES = 80;
// one value's squared error in units of the scale: t = v / s + z, ((t - clamp(rne(t), 0, qmax)))^2; the caller
// multiplies the sum by s^2.  (rne(v / s) + z and rne(v / s + z) agree except at exact ties, where both choices give
// the same error.)
__device__ __forceinline__ float mse_term(float v, float zi, float rsi, float qmax) {
    const float t = fmaf(v, rsi, zi);
    const float d = t - __builtin_amdgcn_fmed3f(rintf(t), 0.f, qmax);
    return d * d;
}
template <typename P, typename R>
__device__ __forceinline__ int mse_search(const double mn, const double mx, const double qmax, const double qs,
                                          P&& partial, R&& reduce) {
    float best = 3.0e38f;
    int ibest = 0;
#pragma unroll 1
    for (int i = 0; i < MSE_CANDIDATES; ++i) {
        double sd, zd;
        grid_params(mn, mx, i, qmax, qs, sd, zd);
        const float si = float(sd);
        const float err = si * si * reduce(partial(float(zd), 1.0f / si));
        if (err < best) { best = err; ibest = i; }
    }
    return ibest;
}

constexpr int PANEL_LDS = (SB * SB + 2 * ROWS * SP + 2 * SB + 3 * ROWS * 8) * 4;

template <int CTRL>
__device__ __forceinline__ float dpp_quad(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
template <int CTRL>
__device__ __forceinline__ double dpp_quad(double v) {
    const uint64_t u = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = uint32_t(__builtin_amdgcn_update_dpp(0, int(uint32_t(u)), CTRL, 0xF, 0xF, true));
    const uint32_t hi = uint32_t(__builtin_amdgcn_update_dpp(0, int(uint32_t(u >> 32)), CTRL, 0xF, 0xF, true));
    return __builtin_bit_cast(double, (uint64_t(hi) << 32) | lo);
}
constexpr int quad_bcast(int o) { return o | (o << 2) | (o << 4) | (o << 6); }
constexpr int QUAD_SWAP1 = 1 | (0 << 2) | (3 << 4) | (2 << 6);   // lanes 0<->1, 2<->3
constexpr int QUAD_SWAP2 = 2 | (3 << 2) | (0 << 4) | (1 << 6);   // lanes 0<->2, 1<->3

// What a block of 128 columns starts from.  The feedback of all earlier columns is kept apart from the weights:
//   sC   (LDS, fp32)  c = -sum_i e_i U_i,col over the finished columns i: the part from earlier super-blocks comes
//                     from the working copy (a.Wf), the part from the earlier blocks of this super-block from the
//                     near update (split-fp16 MFMAs accumulated from zero), the part from the earlier inner blocks
//                     of this block from fp32 MFMAs accumulated from zero; each part is added once in fp32;
//   sE   (LDS, fp32)  an unfinished column holds its ORIGINAL weight w0 (exact: the input is bf16 or fp32); once the
//                     column is finished the slot receives its error e (sC's slot its code).
// The value that is quantized is w0 + c formed in fp64.
//
// DIRECT (block form of the factor): a.U holds U only on its 128 x 128 diagonal blocks and -U_jj R_jk / R_kk
// elsewhere (R = U^-1).  The working copy then accumulates c_k = sum_i (w_i - w^_i) R_ik / R_kk over the finished
// columns i of earlier blocks, where w are the ORIGINAL weights; a block starts from
//   w_b + c Un_bb ,   Un_bb = rows of U_bb divided by their diagonal entries,
// which is the state the sweep with the full U has on entering the block (e = (w - w^) R and
// U_AB = -U_AA R_AB U_BB for finished columns A, remaining columns B).  Inside the block nothing changes; what the
// block passes on is w - w^ measured from the original weights instead of the compensated ones.
template <int GB, bool DIRECT>  // GB: group width seen inside an inner block: 16 (G == 16) or 32 (G = 32, 64, 128)
__device__ __forceinline__ void panel_body(const PanelArgs& a, const int wg, char* psm) {
    float* sU = reinterpret_cast<float*>(psm);   // SB x SB: U[j0 + j][j0 .. j0 + 127], filled by direct loads
    float* sC = sU + SB * SB;                    // ROWS x SP feedback sums / codes (see above)
    float* sE = sC + ROWS * SP;                  // ROWS x SP original weights / errors e
    double* sRd = reinterpret_cast<double*>(sE + ROWS * SP);   // SB reciprocals of the diagonal
    double* sS = sRd + SB;                       // ROWS x 8 scales of the block's groups (fp64; returned rounded to fp32)
    float* sZ = reinterpret_cast<float*>(sS + ROWS * 8);       // ROWS x 8 zero points

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r0 = wg * ROWS;
    const int64_t d_in = a.d_in;
    const int G = 1 << a.lgG;
    // sequential part: quad = row, lane in quad = slice of 8 columns
    const int qrow = tid >> 2, sl = tid & 3;
    const int grow = min(r0 + qrow, a.d_out - 1);
    const bool row_ok = (r0 + qrow) < a.d_out;
    // MFMA accumulator layout: register r of lane l = row (r/4)*8 + (l/32)*4 + r%4, column l%32
    const int lr = (lane >> 5) * 4, lc = lane & 31;
    const double qmax = double(a.qmax), qsd = double(a.qs);
    const float f_d = a.sc->f_d, f_inv = a.sc->f_inv;
    const uint32_t ldsU = uint32_t(uintptr_t((ONECOMP_LDS char*)psm));
    double s = 1.0, rs = 1.0, z = 0.0;
    float lossacc = 0.f;
    bool saturated = false;
    if (a.wide_g >= 0) {
        s = a.s64[grow];
        z = double(a.zeros[int64_t(grow) * a.n_g + a.wide_g]);
        rs = 1.0 / s;
    }

#pragma unroll 1
    for (int b = 0; b < a.nb; ++b) {
        const int j0 = a.s0 + b * SB;
        __syncthreads();   // everybody is done with the previous block's tiles
        if (a.wide_g >= 0 && sl == 0) {   // published by the barriers below, long before the first use
            sS[qrow * 8] = s;
            sZ[qrow * 8] = float(z);
        }
        // ---- U diagonal block -> sU, two rows (1 KB) per wave load, no registers involved
        {
            const float* ub = a.U + int64_t(j0) * d_in + j0;
            __amdgpu_buffer_rsrc_t rsrc =
                __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(ub), 0, int((int64_t(SB - 1) * d_in + SB) * 4), 0x00020000);
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const int row = 2 * (16 * wave + q) + (lane >> 5);
                lds_load16(ldsU + (16 * wave + q) * 1024, uint32_t((int64_t(row) * d_in + (lane & 31) * 4) * 4), rsrc);
            }
        }
        // The original weights of two of the block's eight 32 x 32 tiles, in accumulator layout: row tile 0 / 1 of
        // column tile `wave` (DIRECT: (0, wave) and (1, 3 - wave), the tiles this wave transforms).  Requested here
        // so that they arrive behind the near update; DIRECT keeps them in registers until the block is done.
        float16v w0r[2];
        auto load_w0 = [&](float16v(&dst)[2]) __attribute__((always_inline)) {
            // 32 independent loads in straight-line code (one uniform branch on the element type around them); the
            // workgroup's rows span less than 2^31 elements, so a uniform base and 32-bit lane offsets address them
            int off[2][16];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                const int p = j0 + ((!DIRECT || mt == 0) ? wave : 3 - wave) * 32 + lc;
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    off[mt][r] = (min(r0 + mt * 32 + (r / 4) * 8 + lr + (r % 4), a.d_out - 1) - r0) * int(d_in) + p;
            }
            if (a.w0_bf16) {
                const uint16_t* wp = static_cast<const uint16_t*>(a.W0) + int64_t(r0) * d_in;
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) dst[mt][r] = __uint_as_float(uint32_t(wp[off[mt][r]]) << 16);
            } else {
                const float* wp = static_cast<const float*>(a.W0) + int64_t(r0) * d_in;
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) dst[mt][r] = wp[off[mt][r]];
            }
        };
        load_w0(w0r);
        // ---- feedback sums of this block's columns, wave = column tile: what earlier super-blocks left in the
        // working copy plus the near update from the earlier blocks of this super-block, accumulated from zero
        {
            float16v cf[2], acc[2];
            {
                const float* cbase = a.Wf + int64_t(r0) * d_in;
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int rr = min(r0 + mt * 32 + (r / 4) * 8 + lr + (r % 4), a.d_out - 1) - r0;
                        cf[mt][r] = cbase[rr * int(d_in) + j0 + 32 * wave + lc];
                        acc[mt][r] = 0.f;
                    }
            }
            if (b > 0)
            {
                // rolling window of WIN k-steps of operand fragments (a source block has 8 k-steps)
                constexpr int WIN = 4;
                uint4v win[WIN][6];
                // uniform base pointers + a 32-bit lane offset: the addresses stay in scalar registers
                const uint4v* fh = reinterpret_cast<const uint4v*>(a.Fh) + int64_t(wg) * 3 * 8 * 2 * 64;
                const uint4v* fl = reinterpret_cast<const uint4v*>(a.Fl) + int64_t(wg) * 3 * 8 * 2 * 64;
                const uint4v* bh = reinterpret_cast<const uint4v*>(a.Bh) + (b * (b - 1) / 2) * 8 * 4 * 64 + wave * 64;
                const uint4v* bl = reinterpret_cast<const uint4v*>(a.Bl) + (b * (b - 1) / 2) * 8 * 4 * 64 + wave * 64;
                auto issue = [&](int bp, int ks, uint4v(&d)[6]) __attribute__((always_inline)) {
                    const int fo = (bp * 8 + ks) * 2 * 64, bo = (bp * 8 + ks) * 4 * 64;
                    d[0] = (fl + fo)[lane]; d[1] = (fh + fo)[lane]; d[2] = (fl + fo + 64)[lane]; d[3] = (fh + fo + 64)[lane];
                    d[4] = (bh + bo)[lane]; d[5] = (bl + bo)[lane];
                };
#pragma unroll
                for (int ks = 0; ks < WIN; ++ks) issue(0, ks, win[ks]);
#pragma unroll 1
                for (int bp = 0; bp < b; ++bp) {
                    const bool more = bp + 1 < b;
#pragma unroll
                    for (int ks = 0; ks < 8; ++ks) {
                        uint4v(&cur)[6] = win[ks % WIN];
                        const half8v al0 = __builtin_bit_cast(half8v, cur[0]), ah0 = __builtin_bit_cast(half8v, cur[1]);
                        const half8v al1 = __builtin_bit_cast(half8v, cur[2]), ah1 = __builtin_bit_cast(half8v, cur[3]);
                        const half8v bhv = __builtin_bit_cast(half8v, cur[4]), blv = __builtin_bit_cast(half8v, cur[5]);
                        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(al0, bhv, acc[0], 0, 0, 0);
                        acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(al1, bhv, acc[1], 0, 0, 0);
                        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah0, blv, acc[0], 0, 0, 0);
                        acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah1, blv, acc[1], 0, 0, 0);
                        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah0, bhv, acc[0], 0, 0, 0);
                        acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah1, bhv, acc[1], 0, 0, 0);
                        // refill the slot just consumed: k-step ks + WIN of this source block or of the next
                        if (ks + WIN < 8) issue(bp, ks + WIN, cur);
                        else if (more) issue(bp + 1, ks + WIN - 8, cur);
                    }
                }
            }
            // c = (near update) / (f_d f_u) + (earlier super-blocks): one fp32 rounding
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[mt][r] = __builtin_fmaf(acc[mt][r], f_inv, cf[mt][r]);
            if constexpr (!DIRECT) {
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int o = (mt * 32 + (r / 4) * 8 + lr + (r % 4)) * SP + 32 * wave + lc;
                        sC[o] = acc[mt][r];
                        sE[o] = w0r[mt][r];
                    }
            }
            __builtin_amdgcn_s_waitcnt(wait_vmcnt(0));   // the direct loads into sU have landed
            __syncthreads();
            if (tid < SB) sRd[tid] = 1.0 / double(sU[tid * SB + tid]);
            __syncthreads();
            if constexpr (DIRECT) {
                // c_k / U_kk -> sE (free until the original weights go there), as the A operand of
                // c Un_bb = (c / diag) U_bb
                if (j0 > 0) {
                    const float rd = float(sRd[32 * wave + lc]);
#pragma unroll
                    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            sE[(mt * 32 + (r / 4) * 8 + lr + (r % 4)) * SP + 32 * wave + lc] = acc[mt][r] * rd;
                    __syncthreads();
                }
                // eight 32 x 32 tiles of (c / diag) U_bb, accumulated from zero; column tile nt needs k < 32 (nt + 1)
                // (U_bb is upper triangular), so wave w takes (row tile 0, column tile w) and (1, 3 - w): five chunks
                // of 32 k, 16 MFMAs each.  A chunk's 32 operand values are read before its first MFMA, and the two
                // tiles' chunks alternate so that one tile's LDS reads fall behind the other's MFMAs.
                float16v c0, c1;
#pragma unroll
                for (int r = 0; r < 16; ++r) { c0[r] = 0.f; c1[r] = 0.f; }
                if (j0 > 0) {
                    const int nt0 = wave, nt1 = 3 - wave;
                    const float* ap0 = sE + lc * SP + (lane >> 5);
                    const float* ap1 = sE + (32 + lc) * SP + (lane >> 5);
                    const float* bp0 = sU + (lane >> 5) * SB + nt0 * 32 + lc;
                    const float* bp1 = sU + (lane >> 5) * SB + nt1 * 32 + lc;
                    auto chunk = [&](float16v& c, const float* ap, const float* bp, const int ch) __attribute__((always_inline)) {
                        float av[16], bv[16];
#pragma unroll
                        for (int kk = 0; kk < 16; ++kk) {
                            av[kk] = ap[32 * ch + 2 * kk];
                            bv[kk] = bp[(32 * ch + 2 * kk) * SB];
                        }
#pragma unroll
                        for (int kk = 0; kk < 16; ++kk) c = __builtin_amdgcn_mfma_f32_32x32x2f32(av[kk], bv[kk], c, 0, 0, 0);
                    };
#pragma unroll 1
                    for (int ch = 0; ch < 4; ++ch) {
                        if (ch <= nt0) chunk(c0, ap0, bp0, ch);
                        if (ch <= nt1) chunk(c1, ap1, bp1, ch);
                    }
                    __syncthreads();   // every wave is done reading sE as an operand
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int o0 = ((r / 4) * 8 + lr + (r % 4)) * SP + wave * 32 + lc;
                    const int o1 = (32 + (r / 4) * 8 + lr + (r % 4)) * SP + (3 - wave) * 32 + lc;
                    sC[o0] = c0[r]; sE[o0] = w0r[0][r];
                    sC[o1] = c1[r]; sE[o1] = w0r[1][r];
                }
                __syncthreads();
            }
        }

#pragma unroll 1
        for (int jb = 0; jb < SB; jb += IB) {
            {
                double w[8];
                {
                    const float* cp = sC + qrow * SP + jb + 8 * sl;
                    const float* wp = sE + qrow * SP + jb + 8 * sl;
#pragma unroll
                    for (int i = 0; i < 8; ++i) w[i] = double(wp[i]) + double(cp[i]);
                }
                // row j of the inner block's U triangle (this lane's 8 columns) and 1 / U_jj, one step ahead
                float4v ua[2], ub[2];
                double rdc = sRd[jb], rdn = 0.0;
                const float* up = sU + jb * SB + jb + 8 * sl;
                ua[0] = *reinterpret_cast<const float4v*>(up);
                ua[1] = *reinterpret_cast<const float4v*>(up + 4);
                static_for<0, IB>([&](auto jc) {
                    constexpr int j = decltype(jc)::value;
                    auto step = [&](float4v(&cur)[2], float4v(&nxt)[2]) __attribute__((always_inline)) {
                        if constexpr (j + 1 < IB) {
                            nxt[0] = *reinterpret_cast<const float4v*>(up + (j + 1) * SB);
                            nxt[1] = *reinterpret_cast<const float4v*>(up + (j + 1) * SB + 4);
                            rdn = sRd[jb + j + 1];
                        }
                        if constexpr (j % GB == 0) {
                            const int col = j0 + jb + j;
                            bool fresh;
                            double mn, mx;
                            if constexpr (GB == 16) {
                                // group = the 16 columns held by lanes 2 (j / 16) and 2 (j / 16) + 1 of the quad
                                fresh = true;
                                mn = w[0]; mx = w[0];
#pragma unroll
                                for (int i = 1; i < 8; ++i) { mn = fmin(mn, w[i]); mx = fmax(mx, w[i]); }
                                mn = fmin(mn, dpp_quad<QUAD_SWAP1>(mn));
                                mx = fmax(mx, dpp_quad<QUAD_SWAP1>(mx));
                                mn = dpp_quad<quad_bcast(j / 8)>(mn);
                                mx = dpp_quad<quad_bcast(j / 8)>(mx);
                            } else {
                                fresh = a.wide_g < 0 && (col & (G - 1)) == 0;
                                if (fresh) {   // uniform: the group's G <= 128 columns are unfinished, w0 in sE, c in sC
                                    const float* gc = sC + qrow * SP + jb + sl;
                                    const float* gw = sE + qrow * SP + jb + sl;
                                    mn = double(gw[0]) + double(gc[0]); mx = mn;
                                    for (int c = 4; c < G; c += 4) {
                                        const double v = double(gw[c]) + double(gc[c]);
                                        mn = fmin(mn, v); mx = fmax(mx, v);
                                    }
                                    mn = fmin(mn, dpp_quad<QUAD_SWAP1>(mn));
                                    mx = fmax(mx, dpp_quad<QUAD_SWAP1>(mx));
                                    mn = fmin(mn, dpp_quad<QUAD_SWAP2>(mn));
                                    mx = fmax(mx, dpp_quad<QUAD_SWAP2>(mx));
                                }
                            }
                            if (fresh) {
                                int cand = 0;
                                if constexpr (GB != 16) {
                                    if (a.mse) {   // uniform; this lane's quarter of the group, held in registers
                                        const float* gc = sC + qrow * SP + jb + sl;
                                        const float* gw = sE + qrow * SP + jb + sl;
                                        float gv[32];
#pragma unroll
                                        for (int k = 0; k < 32; ++k) {
                                            const int c = (4 * k) & (G - 1);
                                            gv[k] = float(double(gw[c]) + double(gc[c]));
                                        }
                                        const int n8 = G >> 5;   // batches of 8 values: 1, 2 or 4
                                        const float qmf = a.qmax;
                                        cand = mse_search(mn, mx, qmax, qsd,
                                                   [&](float zi, float rsi) __attribute__((always_inline)) {
                                                       float e0 = 0.f, e1 = 0.f;
#pragma unroll
                                                       for (int k = 0; k < 8; k += 2) {
                                                           e0 += mse_term(gv[k], zi, rsi, qmf);
                                                           e1 += mse_term(gv[k + 1], zi, rsi, qmf);
                                                       }
                                                       if (n8 > 1) {
#pragma unroll
                                                           for (int k = 8; k < 16; k += 2) {
                                                               e0 += mse_term(gv[k], zi, rsi, qmf);
                                                               e1 += mse_term(gv[k + 1], zi, rsi, qmf);
                                                           }
                                                       }
                                                       if (n8 > 2) {
#pragma unroll
                                                           for (int k = 16; k < 32; k += 2) {
                                                               e0 += mse_term(gv[k], zi, rsi, qmf);
                                                               e1 += mse_term(gv[k + 1], zi, rsi, qmf);
                                                           }
                                                       }
                                                       return e0 + e1;
                                                   },
                                                   [&](float x) __attribute__((always_inline)) {
                                                       x += dpp_quad<QUAD_SWAP1>(x);
                                                       return x + dpp_quad<QUAD_SWAP2>(x);
                                                   });
                                    }
                                } else {
                                    if (a.mse) {   // uniform; the group's 16 values sit in two lanes of the quad
                                        float gv[8];
#pragma unroll
                                        for (int k = 0; k < 8; ++k) gv[k] = float(w[k]);
                                        const float qmf = a.qmax;
                                        cand = mse_search(mn, mx, qmax, qsd,
                                                   [&](float zi, float rsi) __attribute__((always_inline)) {
                                                       float e0 = 0.f, e1 = 0.f;
#pragma unroll
                                                       for (int k = 0; k < 8; k += 2) {
                                                           e0 += mse_term(gv[k], zi, rsi, qmf);
                                                           e1 += mse_term(gv[k + 1], zi, rsi, qmf);
                                                       }
                                                       return e0 + e1;
                                                   },
                                                   [&](float x) __attribute__((always_inline)) {
                                                       x += dpp_quad<QUAD_SWAP1>(x);
                                                       return dpp_quad<quad_bcast(j / 8)>(x);
                                                   });
                                    }
                                }
                                grid_params(mn, mx, cand, qmax, qsd, s, z);
                                rs = 1.0 / s;
                                if (sl == 0) {
                                    const int gi = (jb + j) >> a.lgG;
                                    sS[qrow * 8 + gi] = s;
                                    sZ[qrow * 8 + gi] = float(z);
                                    if (row_ok) {
                                        a.scales[int64_t(grow) * a.n_g + (col >> a.lgG)] = float(s);
                                        a.zeros[int64_t(grow) * a.n_g + (col >> a.lgG)] = float(z);
                                    }
                                }
                            }
                        }
                        const double wj = dpp_quad<quad_bcast(j / 8)>(w[j % 8]);
                        // w / s correctly rounded, as the definition's division gives it (an exact tie, possible in a
                        // row's first group where weights and scale are short binary numbers, then falls the same way):
                        // t0 = w * fl(1 / s), residual by FMA, one correction step; no division, no branch
                        const double t0 = wj * rs;
                        const double t = __builtin_fma(__builtin_fma(-t0, s, wj), rs, t0);
                        const double q = fmin(fmax(rint(t) + z, 0.0), qmax);
                        const double e = __builtin_fma(-s, q - z, wj) * rdc;         // (w - s (q - z)) / U_jj
                        // feedback inside the inner block: w_k -= e U_jk.  Columns up to j are finished, updating
                        // them is harmless; in the last slice the finished registers are skipped.
                        // The register the next step broadcasts comes first, and every update is pinned to this step:
                        // left alone, the compiler sinks each register's updates to its next use, a dependent chain
                        // of up to 32 FMAs in front of a decision (and recomputed for each of the four lanes' turns).
#pragma unroll
                        for (int ii = 0; ii < 8; ++ii) {
                            const int i = (j + 1 + ii) % 8;
                            if (j < 24 || i > j % 8) {
                                w[i] = __builtin_fma(-e, double(cur[i / 4][i % 4]), w[i]);
                                asm volatile("" : "+v"(w[i]));
                            }
                        }
                        sE[qrow * SP + jb + j] = float(e);
                        sC[qrow * SP + jb + j] = float(q);
                        rdc = rdn;
                    };
                    if constexpr (j % 2 == 0) step(ua, ub);
                    else step(ub, ua);
                });
            }
            __syncthreads();
            // remaining columns of the block: c_col -= sum_i e_i U[jb+i][col], col >= jb + 32, on 32 x 32 tiles
            // accumulated from zero and then added to the tile in LDS
            const int cs = jb + IB;
            if (cs < SB)
            {
                const int n_tiles = 2 * ((SB - cs) / 32);
                for (int t = wave; t < n_tiles; t += 4) {
                    const int mt = t & 1, nt = t >> 1;
                    float* cp = sC + (mt * 32 + lr) * SP + cs + nt * 32 + lc;
                    float16v c;
#pragma unroll
                    for (int r = 0; r < 16; ++r) c[r] = 0.f;
                    const float* ap = sE + (mt * 32 + lc) * SP + jb + (lane >> 5);
                    const float* bp = sU + (jb + (lane >> 5)) * SB + cs + nt * 32 + lc;
#pragma unroll
                    for (int kk = 0; kk < IB / 2; ++kk)
                        c = __builtin_amdgcn_mfma_f32_32x32x2f32(-ap[2 * kk], bp[2 * kk * SB], c, 0, 0, 0);
#pragma unroll
                    for (int r = 0; r < 16; ++r) cp[((r / 4) * 8 + (r % 4)) * SP] += c[r];
                }
            }
            __syncthreads();
        }

        // ---- block done: loss, residual panels, outputs
        {   // sum of e^2 of this row's quarter of the block, then over the quad
            float acc = 0.f;
            const float* ep = sE + qrow * SP + 32 * sl;
#pragma unroll 8
            for (int c = 0; c < 32; ++c) acc = __builtin_fmaf(ep[c], ep[c], acc);
            acc += dpp_quad<QUAD_SWAP1>(acc);
            acc += dpp_quad<QUAD_SWAP2>(acc);
            lossacc += acc;
        }
        // residual w - w^ = e U_jj, negated, scaled by a power of two and split into fp16 hi + lo
        // (hi = rne(x), lo = rne(x - hi): 22 significant bits); saturated far above anything a sweep of a sane layer
        // produces, and the saturation is reported (the loss then comes back as +infinity).
        auto split8 = [&](auto&& value, short8v& dh, short8v& dl) __attribute__((always_inline)) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float x = value(e);
                saturated |= !(fabsf(x) <= 60000.f);
                x = fminf(fmaxf(x, -60000.f), 60000.f);
                const _Float16 h = (_Float16)x;
                const _Float16 lo = (_Float16)(x - (float)h);
                dh[e] = __builtin_bit_cast(short, h);
                dl[e] = __builtin_bit_cast(short, lo);
            }
        };
        float* sO = sU;   // DIRECT: w - w^ against the original weights, ROWS x SP (the U block is no longer needed)
        if constexpr (DIRECT) {
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                const int col = (mt == 0 ? wave : 3 - wave) * 32 + lc, gi = col >> a.lgG;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int rr = mt * 32 + (r / 4) * 8 + lr + (r % 4);
                    // w0 - s (q - z) with the fp64 scale the sweep used
                    sO[rr * SP + col] = float(__builtin_fma(-sS[rr * 8 + gi], double(sC[rr * SP + col] - sZ[rr * 8 + gi]),
                                                            double(w0r[mt][r])));
                }
            }
            __syncthreads();
        }
        // transposed panel (k-major) for the far update; rows past d_out hold copies of the last row
        for (int it = tid; it < SB * (ROWS / 8); it += 256) {
            const int c = it / (ROWS / 8), r8 = (it % (ROWS / 8)) * 8;
            const float ujj = DIRECT ? 0.f : sU[c * SB + c] * f_d;
            short8v dh, dl;
            if constexpr (DIRECT) split8([&](int e) { return -sO[(r8 + e) * SP + c] * f_d; }, dh, dl);
            else split8([&](int e) { return -sE[(r8 + e) * SP + c] * ujj; }, dh, dl);
            const int64_t off = int64_t(b * SB + c) * a.ldD + r0 + r8;
            *reinterpret_cast<short8v*>(a.Dh + off) = dh;
            *reinterpret_cast<short8v*>(a.Dl + off) = dl;
        }
        // MFMA A-operand fragments for this workgroup's own near updates: lane L of k-step ks, row tile mt holds
        // row mt*32 + L%32, columns ks*16 + 8 (L/32) + 0..7
        if (b + 1 < a.nb)
        {
            for (int it = tid; it < 8 * 2 * 64; it += 256) {
                const int L = it & 63, row = ((it >> 6) & 1) * 32 + (L & 31), c0 = (it >> 7) * 16 + 8 * (L >> 5);
                short8v dh, dl;
                if constexpr (DIRECT) split8([&](int e) { return -sO[row * SP + c0 + e] * f_d; }, dh, dl);
                else split8([&](int e) { return -sE[row * SP + c0 + e] * (sU[(c0 + e) * SB + c0 + e] * f_d); }, dh, dl);
                const int64_t off = ((int64_t(wg) * 3 + b) * (8 * 2 * 64) + it) * 8;
                *reinterpret_cast<short8v*>(a.Fh + off) = dh;
                *reinterpret_cast<short8v*>(a.Fl + off) = dl;
            }
        }
        // W^ = s (q - z) and codes, in sweep order (see unpermute_kernel)
        for (int it = wave; it < ROWS / 2; it += 4) {
            const int rr = it * 2 + (lane >> 5), c4 = (lane & 31) * 4;
            const int gr = r0 + rr;
            if (gr >= a.d_out) continue;
            float qv[4], hv[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int gi = (c4 + e) >> a.lgG;
                qv[e] = sC[rr * SP + c4 + e];
                hv[e] = float(sS[rr * 8 + gi]) * (qv[e] - sZ[rr * 8 + gi]);
            }
            if (a.W_hat) {
                const float4v h = {hv[0], hv[1], hv[2], hv[3]};
                *reinterpret_cast<float4v*>(a.W_hat + int64_t(gr) * d_in + j0 + c4) = h;
            }
            const uint32_t pk = uint32_t(qv[0]) | (uint32_t(qv[1]) << 8) | (uint32_t(qv[2]) << 16) | (uint32_t(qv[3]) << 24);
            *reinterpret_cast<uint32_t*>(a.Q + int64_t(gr) * d_in + j0 + c4) = pk;
        }
        // the fragments written above are read back by other waves of this workgroup (same CU, same L1): a
        // workgroup-scope release, completed by the barrier at the top of the loop
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    }
    if (sl == 0 && row_ok) a.rowloss[grow] += lossacc;
    if (saturated) *a.sat = 1u;
}

// Fragments of the normalized U blocks the panel kernel's near updates multiply with: for super-block S (sbw
// columns wide, gridDim.x = its number of block pairs), block pair p = b (b - 1) / 2 + b' (b' < b), k-step ks,
// column tile nt, lane L:
//   Un[sbw S + 128 b' + 16 ks + 8 (L/32) + e][sbw S + 128 b + 32 nt + L%32] * f_u,  e = 0 .. 7,  fp16 hi and lo.
__global__ __launch_bounds__(256) void nearfrag_kernel(const float* __restrict__ U, int n, const Scalars* __restrict__ sc,
                                                      uint16_t* __restrict__ Bh, uint16_t* __restrict__ Bl, int sbw) {
    const int S = blockIdx.y, p = blockIdx.x;
    const int b = (p >= 3) ? 3 : (p >= 1 ? 2 : 1), bp = p - b * (b - 1) / 2;
    const int k00 = S * sbw + bp * SB, n00 = S * sbw + b * SB;
    if (n00 >= n) return;
    const float f_u = sc->f_u;
    for (int it = threadIdx.x; it < 8 * 4 * 64; it += 256) {
        const int L = it & 63, nt = (it >> 6) & 3, ks = it >> 8;
        const int col = n00 + nt * 32 + (L & 31), k0 = k00 + ks * 16 + 8 * (L >> 5);
        short8v h8, l8;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float dj = U[int64_t(k0 + e) * n + k0 + e];
            float x = U[int64_t(k0 + e) * n + col] / dj * f_u;
            x = fminf(fmaxf(x, -60000.f), 60000.f);
            const _Float16 h = (_Float16)x;
            const _Float16 lo = (_Float16)(x - (float)h);
            h8[e] = __builtin_bit_cast(short, h);
            l8[e] = __builtin_bit_cast(short, lo);
        }
        const int64_t off = ((int64_t(S) * gridDim.x + p) * (8 * 4 * 64) + it) * 8;
        *reinterpret_cast<short8v*>(Bh + off) = h8;
        *reinterpret_cast<short8v*>(Bl + off) = l8;
    }
}

// ------------------------------------------------------------------------------------------
// Operands of the trailing GEMMs (once per layer).  The feedback e_j U_jk is computed as
// (w_j - w^_j) * (U_jk / U_jj): the residual is bounded by the weights and the normalized row by the
// regression coefficients between input channels, so both fit fp16 after a power-of-two scaling taken
// from their maxima, whereas e and U themselves span the scale of 1 / sqrt(H_jj).
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void umax_kernel(const float* __restrict__ U, int n, Scalars* __restrict__ sc) {
    // max_k |U_jk / U_jj| = max_k |U_jk| / |U_jj| exactly: rounding a quotient is monotone in the numerator
    float mm = 0.f;
    for (int j = blockIdx.x; j < n; j += gridDim.x) {   // a workgroup per row, rows strided over the grid
        const float* row = U + int64_t(j) * n;
        float m = 0.f;
        for (int k4 = ((j + 1) & ~3) + 4 * threadIdx.x; k4 < n; k4 += 1024) {
            const float4v v = *reinterpret_cast<const float4v*>(row + k4);
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (k4 + e > j) m = fmaxf(m, fabsf(v[e]));
        }
        m = m / fabsf(row[j]);
        if (!(m < 3.0e38f)) m = 3.0e38f;   // NaN / inf from a failed factorization: keep the scalars finite
        mm = fmaxf(mm, m);
    }
    block_max_to(&sc->max_u_bits, mm);
}

__global__ void scale_kernel(Scalars* sc) {
    // largest magnitudes land at 2^13 (residuals, x8 headroom before saturation) and 2^14 (rows of U)
    const float mw = __uint_as_float(sc->max_w_bits), mu = __uint_as_float(sc->max_u_bits);
    int ew = 0, eu = 0;
    if (mw > 0.f) (void)frexpf(mw, &ew);   // mw = m * 2^ew, 0.5 <= m < 1
    if (mu > 0.f) (void)frexpf(mu, &eu);
    const int sd = max(-60, min(60, 13 - ew)), su = max(-60, min(60, 14 - eu));
    sc->f_d = ldexpf(1.f, sd);
    sc->f_u = ldexpf(1.f, su);
    sc->f_all = ldexpf(1.f, sd + su);
    sc->f_inv = ldexpf(1.f, -(sd + su));
}

__global__ __launch_bounds__(256) void split_kernel(const float* __restrict__ U, int n,
                                                   const Scalars* __restrict__ sc, uint16_t* __restrict__ Uh,
                                                   uint16_t* __restrict__ Ul) {
    const int j = blockIdx.y;
    const int k4 = (blockIdx.x * 256 + threadIdx.x) * 4;
    // the trailing updates read row j only beyond its 128-column block; the rest of Uh / Ul stays unwritten
    if (k4 >= n || k4 < (j / SB + 1) * SB) return;
    const float4v v = *reinterpret_cast<const float4v*>(U + int64_t(j) * n + k4);
    const float dj = U[int64_t(j) * n + j], f_u = sc->f_u;
    short4v h4, l4;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        float x = v[e] / dj * f_u;
        x = fminf(fmaxf(x, -60000.f), 60000.f);
        const _Float16 h = (_Float16)x;
        const _Float16 lo = (_Float16)(x - (float)h);
        h4[e] = __builtin_bit_cast(short, h);
        l4[e] = __builtin_bit_cast(short, lo);
    }
    *reinterpret_cast<short4v*>(Uh + int64_t(j) * n + k4) = h4;
    *reinterpret_cast<short4v*>(Ul + int64_t(j) * n + k4) = l4;
}

// ------------------------------------------------------------------------------------------
// trailing update:  Wf[:, c0 .. c1) += f_inv * D[:, ek .. ek+K) * Un[u0 .. u0+K, c0 .. c1)
// with D = -(w - w^) f_d (stored transposed, Dt[k][row], by the panel kernel) and Un = U_jk / U_jj f_u
// (split_kernel).
//
// fp32 accuracy from fp16 MFMAs: both operands are split x = hi + lo (fp16 each, |lo| <= 2^-11 |hi|) and
// three products are accumulated in fp32, hi*hi + hi*lo + lo*hi; the dropped lo*lo term and the rounding
// of lo are ~2^-22 relative to each product, i.e. the level of fp32 rounding itself.
//
// 128 x 256 tile per workgroup, 4 waves in 2 x 2 (64 x 128 each: 2 x 4 tiles of v_mfma_f32_32x32x16_f16, three
// products each), two workgroups per CU so that one workgroup's read and write of its W tile (the update is
// close to the HBM / MFMA ridge: 384 flop per byte of W at K = 512) overlaps the other's inner loop.
// Both operands are k-major, their fragments come from LDS transpose reads.  Operand tiles go global -> LDS
// directly (lds_load16) in steps of 16 k: four panels (Dt hi, Dt lo, Un hi, Un lo) of 16 rows, 24 KB, in a
// ring of three slots.  16-byte chunk c of panel row r sits at chunk position c ^ ((r & 3) << 2), which spreads
// the four rows of a transpose read over four 64-byte bank groups.
// Half-iteration h:  24 MFMAs on the fragments of k-step h (registers);  LDS -> fragments of k-step h+1;
// loads of k-step h+3 into the slot k-step h was read from;  wait for k-step h+2 + barrier.
// Tiles are ranked so that each XCD (blockIdx % 8) owns a contiguous run, m fastest inside bands of 8 row tiles:
// the workgroups resident on one XCD share their Dt and Un panels through its L2.
// ------------------------------------------------------------------------------------------
namespace tg {
constexpr int TM = 128, TN = 256, KT = 16;
constexpr int A_ROWB = TM * 2, B_ROWB = TN * 2;                     // bytes per panel row
constexpr int A_PANELB = KT * A_ROWB, B_PANELB = KT * B_ROWB;       // 4 KB, 8 KB
constexpr int OFF_AH = 0, OFF_AL = A_PANELB, OFF_BH = 2 * A_PANELB, OFF_BL = 2 * A_PANELB + B_PANELB;
constexpr int STAGEB = 2 * A_PANELB + 2 * B_PANELB;                 // 24 KB
constexpr size_t LDS_BYTES = size_t(3) * STAGEB;                    // 72 KB with 3 slots: two workgroups per CU
}  // namespace tg

struct TrailArgs {
    float* Wf;
    const uint16_t *Dh, *Dl;   // [SBIG x ldD] fp16 bits
    const uint16_t *Uh, *Ul;   // [d_in x d_in] fp16 bits
    const Scalars* sc;
    int d_out, ldD, d_in;
    int ek, K, u0, c0, c1;     // K % 32 == 0, c0 % 8 == 0, c1 % 8 == 0
    int n_mt, n_nt, chunk;
};

// FROM_ZERO: the accumulators start at zero and the product is added to the tile of C once, at the end, with one
// fp32 rounding (the sweep: every rounding inside the MFMA chain then happens at the size of the increment, not of
// the sum it joins).  Otherwise the tile of C is loaded, scaled, into the accumulators before the loop.
template <int NBUF, bool FROM_ZERO>   // NBUF: slots of the LDS ring
__device__ __forceinline__ void trailing_tile(const TrailArgs& a, const int bid, char* tl) {
    using namespace tg;
    int mt_, nt_;
    if (!plan::trail_tile(bid, a.chunk, a.n_mt, a.n_nt, mt_, nt_)) return;
    const int m0 = mt_ * TM;
    const int n0 = a.c0 + nt_ * TN;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave >> 1, wc = wave & 1;
    const int d_out = a.d_out, c1 = a.c1;
    const int64_t d_in = a.d_in;
    const uint32_t lds0 = uint32_t(uintptr_t((ONECOMP_LDS char*)tl));

    // this wave's six 1 KB loads per k-step: Dt panels rows 4 wave .. 4 wave + 3 (one load each), Un panels the
    // same rows (two loads of two rows each)
    uint32_t voff_a, voff_b[2];
    {
        const int row = 4 * wave + (lane >> 4);
        const int c = (lane & 15) ^ ((row & 3) << 2);
        voff_a = (m0 + c * 8 < a.ldD) ? uint32_t((row * a.ldD + m0 + c * 8) * 2) : LDS_DMA_OOB;
    }
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int row = 4 * wave + 2 * q + (lane >> 5);
        const int c = (lane & 31) ^ ((row & 3) << 2);
        voff_b[q] = (n0 + c * 8 < c1) ? uint32_t((int64_t(row) * d_in + n0 + c * 8) * 2) : LDS_DMA_OOB;
    }
    const int n_kb = a.K / KT;
    struct Desc {
        __amdgpu_buffer_rsrc_t ah, al, bh, bl;
    };
    auto make_desc = [&](int kb, bool live) __attribute__((always_inline)) {
        Desc d;
        if (!live) kb = 0;
        const int64_t ea = (int64_t(a.ek) + kb * KT) * a.ldD, eb = (int64_t(a.u0) + kb * KT) * d_in;
        const int ra = live ? KT * a.ldD * 2 : 0, rb = live ? int(KT * d_in * 2) : 0;
        d.ah = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(a.Dh + ea), 0, ra, 0x00020000);
        d.al = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(a.Dl + ea), 0, ra, 0x00020000);
        d.bh = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(a.Uh + eb), 0, rb, 0x00020000);
        d.bl = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(a.Ul + eb), 0, rb, 0x00020000);
        return d;
    };
    // load number i (0..5) of a k-step into the slot at LDS byte address dst
    auto gload1 = [&](const Desc& d, uint32_t dst, int i) __attribute__((always_inline)) {
        if (i == 0) lds_load16(dst + OFF_AH + wave * 1024, voff_a, d.ah);
        else if (i == 1) lds_load16(dst + OFF_AL + wave * 1024, voff_a, d.al);
        else if (i == 2) lds_load16(dst + OFF_BH + wave * 2048, voff_b[0], d.bh);
        else if (i == 3) lds_load16(dst + OFF_BH + wave * 2048 + 1024, voff_b[1], d.bh);
        else if (i == 4) lds_load16(dst + OFF_BL + wave * 2048, voff_b[0], d.bl);
        else lds_load16(dst + OFF_BL + wave * 2048 + 1024, voff_b[1], d.bl);
    };

    // transpose-read addressing: within 16 lanes, lane 4 k + c reads 8 bytes of panel row k at byte 8 c of a
    // 32-byte column group; two reads (rows +0 and +4) make one MFMA operand (k = 8 (lane / 32) + 0..7)
    const int i16 = lane & 15, g16 = (lane >> 4) & 1, kb8 = lane >> 5;
    const int kq = i16 >> 2;
    const int lo = (2 * g16 + ((i16 & 3) >> 1)) * 16 + (i16 & 1) * 8;
    int fa[2], fb[4];
#pragma unroll
    for (int m = 0; m < 2; ++m) fa[m] = OFF_AH + (kb8 * 8 + kq) * A_ROWB + (((wr * 2 + m) ^ kq) << 6) + lo;
#pragma unroll
    for (int n = 0; n < 4; ++n) fb[n] = OFF_BH + (kb8 * 8 + kq) * B_ROWB + wc * 256 + ((n ^ kq) << 6) + lo;

    struct Frags {
        half8v ah[2], al[2], bh[4], bl[4];
    };
    auto rd2 = [&](const char* p, int rowb) __attribute__((always_inline)) {
        short4v x0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((ONECOMP_LDS short4v*)(p));
        short4v x1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((ONECOMP_LDS short4v*)(p + 4 * rowb));
        return __builtin_bit_cast(half8v, __builtin_shufflevector(x0, x1, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    // fragment r (0..11) of the slot at tl + sb, in the order the MFMAs use them
    auto rd = [&](Frags& f, int r, int sb) __attribute__((always_inline)) {
        const char* s = tl + sb;
        if (r == 0) f.al[0] = rd2(s + fa[0] + A_PANELB, A_ROWB);
        else if (r <= 4) f.bh[r - 1] = rd2(s + fb[r - 1], B_ROWB);
        else if (r == 5) f.ah[0] = rd2(s + fa[0], A_ROWB);
        else if (r <= 9) f.bl[r - 6] = rd2(s + fb[r - 6] + B_PANELB, B_ROWB);
        else if (r == 10) f.al[1] = rd2(s + fa[1] + A_PANELB, A_ROWB);
        else f.ah[1] = rd2(s + fa[1], A_ROWB);
    };

    // prologue: k-steps 0 .. 2 in flight, then the W tile (scaled by the exact power of two f_d f_u) straight into
    // the accumulators; register r of lane l is row (r/4)*8 + (l/32)*4 + r%4, column l%32 of a 32 x 32 tile
    for (int kb = 0; kb < NBUF; ++kb)
        if (kb < n_kb) {
            const Desc d = make_desc(kb, true);
#pragma unroll
            for (int i = 0; i < 6; ++i) gload1(d, lds0 + kb * STAGEB, i);
        }
    const float f_all = a.sc->f_all, f_inv = a.sc->f_inv;
    float16v acc[2][4];
    const int lr = (lane >> 5) * 4, lc = lane & 31;
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int n = 0; n < 4; ++n)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                if constexpr (FROM_ZERO) {
                    acc[m][n][r] = 0.f;
                } else {
                    const int rr = min(m0 + wr * 64 + m * 32 + (r / 4) * 8 + lr + (r % 4), d_out - 1);
                    const int cc = min(n0 + wc * 128 + n * 32 + lc, c1 - 1);
                    acc[m][n][r] = a.Wf[int64_t(rr) * d_in + cc] * f_all;
                }
            }
    __builtin_amdgcn_s_waitcnt(wait_vmcnt(0));
    __syncthreads();
    Frags Fc, FH;
#pragma unroll
    for (int r = 0; r < 12; ++r) rd(Fc, r, 0);
    __syncthreads();   // slot 0 is overwritten by the loads of the first half-iteration

    // the 24 MFMAs of one k-step: per row tile m the products lo*hi, hi*lo, hi*hi against the four column tiles,
    // consecutive MFMAs on different accumulators; `between(i)` is placed behind MFMA i
    auto mma = [&](const Frags& f, auto&& between) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 24; ++i) {
            const int m = i / 12, p = (i % 12) / 4, n = i % 4;
            if (p == 0) acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_f16(f.al[m], f.bh[n], acc[m][n], 0, 0, 0);
            else if (p == 1) acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_f16(f.ah[m], f.bl[n], acc[m][n], 0, 0, 0);
            else acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_f16(f.ah[m], f.bh[n], acc[m][n], 0, 0, 0);
            between(i);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    int s0 = 0;   // slot of k-step kb
#pragma unroll 1
    for (int kb = 0; kb < n_kb; kb += 2) {
        const int s1 = (s0 == NBUF - 1) ? 0 : s0 + 1, s2 = (s1 == NBUF - 1) ? 0 : s1 + 1;
        // Loads and fragment reads past the last k-step are not branched around: the loads get an empty
        // descriptor (they deposit zeros into a slot nobody reads again), the reads fetch stale data nobody uses.
        {   // k-step kb from Fc; fragments of kb+1 -> FH; loads of kb+NBUF -> slot s0
            const Desc d = make_desc(kb + NBUF, kb + NBUF < n_kb);
            const uint32_t dst = lds0 + s0 * STAGEB;
            const int sb = s1 * STAGEB;
            mma(Fc, [&](int i) __attribute__((always_inline)) {
                if ((i & 1) == 0) rd(FH, i / 2, sb);
                else if (i < 12) gload1(d, dst, i / 2);
            });
            __builtin_amdgcn_s_waitcnt(wait_vmcnt(6 * (NBUF - 2)));   // k-step kb+2 has landed
            __syncthreads();
        }
        {   // k-step kb+1 from FH; fragments of kb+2 -> Fc; loads of kb+1+NBUF -> slot s1
            const Desc d = make_desc(kb + 1 + NBUF, kb + 1 + NBUF < n_kb);
            const uint32_t dst = lds0 + s1 * STAGEB;
            const int sb = s2 * STAGEB;
            mma(FH, [&](int i) __attribute__((always_inline)) {
                if ((i & 1) == 0) rd(Fc, i / 2, sb);
                else if (i < 12) gload1(d, dst, i / 2);
            });
            __builtin_amdgcn_s_waitcnt(wait_vmcnt(6 * (NBUF - 2)));   // k-step kb+3 has landed
            __syncthreads();
        }
        s0 = s2;
    }
    __builtin_amdgcn_s_waitcnt(wait_vmcnt(0));   // no LDS write may be in flight when the workgroup ends
    // uniform branch: interior tiles store without per-element masks
    if ((m0 + TM <= d_out) && (n0 + TN <= c1)) {
        float* wp = a.Wf + int64_t(m0 + wr * 64 + lr) * d_in + n0 + wc * 128 + lc;
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            if constexpr (FROM_ZERO) {
                // the tile's current values: 32 independent loads at a time (the operand registers are free now)
#pragma unroll
                for (int n2 = 0; n2 < 4; n2 += 2) {
                    float16v old[2];
#pragma unroll
                    for (int n = 0; n < 2; ++n)
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            old[n][r] = wp[int64_t(m * 32 + (r / 4) * 8 + (r % 4)) * d_in + (n2 + n) * 32];
#pragma unroll
                    for (int n = 0; n < 2; ++n)
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            wp[int64_t(m * 32 + (r / 4) * 8 + (r % 4)) * d_in + (n2 + n) * 32] =
                                __builtin_fmaf(acc[m][n2 + n][r], f_inv, old[n][r]);
                }
            } else {
#pragma unroll
                for (int n = 0; n < 4; ++n)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        wp[int64_t(m * 32 + (r / 4) * 8 + (r % 4)) * d_in + n * 32] = acc[m][n][r] * f_inv;
            }
        }
    } else {
#pragma unroll
        for (int m = 0; m < 2; ++m)
#pragma unroll
            for (int n = 0; n < 4; ++n)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int rr = m0 + wr * 64 + m * 32 + (r / 4) * 8 + lr + (r % 4);
                    const int cc = n0 + wc * 128 + n * 32 + lc;
                    if (rr < d_out && cc < c1) {
                        float* q = a.Wf + int64_t(rr) * d_in + cc;
                        if constexpr (FROM_ZERO) *q = __builtin_fmaf(acc[m][n][r], f_inv, *q);
                        else *q = acc[m][n][r] * f_inv;
                    }
                }
    }
}

template <bool FROM_ZERO>
__global__ __launch_bounds__(256, 2) void trailing_kernel(TrailArgs a) {
    extern __shared__ __attribute__((aligned(1024))) char dyn_lds[];
    trailing_tile<3, FROM_ZERO>(a, blockIdx.x, dyn_lds);
}

// One launch = the panel sweep of a super-block next to the far update of the previous super-block on the
// columns beyond the panel's.  The panel needs only 64 rows' worth of workgroups, far fewer than there are CUs, and
// its workgroups are the first of the grid, so they are resident from the start; the update's tiles fill the other
// CUs, and all of them once the panel is done.  The two parts touch disjoint columns of the working copy, and the
// panel writes the residual panels of its own super-block into the buffer the update does not read.
template <int GB, bool DIRECT>
__global__ __launch_bounds__(256) void panel_far_kernel(PanelArgs pa, TrailArgs ta, int n_panel) {
    extern __shared__ __attribute__((aligned(1024))) char dyn_lds[];
    if (int(blockIdx.x) < n_panel) panel_body<GB, DIRECT>(pa, blockIdx.x, dyn_lds);
    else trailing_tile<3, true>(ta, blockIdx.x - n_panel, dyn_lds);
}

// Scale and zero-point of one wide group (columns g0 .. g0 + G - 1 of every row) from its current values
// w0 + c in fp64: W0 the weights in sweep order, C the working copy (accumulated feedback; nullptr = none, the
// first group of a row or one group per row), which the caller guarantees to be complete for these columns: the far
// updates of all earlier super-blocks have run.  One workgroup per row; the fp64 scale goes to s64[row].
template <typename T>
__global__ __launch_bounds__(256) void group_params_kernel(const T* __restrict__ W0, const float* __restrict__ C, int d_out,
                                                          int d_in, int g0, int G, float qmax, float qs, int mse, int n_g,
                                                          int g_idx, float* __restrict__ scales, float* __restrict__ zeros,
                                                          double* __restrict__ s64) {
    __shared__ double smn[256], smx[256];
    __shared__ float sred[256];
    for (int64_t r = blockIdx.x; r < d_out; r += gridDim.x) {
        const T* row = W0 + r * d_in + g0;
        const float* crow = C ? C + r * d_in + g0 : nullptr;
        auto value = [&](int c) __attribute__((always_inline)) {
            return double(to_f32<T>(row[c])) + (crow ? double(crow[c]) : 0.0);
        };
        double mn = value(0), mx = mn;
        for (int c = threadIdx.x; c < G; c += 256) {
            const double v = value(c);
            mn = fmin(mn, v); mx = fmax(mx, v);
        }
        smn[threadIdx.x] = mn; smx[threadIdx.x] = mx;
        __syncthreads();
        for (int w = 128; w > 0; w >>= 1) {
            if (int(threadIdx.x) < w) {
                smn[threadIdx.x] = fmin(smn[threadIdx.x], smn[threadIdx.x + w]);
                smx[threadIdx.x] = fmax(smx[threadIdx.x], smx[threadIdx.x + w]);
            }
            __syncthreads();
        }
        mn = smn[0]; mx = smx[0];
        __syncthreads();
        int cand = 0;
        if (mse) {   // uniform; the row's values are re-read from cache for every candidate
            cand = mse_search(mn, mx, double(qmax), double(qs),
                       [&](float zi, float rsi) __attribute__((always_inline)) {
                           float e = 0.f;
                           for (int c = threadIdx.x; c < G; c += 256) e += mse_term(float(value(c)), zi, rsi, qmax);
                           return e;
                       },
                       [&](float x) __attribute__((always_inline)) {   // workgroup sum, the same value in every thread
                           x += dpp_quad<QUAD_SWAP1>(x);
                           x += dpp_quad<QUAD_SWAP2>(x);
                           sred[threadIdx.x] = x;
                           __syncthreads();
                           float t = 0.f;
                           for (int w = 0; w < 256; w += 4) t += sred[w];
                           __syncthreads();
                           return t;
                       });
        }
        double s, z;
        grid_params(mn, mx, cand, double(qmax), double(qs), s, z);
        if (threadIdx.x == 0) {
            scales[r * n_g + g_idx] = float(s);
            zeros[r * n_g + g_idx] = float(z);
            s64[r] = s;
        }
    }
}

// Column order (activation ordering): the sweep stages its codes in sweep order (coalesced rows); the caller's
// arrays are then written in ORIGINAL column order, coalesced, gathering from the staged row (a row is a few KB and
// stays in cache).  W^ is recomputed as s (q - z), the same fp32 operations the sweep used.
__global__ __launch_bounds__(256) void inv_perm_kernel(const int32_t* __restrict__ perm, int n, int32_t* __restrict__ inv) {
    const int p = blockIdx.x * 256 + threadIdx.x;
    if (p < n) inv[perm[p]] = p;
}

__global__ __launch_bounds__(256) void unpermute_kernel(const uint8_t* __restrict__ Qs, const float* __restrict__ scales,
                                                       const float* __restrict__ zeros, const int32_t* __restrict__ inv,
                                                       int d_out, int d_in, int G, int n_g, uint8_t* __restrict__ Q,
                                                       float* __restrict__ W_hat) {
    for (int64_t r = blockIdx.y; r < d_out; r += gridDim.y) {
        const int oc = (blockIdx.x * 256 + threadIdx.x) * 4;   // d_in % 128 == 0: whole groups of 4 columns
        if (oc >= d_in) continue;
        const int4 pv = *reinterpret_cast<const int4*>(inv + oc);
        const int ps[4] = {pv.x, pv.y, pv.z, pv.w};
        uint32_t pk = 0;
        float4v h;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t q = Qs[r * d_in + ps[e]];
            const int g = ps[e] / G;
            h[e] = scales[r * n_g + g] * (float(q) - zeros[r * n_g + g]);
            pk |= q << (8 * e);
        }
        *reinterpret_cast<uint32_t*>(Q + r * d_in + oc) = pk;
        if (W_hat) *reinterpret_cast<float4v*>(W_hat + r * d_in + oc) = h;
    }
}

// loss = sum of the per-row sums, fixed order; +infinity if a residual was saturated on its way into the fp16
// operands of the feedback products (the codes of later columns are then not those of the sweep).  One workgroup.
__global__ __launch_bounds__(1024) void loss_kernel(const float* __restrict__ rowloss, int d_out,
                                                   const uint32_t* __restrict__ sat, float* __restrict__ loss) {
    __shared__ double part[1024];
    double s = 0.0;
    for (int i = threadIdx.x; i < d_out; i += 1024) s += double(rowloss[i]);
    part[threadIdx.x] = s;
    __syncthreads();
    for (int w = 512; w > 0; w >>= 1) {
        if (threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) *loss = *sat ? __builtin_inff() : float(part[0]);
}

struct SweepWs {
    float* Wf;        // [d_out x d_in] working copy, sweep order
    uint16_t* Dh;     // 2 x [SBIG x ldD] scaled negated residuals of a super-block, transposed, fp16 hi; two buffers:
    uint16_t* Dl;     // one is read by the far update while the next super-block fills the other       fp16 lo
    uint16_t* Uh;     // [d_in x d_in] scaled rows U_jk / U_jj, fp16 hi
    uint16_t* Ul;     //                                        fp16 lo
    float* rowloss;   // [d_out]
    uint16_t *Fh, *Fl;   // panel kernel: residual fragments, [workgroups][3 x 8 x 2 x 64 x 8]
    uint16_t *Bh, *Bl;   // panel kernel: fragments of the normalized U blocks, [super-blocks][6 x 8 x 4 x 64 x 8]
    Scalars* sc;
    uint8_t* Qs;         // [d_out x d_in] codes in sweep order (used under a column order)
    int32_t* inv;        // [d_in] inverse of the column order
    float* W0p;          // [d_out x d_in] the weights gathered into sweep order (used under a column order)
    double* s64;         // [d_out] fp64 scale of the wide group being swept
};

constexpr size_t F_PER_WG = size_t(3) * 8 * 2 * 64 * 8 * 2;    // bytes of Fh (or Fl) per workgroup of the panel kernel
constexpr size_t B_PER_SB = size_t(6) * 8 * 4 * 64 * 8 * 2;    // bytes of Bh (or Bl) per super-block

// leading dimension of the transposed residual panels: whole 64-row workgroups of the panel kernel
inline int64_t ld_d(int64_t d_out) { return ceil_div(d_out, ROWS) * ROWS; }

SweepWs carve(void* ws, int64_t d_out, int64_t d_in) {
    char* p = static_cast<char*>(ws);
    SweepWs w;
    w.Wf = reinterpret_cast<float*>(p); p += align_up(size_t(d_out) * d_in * sizeof(float), 256);   // feedback sums c
    w.Dh = reinterpret_cast<uint16_t*>(p); p += 2 * size_t(SBIG) * ld_d(d_out) * 2;
    w.Dl = reinterpret_cast<uint16_t*>(p); p += 2 * size_t(SBIG) * ld_d(d_out) * 2;
    w.Uh = reinterpret_cast<uint16_t*>(p); p += align_up(size_t(d_in) * d_in * 2, 256);
    w.Ul = reinterpret_cast<uint16_t*>(p); p += align_up(size_t(d_in) * d_in * 2, 256);
    w.rowloss = reinterpret_cast<float*>(p); p += align_up(size_t(d_out) * sizeof(float), 256);
    const size_t fb = size_t(ceil_div(d_out, ROWS)) * F_PER_WG, bb = size_t(ceil_div(d_in, SBIG)) * B_PER_SB;
    w.Fh = reinterpret_cast<uint16_t*>(p); p += fb;
    w.Fl = reinterpret_cast<uint16_t*>(p); p += fb;
    w.Bh = reinterpret_cast<uint16_t*>(p); p += bb;
    w.Bl = reinterpret_cast<uint16_t*>(p); p += bb;
    w.sc = reinterpret_cast<Scalars*>(p); p += 256;
    w.Qs = reinterpret_cast<uint8_t*>(p); p += align_up(size_t(d_out) * d_in, 256);
    w.inv = reinterpret_cast<int32_t*>(p); p += align_up(size_t(d_in) * sizeof(int32_t), 256);
    w.W0p = reinterpret_cast<float*>(p); p += align_up(size_t(d_out) * d_in * sizeof(float), 256);
    w.s64 = reinterpret_cast<double*>(p);
    return w;
}

template <int GB, bool DIRECT>
onecomp_status launch_panel(const PanelArgs& pa, const TrailArgs& ta, int far_wgs, hipStream_t stream) {
    static std::atomic<uint64_t> lds_ok{0};
    if (allow_dynamic_lds(reinterpret_cast<const void*>(&panel_far_kernel<GB, DIRECT>), PANEL_LDS, lds_ok) != ONECOMP_OK)
        return ONECOMP_ERR_HIP;
    const int n_panel = int(ceil_div(pa.d_out, ROWS));
    hipLaunchKernelGGL((panel_far_kernel<GB, DIRECT>), dim3(unsigned(n_panel + far_wgs)), dim3(256), PANEL_LDS, stream,
                       pa, ta, n_panel);
    ONECOMP_CHECK_LAUNCH();
    return ONECOMP_OK;
}

}  // namespace

size_t sweep_workspace_bytes(int64_t d_out, int64_t d_in, int block) {
    (void)block;
    return align_up(size_t(d_out) * d_in * sizeof(float), 256) + 4 * size_t(SBIG) * ld_d(d_out) * 2 +
           2 * align_up(size_t(d_in) * d_in * 2, 256) + align_up(size_t(d_out) * sizeof(float), 256) +
           2 * size_t(ceil_div(d_out, ROWS)) * F_PER_WG + 2 * size_t(ceil_div(d_in, SBIG)) * B_PER_SB + 256 +
           align_up(size_t(d_out) * d_in, 256) + align_up(size_t(d_in) * sizeof(int32_t), 256) +
           align_up(size_t(d_out) * d_in * sizeof(float), 256) + align_up(size_t(d_out) * sizeof(double), 256);
}

// C[:, c0 .. c1) += f_inv * (D[ek .. ek + K, :])^T * B[u0 .. u0 + K, c0 .. c1): the split-fp16 product of the sweep's
// trailing update, for other callers (see the declaration).
onecomp_status split_update(float* C, int64_t d_out, int64_t d_in, const uint16_t* Dh, const uint16_t* Dl, int64_t ldD,
                            const uint16_t* Bh, const uint16_t* Bl, const Scalars* sc, int ek, int K, int u0, int c0,
                            int c1, hipStream_t stream) {
    if (c1 <= c0 || K <= 0) return ONECOMP_OK;
    static std::atomic<uint64_t> lds_ok{0};
    if (allow_dynamic_lds(reinterpret_cast<const void*>(&trailing_kernel<false>), int(tg::LDS_BYTES), lds_ok) != ONECOMP_OK)
        return ONECOMP_ERR_HIP;
    TrailArgs t;
    t.Wf = C; t.Dh = Dh; t.Dl = Dl; t.Uh = Bh; t.Ul = Bl; t.sc = sc;
    t.d_out = int(d_out); t.ldD = int(ldD); t.d_in = int(d_in);
    t.ek = ek; t.K = K; t.u0 = u0; t.c0 = c0; t.c1 = c1;
    t.n_mt = int(ceil_div(d_out, tg::TM));
    t.n_nt = int(ceil_div(c1 - c0, tg::TN));
    t.chunk = int(ceil_div(int64_t(t.n_mt) * t.n_nt, 8));
    hipLaunchKernelGGL(trailing_kernel<false>, dim3(unsigned(t.chunk * 8)), dim3(256), tg::LDS_BYTES, stream, t);
    ONECOMP_CHECK_LAUNCH();
    return ONECOMP_OK;
}

int64_t split_update_ld(int64_t d_out) { return ld_d(d_out); }

onecomp_status sweep_run(const void* W, onecomp_dtype w_dtype, int64_t d_out, int64_t d_in, const float* U,
                         int form, const int32_t* perm, int bits, int group_size, int block, int grid, uint8_t* Q,
                         float* scales, float* zeros, float* W_hat, float* loss, void* workspace, hipStream_t stream) {
    (void)block;
    const bool direct = form == ONECOMP_FACTOR_BLOCK;   // block form of the factor: see panel_body
    // Wide groups whose parameters can be fixed before the sweep enters them: one group per row (its values are the
    // original weights), or groups made of whole super-blocks (all earlier feedback has reached the working copy
    // once the previous super-block's far update is complete).  These run through the panel kernel.
    const bool wide_static = group_size > SB;
    // super-block width: 512 columns, or for wide groups the largest of 512 / 384 / 256 / 128 that divides the group,
    // so that a group is a run of whole super-blocks
    const int sbw = plan::sweep_superblock_width(group_size, d_in);
    const int sb_pairs = (sbw / SB) * (sbw / SB - 1) / 2;   // block pairs (b' < b) inside a super-block
    if (direct && group_size > SB && group_size != d_in) return ONECOMP_ERR_UNSUPPORTED;
    SweepWs w = carve(workspace, d_out, d_in);
    hipLaunchKernelGGL(init_scalars_kernel, dim3(1), dim3(1), 0, stream, w.sc);
    ONECOMP_CHECK_LAUNCH();
    dim3 lgrid{unsigned(d_out < 1024 ? d_out : 1024)};
    if (w_dtype == ONECOMP_BF16)
        hipLaunchKernelGGL(load_kernel<uint16_t>, lgrid, dim3(256), 0, stream, static_cast<const uint16_t*>(W), d_out,
                           d_in, perm, w.Wf, w.rowloss, w.sc, perm ? w.W0p : nullptr);
    else
        hipLaunchKernelGGL(load_kernel<float>, lgrid, dim3(256), 0, stream, static_cast<const float*>(W), d_out, d_in,
                           perm, w.Wf, w.rowloss, w.sc, perm ? w.W0p : nullptr);
    ONECOMP_CHECK_LAUNCH();
    hipLaunchKernelGGL(umax_kernel, dim3(unsigned(d_in < 1024 ? d_in : 1024)), dim3(256), 0, stream, U,
                       int(d_in), w.sc);
    ONECOMP_CHECK_LAUNCH();
    hipLaunchKernelGGL(scale_kernel, dim3(1), dim3(1), 0, stream, w.sc);
    ONECOMP_CHECK_LAUNCH();
    hipLaunchKernelGGL(split_kernel, dim3(unsigned(ceil_div(d_in, 1024)), unsigned(d_in)), dim3(256), 0, stream, U,
                       int(d_in), w.sc, w.Uh, w.Ul);
    ONECOMP_CHECK_LAUNCH();

    static std::atomic<uint64_t> lds_ok{0};
    if (allow_dynamic_lds(reinterpret_cast<const void*>(&trailing_kernel<true>), int(tg::LDS_BYTES), lds_ok) != ONECOMP_OK)
        return ONECOMP_ERR_HIP;
    TrailArgs t;
    t.Wf = w.Wf; t.Dh = w.Dh; t.Dl = w.Dl; t.Uh = w.Uh; t.Ul = w.Ul; t.sc = w.sc;
    t.ek = 0; t.K = 0; t.u0 = 0; t.c0 = 0; t.c1 = 0; t.n_nt = 0; t.chunk = 0;
    t.d_out = int(d_out); t.ldD = int(ld_d(d_out)); t.d_in = int(d_in);
    t.n_mt = int(ceil_div(d_out, tg::TM));
    // fills t for Wf[:, c0 .. c1) += residual columns ek .. ek+K of buffer `buf` times rows u0 .. u0+K of Un;
    // returns the number of workgroups (0: nothing to do)
    const size_t d_buf = size_t(SBIG) * ld_d(d_out);
    auto set_trailing = [&](int buf, int ek, int K, int u0, int c0, int c1) -> int {
        if (c1 <= c0) return 0;
        t.Dh = w.Dh + buf * d_buf; t.Dl = w.Dl + buf * d_buf;
        t.ek = ek; t.K = K; t.u0 = u0; t.c0 = c0; t.c1 = c1;
        t.n_nt = int(ceil_div(c1 - c0, tg::TN));
        t.chunk = int(ceil_div(int64_t(t.n_mt) * t.n_nt, 8));
        return t.chunk * 8;
    };
    auto trailing = [&](int buf, int ek, int K, int u0, int c0, int c1) -> onecomp_status {
        const int wgs = set_trailing(buf, ek, K, u0, c0, c1);
        if (wgs == 0) return ONECOMP_OK;
        hipLaunchKernelGGL(trailing_kernel<true>, dim3(unsigned(wgs)), dim3(256), tg::LDS_BYTES, stream, t);
        ONECOMP_CHECK_LAUNCH();
        return ONECOMP_OK;
    };

    onecomp_status st;
    {
        // Groups no wider than a block: one launch sweeps a super-block of 512 columns (the feedback between its
        // blocks is applied inside the panel kernel).  The columns beyond a super-block receive its feedback once,
        // with K = its width: first those of the next super-block, then, in the same launch as the next panel,
        // the rest.
        if (sb_pairs > 0) {
            hipLaunchKernelGGL(nearfrag_kernel, dim3(unsigned(sb_pairs), unsigned(ceil_div(d_in, sbw))), dim3(256), 0,
                               stream, U, int(d_in), w.sc, w.Bh, w.Bl, sbw);
            ONECOMP_CHECK_LAUNCH();
        }
        PanelArgs pa;
        pa.Wf = w.Wf; pa.U = U;
        // where the panel finds the original weights in sweep order: under a column order, the gathered fp32 copy
        pa.W0 = perm ? static_cast<const void*>(w.W0p) : W;
        pa.w0_bf16 = !perm && w_dtype == ONECOMP_BF16;
        pa.s64 = w.s64; pa.sat = sat_flag(w.sc);
        pa.Q = perm ? w.Qs : Q; pa.scales = scales; pa.zeros = zeros; pa.W_hat = perm ? nullptr : W_hat;
        pa.Fh = w.Fh; pa.Fl = w.Fl; pa.sc = w.sc; pa.rowloss = w.rowloss;
        pa.d_out = int(d_out); pa.d_in = int(d_in); pa.n_g = int(d_in / group_size); pa.ldD = int(ld_d(d_out));
        pa.lgG = 0;
        while ((1 << pa.lgG) < group_size) ++pa.lgG;
        if (wide_static) pa.lgG = 7;
        pa.wide_g = -1;
        const bool symmetric = grid == ONECOMP_GRID_SYMMETRIC || grid == ONECOMP_GRID_SYMMETRIC_MSE;
        pa.mse = grid == ONECOMP_GRID_MINMAX_MSE || grid == ONECOMP_GRID_SYMMETRIC_MSE;
        pa.qs = symmetric ? float((1 << (bits - 1)) - 1) : 0.f;
        pa.qmax = symmetric ? 2.f * pa.qs : float((1 << bits) - 1);
        int buf = 0, p0 = 0, p1 = 0;   // previous super-block: residual buffer and column range
        for (int s0 = 0; s0 < d_in; s0 += sbw) {
            const int s1 = int(d_in < int64_t(s0) + sbw ? d_in : int64_t(s0) + sbw);
            int far_wgs = 0;
            const bool group_start = wide_static && s0 % group_size == 0;
            if (s0 > 0 && group_start) {   // every later column must be current before the group's range is taken
                if ((st = trailing(buf ^ 1, 0, p1 - p0, p0, s0, int(d_in))) != ONECOMP_OK) return st;
            } else if (s0 > 0) {
                if ((st = trailing(buf ^ 1, 0, p1 - p0, p0, s0, s1)) != ONECOMP_OK) return st;
                far_wgs = set_trailing(buf ^ 1, 0, p1 - p0, p0, s1, int(d_in));
            }
            if (group_start) {
                const dim3 pgrid{unsigned(d_out < 2048 ? d_out : 2048)};
                const int g_idx = s0 / group_size;
                // the feedback of the earlier columns (none before the first group; the block form only takes one
                // group per row, whose grid comes from the original weights)
                const float* cur = (direct || s0 == 0) ? nullptr : w.Wf;
                if (pa.w0_bf16)
                    hipLaunchKernelGGL(group_params_kernel<uint16_t>, pgrid, dim3(256), 0, stream,
                                       static_cast<const uint16_t*>(pa.W0), cur, int(d_out), int(d_in), s0, group_size,
                                       pa.qmax, pa.qs, pa.mse, pa.n_g, g_idx, scales, zeros, w.s64);
                else
                    hipLaunchKernelGGL(group_params_kernel<float>, pgrid, dim3(256), 0, stream,
                                       static_cast<const float*>(pa.W0), cur, int(d_out), int(d_in), s0, group_size,
                                       pa.qmax, pa.qs, pa.mse, pa.n_g, g_idx, scales, zeros, w.s64);
                ONECOMP_CHECK_LAUNCH();
            }
            if (wide_static) pa.wide_g = s0 / group_size;
            pa.s0 = s0; pa.nb = (s1 - s0) / SB;
            pa.Dh = w.Dh + buf * d_buf; pa.Dl = w.Dl + buf * d_buf;
            pa.Bh = w.Bh + size_t(s0 / sbw) * sb_pairs * (8 * 4 * 64 * 8);
            pa.Bl = w.Bl + size_t(s0 / sbw) * sb_pairs * (8 * 4 * 64 * 8);
            if (group_size == 16 && direct) st = launch_panel<16, true>(pa, t, far_wgs, stream);
            else if (group_size == 16) st = launch_panel<16, false>(pa, t, far_wgs, stream);
            else if (direct) st = launch_panel<32, true>(pa, t, far_wgs, stream);
            else st = launch_panel<32, false>(pa, t, far_wgs, stream);
            if (st != ONECOMP_OK) return st;
            buf ^= 1; p0 = s0; p1 = s1;
        }
    }
    if (perm) {
        hipLaunchKernelGGL(inv_perm_kernel, dim3(unsigned(ceil_div(d_in, 256))), dim3(256), 0, stream, perm, int(d_in),
                           w.inv);
        ONECOMP_CHECK_LAUNCH();
        hipLaunchKernelGGL(unpermute_kernel, dim3(unsigned(ceil_div(d_in, 1024)), unsigned(d_out < 4096 ? d_out : 4096)),
                           dim3(256), 0, stream, w.Qs, scales, zeros, w.inv, int(d_out), int(d_in), group_size,
                           int(d_in / group_size), Q, W_hat);
        ONECOMP_CHECK_LAUNCH();
    }
    hipLaunchKernelGGL(loss_kernel, dim3(1), dim3(1024), 0, stream, w.rowloss, int(d_out), sat_flag(w.sc), loss);
    ONECOMP_CHECK_LAUNCH();
    return ONECOMP_OK;
}

}  // namespace onecomp
