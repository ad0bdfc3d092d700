// Column sweep of the layer-wise quantizer (Sec. 4.2 of the paper: quantize one column, propagate its
// residual to the columns not yet quantized) on the per-group asymmetric min-max grid (Eq. (1), (2), (4)).
//
// Per output row, for sweep positions j = 0 .. d_in-1:
//   group start:  s = (max - min) / (2^b - 1) of the current values of the group (1 if max == min),
//                 z = clamp(rne(-min / s), 0, 2^b - 1)
//   q = clamp(rne(w_j / s) + z, 0, 2^b - 1),  w^ = s (q - z),  e = (w_j - w^) / U_jj
//   (w_j / s and the division by U_jj are multiplications by correctly rounded reciprocals),
//   w_k -= e U_jk for k > j.
//
// gfx950 schedule (lazy batch of B = 128 columns inside super-blocks of 512, right-looking):
//   block kernel    one LANE per output row: the row's 128 current values live in registers, the 128
//                   dependent column steps are fully unrolled, so there is no cross-lane traffic at all in
//                   the sequential part; group min / max are in-register reductions.  The 128 x 128
//                   diagonal block of U sits in LDS and is read with wave-uniform (broadcast) addresses.
//                   Tiles of W / E / W^ / codes move between HBM and registers through LDS so that every
//                   global access is a coalesced row segment.
//   trailing kernel W[:, cols] -= E U[rows, cols] as a split-fp16 MFMA GEMM (three v_mfma_f32_32x32x16_f16 products
//                   per term, fp32 accuracy), 128 x 256 tile per workgroup, the W tile is loaded straight into
//                   the accumulators.  Two levels: after each 128-column block only the rest of its 512-column
//                   super-block is updated (K = 128); the columns beyond are updated once per super-block
//                   (K = 512), which cuts the read-modify-write traffic on W four-fold.
//   The loss is the sum of e^2 (equal to tr((W-W^) Hd (W-W^)^T) because U Hd U^T = I), kept per row and
//   reduced in a fixed order.
#include "common.hpp"
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
constexpr int ROWS = 64;       // rows per workgroup of the block kernel (one wave)
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

// Device scalars of one sweep: maxima (as the bit patterns of non-negative floats, which order like unsigned
// integers, so an integer atomic max is exact and order independent) and the power-of-two scales derived from them.
struct Scalars {
    uint32_t max_w_bits;   // max |W|
    uint32_t max_u_bits;   // max |U_jk / U_jj| over the strict upper triangle
    float f_d;             // residuals are stored as fp16 of  -(w - w^) * f_d
    float f_u;             // rows of U are stored as fp16 of  U_jk / U_jj * f_u
    float f_all;           // f_d * f_u
    float f_inv;           // 1 / (f_d * f_u)
};

__global__ void init_scalars_kernel(Scalars* sc) {
    sc->max_w_bits = 0u;
    sc->max_u_bits = 0u;
}

__device__ inline void block_max_to(uint32_t* dst, float v) {
    // wave maximum by butterfly shuffles, then one atomic per wave
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    if ((threadIdx.x & 63) == 0) atomicMax(dst, __float_as_uint(v));
}

template <typename T>
__global__ __launch_bounds__(256) void load_kernel(const T* __restrict__ W, int64_t d_in,
                                                  const int32_t* __restrict__ perm, float* __restrict__ Wf,
                                                  float* __restrict__ rowloss, Scalars* __restrict__ sc) {
    // one workgroup per row: few atomics on the shared maximum
    const int64_t r = blockIdx.x;
    if (threadIdx.x == 0) rowloss[r] = 0.f;
    float m = 0.f;
    for (int p = threadIdx.x; p < d_in; p += 256) {
        const int c = perm ? perm[p] : p;
        const float v = to_f32<T>(W[r * d_in + c]);
        Wf[r * d_in + p] = v;
        m = fmaxf(m, fabsf(v));
    }
    block_max_to(&sc->max_w_bits, m);
}

// ------------------------------------------------------------------------------------------
// block kernel
// ------------------------------------------------------------------------------------------
struct BlockArgs {
    float* Wf;              // [d_out x d_in] working copy, sweep order
    const float* U;         // [d_in x d_in]
    const int32_t* perm;    // or nullptr
    uint8_t* Q;             // [d_out x d_in] original order
    float* scales;          // [d_out x n_g]
    float* zeros;
    float* W_hat;           // or nullptr
    uint16_t* Eh;           // [d_out x SBIG] -(w - w^) * f_d split into fp16 hi + lo, columns e_col .. e_col+127 written
    uint16_t* El;
    const Scalars* sc;
    int e_col;
    float* rowloss;         // [d_out]
    int d_out, d_in, j0, G, n_g;
    float qmax;
};

constexpr int IB = 32;          // columns swept in registers at a time
constexpr int QP = SB + 4;      // byte pitch of the code tile
constexpr int BLOCK_THREADS = 256;

// One workgroup = 64 rows x 128 columns.  The block is swept in 4 inner blocks of 32 columns:
//   wave 0, one lane per row, runs the 32 dependent column steps of the inner block in registers;
//   then all 4 waves apply the inner block's 32 errors to the block's remaining columns (kept in LDS),
//   each wave taking every fourth group of 4 columns, lane = row.
template <int GB>  // group width seen inside an inner block: 16 (G == 16) or 32 (G >= 32)
__global__ __launch_bounds__(BLOCK_THREADS) void block_kernel(BlockArgs a) {
    extern __shared__ __attribute__((aligned(16))) float smem[];
    float* sU = smem;                      // SB x SB, row j holds U[j0+j][j0 .. j0+127]
    float* sRd = sU + SB * SB;             // SB reciprocals of the diagonal
    float* sW = sRd + SB;                  // ROWS x SP : current values; a finished column holds its W^
    float* sE = sW + ROWS * SP;            // ROWS x SP : errors e
    uint8_t* sQ = reinterpret_cast<uint8_t*>(sE + ROWS * SP);  // ROWS x QP bytes

    const int tid = threadIdx.x, l = tid & 63, wave = tid >> 6;
    const int r0 = blockIdx.x * ROWS;
    const int j0 = a.j0;
    const int64_t d_in = a.d_in;

    // U block (coalesced rows) and reciprocal diagonal
    for (int e = tid; e < SB * SB / 4; e += BLOCK_THREADS) {
        const int rr = e / (SB / 4), c4 = (e % (SB / 4)) * 4;
        *reinterpret_cast<float4v*>(sU + rr * SB + c4) =
            *reinterpret_cast<const float4v*>(a.U + (int64_t(j0) + rr) * d_in + j0 + c4);
    }
    if (tid < SB) sRd[tid] = 1.0f / a.U[(int64_t(j0) + tid) * d_in + j0 + tid];
    // W tile: every wave instruction covers 2 rows x 512 B
    for (int it = wave; it < ROWS / 2; it += 4) {
        const int rr = it * 2 + (l >> 5), c4 = (l & 31) * 4;
        const int gr = min(r0 + rr, a.d_out - 1);
        const float4v v = *reinterpret_cast<const float4v*>(a.Wf + int64_t(gr) * d_in + j0 + c4);
        sW[rr * SP + c4 + 0] = v[0]; sW[rr * SP + c4 + 1] = v[1];
        sW[rr * SP + c4 + 2] = v[2]; sW[rr * SP + c4 + 3] = v[3];
    }
    __syncthreads();

    const int row = min(r0 + l, a.d_out - 1);
    const bool row_ok = (r0 + l) < a.d_out;
    const float qmax = a.qmax;
    float s = 1.f, rs = 1.f, z = 0.f, loss = 0.f;
    if (wave == 0 && (j0 % a.G) != 0) {  // block continues a group wider than the block
        s = a.scales[int64_t(row) * a.n_g + j0 / a.G];
        z = a.zeros[int64_t(row) * a.n_g + j0 / a.G];
        rs = 1.0f / s;
    }

#pragma unroll 1
    for (int jb = 0; jb < SB; jb += IB) {
        if (wave == 0) {
            float w[IB];
            static_for<0, IB>([&](auto cc) { w[decltype(cc)::value] = sW[l * SP + jb + decltype(cc)::value]; });
            // Row j of the inner block's U triangle (and 1 / U_jj) is read one step ahead of its use: the reads
            // do not depend on the sequential chain, so their LDS latency hides behind the previous step.
            float4v ua[IB / 4], ub[IB / 4];
            float rdc = sRd[jb], rdn = 0.f;
            auto load_row = [&](float4v(&dst)[IB / 4], auto jc) __attribute__((always_inline)) {
                constexpr int j = decltype(jc)::value;
                static_for<(j + 1) / 4, IB / 4>([&](auto gc) {
                    constexpr int g = decltype(gc)::value;
                    dst[g] = *reinterpret_cast<const float4v*>(sU + (jb + j) * SB + jb + 4 * g);
                });
            };
            load_row(ua, std::integral_constant<int, 0>{});
            static_for<0, IB>([&](auto jc) {
                constexpr int j = decltype(jc)::value;
                auto step = [&](float4v(&cur)[IB / 4], float4v(&nxt)[IB / 4]) __attribute__((always_inline)) {
                    if constexpr (j + 1 < IB) {
                        load_row(nxt, std::integral_constant<int, j + 1>{});
                        rdn = sRd[jb + j + 1];
                    }
                    if constexpr (j % GB == 0) {
                        const int col = j0 + jb + j;
                        bool fresh;
                        float mn, mx;
                        if constexpr (GB == 16) {
                            fresh = true;
                            mn = w[j]; mx = w[j];
                            static_for<j + 1, j + 16>([&](auto cc) {
                                mn = fminf(mn, w[decltype(cc)::value]);
                                mx = fmaxf(mx, w[decltype(cc)::value]);
                            });
                        } else {
                            fresh = (col % a.G) == 0;
                            if (fresh) {
                                // the group's columns inside this block are current in LDS; a group wider than
                                // the block continues in the working copy (already updated by earlier blocks)
                                const int in_blk = min(a.G, SB - jb);
                                mn = mx = sW[l * SP + jb];
                                for (int c = 1; c < in_blk; ++c) {
                                    const float v = sW[l * SP + jb + c];
                                    mn = fminf(mn, v); mx = fmaxf(mx, v);
                                }
                                const float* wr = a.Wf + int64_t(row) * d_in + j0;
                                for (int c = SB; c < a.G; ++c) { const float v = wr[c]; mn = fminf(mn, v); mx = fmaxf(mx, v); }
                            }
                        }
                        if (fresh) {
                            s = (mx - mn) / qmax;
                            if (s == 0.f) s = 1.f;
                            rs = 1.0f / s;
                            z = fminf(fmaxf(rintf(-mn / s), 0.f), qmax);
                            if (row_ok) {
                                a.scales[int64_t(row) * a.n_g + col / a.G] = s;
                                a.zeros[int64_t(row) * a.n_g + col / a.G] = z;
                            }
                        }
                    }
                    const float wj = w[j];
                    const float q = fminf(fmaxf(rintf(wj * rs) + z, 0.f), qmax);   // w / s as w * fl(1 / s)
                    const float wh = s * (q - z);
                    const float e = (wj - wh) * rdc;
                    // feedback inside the inner block: w_k -= e U_jk, j < k < 32; the next column first, it
                    // heads the next step's dependency chain
                    static_for<(j + 1) / 4, IB / 4>([&](auto gc) {
                        constexpr int g = decltype(gc)::value;
                        constexpr int c4 = 4 * g;
                        if constexpr (c4 + 0 > j) w[c4 + 0] = __builtin_fmaf(-e, cur[g][0], w[c4 + 0]);
                        if constexpr (c4 + 1 > j) w[c4 + 1] = __builtin_fmaf(-e, cur[g][1], w[c4 + 1]);
                        if constexpr (c4 + 2 > j) w[c4 + 2] = __builtin_fmaf(-e, cur[g][2], w[c4 + 2]);
                        if constexpr (c4 + 3 > j) w[c4 + 3] = __builtin_fmaf(-e, cur[g][3], w[c4 + 3]);
                    });
                    loss += e * e;
                    sE[l * SP + jb + j] = e;
                    sW[l * SP + jb + j] = wh;
                    sQ[l * QP + jb + j] = uint8_t(q);
                    rdc = rdn;
                };
                if constexpr (j % 2 == 0) step(ua, ub);
                else step(ub, ua);
            });
        }
        __syncthreads();
        // remaining columns of the block: w_c -= sum_i e_i U[jb+i][c], c >= jb + 32
        const int cs = jb + IB;
        if (cs < SB) {
            float ev[IB];
            static_for<0, IB>([&](auto ic) { ev[decltype(ic)::value] = sE[l * SP + jb + decltype(ic)::value]; });
            for (int c = cs + 4 * wave; c < SB; c += 16) {
                float a0 = sW[l * SP + c + 0], a1 = sW[l * SP + c + 1], a2 = sW[l * SP + c + 2], a3 = sW[l * SP + c + 3];
                static_for<0, IB>([&](auto ic) {
                    constexpr int i = decltype(ic)::value;
                    const float4v u = *reinterpret_cast<const float4v*>(sU + (jb + i) * SB + c);
                    a0 = __builtin_fmaf(-ev[i], u[0], a0);
                    a1 = __builtin_fmaf(-ev[i], u[1], a1);
                    a2 = __builtin_fmaf(-ev[i], u[2], a2);
                    a3 = __builtin_fmaf(-ev[i], u[3], a3);
                });
                sW[l * SP + c + 0] = a0; sW[l * SP + c + 1] = a1; sW[l * SP + c + 2] = a2; sW[l * SP + c + 3] = a3;
            }
        }
        __syncthreads();
    }
    if (wave == 0 && row_ok) a.rowloss[row] += loss;

    // tiles out: E (dense), W^ and codes (original column order)
    for (int it = wave; it < ROWS / 2; it += 4) {
        const int rr = it * 2 + (l >> 5), c4 = (l & 31) * 4;
        const int gr = r0 + rr;
        if (gr >= a.d_out) continue;
        // residual w - w^ = e U_jj, negated, scaled by a power of two and split into fp16 hi + lo
        // (hi = rne(x), lo = rne(x - hi): 22 significant bits); saturated far above anything a sweep produces
        short4v eh, el;
        const float f_d = a.sc->f_d;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float x = -sE[rr * SP + c4 + e] * sU[(c4 + e) * SB + c4 + e] * f_d;
            x = fminf(fmaxf(x, -60000.f), 60000.f);
            const _Float16 h = (_Float16)x;
            const _Float16 lo = (_Float16)(x - (float)h);
            eh[e] = __builtin_bit_cast(short, h);
            el[e] = __builtin_bit_cast(short, lo);
        }
        *reinterpret_cast<short4v*>(a.Eh + int64_t(gr) * SBIG + a.e_col + c4) = eh;
        *reinterpret_cast<short4v*>(a.El + int64_t(gr) * SBIG + a.e_col + c4) = el;
        if (!a.perm) {
            if (a.W_hat) {
                float4v h;
                h[0] = sW[rr * SP + c4 + 0]; h[1] = sW[rr * SP + c4 + 1];
                h[2] = sW[rr * SP + c4 + 2]; h[3] = sW[rr * SP + c4 + 3];
                *reinterpret_cast<float4v*>(a.W_hat + int64_t(gr) * d_in + j0 + c4) = h;
            }
            *reinterpret_cast<uint32_t*>(a.Q + int64_t(gr) * d_in + j0 + c4) =
                *reinterpret_cast<const uint32_t*>(sQ + rr * QP + c4);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int oc = a.perm[j0 + c4 + e];
                if (a.W_hat) a.W_hat[int64_t(gr) * d_in + oc] = sW[rr * SP + c4 + e];
                a.Q[int64_t(gr) * d_in + oc] = sQ[rr * QP + c4 + e];
            }
        }
    }
}

constexpr size_t BLOCK_LDS = (size_t(SB) * SB + SB + 2 * size_t(ROWS) * SP) * sizeof(float) + size_t(ROWS) * QP;

// ------------------------------------------------------------------------------------------
// Operands of the trailing GEMMs (once per layer).  The feedback e_j U_jk is computed as
// (w_j - w^_j) * (U_jk / U_jj): the residual is bounded by the weights and the normalized row by the
// regression coefficients between input channels, so both fit fp16 after a power-of-two scaling taken
// from their maxima, whereas e and U themselves span the scale of 1 / sqrt(H_jj).
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void umax_kernel(const float* __restrict__ U, int n, Scalars* __restrict__ sc) {
    const int j = blockIdx.x;   // one workgroup per row
    const float dj = U[int64_t(j) * n + j];
    float m = 0.f;
    for (int k = j + 1 + threadIdx.x; k < n; k += 256) m = fmaxf(m, fabsf(U[int64_t(j) * n + k] / dj));
    if (!(m < 3.0e38f)) m = 3.0e38f;   // NaN / inf from a failed factorization: keep the scalars finite
    block_max_to(&sc->max_u_bits, m);
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
    if (k4 >= n) return;
    const float4v v = *reinterpret_cast<const float4v*>(U + int64_t(j) * n + k4);
    const float dj = U[int64_t(j) * n + j], f_u = sc->f_u;
    short4v h4, l4;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        float x = (k4 + e > j) ? v[e] / dj * f_u : 0.f;
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
// with D = -(w - w^) f_d and Un = U_jk / U_jj f_u as written by the block kernel and split_kernel.
//
// fp32 accuracy from fp16 MFMAs: both operands are split x = hi + lo (fp16 each, |lo| <= 2^-11 |hi|) and
// three products are accumulated in fp32, hi*hi + hi*lo + lo*hi; the dropped lo*lo term and the rounding
// of lo are ~2^-22 relative to each product, i.e. the level of fp32 rounding itself.
// 128 x 256 tile per workgroup, 4 waves in 2 x 2 (64 x 128 each: 2 x 4 tiles of v_mfma_f32_32x32x16_f16),
// the W tile is loaded (scaled) into the accumulators and written back once.  D is k-contiguous (plain 16-byte LDS
// reads); U is k-major, its fragments come from LDS transpose reads.  LDS double-buffered, K step 32.
// ------------------------------------------------------------------------------------------
namespace tg {
constexpr int TM = 128, TN = 256, TK = 32;
constexpr int PA = TK + 8;            // bf16 elements per A row in LDS (80 B: 16 rows hit 16 distinct 16-byte bank groups)
constexpr int PB = TN + 32;           // bf16 elements per B row in LDS (+64 B, as in the Gram kernels)
constexpr int A_ELEMS = TM * PA, B_ELEMS = TK * PB;
constexpr int STAGE = 2 * A_ELEMS + 2 * B_ELEMS;   // hi and lo of both operands
constexpr size_t LDS_BYTES = size_t(2) * STAGE * 2;
}  // namespace tg

__global__ __launch_bounds__(256) void trailing_kernel(float* __restrict__ Wf, const uint16_t* __restrict__ Eh,
                                                       const uint16_t* __restrict__ El,
                                                       const uint16_t* __restrict__ Uh,
                                                       const uint16_t* __restrict__ Ul,
                                                       const Scalars* __restrict__ sc, int d_out, int64_t d_in,
                                                       int ek, int K, int u0, int c0, int c1) {
    using namespace tg;
    extern __shared__ __attribute__((aligned(16))) uint16_t tl[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1;
    const int m0 = blockIdx.y * TM;
    const int n0 = c0 + blockIdx.x * TN;

    // global -> register staging: A tile 128 rows x 32 k (4 chunks of 16 B per row), B tile 32 k x 256 n (32 chunks per row)
    int a_row[2], a_kc[2], b_kr[4], b_nc[4];
#pragma unroll
    for (int i = 0; i < 2; ++i) { const int id = tid + 256 * i; a_row[i] = id >> 2; a_kc[i] = (id & 3) * 8; }
#pragma unroll
    for (int i = 0; i < 4; ++i) { const int id = tid + 256 * i; b_kr[i] = id >> 5; b_nc[i] = (id & 31) * 8; }
    uint4v rah[2], ral[2], rbh[4], rbl[4];
    auto gload = [&](int k0) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int64_t off = int64_t(min(m0 + a_row[i], d_out - 1)) * SBIG + ek + k0 + a_kc[i];
            rah[i] = *reinterpret_cast<const uint4v*>(Eh + off);
            ral[i] = *reinterpret_cast<const uint4v*>(El + off);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int col = min(n0 + b_nc[i], c1 - 8);     // ragged right edge: duplicate columns, never stored
            const int64_t off = (int64_t(u0) + k0 + b_kr[i]) * d_in + col;
            rbh[i] = *reinterpret_cast<const uint4v*>(Uh + off);
            rbl[i] = *reinterpret_cast<const uint4v*>(Ul + off);
        }
    };
    auto lwrite = [&](int st) __attribute__((always_inline)) {
        uint16_t* base = tl + st * STAGE;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            *reinterpret_cast<uint4v*>(base + a_row[i] * PA + a_kc[i]) = rah[i];
            *reinterpret_cast<uint4v*>(base + A_ELEMS + a_row[i] * PA + a_kc[i]) = ral[i];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            *reinterpret_cast<uint4v*>(base + 2 * A_ELEMS + b_kr[i] * PB + b_nc[i]) = rbh[i];
            *reinterpret_cast<uint4v*>(base + 2 * A_ELEMS + B_ELEMS + b_kr[i] * PB + b_nc[i]) = rbl[i];
        }
    };

    gload(0);
    // accumulators start as the W tile times f_d f_u (a power of two: exact), so the tile is in flight together
    // with the first operand tiles; register r of lane l is row (r/4)*8 + (l/32)*4 + r%4, column l%32
    const float f_all = sc->f_all, f_inv = sc->f_inv;
    float16v acc[2][4];
    const int lr = (lane >> 5) * 4, lc = lane & 31;
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int n = 0; n < 4; ++n)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int rr = min(m0 + wr * 64 + m * 32 + (r / 4) * 8 + lr + (r % 4), d_out - 1);
                const int cc = min(n0 + wc * 128 + n * 32 + lc, c1 - 1);
                acc[m][n][r] = Wf[int64_t(rr) * d_in + cc] * f_all;
            }
    lwrite(0);
    __syncthreads();

    const int a_off = (wr * 64 + lc) * PA + (lane >> 5) * 8;                      // + m*32*PA + kq*16
    const int i16 = lane & 15, g16 = (lane >> 4) & 1, kb8 = lane >> 5;
    const int b_off = (kb8 * 8 + (i16 >> 2)) * PB + g16 * 16 + (i16 & 3) * 4 + wc * 128;   // + kq*16*PB + n*32
    const int n_st = K / TK;
#pragma unroll 1
    for (int st = 0; st < n_st; ++st) {
        const int cur = st & 1;
        if (st + 1 < n_st) gload((st + 1) * TK);
        const uint16_t* base = tl + cur * STAGE;
#pragma unroll
        for (int kq = 0; kq < 2; ++kq) {
            half8v ah[2], al[2], bh[4], bl[4];
#pragma unroll
            for (int m = 0; m < 2; ++m) {
                const uint16_t* pa = base + a_off + m * 32 * PA + kq * 16;
                ah[m] = __builtin_bit_cast(half8v, *reinterpret_cast<const uint4v*>(pa));
                al[m] = __builtin_bit_cast(half8v, *reinterpret_cast<const uint4v*>(pa + A_ELEMS));
            }
#pragma unroll
            for (int n = 0; n < 4; ++n) {
                const uint16_t* pb = base + 2 * A_ELEMS + b_off + kq * 16 * PB + n * 32;
                short4v h0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((ONECOMP_LDS short4v*)(pb));
                short4v h1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((ONECOMP_LDS short4v*)(pb + 4 * PB));
                short4v l0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((ONECOMP_LDS short4v*)(pb + B_ELEMS));
                short4v l1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((ONECOMP_LDS short4v*)(pb + B_ELEMS + 4 * PB));
                bh[n] = __builtin_bit_cast(half8v, __builtin_shufflevector(h0, h1, 0, 1, 2, 3, 4, 5, 6, 7));
                bl[n] = __builtin_bit_cast(half8v, __builtin_shufflevector(l0, l1, 0, 1, 2, 3, 4, 5, 6, 7));
            }
#pragma unroll
            for (int m = 0; m < 2; ++m)
#pragma unroll
                for (int n = 0; n < 4; ++n) {
                    acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_f16(al[m], bh[n], acc[m][n], 0, 0, 0);
                    acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah[m], bl[n], acc[m][n], 0, 0, 0);
                    acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah[m], bh[n], acc[m][n], 0, 0, 0);
                }
        }
        if (st + 1 < n_st) lwrite(cur ^ 1);
        __syncthreads();
    }
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int n = 0; n < 4; ++n)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int rr = m0 + wr * 64 + m * 32 + (r / 4) * 8 + lr + (r % 4);
                const int cc = n0 + wc * 128 + n * 32 + lc;
                if (rr < d_out && cc < c1) Wf[int64_t(rr) * d_in + cc] = acc[m][n][r] * f_inv;
            }
}

// loss = sum of the per-row sums, fixed order.  One workgroup.
__global__ __launch_bounds__(1024) void loss_kernel(const float* __restrict__ rowloss, int d_out,
                                                   float* __restrict__ loss) {
    __shared__ double part[1024];
    double s = 0.0;
    for (int i = threadIdx.x; i < d_out; i += 1024) s += double(rowloss[i]);
    part[threadIdx.x] = s;
    __syncthreads();
    for (int w = 512; w > 0; w >>= 1) {
        if (threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) *loss = float(part[0]);
}

struct SweepWs {
    float* Wf;        // [d_out x d_in] working copy, sweep order
    uint16_t* Eh;     // [d_out x SBIG] scaled negated residuals of the current super-block, fp16 hi
    uint16_t* El;     //                                                                     fp16 lo
    uint16_t* Uh;     // [d_in x d_in] scaled rows U_jk / U_jj, fp16 hi
    uint16_t* Ul;     //                                        fp16 lo
    float* rowloss;   // [d_out]
    Scalars* sc;
};

SweepWs carve(void* ws, int64_t d_out, int64_t d_in) {
    char* p = static_cast<char*>(ws);
    SweepWs w;
    w.Wf = reinterpret_cast<float*>(p); p += align_up(size_t(d_out) * d_in * sizeof(float), 256);
    w.Eh = reinterpret_cast<uint16_t*>(p); p += align_up(size_t(d_out) * SBIG * 2, 256);
    w.El = reinterpret_cast<uint16_t*>(p); p += align_up(size_t(d_out) * SBIG * 2, 256);
    w.Uh = reinterpret_cast<uint16_t*>(p); p += align_up(size_t(d_in) * d_in * 2, 256);
    w.Ul = reinterpret_cast<uint16_t*>(p); p += align_up(size_t(d_in) * d_in * 2, 256);
    w.rowloss = reinterpret_cast<float*>(p); p += align_up(size_t(d_out) * sizeof(float), 256);
    w.sc = reinterpret_cast<Scalars*>(p);
    return w;
}

template <int GB>
onecomp_status launch_block(const BlockArgs& a, hipStream_t stream) {
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&block_kernel<GB>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, int(BLOCK_LDS)) != hipSuccess)
            return ONECOMP_ERR_HIP;
        attr_set = true;
    }
    hipLaunchKernelGGL(block_kernel<GB>, dim3(unsigned(ceil_div(a.d_out, ROWS))), dim3(BLOCK_THREADS), BLOCK_LDS, stream,
                       a);
    ONECOMP_CHECK_LAUNCH();
    return ONECOMP_OK;
}

}  // namespace

size_t sweep_workspace_bytes(int64_t d_out, int64_t d_in, int block) {
    (void)block;
    return align_up(size_t(d_out) * d_in * sizeof(float), 256) + 2 * align_up(size_t(d_out) * SBIG * 2, 256) +
           2 * align_up(size_t(d_in) * d_in * 2, 256) + align_up(size_t(d_out) * sizeof(float), 256) + 256;
}

onecomp_status sweep_run(const void* W, onecomp_dtype w_dtype, int64_t d_out, int64_t d_in, const float* U,
                         const int32_t* perm, int bits, int group_size, int block, uint8_t* Q, float* scales,
                         float* zeros, float* W_hat, float* loss, void* workspace, hipStream_t stream) {
    (void)block;
    SweepWs w = carve(workspace, d_out, d_in);
    hipLaunchKernelGGL(init_scalars_kernel, dim3(1), dim3(1), 0, stream, w.sc);
    ONECOMP_CHECK_LAUNCH();
    dim3 lgrid{unsigned(d_out)};
    if (w_dtype == ONECOMP_BF16)
        hipLaunchKernelGGL(load_kernel<uint16_t>, lgrid, dim3(256), 0, stream, static_cast<const uint16_t*>(W), d_in,
                           perm, w.Wf, w.rowloss, w.sc);
    else
        hipLaunchKernelGGL(load_kernel<float>, lgrid, dim3(256), 0, stream, static_cast<const float*>(W), d_in, perm,
                           w.Wf, w.rowloss, w.sc);
    ONECOMP_CHECK_LAUNCH();
    hipLaunchKernelGGL(umax_kernel, dim3(unsigned(d_in)), dim3(256), 0, stream, U,
                       int(d_in), w.sc);
    ONECOMP_CHECK_LAUNCH();
    hipLaunchKernelGGL(scale_kernel, dim3(1), dim3(1), 0, stream, w.sc);
    ONECOMP_CHECK_LAUNCH();
    hipLaunchKernelGGL(split_kernel, dim3(unsigned(ceil_div(d_in, 1024)), unsigned(d_in)), dim3(256), 0, stream, U,
                       int(d_in), w.sc, w.Uh, w.Ul);
    ONECOMP_CHECK_LAUNCH();

    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&trailing_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, int(tg::LDS_BYTES)) != hipSuccess)
            return ONECOMP_ERR_HIP;
        attr_set = true;
    }
    auto trailing = [&](int ek, int K, int u0, int c0, int c1) -> onecomp_status {
        if (c1 <= c0) return ONECOMP_OK;
        dim3 grid(unsigned(ceil_div(c1 - c0, tg::TN)), unsigned(ceil_div(d_out, tg::TM)));
        hipLaunchKernelGGL(trailing_kernel, grid, dim3(256), tg::LDS_BYTES, stream, w.Wf, w.Eh, w.El, w.Uh, w.Ul, w.sc,
                           int(d_out), d_in, ek, K, u0, c0, c1);
        ONECOMP_CHECK_LAUNCH();
        return ONECOMP_OK;
    };

    BlockArgs a;
    a.Wf = w.Wf; a.U = U; a.perm = perm; a.Q = Q; a.scales = scales; a.zeros = zeros; a.W_hat = W_hat;
    a.Eh = w.Eh; a.El = w.El; a.sc = w.sc; a.rowloss = w.rowloss;
    a.d_out = int(d_out); a.d_in = int(d_in); a.G = group_size; a.n_g = int(d_in / group_size);
    a.qmax = float((1 << bits) - 1);
    onecomp_status st;
    // two-level lazy batch: inside a super-block of up to 512 columns every 128-column block updates the rest
    // of the super-block; the columns beyond it are updated once per super-block with K = its width
    for (int s0 = 0; s0 < d_in; s0 += SBIG) {
        const int s1 = int(d_in < int64_t(s0) + SBIG ? d_in : int64_t(s0) + SBIG);
        for (int j0 = s0; j0 < s1; j0 += SB) {
            a.j0 = j0;
            a.e_col = j0 - s0;
            if (group_size == 16) st = launch_block<16>(a, stream);
            else st = launch_block<32>(a, stream);
            if (st != ONECOMP_OK) return st;
            if ((st = trailing(j0 - s0, SB, j0, j0 + SB, s1)) != ONECOMP_OK) return st;
        }
        if ((st = trailing(0, s1 - s0, s0, s1, int(d_in))) != ONECOMP_OK) return st;
    }
    hipLaunchKernelGGL(loss_kernel, dim3(1), dim3(1024), 0, stream, w.rowloss, int(d_out), loss);
    ONECOMP_CHECK_LAUNCH();
    return ONECOMP_OK;
}

}  // namespace onecomp
