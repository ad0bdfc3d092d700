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
// gfx950 schedule (lazy batch of B = 128 columns, right-looking):
//   block kernel    one LANE per output row: the row's 128 current values live in registers, the 128
//                   dependent column steps are fully unrolled, so there is no cross-lane traffic at all in
//                   the sequential part; group min / max are in-register reductions.  The 128 x 128
//                   diagonal block of U sits in LDS and is read with wave-uniform (broadcast) addresses.
//                   Tiles of W / E / W^ / codes move between HBM and registers through LDS so that every
//                   global access is a coalesced row segment.
//   trailing kernel W[:, rest] -= E_blk U[blk, rest] as an fp32 MFMA GEMM (v_mfma_f32_32x32x2_f32), 128 x 128
//                   tile per workgroup, the W tile is loaded straight into the accumulators.
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

template <typename T>
__global__ __launch_bounds__(256) void load_kernel(const T* __restrict__ W, int64_t d_in,
                                                  const int32_t* __restrict__ perm, float* __restrict__ Wf,
                                                  float* __restrict__ rowloss) {
    const int64_t r = blockIdx.y;
    const int p = blockIdx.x * 256 + threadIdx.x;
    if (p == 0) rowloss[r] = 0.f;
    if (p >= d_in) return;
    const int c = perm ? perm[p] : p;
    Wf[r * d_in + p] = to_f32<T>(W[r * d_in + c]);
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
    float* E;               // [d_out x SB] errors of this block
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
        float4v v;
        v[0] = sE[rr * SP + c4 + 0]; v[1] = sE[rr * SP + c4 + 1];
        v[2] = sE[rr * SP + c4 + 2]; v[3] = sE[rr * SP + c4 + 3];
        *reinterpret_cast<float4v*>(a.E + int64_t(gr) * SB + c4) = v;
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
// trailing update:  Wf[:, c0 + 0 .. ncols) -= E[:, 0..128) * U[j0 .. j0+128, c0 ..)      fp32 MFMA
// ------------------------------------------------------------------------------------------
constexpr int TT = 128, TK = 32, TPA = TK + 1, TPB = TT + 4;

__global__ __launch_bounds__(256) void trailing_kernel(float* __restrict__ Wf, const float* __restrict__ E,
                                                       const float* __restrict__ U, int d_out, int64_t d_in, int j0,
                                                       int c0) {
    __shared__ __attribute__((aligned(16))) float sA[2][TT * TPA];
    __shared__ __attribute__((aligned(16))) float sB[2][TK * TPB];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1;
    const int m0 = blockIdx.y * TT;
    const int64_t n0 = int64_t(c0) + int64_t(blockIdx.x) * TT;

    float4v ra[4], rb[4];
    auto gload = [&](int k0) {
#pragma unroll
        for (int n = 0; n < 4; ++n) {
            const int id = tid + 256 * n;
            const int rr = min(m0 + id / 8, d_out - 1), ks = (id % 8) * 4;
            ra[n] = *reinterpret_cast<const float4v*>(E + int64_t(rr) * SB + k0 + ks);
            const int kr = id / 32, cs = (id % 32) * 4;
            rb[n] = *reinterpret_cast<const float4v*>(U + (int64_t(j0) + k0 + kr) * d_in + n0 + cs);
        }
    };
    auto lstore = [&](int st) {
#pragma unroll
        for (int n = 0; n < 4; ++n) {
            const int id = tid + 256 * n;
            float* pa = &sA[st][(id / 8) * TPA + (id % 8) * 4];
            pa[0] = -ra[n][0]; pa[1] = -ra[n][1]; pa[2] = -ra[n][2]; pa[3] = -ra[n][3];
            *reinterpret_cast<float4v*>(&sB[st][(id / 32) * TPB + (id % 32) * 4]) = rb[n];
        }
    };

    gload(0);
    // accumulators start as the W tile: register r of lane l is row (r/4)*8 + (l/32)*4 + r%4, column l%32
    float16v acc[2][2];
    const int lr = (lane >> 5) * 4, lc = lane & 31;
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int n = 0; n < 2; ++n)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int rr = min(m0 + wr * 64 + m * 32 + (r / 4) * 8 + lr + (r % 4), d_out - 1);
                acc[m][n][r] = Wf[int64_t(rr) * d_in + n0 + wc * 64 + n * 32 + lc];
            }
    lstore(0);
    __syncthreads();
    const int kl = lane >> 5;
#pragma unroll 1
    for (int ks = 0; ks < SB / TK; ++ks) {
        const int st = ks & 1;
        if (ks + 1 < SB / TK) gload((ks + 1) * TK);
#pragma unroll
        for (int k2 = 0; k2 < TK; k2 += 2) {
            float av[2], bv[2];
#pragma unroll
            for (int m = 0; m < 2; ++m) av[m] = sA[st][(wr * 64 + m * 32 + lc) * TPA + k2 + kl];
#pragma unroll
            for (int n = 0; n < 2; ++n) bv[n] = sB[st][(k2 + kl) * TPB + wc * 64 + n * 32 + lc];
#pragma unroll
            for (int m = 0; m < 2; ++m)
#pragma unroll
                for (int n = 0; n < 2; ++n)
                    acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[m], bv[n], acc[m][n], 0, 0, 0);
        }
        if (ks + 1 < SB / TK) lstore(st ^ 1);
        __syncthreads();
    }
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int n = 0; n < 2; ++n)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int rr = m0 + wr * 64 + m * 32 + (r / 4) * 8 + lr + (r % 4);
                if (rr < d_out) Wf[int64_t(rr) * d_in + n0 + wc * 64 + n * 32 + lc] = acc[m][n][r];
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
    float* Wf;
    float* E;
    float* rowloss;
};

SweepWs carve(void* ws, int64_t d_out, int64_t d_in) {
    char* p = static_cast<char*>(ws);
    SweepWs w;
    w.Wf = reinterpret_cast<float*>(p); p += align_up(size_t(d_out) * d_in * sizeof(float), 256);
    w.E = reinterpret_cast<float*>(p); p += align_up(size_t(d_out) * SB * sizeof(float), 256);
    w.rowloss = reinterpret_cast<float*>(p);
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
    return align_up(size_t(d_out) * d_in * sizeof(float), 256) + align_up(size_t(d_out) * SB * sizeof(float), 256) +
           align_up(size_t(d_out) * sizeof(float), 256);
}

onecomp_status sweep_run(const void* W, onecomp_dtype w_dtype, int64_t d_out, int64_t d_in, const float* U,
                         const int32_t* perm, int bits, int group_size, int block, uint8_t* Q, float* scales,
                         float* zeros, float* W_hat, float* loss, void* workspace, hipStream_t stream) {
    (void)block;
    SweepWs w = carve(workspace, d_out, d_in);
    dim3 lgrid(unsigned(ceil_div(d_in, 256)), unsigned(d_out));
    if (w_dtype == ONECOMP_BF16)
        hipLaunchKernelGGL(load_kernel<uint16_t>, lgrid, dim3(256), 0, stream, static_cast<const uint16_t*>(W), d_in,
                           perm, w.Wf, w.rowloss);
    else
        hipLaunchKernelGGL(load_kernel<float>, lgrid, dim3(256), 0, stream, static_cast<const float*>(W), d_in, perm,
                           w.Wf, w.rowloss);
    ONECOMP_CHECK_LAUNCH();

    BlockArgs a;
    a.Wf = w.Wf; a.U = U; a.perm = perm; a.Q = Q; a.scales = scales; a.zeros = zeros; a.W_hat = W_hat;
    a.E = w.E; a.rowloss = w.rowloss;
    a.d_out = int(d_out); a.d_in = int(d_in); a.G = group_size; a.n_g = int(d_in / group_size);
    a.qmax = float((1 << bits) - 1);
    for (int j0 = 0; j0 < d_in; j0 += SB) {
        a.j0 = j0;
        onecomp_status st;
        if (group_size == 16) st = launch_block<16>(a, stream);
        else st = launch_block<32>(a, stream);
        if (st != ONECOMP_OK) return st;
        const int64_t rest = d_in - j0 - SB;
        if (rest > 0) {
            dim3 grid(unsigned(rest / TT), unsigned(ceil_div(d_out, TT)));
            hipLaunchKernelGGL(trailing_kernel, grid, dim3(256), 0, stream, w.Wf, w.E, U, int(d_out), d_in, j0,
                               j0 + SB);
            ONECOMP_CHECK_LAUNCH();
        }
    }
    hipLaunchKernelGGL(loss_kernel, dim3(1), dim3(1024), 0, stream, w.rowloss, int(d_out), loss);
    ONECOMP_CHECK_LAUNCH();
    return ONECOMP_OK;
}

}  // namespace onecomp
