// extern "C" boundary: argument checks, then dispatch to the kernel launchers.  See include/onecomp.h.
#include "common.hpp"
#include <dlfcn.h>
#include <cstdlib>

using namespace onecomp;

namespace {
inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// Named host ranges around the entry points for a profiler's marker trace (rocprofv3 --marker-trace), off unless the
// environment holds ONECOMP_ROCTX=1 when the first entry point is called: then the ROCTx library is looked up at run
// time (the library does not link against it) and every call pushes a range with its own name.  The launches are
// asynchronous, so a range covers the argument checks and the enqueueing, not the kernels' run time.
struct Roctx {
    int (*push)(const char*) = nullptr;
    int (*pop)() = nullptr;
};
const Roctx& roctx() {
    static const Roctx r = [] {
        Roctx x;
        const char* e = std::getenv("ONECOMP_ROCTX");
        if (!e || e[0] != '1' || e[1] != 0) return x;
        for (const char* lib : {"librocprofiler-sdk-roctx.so.1", "librocprofiler-sdk-roctx.so", "libroctx64.so.4", "libroctx64.so"}) {
            void* h = dlopen(lib, RTLD_NOW | RTLD_LOCAL);
            if (!h) continue;
            x.push = reinterpret_cast<int (*)(const char*)>(dlsym(h, "roctxRangePushA"));
            x.pop = reinterpret_cast<int (*)()>(dlsym(h, "roctxRangePop"));
            if (x.push && x.pop) return x;
            x = Roctx();
        }
        return x;
    }();
    return r;
}
struct ApiRange {
    const Roctx& r;
    explicit ApiRange(const char* name) : r(roctx()) { if (r.push) r.push(name); }
    ~ApiRange() { if (r.push) r.pop(); }
    ApiRange(const ApiRange&) = delete;
    ApiRange& operator=(const ApiRange&) = delete;
};
}  // namespace

#define ONECOMP_API __attribute__((visibility("default")))
extern "C" {

ONECOMP_API size_t onecomp_accumulate_workspace_bytes(onecomp_dtype x_dtype, int64_t d_in) {
    if (x_dtype != ONECOMP_BF16 || d_in <= 0 || d_in % 16 != 0 || d_in > (1 << 20)) return 0;
    return gram_workspace_bytes(d_in);
}

ONECOMP_API onecomp_status onecomp_hessian_accumulate_ws(const void* X, onecomp_dtype x_dtype, int64_t n_tokens,
                                                         int64_t d_in, int64_t ldx, float* H, void* workspace,
                                                         size_t workspace_bytes, void* hip_stream) {
    const ApiRange range("onecomp_hessian_accumulate_ws");
    if (x_dtype != ONECOMP_F32 && x_dtype != ONECOMP_BF16) return ONECOMP_ERR_UNSUPPORTED;
    if (!H || d_in <= 0 || n_tokens < 0 || ldx < d_in) return ONECOMP_ERR_INVALID_ARG;
    if (d_in % 16 != 0 || d_in > (1 << 20)) return ONECOMP_ERR_INVALID_ARG;
    if (workspace && !aligned(workspace, 256)) return ONECOMP_ERR_WORKSPACE;
    if (n_tokens == 0) return ONECOMP_OK;
    if (!X) return ONECOMP_ERR_INVALID_ARG;
    const size_t esz = (x_dtype == ONECOMP_BF16) ? 2 : 4;
    if (!aligned(X, 16) || (size_t(ldx) * esz) % 16 != 0 || !aligned(H, 16)) return ONECOMP_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (x_dtype == ONECOMP_BF16)
        return gram_accumulate_bf16(X, n_tokens, d_in, ldx, H, workspace, workspace ? workspace_bytes : 0, s);
    return gram_accumulate_f32(X, n_tokens, d_in, ldx, H, s);
}

ONECOMP_API onecomp_status onecomp_accumulate_describe(onecomp_dtype x_dtype, int64_t n_tokens, int64_t d_in, int64_t ldx,
                                                       size_t workspace_bytes, int32_t* out3) {
    if (x_dtype != ONECOMP_F32 && x_dtype != ONECOMP_BF16) return ONECOMP_ERR_UNSUPPORTED;
    if (!out3 || d_in <= 0 || n_tokens < 0 || ldx < d_in) return ONECOMP_ERR_INVALID_ARG;
    if (d_in % 16 != 0 || d_in > (1 << 20)) return ONECOMP_ERR_INVALID_ARG;
    GramPlanInfo info{128, 128, 1};
    if (x_dtype == ONECOMP_BF16) {
        const onecomp_status st = gram_accumulate_bf16(nullptr, n_tokens, d_in, ldx, nullptr, nullptr, workspace_bytes,
                                                       nullptr, &info);
        if (st != ONECOMP_OK) return st;
    }
    out3[0] = info.tile_rows;
    out3[1] = info.tile_cols;
    out3[2] = info.launches;
    return ONECOMP_OK;
}

ONECOMP_API onecomp_status onecomp_hessian_accumulate(const void* X, onecomp_dtype x_dtype, int64_t n_tokens, int64_t d_in,
                                          int64_t ldx, float* H, void* hip_stream) {
    return onecomp_hessian_accumulate_ws(X, x_dtype, n_tokens, d_in, ldx, H, nullptr, 0, hip_stream);
}

ONECOMP_API size_t onecomp_factor_workspace_bytes(int64_t d_in) {
    if (d_in <= 0 || d_in % 16 != 0 || d_in > 46336) return 0;
    return factor_workspace_bytes(d_in);
}

ONECOMP_API onecomp_status onecomp_hessian_factor_form(const float* H, int64_t d_in, float damp, int act_order,
                                                       onecomp_factor_form form, int32_t* perm_out, float* F_out,
                                                       int32_t* info, void* workspace, size_t workspace_bytes,
                                                       void* hip_stream) {
    const ApiRange range("onecomp_hessian_factor_form");
    if (form != ONECOMP_FACTOR_INVERSE && form != ONECOMP_FACTOR_BLOCK) return ONECOMP_ERR_UNSUPPORTED;
    if (!H || !F_out || !info || d_in <= 0) return ONECOMP_ERR_INVALID_ARG;
    if (d_in % 16 != 0 || d_in > 46336) return ONECOMP_ERR_INVALID_ARG;
    if (form == ONECOMP_FACTOR_BLOCK && d_in % 128 != 0) return ONECOMP_ERR_UNSUPPORTED;
    if (!(damp >= 0.0f)) return ONECOMP_ERR_INVALID_ARG;
    if (act_order && !perm_out) return ONECOMP_ERR_INVALID_ARG;
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < factor_workspace_bytes(d_in))
        return ONECOMP_ERR_WORKSPACE;
    return factor_run(H, d_in, damp, act_order, int(form), perm_out, F_out, info, workspace,
                      static_cast<hipStream_t>(hip_stream));
}

ONECOMP_API onecomp_status onecomp_hessian_factor(const float* H, int64_t d_in, float damp, int act_order, int32_t* perm_out,
                                      float* U, int32_t* info, void* workspace, size_t workspace_bytes,
                                      void* hip_stream) {
    return onecomp_hessian_factor_form(H, d_in, damp, act_order, ONECOMP_FACTOR_INVERSE, perm_out, U, info, workspace,
                                       workspace_bytes, hip_stream);
}

ONECOMP_API size_t onecomp_quantize_workspace_bytes(int64_t d_out, int64_t d_in, int block_size) {
    if (d_out <= 0 || d_in <= 0 || block_size != 128 || d_in % 128 != 0) return 0;
    return sweep_workspace_bytes(d_out, d_in, block_size);
}

ONECOMP_API onecomp_status onecomp_quantize_layer_form(const void* W, onecomp_dtype w_dtype, int64_t d_out,
                                                       int64_t d_in, const float* F, onecomp_factor_form form,
                                                       const int32_t* perm, int bits, int group_size, int block_size,
                                                       onecomp_grid grid, uint8_t* Q_codes, float* scales,
                                                       float* zeros, float* W_hat, float* loss, void* workspace,
                                                       size_t workspace_bytes, void* hip_stream) {
    const ApiRange range("onecomp_quantize_layer_form");
    const float* U = F;
    if (w_dtype != ONECOMP_F32 && w_dtype != ONECOMP_BF16) return ONECOMP_ERR_UNSUPPORTED;
    if (grid != ONECOMP_GRID_MINMAX && grid != ONECOMP_GRID_SYMMETRIC && grid != ONECOMP_GRID_MINMAX_MSE &&
        grid != ONECOMP_GRID_SYMMETRIC_MSE)
        return ONECOMP_ERR_UNSUPPORTED;
    if (form != ONECOMP_FACTOR_INVERSE && form != ONECOMP_FACTOR_BLOCK) return ONECOMP_ERR_UNSUPPORTED;
    if (!W || !U || !Q_codes || !scales || !zeros || !loss) return ONECOMP_ERR_INVALID_ARG;
    if (d_out <= 0 || d_in <= 0 || d_out > (1 << 24) || d_in > 65535) return ONECOMP_ERR_INVALID_ARG;
    if (bits != 2 && bits != 3 && bits != 4 && bits != 8) return ONECOMP_ERR_UNSUPPORTED;
    if (block_size != 128) return ONECOMP_ERR_UNSUPPORTED;
    if (group_size <= 0 || d_in % block_size != 0 || d_in % group_size != 0) return ONECOMP_ERR_INVALID_ARG;
    if (group_size % 16 != 0) return ONECOMP_ERR_UNSUPPORTED;
    if (block_size % group_size != 0 && group_size % block_size != 0) return ONECOMP_ERR_INVALID_ARG;
    if (form == ONECOMP_FACTOR_BLOCK && group_size > block_size && group_size != d_in) return ONECOMP_ERR_UNSUPPORTED;
    if (!aligned(W, 16) || !aligned(U, 16) || !aligned(Q_codes, 4) || (W_hat && !aligned(W_hat, 16)))
        return ONECOMP_ERR_INVALID_ARG;
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < sweep_workspace_bytes(d_out, d_in, block_size))
        return ONECOMP_ERR_WORKSPACE;
    return sweep_run(W, w_dtype, d_out, d_in, U, int(form), perm, bits, group_size, block_size, int(grid), Q_codes,
                     scales, zeros, W_hat, loss, workspace, static_cast<hipStream_t>(hip_stream));
}

ONECOMP_API onecomp_status onecomp_quantize_layer_grid(const void* W, onecomp_dtype w_dtype, int64_t d_out,
                                                       int64_t d_in, const float* U, const int32_t* perm, int bits,
                                                       int group_size, int block_size, onecomp_grid grid,
                                                       uint8_t* Q_codes, float* scales, float* zeros, float* W_hat,
                                                       float* loss, void* workspace, size_t workspace_bytes,
                                                       void* hip_stream) {
    return onecomp_quantize_layer_form(W, w_dtype, d_out, d_in, U, ONECOMP_FACTOR_INVERSE, perm, bits, group_size,
                                       block_size, grid, Q_codes, scales, zeros, W_hat, loss, workspace, workspace_bytes,
                                       hip_stream);
}

ONECOMP_API onecomp_status onecomp_quantize_layer(const void* W, onecomp_dtype w_dtype, int64_t d_out, int64_t d_in,
                                      const float* U, const int32_t* perm, int bits, int group_size, int block_size,
                                      uint8_t* Q_codes, float* scales, float* zeros, float* W_hat, float* loss,
                                      void* workspace, size_t workspace_bytes, void* hip_stream) {
    return onecomp_quantize_layer_grid(W, w_dtype, d_out, d_in, U, perm, bits, group_size, block_size,
                                       ONECOMP_GRID_MINMAX, Q_codes, scales, zeros, W_hat, loss, workspace,
                                       workspace_bytes, hip_stream);
}

ONECOMP_API onecomp_status onecomp_crossgram_accumulate(const void* X_hat, const void* X, onecomp_dtype x_dtype,
                                                        int64_t n_tokens, int64_t d_in, int64_t ldxh, int64_t ldx,
                                                        float* G, void* hip_stream) {
    const ApiRange range("onecomp_crossgram_accumulate");
    if (x_dtype != ONECOMP_BF16) return ONECOMP_ERR_UNSUPPORTED;
    if (!G || d_in <= 0 || n_tokens < 0 || ldxh < d_in || ldx < d_in) return ONECOMP_ERR_INVALID_ARG;
    if (d_in % 16 != 0 || d_in > (1 << 20)) return ONECOMP_ERR_INVALID_ARG;
    if (n_tokens == 0) return ONECOMP_OK;
    if (!X_hat || !X) return ONECOMP_ERR_INVALID_ARG;
    if (!aligned(X_hat, 16) || !aligned(X, 16) || (ldxh * 2) % 16 != 0 || (ldx * 2) % 16 != 0 || !aligned(G, 16))
        return ONECOMP_ERR_INVALID_ARG;
    // the kernel addresses a step of 16 token rows with 32-bit byte offsets
    if (ldxh * 64 >= (int64_t(1) << 31) || ldx * 64 >= (int64_t(1) << 31)) return ONECOMP_ERR_UNSUPPORTED;
    return gram_cross_accumulate_bf16(X_hat, X, n_tokens, d_in, ldxh, ldx, G, static_cast<hipStream_t>(hip_stream));
}

ONECOMP_API size_t onecomp_qep_workspace_bytes(int64_t d_out, int64_t d_in) {
    if (d_out <= 0 || d_in <= 0 || d_in % 16 != 0 || d_in > 65535 || d_out > (1 << 24)) return 0;
    return qep_workspace_bytes(d_out, d_in);
}

ONECOMP_API onecomp_status onecomp_qep_target(const void* W, onecomp_dtype w_dtype, int64_t d_out, int64_t d_in,
                                              const float* G, const float* H, const float* U, const int32_t* perm,
                                              float alpha, float* W_star, void* workspace, size_t workspace_bytes,
                                              void* hip_stream) {
    const ApiRange range("onecomp_qep_target");
    if (w_dtype != ONECOMP_F32 && w_dtype != ONECOMP_BF16) return ONECOMP_ERR_UNSUPPORTED;
    if (!W || !G || !H || !U || !W_star) return ONECOMP_ERR_INVALID_ARG;
    if (d_out <= 0 || d_in <= 0 || d_in % 16 != 0 || d_in > 65535 || d_out > (1 << 24)) return ONECOMP_ERR_INVALID_ARG;
    if (!(alpha >= 0.0f && alpha <= 1.0f)) return ONECOMP_ERR_INVALID_ARG;
    if (static_cast<const void*>(W_star) == W) return ONECOMP_ERR_INVALID_ARG;
    if (!aligned(W, 16) || !aligned(G, 16) || !aligned(H, 16) || !aligned(U, 16) || !aligned(W_star, 16))
        return ONECOMP_ERR_INVALID_ARG;
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < qep_workspace_bytes(d_out, d_in))
        return ONECOMP_ERR_WORKSPACE;
    return qep_target_run(W, w_dtype, d_out, d_in, G, H, U, perm, alpha, W_star, workspace,
                          static_cast<hipStream_t>(hip_stream));
}

ONECOMP_API size_t onecomp_jointq_workspace_bytes(int64_t d_out, int64_t d_in, int group_size) {
    if (d_out <= 0 || d_in <= 0 || group_size <= 0 || group_size % 16 != 0 || d_in % group_size != 0) return 0;
    if (group_size > 128 && group_size % 128 != 0) return 0;
    return jointq_workspace_bytes(d_out, d_in, group_size);
}

ONECOMP_API onecomp_status onecomp_jointq_refine(const void* W, onecomp_dtype w_dtype, int64_t d_out, int64_t d_in,
                                                 const float* H, const int32_t* perm, float lam, int bits,
                                                 int group_size,
                                                 onecomp_grid grid, int n_pass, int max_scans, uint8_t* Q_codes,
                                                 float* scales, const float* zeros, float* W_hat, float* objective,
                                                 int32_t* n_moves, void* workspace, size_t workspace_bytes,
                                                 void* hip_stream) {
    const ApiRange range("onecomp_jointq_refine");
    if (w_dtype != ONECOMP_F32 && w_dtype != ONECOMP_BF16) return ONECOMP_ERR_UNSUPPORTED;
    if (grid != ONECOMP_GRID_MINMAX && grid != ONECOMP_GRID_SYMMETRIC && grid != ONECOMP_GRID_MINMAX_MSE &&
        grid != ONECOMP_GRID_SYMMETRIC_MSE)
        return ONECOMP_ERR_UNSUPPORTED;
    if (bits != 2 && bits != 3 && bits != 4 && bits != 8) return ONECOMP_ERR_UNSUPPORTED;
    if (!W || !H || !Q_codes || !scales || !zeros || !objective || !n_moves) return ONECOMP_ERR_INVALID_ARG;
    if (d_out <= 0 || d_in <= 0 || d_out > (1 << 24) || d_in > (1 << 20)) return ONECOMP_ERR_INVALID_ARG;
    if (!(lam >= 0.0f) || n_pass < 0 || max_scans < 1) return ONECOMP_ERR_INVALID_ARG;
    if (group_size <= 0 || d_in % 16 != 0 || d_in % group_size != 0) return ONECOMP_ERR_INVALID_ARG;
    if (group_size % 16 != 0 || (group_size > 128 && group_size % 128 != 0)) return ONECOMP_ERR_UNSUPPORTED;
    if (!aligned(W, 16) || !aligned(H, 16) || !aligned(Q_codes, 4) || (W_hat && !aligned(W_hat, 16)))
        return ONECOMP_ERR_INVALID_ARG;
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < jointq_workspace_bytes(d_out, d_in, group_size))
        return ONECOMP_ERR_WORKSPACE;
    return jointq_run(W, w_dtype, d_out, d_in, H, perm, lam, bits, group_size, int(grid), n_pass, max_scans, Q_codes, scales,
                      zeros, W_hat, objective, n_moves, workspace, static_cast<hipStream_t>(hip_stream));
}

ONECOMP_API size_t onecomp_sensitivity_workspace_bytes(void) { return sensitivity_workspace_bytes(); }

ONECOMP_API onecomp_status onecomp_rtn_sensitivity(const void* W, onecomp_dtype w_dtype, int64_t d_out, int64_t d_in,
                                                   const float* a_diag, const float* b_diag, int bits, int group_size,
                                                   onecomp_grid grid, float* err, void* workspace,
                                                   size_t workspace_bytes, void* hip_stream) {
    const ApiRange range("onecomp_rtn_sensitivity");
    if (w_dtype != ONECOMP_F32 && w_dtype != ONECOMP_BF16) return ONECOMP_ERR_UNSUPPORTED;
    if (grid != ONECOMP_GRID_MINMAX && grid != ONECOMP_GRID_SYMMETRIC) return ONECOMP_ERR_UNSUPPORTED;
    if (bits != 2 && bits != 3 && bits != 4 && bits != 8) return ONECOMP_ERR_UNSUPPORTED;
    if (!W || !a_diag || !err) return ONECOMP_ERR_INVALID_ARG;
    if (d_out <= 0 || d_in <= 0 || d_out > (1 << 24) || d_in > (1 << 24)) return ONECOMP_ERR_INVALID_ARG;
    if (group_size <= 0 || d_in % group_size != 0) return ONECOMP_ERR_INVALID_ARG;
    if (group_size % 16 != 0) return ONECOMP_ERR_UNSUPPORTED;
    if (!aligned(W, 16) || !aligned(a_diag, 16)) return ONECOMP_ERR_INVALID_ARG;   // 16-byte vector loads
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < sensitivity_workspace_bytes())
        return ONECOMP_ERR_WORKSPACE;
    return sensitivity_run(W, w_dtype, d_out, d_in, a_diag, b_diag, bits, group_size, int(grid), err, workspace,
                           static_cast<hipStream_t>(hip_stream));
}

ONECOMP_API onecomp_status onecomp_rtn_sensitivity_static(const void* W, onecomp_dtype w_dtype, int64_t d_out,
                                                          int64_t d_in, const float* a_diag, const float* b_diag,
                                                          int bits, int group_size, onecomp_grid grid, float* err,
                                                          void* hip_stream) {
    const ApiRange range("onecomp_rtn_sensitivity_static");
    if (w_dtype != ONECOMP_F32 && w_dtype != ONECOMP_BF16) return ONECOMP_ERR_UNSUPPORTED;
    if (grid != ONECOMP_GRID_MINMAX && grid != ONECOMP_GRID_SYMMETRIC) return ONECOMP_ERR_UNSUPPORTED;
    if (bits != 2 && bits != 3 && bits != 4 && bits != 8) return ONECOMP_ERR_UNSUPPORTED;
    if (!W || !a_diag || !err) return ONECOMP_ERR_INVALID_ARG;
    // the built-in scratch holds one partial sum per workgroup of a grid capped at 2048 workgroups, which covers every
    // size up to the limits below; anything beyond them is rejected here, before any launch
    if (d_out <= 0 || d_in <= 0 || d_out > (1 << 24) || d_in > (1 << 24)) return ONECOMP_ERR_INVALID_ARG;
    if (group_size <= 0 || d_in % group_size != 0) return ONECOMP_ERR_INVALID_ARG;
    if (group_size % 16 != 0) return ONECOMP_ERR_UNSUPPORTED;
    if (!aligned(W, 16) || !aligned(a_diag, 16)) return ONECOMP_ERR_INVALID_ARG;
    return sensitivity_run_static(W, w_dtype, d_out, d_in, a_diag, b_diag, bits, group_size, int(grid), err,
                                  static_cast<hipStream_t>(hip_stream));
}

ONECOMP_API onecomp_status onecomp_mfma_rate_probe(int kind, int waves_per_simd, int random_operands, int64_t iters,
                                                   float* sink, double* flops_out, void* hip_stream) {
    if (kind != 0 && kind != 1) return ONECOMP_ERR_UNSUPPORTED;
    if (waves_per_simd != 1 && waves_per_simd != 2) return ONECOMP_ERR_UNSUPPORTED;
    if (random_operands != 0 && random_operands != 1) return ONECOMP_ERR_INVALID_ARG;
    if (!sink || !flops_out || iters <= 0 || iters > (int64_t(1) << 24)) return ONECOMP_ERR_INVALID_ARG;
    const ApiRange range("onecomp_mfma_rate_probe");
    return mfma_rate_probe(kind, waves_per_simd, random_operands, iters, sink, flops_out,
                           static_cast<hipStream_t>(hip_stream));
}

ONECOMP_API const char* onecomp_status_string(onecomp_status status) {
    switch (status) {
        case ONECOMP_OK: return "ok";
        case ONECOMP_ERR_INVALID_ARG: return "invalid argument";
        case ONECOMP_ERR_UNSUPPORTED: return "unsupported dtype, bit width, group size or block size";
        case ONECOMP_ERR_NOT_POSDEF: return "matrix is not positive definite";
        case ONECOMP_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case ONECOMP_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

ONECOMP_API int onecomp_version(void) { return 100; }

}  // extern "C"
