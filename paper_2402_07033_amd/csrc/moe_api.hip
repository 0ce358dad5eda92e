// C ABI of libmoe_hip (include/moe.h): argument validation on the host, then
// dispatch to the kernel launchers.  Nothing is enqueued when validation fails.
#include "moe_internal.h"

// mean rows per expert up to which AUTO takes the weight-streaming grouped GEMM
#ifndef MOE_MID_MAX_ROWS
#define MOE_MID_MAX_ROWS 10
#endif

static inline bool dims_ok(int d) { return d >= 64 && d % 64 == 0 && d <= (1 << 20); }
static inline bool tek_ok(int T, int E, int k) {
    return T >= 0 && E >= 1 && E <= MOE_MAX_E && k >= 1 && k <= MOE_MAX_K && k <= E &&
           (long long)T * k < MOE_MAX_N;
}
static inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// Do two byte ranges overlap?
static inline bool ranges_overlap(const void* a, size_t an, const void* b, size_t bn) {
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a && b && a0 < b0 + bn && b0 < a0 + an;
}

// AUTO's choice of kernel family (measured crossovers, Mixtral shape and the 16-expert shape,
// Zipf-skewed routing; with balanced routing each kernel stays ahead somewhat longer than its
// limit here):
//   up to 72 routed rows the decode kernels, which stream each active expert once per
//   16-row tile at ~6.5 TB/s;
//   up to MOE_MID_MAX_ROWS rows per expert on average the weight-streaming grouped GEMM
//   (many experts with a handful of rows each: 11 % ahead at 6 rows per expert, 5 % behind
//   at 12; with 8 experts the window is 73..80 rows, so this is a path of E >= 16 layers);
//   above that the LDS-tiled grouped GEMM, whose smaller tiles stream the weights too.
int moe_ffn_auto_path(int N, int E, int d, int f) {
    if (N <= 72 && moe_ffn_stream_supported(d, f)) return MOE_FFN_STREAM;
    if ((long long)N <= (long long)MOE_MID_MAX_ROWS * E && moe_ffn_mid_supported(N, E, d, f))
        return MOE_FFN_MID;
    return MOE_FFN_GROUPED;
}

// moe_expert_ffn and its variants: validation, then the kernel family.  With `perm` the
// batched row i is read as xg[perm[i] / k] (xg is then the token array).
static int ffn_dispatch(const moe_weights_t* W, const void* xg, moe_dtype_t act_dtype,
                        const int32_t* perm, int k, const int32_t* offsets, int N, void* workspace,
                        size_t workspace_bytes, float* yg, int path, void* stream) {
    if (!W || N < 0 || N >= MOE_MAX_N) return MOE_ERR_INVALID_ARG;
    if (act_dtype != MOE_F32 && act_dtype != MOE_BF16) return MOE_ERR_INVALID_ARG;
    if (path != MOE_FFN_AUTO && path != MOE_FFN_STREAM && path != MOE_FFN_GROUPED &&
        path != MOE_FFN_MID)
        return MOE_ERR_INVALID_ARG;
    if (!offsets) return MOE_ERR_INVALID_ARG;
    if (N == 0) return MOE_OK;
    if (!xg || !yg || !moe_aligned16(xg) || !moe_aligned16(yg)) return MOE_ERR_INVALID_ARG;
    if (!workspace || (((uintptr_t)workspace) & 255u)) return MOE_ERR_WORKSPACE;
    if (workspace_bytes < moe_expert_ffn_workspace(N, W->E, W->d, W->f, act_dtype))
        return MOE_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;

    if (W->dtype == MOE_F32) {
        if (act_dtype != MOE_F32 || path != MOE_FFN_AUTO) return MOE_ERR_UNSUPPORTED;
        return moe_ffn_f32_launch(W, (const float*)xg, perm, k, offsets, N, workspace, yg, s);
    }
    if (path == MOE_FFN_AUTO) path = moe_ffn_auto_path(N, W->E, W->d, W->f);
    if (path == MOE_FFN_STREAM)
        return moe_ffn_stream_launch(W, xg, act_dtype, perm, k, offsets, N, workspace, yg, nullptr, s);
    if (path == MOE_FFN_MID)
        return moe_ffn_mid_launch(W, xg, act_dtype, perm, k, offsets, N, workspace, yg, s);
    return moe_ffn_grouped_launch(W, xg, act_dtype, perm, k, offsets, N, workspace, yg, s);
}

extern "C" {

const char* moe_status_string(int status) {
    switch (status) {
        case MOE_OK: return "ok";
        case MOE_ERR_INVALID_ARG: return "invalid argument";
        case MOE_ERR_UNSUPPORTED: return "unsupported shape or dtype";
        case MOE_ERR_WORKSPACE: return "workspace missing or too small";
        case MOE_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

int moe_route(const float* logits, int T, int E, int k, int32_t* idx, float* weights,
              void* stream) {
    if (!tek_ok(T, E, k)) return MOE_ERR_INVALID_ARG;
    if (T == 0) return MOE_OK;
    if (!logits || !idx || !weights) return MOE_ERR_INVALID_ARG;
    if (!moe_aligned16(logits) || !moe_aligned16(idx) || !moe_aligned16(weights))
        return MOE_ERR_INVALID_ARG;
    return moe_route_launch(logits, T, E, k, idx, weights, (hipStream_t)stream);
}

int moe_permute(const int32_t* idx, int T, int E, int k, const void* x, int d,
                moe_dtype_t x_dtype, int32_t* counts, int32_t* offsets, int32_t* perm,
                int32_t* inv_perm, void* xg, void* stream) {
    if (!tek_ok(T, E, k)) return MOE_ERR_INVALID_ARG;
    if (!counts || !offsets) return MOE_ERR_INVALID_ARG;
    if (T > 0 && (!idx || !perm || !inv_perm)) return MOE_ERR_INVALID_ARG;
    if ((x == nullptr) != (xg == nullptr)) return MOE_ERR_INVALID_ARG;
    if (x) {
        if (!dims_ok(d) || (x_dtype != MOE_F32 && x_dtype != MOE_BF16)) return MOE_ERR_INVALID_ARG;
        if (!moe_aligned16(x) || !moe_aligned16(xg)) return MOE_ERR_INVALID_ARG;
    }
    if (!moe_aligned16(idx) || !moe_aligned16(perm) || !moe_aligned16(inv_perm))
        return MOE_ERR_INVALID_ARG;
    // T == 0 still writes counts = 0 and offsets = 0.
    return moe_permute_launch(idx, T, E, k, T > 0 ? x : nullptr, d, x_dtype, counts, offsets, perm,
                              inv_perm, xg, (hipStream_t)stream);
}

int moe_weights_pack(const void* w1, const void* w3, const void* w2, int E, int d, int f,
                     moe_dtype_t w_dtype, moe_weights_t** out, void* stream) {
    if (!out) return MOE_ERR_INVALID_ARG;
    *out = nullptr;
    if (!w1 || !w3 || !w2 || E < 1 || E > MOE_MAX_E || !dims_ok(d) || !dims_ok(f))
        return MOE_ERR_INVALID_ARG;
    if (w_dtype != MOE_F32 && w_dtype != MOE_BF16) return MOE_ERR_INVALID_ARG;
    if (!moe_aligned16(w1) || !moe_aligned16(w3) || !moe_aligned16(w2)) return MOE_ERR_INVALID_ARG;
    return moe_weights_pack_impl(w1, w3, w2, E, d, f, w_dtype, out, (hipStream_t)stream);
}

int moe_weights_free(moe_weights_t* w) { return moe_weights_free_impl(w); }

size_t moe_weights_bytes(const moe_weights_t* w) { return w ? w->bytes : 0; }

size_t moe_expert_ffn_workspace(int N, int E, int d, int f, moe_dtype_t act_dtype) {
    if (N < 0 || N >= MOE_MAX_N || E < 1 || E > MOE_MAX_E || !dims_ok(d) || !dims_ok(f)) return 0;
    if (act_dtype != MOE_F32 && act_dtype != MOE_BF16) return 0;
    size_t need = moe_ffn_f32_workspace(N, E, d, f);
    const size_t s = moe_ffn_stream_workspace(N, E, d, f);
    const size_t g = moe_ffn_grouped_workspace(N, E, d, f);
    const size_t m = moe_ffn_mid_workspace(N, E, d, f);
    if (s > need) need = s;
    if (g > need) need = g;
    if (m > need) need = m;
    return align256(need) + 256;
}

int moe_expert_ffn_path(const moe_weights_t* W, const void* xg, moe_dtype_t act_dtype,
                        const int32_t* offsets, int N, void* workspace, size_t workspace_bytes,
                        float* yg, int path, void* stream) {
    return ffn_dispatch(W, xg, act_dtype, nullptr, 1, offsets, N, workspace, workspace_bytes, yg,
                        path, stream);
}

int moe_expert_ffn_tokens(const moe_weights_t* W, const void* x, moe_dtype_t act_dtype, int T,
                          int k, const int32_t* perm, const int32_t* offsets, void* workspace,
                          size_t workspace_bytes, float* yg, void* stream) {
    if (!W || !tek_ok(T, W->E, k)) return MOE_ERR_INVALID_ARG;
    if (T > 0 && (!perm || !moe_aligned16(perm))) return MOE_ERR_INVALID_ARG;
    return ffn_dispatch(W, x, act_dtype, perm, k, offsets, T * k, workspace, workspace_bytes, yg,
                        MOE_FFN_AUTO, stream);
}

int moe_expert_ffn(const moe_weights_t* W, const void* xg, moe_dtype_t act_dtype,
                   const int32_t* offsets, int N, void* workspace, size_t workspace_bytes,
                   float* yg, void* stream) {
    return moe_expert_ffn_path(W, xg, act_dtype, offsets, N, workspace, workspace_bytes, yg,
                               MOE_FFN_AUTO, stream);
}

int moe_expert_ffn_plan(int N, int E, int d, int f, moe_dtype_t w_dtype, int path,
                        moe_ffn_plan_t* plan) {
    if (!plan || N < 0 || N >= MOE_MAX_N || E < 1 || E > MOE_MAX_E || !dims_ok(d) || !dims_ok(f))
        return MOE_ERR_INVALID_ARG;
    if (w_dtype != MOE_F32 && w_dtype != MOE_BF16) return MOE_ERR_INVALID_ARG;
    if (path != MOE_FFN_AUTO && path != MOE_FFN_STREAM && path != MOE_FFN_GROUPED &&
        path != MOE_FFN_MID)
        return MOE_ERR_INVALID_ARG;
    *plan = moe_ffn_plan_t{};
    plan->n_parts = 1;
    if (w_dtype == MOE_F32) {
        if (path != MOE_FFN_AUTO) return MOE_ERR_UNSUPPORTED;
        plan->path = MOE_FFN_AUTO;  // the all-fp32 kernels are no family of their own
        return MOE_OK;
    }
    if (path == MOE_FFN_AUTO) path = moe_ffn_auto_path(N, E, d, f);
    plan->path = path;
    if (path == MOE_FFN_STREAM) {
        if (!moe_ffn_stream_supported(d, f)) return MOE_ERR_UNSUPPORTED;
        plan->n_parts = moe_ffn_stream_parts(N, d, f);
    } else if (path == MOE_FFN_MID) {
        if (!moe_ffn_mid_supported(N, E, d, f)) return MOE_ERR_UNSUPPORTED;
    } else {
        return moe_ffn_grouped_plan(N, E, d, f, plan);
    }
    return MOE_OK;
}

int moe_expert_ffn_parts(const moe_weights_t* W, const void* xg, moe_dtype_t act_dtype,
                         const int32_t* offsets, int N, void* workspace, size_t workspace_bytes,
                         float* yg_parts, int max_parts, int* n_parts, void* stream) {
    if (!W || !n_parts || max_parts < 1) return MOE_ERR_INVALID_ARG;
    *n_parts = 1;
    if (N < 0 || N >= MOE_MAX_N) return MOE_ERR_INVALID_ARG;
    const bool stream_path = W->dtype == MOE_BF16 && moe_ffn_auto_path(N, W->E, W->d, W->f) == MOE_FFN_STREAM;
    if (!stream_path || N == 0)
        return moe_expert_ffn_path(W, xg, act_dtype, offsets, N, workspace, workspace_bytes,
                                   yg_parts, MOE_FFN_AUTO, stream);
    if (act_dtype != MOE_F32 && act_dtype != MOE_BF16) return MOE_ERR_INVALID_ARG;
    if (!offsets || !xg || !yg_parts || !moe_aligned16(xg) || !moe_aligned16(yg_parts))
        return MOE_ERR_INVALID_ARG;
    if (moe_ffn_stream_parts(N, W->d, W->f) > max_parts) return MOE_ERR_INVALID_ARG;
    if (!workspace || (((uintptr_t)workspace) & 255u)) return MOE_ERR_WORKSPACE;
    if (workspace_bytes < moe_expert_ffn_workspace(N, W->E, W->d, W->f, act_dtype))
        return MOE_ERR_WORKSPACE;
    return moe_ffn_stream_launch(W, xg, act_dtype, nullptr, 1, offsets, N, workspace, yg_parts, n_parts,
                                 (hipStream_t)stream);
}

int moe_combine_parts(const float* yg_parts, int n_parts, const int32_t* inv_perm,
                      const float* weights, int T, int k, int d, float* y, int residual,
                      float* yg, void* stream) {
    if (T < 0 || k < 1 || k > MOE_MAX_K || (long long)T * k >= MOE_MAX_N || !dims_ok(d) ||
        n_parts < 1 || n_parts > 1024)
        return MOE_ERR_INVALID_ARG;
    if (T == 0) return MOE_OK;
    if (!yg_parts || !inv_perm || !weights || !y) return MOE_ERR_INVALID_ARG;
    if (!moe_aligned16(yg_parts) || !moe_aligned16(y) || (yg && !moe_aligned16(yg)))
        return MOE_ERR_INVALID_ARG;
    const size_t slab = (size_t)T * k * d * sizeof(float);
    if (ranges_overlap(y, (size_t)T * d * sizeof(float), yg_parts, slab * n_parts) ||
        ranges_overlap(yg, slab, yg_parts, slab * n_parts))
        return MOE_ERR_INVALID_ARG;
    return moe_combine_parts_launch(yg_parts, n_parts, (size_t)T * k * d, inv_perm, weights, T, k, d,
                                    y, residual != 0, yg, (hipStream_t)stream);
}

int moe_decode_layer(const moe_weights_t* W, const float* x, const float* logits, int T, int k,
                     int32_t* idx, float* weights, int32_t* counts, int32_t* offsets,
                     int32_t* perm, int32_t* inv_perm, float* xg, void* workspace,
                     size_t workspace_bytes, float* yg, float* y, void* stream) {
    if (!W) return MOE_ERR_INVALID_ARG;
    if (!tek_ok(T, W->E, k)) return MOE_ERR_INVALID_ARG;
    if (!x || !logits || !idx || !weights || !counts || !offsets || !perm || !inv_perm || !y)
        return MOE_ERR_INVALID_ARG;
    if (!moe_aligned16(x) || !moe_aligned16(y) || !moe_aligned16(logits) || !moe_aligned16(idx) ||
        !moe_aligned16(weights) || (xg && !moe_aligned16(xg)) || (yg && !moe_aligned16(yg)))
        return MOE_ERR_INVALID_ARG;
    if (W->dtype != MOE_BF16 || !moe_ffn_stream_decode_supported(T, W->E, k, W->d, W->f))
        return MOE_ERR_UNSUPPORTED;
    const int N = T * k;
    if (!workspace || (((uintptr_t)workspace) & 255u)) return MOE_ERR_WORKSPACE;
    if (workspace_bytes < moe_expert_ffn_workspace(N, W->E, W->d, W->f, MOE_F32))
        return MOE_ERR_WORKSPACE;
    // every workgroup of the first kernel reads x and logits while one writes the outputs
    const size_t xb = (size_t)T * W->d * sizeof(float), nb = (size_t)N * W->d * sizeof(float);
    if (ranges_overlap(x, xb, xg, nb) || ranges_overlap(x, xb, y, xb) ||
        ranges_overlap(logits, (size_t)T * W->E * 4, weights, (size_t)N * 4))
        return MOE_ERR_INVALID_ARG;
    const float* parts = nullptr;
    int n_parts = 1;
    size_t stride = 0;
    int rc = moe_ffn_stream_decode_launch(W, x, logits, T, k, idx, weights, counts, offsets, perm,
                                          inv_perm, xg, workspace, y, yg, &parts, &n_parts, &stride,
                                          (hipStream_t)stream);
    if (rc != MOE_OK || n_parts == 0) return rc;  // 0 parts: the second kernel combined already
    return moe_combine_parts_launch(parts, n_parts, stride, inv_perm, weights, T, k, W->d, y, false,
                                    yg, (hipStream_t)stream);
}

int moe_decode_block(const moe_weights_t* W, const float* x_in, const float* gate_sums,
                     int n_shares, float eps, float* logits, int T, int k, int32_t* idx,
                     float* weights, int32_t* counts, int32_t* offsets, int32_t* perm,
                     int32_t* inv_perm, void* workspace, size_t workspace_bytes, float* x_out,
                     const float* w_gate_next, float* gate_sums_next, void* stream) {
    if (!W) return MOE_ERR_INVALID_ARG;
    if (!tek_ok(T, W->E, k) || T < 1) return MOE_ERR_INVALID_ARG;
    if (!x_in || !logits || !idx || !weights || !counts || !offsets || !perm || !inv_perm || !x_out)
        return MOE_ERR_INVALID_ARG;
    if (gate_sums && (n_shares < 1 || !(eps >= 0.f) || !moe_aligned16(gate_sums)))
        return MOE_ERR_INVALID_ARG;
    if (w_gate_next && (!gate_sums_next || !moe_aligned16(gate_sums_next))) return MOE_ERR_INVALID_ARG;
    if (!moe_aligned16(x_in) || !moe_aligned16(x_out) || !moe_aligned16(logits) ||
        !moe_aligned16(idx) || !moe_aligned16(weights))
        return MOE_ERR_INVALID_ARG;
    if (W->dtype != MOE_BF16 || !moe_ffn_stream_block_supported(T, W->E, k, W->d, W->f))
        return MOE_ERR_UNSUPPORTED;
    if (gate_sums && n_shares > W->d / 16 && n_shares > 1) return MOE_ERR_INVALID_ARG;
    const int N = T * k;
    if (!workspace || (((uintptr_t)workspace) & 255u)) return MOE_ERR_WORKSPACE;
    if (workspace_bytes < moe_expert_ffn_workspace(N, W->E, W->d, W->f, MOE_F32))
        return MOE_ERR_WORKSPACE;
    // x_out may be x_in itself (every element is read and written by the same lane), nothing else
    const size_t xb = (size_t)T * W->d * sizeof(float), lb = (size_t)T * W->E * sizeof(float);
    const size_t share = (size_t)moe_ffn_stream_gate_stride(T, W->E) * sizeof(float);
    const size_t sb_in = share * (size_t)(gate_sums ? n_shares : 0), sb_out = share * (size_t)(W->d / 16);
    if (x_out != x_in && ranges_overlap(x_in, xb, x_out, xb)) return MOE_ERR_INVALID_ARG;
    if (ranges_overlap(logits, lb, weights, (size_t)N * 4) || ranges_overlap(x_out, xb, logits, lb) ||
        ranges_overlap(gate_sums, sb_in, gate_sums_next, sb_out) ||
        ranges_overlap(x_out, xb, gate_sums_next, sb_out) || ranges_overlap(x_out, xb, gate_sums, sb_in) ||
        ranges_overlap(logits, lb, gate_sums_next, sb_out) || ranges_overlap(logits, lb, gate_sums, sb_in))
        return MOE_ERR_INVALID_ARG;
    return moe_ffn_stream_block_launch(W, x_in, gate_sums, n_shares, eps, logits, T, k, idx, weights,
                                       counts, offsets, perm, inv_perm, workspace, x_out, w_gate_next,
                                       gate_sums_next, (hipStream_t)stream);
}

int moe_combine(const float* yg, const int32_t* inv_perm, const float* weights, int T, int k,
                int d, float* y, void* stream) {
    if (T < 0 || k < 1 || k > MOE_MAX_K || (long long)T * k >= MOE_MAX_N || !dims_ok(d))
        return MOE_ERR_INVALID_ARG;
    if (T == 0) return MOE_OK;
    if (!yg || !inv_perm || !weights || !y) return MOE_ERR_INVALID_ARG;
    if (!moe_aligned16(yg) || !moe_aligned16(y)) return MOE_ERR_INVALID_ARG;
    return moe_combine_launch(yg, inv_perm, weights, T, k, d, y, (hipStream_t)stream);
}

int moe_rmsnorm(const float* x, int T, int d, float eps, float* h, void* stream) {
    if (T < 0 || !dims_ok(d) || !(eps >= 0.f)) return MOE_ERR_INVALID_ARG;
    if (T == 0) return MOE_OK;
    if (!x || !h) return MOE_ERR_INVALID_ARG;
    return moe_rmsnorm_launch(x, T, d, eps, h, (hipStream_t)stream);
}

int moe_router_logits(const float* h, const float* w_gate, int T, int d, int E, float* logits,
                      void* stream) {
    if (T < 0 || !dims_ok(d) || E < 1 || E > MOE_MAX_E) return MOE_ERR_INVALID_ARG;
    if (T == 0) return MOE_OK;
    if (!h || !w_gate || !logits) return MOE_ERR_INVALID_ARG;
    if (moe_norm_logits_supported(E) && moe_aligned16(h))
        return moe_norm_logits_launch(false, h, w_gate, T, d, E, 0.f, nullptr, logits, nullptr,
                                      (hipStream_t)stream);
    return moe_router_logits_launch(h, w_gate, T, d, E, logits, (hipStream_t)stream);
}

int moe_rmsnorm_router_logits(const float* x, const float* w_gate, int T, int d, int E, float eps,
                              float* h, float* logits, void* stream) {
    if (T < 0 || !dims_ok(d) || E < 1 || E > MOE_MAX_E || !(eps >= 0.f)) return MOE_ERR_INVALID_ARG;
    if (T == 0) return MOE_OK;
    if (!x || !w_gate || !h || !logits || !moe_aligned16(x) || !moe_aligned16(h))
        return MOE_ERR_INVALID_ARG;
    if (!moe_norm_logits_supported(E)) return MOE_ERR_UNSUPPORTED;
    return moe_norm_logits_launch(true, x, w_gate, T, d, E, eps, h, logits, nullptr,
                                  (hipStream_t)stream);
}

int moe_gate_sums(const float* x, const float* w_gate, int T, int d, int E, float* sums,
                  void* stream) {
    if (T < 0 || !dims_ok(d) || E < 1 || E > MOE_MAX_E) return MOE_ERR_INVALID_ARG;
    if (T == 0) return MOE_OK;
    if (!x || !w_gate || !sums || !moe_aligned16(x) || !moe_aligned16(sums)) return MOE_ERR_INVALID_ARG;
    if (!moe_norm_logits_supported(E)) return MOE_ERR_UNSUPPORTED;
    return moe_norm_logits_launch(true, x, w_gate, T, d, E, 0.f, nullptr, nullptr, sums,
                                  (hipStream_t)stream);
}

size_t moe_gate_sums_stride(int T, int E) {
    if (T < 1 || E < 1 || E > MOE_MAX_E) return 0;
    return (size_t)moe_ffn_stream_gate_stride(T, E);
}

int moe_decode_block_supported(int T, int E, int k, int d, int f, moe_dtype_t w_dtype) {
    if (!tek_ok(T, E, k) || T < 1 || !dims_ok(d) || !dims_ok(f)) return 0;
    return (w_dtype == MOE_BF16 && moe_ffn_stream_block_supported(T, E, k, d, f)) ? 1 : 0;
}

int moe_residual_add(float* x, const float* y, int T, int d, void* stream) {
    if (T < 0 || !dims_ok(d)) return MOE_ERR_INVALID_ARG;
    if (T == 0) return MOE_OK;
    if (!x || !y || !moe_aligned16(x) || !moe_aligned16(y)) return MOE_ERR_INVALID_ARG;
    return moe_residual_add_launch(x, y, T, d, (hipStream_t)stream);
}

int moe_route_permute(const float* logits, int T, int E, int k, const float* x, int d,
                      int32_t* idx, float* weights, int32_t* counts, int32_t* offsets,
                      int32_t* perm, int32_t* inv_perm, float* xg, void* stream) {
    if (!tek_ok(T, E, k) || !dims_ok(d)) return MOE_ERR_INVALID_ARG;
    if (!logits || !x || !idx || !weights || !counts || !offsets || !perm || !inv_perm || !xg)
        return MOE_ERR_INVALID_ARG;
    if (!moe_aligned16(x) || !moe_aligned16(xg)) return MOE_ERR_INVALID_ARG;
    if (ranges_overlap(x, (size_t)T * d * sizeof(float), xg, (size_t)T * k * d * sizeof(float)))
        return MOE_ERR_INVALID_ARG;
    if (T < 1 || T > 16 || E > 16) return MOE_ERR_UNSUPPORTED;
    return moe_gate_small_launch(false, x, nullptr, logits, T, d, E, k, 0.f, nullptr, nullptr, idx,
                                 weights, counts, offsets, perm, inv_perm, xg, nullptr, 1, nullptr,
                                 nullptr, 0, nullptr, (hipStream_t)stream);
}

int moe_norm_route_permute(const float* x, const float* w_gate, int T, int d, int E, int k,
                           float eps, float* h, float* logits, int32_t* idx, float* weights,
                           int32_t* counts, int32_t* offsets, int32_t* perm,
                           int32_t* inv_perm, float* xg, void* stream) {
    if (!tek_ok(T, E, k) || !dims_ok(d) || !(eps >= 0.f)) return MOE_ERR_INVALID_ARG;
    if (!x || !w_gate || !h || !logits || !idx || !weights || !counts || !offsets || !perm ||
        !inv_perm || !xg)
        return MOE_ERR_INVALID_ARG;
    if (!moe_aligned16(x) || !moe_aligned16(xg) || !moe_aligned16(h) || !moe_aligned16(w_gate))
        return MOE_ERR_INVALID_ARG;
    // every workgroup reads x while workgroup 0 writes h and the workgroups share xg
    const size_t xb = (size_t)T * d * sizeof(float);
    if (ranges_overlap(x, xb, h, xb) || ranges_overlap(x, xb, xg, xb * k))
        return MOE_ERR_INVALID_ARG;
    if (T < 1 || T > 4 || E > 16) return MOE_ERR_UNSUPPORTED;
    return moe_gate_small_launch(true, x, w_gate, nullptr, T, d, E, k, eps, h, logits, idx, weights,
                                 counts, offsets, perm, inv_perm, xg, nullptr, 1, nullptr, nullptr, 0,
                                 nullptr, (hipStream_t)stream);
}

int moe_combine_norm_route_permute(const float* yg_prev, int n_parts_prev,
                                   const int32_t* inv_perm_prev,
                                   const float* weights_prev, int k_prev, const float* x_in,
                                   float* x_out, const float* w_gate, int T, int d, int E, int k,
                                   float eps, float* h, float* logits, int32_t* idx, float* weights,
                                   int32_t* counts, int32_t* offsets, int32_t* perm,
                                   int32_t* inv_perm, float* xg, void* stream) {
    if (!tek_ok(T, E, k) || !dims_ok(d) || !(eps >= 0.f) || k_prev < 1 || k_prev > MOE_MAX_K)
        return MOE_ERR_INVALID_ARG;
    if (!yg_prev || !inv_perm_prev || !weights_prev || !x_in || !x_out || !w_gate || !h || !logits ||
        !idx || !weights || !counts || !offsets || !perm || !inv_perm || !xg)
        return MOE_ERR_INVALID_ARG;
    if (!moe_aligned16(x_in) || !moe_aligned16(x_out) || !moe_aligned16(xg) || !moe_aligned16(h) ||
        !moe_aligned16(yg_prev) || !moe_aligned16(w_gate))
        return MOE_ERR_INVALID_ARG;
    if (n_parts_prev < 1) return MOE_ERR_INVALID_ARG;
    // every workgroup reads the inputs while workgroup 0 writes the outputs
    const size_t xb = (size_t)T * d * sizeof(float);
    const size_t ygb = xb * k_prev * n_parts_prev;
    if (ranges_overlap(x_in, xb, x_out, xb) || ranges_overlap(x_in, xb, h, xb) ||
        ranges_overlap(x_in, xb, xg, xb * k) || ranges_overlap(yg_prev, ygb, xg, xb * k) ||
        ranges_overlap(yg_prev, ygb, h, xb) || ranges_overlap(yg_prev, ygb, x_out, xb) ||
        ranges_overlap(inv_perm_prev, (size_t)T * k_prev * 4, inv_perm, (size_t)T * k * 4) ||
        ranges_overlap(weights_prev, (size_t)T * k_prev * 4, weights, (size_t)T * k * 4))
        return MOE_ERR_INVALID_ARG;
    if (T < 1 || T > 4 || E > 16) return MOE_ERR_UNSUPPORTED;
    return moe_gate_small_launch(true, x_in, w_gate, nullptr, T, d, E, k, eps, h, logits, idx,
                                 weights, counts, offsets, perm, inv_perm, xg, yg_prev, n_parts_prev,
                                 inv_perm_prev, weights_prev, k_prev, x_out, (hipStream_t)stream);
}

int moe_combine_residual(const float* yg, const int32_t* inv_perm, const float* weights, int T,
                         int k, int d, float* x, void* stream) {
    if (T < 0 || k < 1 || k > MOE_MAX_K || (long long)T * k >= MOE_MAX_N || !dims_ok(d))
        return MOE_ERR_INVALID_ARG;
    if (T == 0) return MOE_OK;
    if (!yg || !inv_perm || !weights || !x) return MOE_ERR_INVALID_ARG;
    if (!moe_aligned16(yg) || !moe_aligned16(x)) return MOE_ERR_INVALID_ARG;
    return moe_combine_residual_launch(yg, inv_perm, weights, T, k, d, x, (hipStream_t)stream);
}

}  // extern "C"
