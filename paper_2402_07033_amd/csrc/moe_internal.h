// Internal declarations shared by the translation units of libmoe_hip.
// Nothing here is part of the C ABI (see include/moe.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "moe.h"

#define MOE_MAX_E 64
#define MOE_MAX_K 8
#define MOE_MAX_N (1 << 24)
#define MOE_MAX_DEVICES 64  // per-device tables of one-time set-up

// bf16 weights are stored in "fragment order": the unit is the operand tile of
// one v_mfma_f32_16x16x32_bf16 -- 16 output features (rows of W^T) by 32
// reduction indices -- laid out exactly as the 64 lanes hold it: lane l owns
// feature (l % 16) and the 8 consecutive reduction indices 8*(l / 16) .. +7,
// as one 16-byte chunk at byte offset 16*l.  A fragment is 1 KiB, so a
// wavefront fetches it with one fully coalesced 16-byte-per-lane load.
//   w13 : [E][f/16][2 (w1,w3)][d/32] fragments   (reduction over d)
//   w2  : [E][d/16][f/32]           fragments   (reduction over f)
#define MOE_FRAG_BYTES 1024
#define MOE_FRAG_ELEMS 512

struct moe_weights {
    int E, d, f;
    moe_dtype_t dtype;
    int device;
    // bf16: fragment-ordered w13 and w2.  fp32: w1f/w3f/w2f plain copies.
    void* w13;
    void* w2;
    float* w1f;
    float* w3f;
    float* w2f;
    size_t bytes;
};

static inline bool moe_aligned16(const void* p) { return (((uintptr_t)p) & 15u) == 0; }

#define MOE_HIP_TRY(expr)                       \
    do {                                        \
        if ((expr) != hipSuccess) {             \
            (void)hipGetLastError();            \
            return MOE_ERR_HIP;                 \
        }                                       \
    } while (0)

static inline int moe_launch_status() {
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

// Event recorded between the two projections of moe_expert_ffn (measurement hook of
// moe_probe.h), or null: one relaxed atomic load per call when it is off.
void moe_record_mid_event(hipStream_t s);

// Current device, or -1 (on a HIP error, or an ordinal beyond MOE_MAX_DEVICES).
int moe_current_device();
// Number of compute units of the current device (cached per device; 256 on MI355X).
int moe_num_cus();

// AUTO's choice among MOE_FFN_STREAM / MID / GROUPED for bf16 weights (moe_api.hip).
int moe_ffn_auto_path(int N, int E, int d, int f);

// ---- expert FFN kernel families (each returns a moe_status_t) ----------------
size_t moe_ffn_f32_workspace(int N, int E, int d, int f);
// All launchers: with `perm` (device, or null) the batched row i of the activations is read
// as xg[perm[i] / k], i.e. xg is the token array and no gathered copy exists.
int moe_ffn_f32_launch(const moe_weights* W, const float* xg, const int32_t* perm, int k,
                       const int32_t* offsets, int N, void* ws, float* yg, hipStream_t s);

bool moe_ffn_stream_supported(int d, int f);
size_t moe_ffn_stream_workspace(int N, int E, int d, int f);
int moe_ffn_stream_parts(int N, int d, int f);  // slabs the second projection leaves (0: unsupported)
int moe_ffn_stream_launch(const moe_weights* W, const void* xg, moe_dtype_t act_dtype,
                          const int32_t* perm, int k, const int32_t* offsets, int N, void* ws,
                          float* out, int* n_parts, hipStream_t s);
bool moe_ffn_stream_decode_supported(int T, int E, int k, int d, int f);
int moe_ffn_stream_decode_launch(const moe_weights* W, const float* x, const float* logits, int T,
                                 int k, int32_t* idx, float* weights, int32_t* counts,
                                 int32_t* offsets, int32_t* perm, int32_t* inv_perm, float* xg,
                                 void* ws, float* y, float* yg, const float** parts, int* n_parts,
                                 size_t* part_stride, hipStream_t s);

bool moe_ffn_stream_block_supported(int T, int E, int k, int d, int f);
int moe_ffn_stream_gate_stride(int T, int E);  // floats per share of the gating sums
int moe_ffn_stream_block_launch(const moe_weights* W, const float* x_in, const float* gate_sums,
                                int n_shares, float eps, float* logits, int T, int k, int32_t* idx,
                                float* weights, int32_t* counts, int32_t* offsets, int32_t* perm,
                                int32_t* inv_perm, void* ws, float* x_out, const float* w_gate_next,
                                float* gate_sums_next, hipStream_t s);

size_t moe_ffn_grouped_workspace(int N, int E, int d, int f);
int moe_ffn_grouped_plan(int N, int E, int d, int f, moe_ffn_plan_t* plan);  // fills the tile fields
int moe_ffn_grouped_launch(const moe_weights* W, const void* xg, moe_dtype_t act_dtype,
                           const int32_t* perm, int k, const int32_t* offsets, int N, void* ws,
                           float* yg, hipStream_t s);

bool moe_ffn_mid_supported(int N, int E, int d, int f);
size_t moe_ffn_mid_workspace(int N, int E, int d, int f);
int moe_ffn_mid_launch(const moe_weights* W, const void* xg, moe_dtype_t act_dtype,
                       const int32_t* perm, int k, const int32_t* offsets, int N, void* ws,
                       float* yg, hipStream_t s);

// ---- small device helpers ------------------------------------------------------
#ifdef __HIPCC__
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

// fp32 -> bf16 bits, round to nearest even (finite inputs).
__device__ __forceinline__ unsigned moe_bf16_rne(float v) {
    unsigned u = __float_as_uint(v);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ float moe_bf16_to_f32(unsigned bits) {
    return __uint_as_float(bits << 16);
}
__device__ __forceinline__ unsigned moe_pack_bf16x2(float lo, float hi) {
    return moe_bf16_rne(lo) | (moe_bf16_rne(hi) << 16);
}
#endif

// ---- launchers of the small kernels (moe_route_permute.hip, moe_weights.hip) ----
int moe_route_launch(const float* logits, int T, int E, int k, int32_t* idx, float* weights,
                     hipStream_t s);
int moe_permute_launch(const int32_t* idx, int T, int E, int k, const void* x, int d,
                       moe_dtype_t x_dtype, int32_t* counts, int32_t* offsets, int32_t* perm,
                       int32_t* inv_perm, void* xg, hipStream_t s);
int moe_combine_launch(const float* yg, const int32_t* inv_perm, const float* weights, int T, int k,
                       int d, float* y, hipStream_t s);
int moe_rmsnorm_launch(const float* x, int T, int d, float eps, float* h, hipStream_t s);
int moe_router_logits_launch(const float* h, const float* w_gate, int T, int d, int E,
                             float* logits, hipStream_t s);
int moe_residual_add_launch(float* x, const float* y, int T, int d, hipStream_t s);
bool moe_norm_logits_supported(int E);
int moe_norm_logits_launch(bool norm, const float* x, const float* w_gate, int T, int d, int E,
                           float eps, float* h, float* logits, float* sums, hipStream_t s);
int moe_weights_pack_impl(const void* w1, const void* w3, const void* w2, int E, int d, int f,
                          moe_dtype_t w_dtype, moe_weights** out, hipStream_t s);
int moe_weights_free_impl(moe_weights* W);
int moe_weights_repack_impl(moe_weights* W, const void* w1, const void* w3, const void* w2,
                            hipStream_t s);
int moe_gate_small_launch(bool norm, const float* x, const float* w_gate, const float* logits_in,
                          int T, int d, int E, int k, float eps, float* h_out, float* logits_out,
                          int32_t* idx, float* weights, int32_t* counts, int32_t* offsets,
                          int32_t* perm, int32_t* inv_perm, float* xg, const float* yg_prev,
                          int n_parts_prev, const int32_t* inv_perm_prev, const float* weights_prev,
                          int k_prev, float* x_out, hipStream_t s);
int moe_combine_residual_launch(const float* yg, const int32_t* inv_perm, const float* weights, int T,
                                int k, int d, float* x, hipStream_t s);
// y[t] = sum_j w[t,j] * (sum_p parts[p][inv_perm[t*k+j]]), parts `part_stride` floats apart;
// yg_out (or null) receives the summed rows.
// residual: y[t] += ... instead of y[t] = ...
int moe_combine_parts_launch(const float* parts, int n_parts, size_t part_stride,
                             const int32_t* inv_perm, const float* weights, int T, int k, int d,
                             float* y, bool residual, float* yg_out, hipStream_t s);
