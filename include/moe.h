/*
 * libmoe_hip -- C ABI of the MoE expert-layer hot path for AMD MI355X (gfx950).
 *
 * The layer is the computation Fiddler (arXiv 2402.07033) schedules: the
 * gating function selects the experts of every token (Sec. 2.1, Sec. 3.3
 * "Execution"), tokens are batched per expert (the inp_size array of
 * Algorithm 1), every expert that received tokens runs its feed-forward block
 * (three d x f matrices per expert, Sec. 3.2; SiLU activation, Sec. 2.2;
 * experts with zero tokens are skipped, Algorithm 1), and the expert outputs
 * return to the token stream.  All experts are resident in device memory,
 * i.e. every expert is case (a) of Sec. 3.2.
 *
 * Conventions (all entry points):
 *   - Every data pointer is a DEVICE pointer owned by the caller unless the
 *     comment says HOST.  The library never frees caller memory and allocates
 *     device memory only in moe_weights_pack (released by moe_weights_free).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue work on it and return; there is no host synchronisation
 *     and no device-to-host copy inside any call except where stated.
 *   - Return value: MOE_OK (0) or a negative moe_status_t.  Arguments are
 *     validated on the host before anything is launched; on error nothing has
 *     been enqueued.  No exception or abort crosses the boundary.
 *   - Row-major arrays; pointers must be 16-byte aligned.
 *   - Domain: 1 <= k <= 8, k <= E <= 64, T >= 0 (T == 0 is a no-op),
 *     T*k < 2^24, d and f multiples of 64.
 */
#ifndef MOE_H_
#define MOE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { MOE_F32 = 0, MOE_BF16 = 1 } moe_dtype_t;

typedef enum {
    MOE_OK = 0,
    MOE_ERR_INVALID_ARG = -1, /* null/misaligned pointer, size out of the domain */
    MOE_ERR_UNSUPPORTED = -2, /* valid request this build has no kernel for */
    MOE_ERR_WORKSPACE = -3,   /* workspace missing or too small */
    MOE_ERR_HIP = -4          /* a HIP runtime call failed (allocation, launch) */
} moe_status_t;

/* Which expert-FFN kernels to run.  AUTO picks from N, E and the shape: STREAM up to 72 routed
 * rows, MID up to 10 rows per expert on average, GROUPED above. */
typedef enum {
    MOE_FFN_AUTO = 0,
    MOE_FFN_STREAM = 1, /* decode: weight-streaming MFMA kernels, <=16 rows per pass */
    MOE_FFN_GROUPED = 2, /* prefill: grouped LDS-tiled MFMA GEMM */
    MOE_FFN_MID = 3      /* a handful of rows for each of many experts: weight-streaming grouped GEMM */
} moe_ffn_path_t;

typedef struct moe_weights moe_weights_t; /* opaque, library-owned */

/* Human-readable name of a status code (static storage, never NULL). */
const char* moe_status_string(int status);

/*
 * Gating (Sec. 2.1; Sec. 3.3 "Execution": the gating function tells which
 * experts each token uses).  For every token t the k largest of logits[t,:]
 * are selected on the raw fp32 values; a larger logit comes first and among
 * equal logits (+0.0 == -0.0) the lower expert index comes first.  weights is
 * the softmax over the k selected logits (the full softmax renormalised over
 * the winners), fp32.
 *   logits  [T,E] fp32, finite (NaN/Inf: result unspecified)
 *   idx     [T,k] int32 out, expert ids in the order described above
 *   weights [T,k] fp32 out
 */
int moe_route(const float* logits, int T, int E, int k, int32_t* idx, float* weights,
              void* stream);

/*
 * Per-expert batching (Algorithm 1's inp_size; Sec. 3.3).  With flat slots
 * p = t*k + j and e_p = idx[p]:
 *   counts[e]  = number of slots routed to e          (inp_size)
 *   offsets    = exclusive scan of counts, offsets[E] = T*k
 *   perm       = stable ordering of the slots by expert: perm[i] = p
 *   inv_perm   = its inverse: inv_perm[p] = i
 *   xg[i,:]    = x[perm[i] / k, :]  (bit copy, same dtype as x)
 * All index outputs are int32 and unique, hence bit-reproducible.
 *   idx [T,k] int32 with 0 <= idx < E (values outside are undefined behaviour
 *   of the outputs but never of memory: they are clamped for addressing)
 *   x   [T,d] of x_dtype, xg [T*k,d] out; x and xg may both be NULL to skip
 *   the row gather.
 */
int moe_permute(const int32_t* idx, int T, int E, int k, const void* x, int d,
                moe_dtype_t x_dtype, int32_t* counts, int32_t* offsets, int32_t* perm,
                int32_t* inv_perm, void* xg, void* stream);

/*
 * One-time repack of a layer's expert matrices (Sec. 3.2: w1, w3 [d,f] and
 * w2 [f,d] per expert, stacked over experts; y = (silu(x.w1) * (x.w3)) . w2)
 * into the layout the kernels stream.  The sources are read on `stream` and
 * may be freed once the stream has passed this call.
 *   w_dtype MOE_BF16: device copy in MFMA-fragment order, same byte count.
 *   w_dtype MOE_F32 : plain device copy.
 * *out receives a handle owned by the library; release with moe_weights_free
 * (which synchronises the device).  Allocates device memory.
 */
int moe_weights_pack(const void* w1, const void* w3, const void* w2, int E, int d, int f,
                     moe_dtype_t w_dtype, moe_weights_t** out, void* stream);
int moe_weights_free(moe_weights_t* w);
/* Device bytes held by a packed handle (0 for NULL). HOST query. */
size_t moe_weights_bytes(const moe_weights_t* w);

/* Bytes of scratch moe_expert_ffn needs for N rows (any path). HOST query;
 * returns 0 for arguments outside the domain. */
size_t moe_expert_ffn_workspace(int N, int E, int d, int f, moe_dtype_t act_dtype);

/*
 * Expert feed-forward over the batched rows (Sec. 3.2 case (a); Algorithm 1
 * loop over experts, skipping empty ones).  For each expert e and each row i
 * in [offsets[e], offsets[e+1]):
 *     yg[i,:] = ( silu(xg[i,:] . w1_e) * (xg[i,:] . w3_e) ) . w2_e
 * with fp32 accumulation.  offsets is read on the device: the call never
 * learns the per-expert sizes on the host.
 *   W         packed handle (bf16 or fp32 weights)
 *   xg        [N,d] of act_dtype (fp32 weights need fp32 activations)
 *   offsets   [E+1] int32 DEVICE, offsets[0] = 0, non-decreasing, offsets[E] = N
 *   workspace >= moe_expert_ffn_workspace(...) bytes, 256-byte aligned; contents
 *             are scratch (may be reused by the next call on the same stream)
 *   yg        [N,d] fp32 out
 * bf16-weight kernels multiply on the bf16 matrix cores: fp32 activations are
 * split into bf16 high and low parts (STREAM path, ~2^-16 relative) or rounded
 * to bf16 (GROUPED path); the intermediate silu(a)*b is kept in fp32 (STREAM)
 * or bf16 (GROUPED).  Every path adds its partial sums in a fixed order: the
 * same inputs give the same bits on every run.
 */
int moe_expert_ffn(const moe_weights_t* W, const void* xg, moe_dtype_t act_dtype,
                   const int32_t* offsets, int N, void* workspace, size_t workspace_bytes,
                   float* yg, void* stream);
/* Same, with the kernel family forced (for tests and measurements).  Returns
 * MOE_ERR_UNSUPPORTED if that family cannot run the shape. */
int moe_expert_ffn_path(const moe_weights_t* W, const void* xg, moe_dtype_t act_dtype,
                        const int32_t* offsets, int N, void* workspace,
                        size_t workspace_bytes, float* yg, int path, void* stream);

/*
 * moe_expert_ffn without the gathered copy (Sec. 3.3: the experts consume the tokens the
 * gate sent them; where those rows live is an implementation matter): the kernels read the
 * batched row i as x[perm[i] / k, :], so moe_permute can be called without x / xg and the
 * N x d copy is never written or read back.  Same results as moe_expert_ffn on the xg that
 * moe_permute would have produced, bit for bit.
 *   x [T,d] of act_dtype; perm [T*k] int32 as written by moe_permute; offsets as above;
 *   workspace >= moe_expert_ffn_workspace(T*k, ...); yg [T*k,d] fp32 out
 */
int moe_expert_ffn_tokens(const moe_weights_t* W, const void* x, moe_dtype_t act_dtype, int T,
                          int k, const int32_t* perm, const int32_t* offsets, void* workspace,
                          size_t workspace_bytes, float* yg, void* stream);

/*
 * moe_expert_ffn for callers that cannot allocate device memory and have no workspace to
 * pass: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, kernels and results as moe_expert_ffn; the scratch is a static device
 * array of moe_expert_ffn_noalloc_max_bytes() = 32 MiB inside the library (one copy per GPU,
 * held until the process ends).  The call allocates nothing and frees nothing.
 *   Returns MOE_ERR_WORKSPACE when the kernel family that would run needs more scratch
 *   than that (decode-sized calls fit: the Mixtral shape needs 120 KiB per routed row;
 *   prefill-sized calls do not -- they take moe_expert_ffn with a caller's workspace).
 *   All calls on one GPU share the array: calls that overlap in time on one GPU (different
 *   streams, different host threads) race; serialise them.  Nothing in the array has to
 *   survive between calls and nothing has to be zero at the start of one.
 */
int moe_expert_ffn_noalloc(const moe_weights_t* W, const void* xg, moe_dtype_t act_dtype,
                           const int32_t* offsets, int N, float* yg, void* stream);
size_t moe_expert_ffn_noalloc_max_bytes(void);

/*
 * What moe_expert_ffn_path would run for these sizes (HOST query; nothing is launched).
 *   path     the kernel family (AUTO resolved; MOE_FFN_AUTO for fp32 weights, which have
 *            one kernel pair of their own)
 *   n_parts  reduction parts of the second projection that moe_expert_ffn_parts leaves
 *            unsummed (1 unless STREAM)
 *   up_* / down_*  GROUPED: token rows x output features of the workgroup tile of the
 *            first / second projection (0 otherwise).  The first projection's features
 *            count w1 and w3 columns together.
 * Returns MOE_ERR_UNSUPPORTED if a forced family cannot run the shape.
 */
typedef struct {
    int path;
    int n_parts;
    int up_tile_rows, up_tile_features;
    int down_tile_rows, down_tile_features;
} moe_ffn_plan_t;
int moe_expert_ffn_plan(int N, int E, int d, int f, moe_dtype_t w_dtype, int path,
                        moe_ffn_plan_t* plan);

/*
 * moe_expert_ffn for a consumer that adds the second projection's reduction parts itself
 * (moe_combine_parts, moe_combine_norm_route_permute): the decode kernels cut the long
 * reduction over f into parts and a separate launch would otherwise add them.
 *   yg_parts  [max_parts][N,d] fp32 out: slab p holds part p's partial sums; the layer's
 *             yg is slab 0 + slab 1 + ... in that order
 *   n_parts   HOST out: slabs written (1 for every path but STREAM: then slab 0 is yg)
 * MOE_ERR_INVALID_ARG if the shape needs more than max_parts (see moe_expert_ffn_plan).
 */
int moe_expert_ffn_parts(const moe_weights_t* W, const void* xg, moe_dtype_t act_dtype,
                         const int32_t* offsets, int N, void* workspace, size_t workspace_bytes,
                         float* yg_parts, int max_parts, int* n_parts, void* stream);

/*
 * Expert outputs return to token order, weighted by the gate (Sec. 3.2 names
 * the return of expert outputs; the weighting is the Mixtral layer's):
 *     y[t,:] = sum_{j=0..k-1, ascending} weights[t,j] * yg[inv_perm[t*k+j], :]
 *   yg [T*k,d] fp32, inv_perm [T*k] int32, weights [T,k] fp32, y [T,d] fp32 out
 */
int moe_combine(const float* yg, const int32_t* inv_perm, const float* weights, int T, int k,
                int d, float* y, void* stream);
/*
 * The same over unsummed reduction parts (see moe_expert_ffn_parts), in one launch:
 *     v_j    = yg_parts[0][inv_perm[t*k+j], :] + yg_parts[1][...] + ...   (part order)
 *     y[t,:] = (residual ? y[t,:] : 0) + sum_j weights[t,j] * v_j
 *   yg_parts [n_parts][T*k,d] fp32; yg [T*k,d] fp32 out or NULL: receives the summed rows;
 *   y, yg must not overlap yg_parts.
 */
int moe_combine_parts(const float* yg_parts, int n_parts, const int32_t* inv_perm,
                      const float* weights, int T, int k, int d, float* y, int residual,
                      float* yg, void* stream);

/*
 * One decode step of the layer in three launches (Sec. 3.3 "Execution" for a handful of
 * tokens, where every launch is a few percent of the step): the first-projection kernel runs
 * the gating function and the per-expert batching in its prologue and reads the token rows
 * directly, the second projection leaves its reduction parts, and the combine adds them.
 * With at most four routed rows (one token of a top-2 layer: Sec. 4.1, scenario (a)) the
 * second projection finishes its reduction and the combine inside its workgroups: two
 * launches.
 * Same results as moe_route + moe_permute + moe_expert_ffn + moe_combine: index outputs bit
 * for bit, y and yg in the same fixed summation order.
 *   x [T,d] fp32, logits [T,E] fp32; bf16 weights; 1 <= T <= 16, E <= 16, T*k <= 64 and a
 *   shape the STREAM family supports (MOE_ERR_UNSUPPORTED otherwise)
 *   idx, weights, counts, offsets, perm, inv_perm: as moe_route / moe_permute, all written
 *   xg [T*k,d] fp32 out or NULL, yg [T*k,d] fp32 out or NULL: written only when given
 *   workspace >= moe_expert_ffn_workspace(T*k, E, d, f, MOE_F32)
 *   y [T,d] fp32 out.  Outputs must not overlap x or logits.
 */
int moe_decode_layer(const moe_weights_t* W, const float* x, const float* logits, int T, int k,
                     int32_t* idx, float* weights, int32_t* counts, int32_t* offsets,
                     int32_t* perm, int32_t* inv_perm, float* xg, void* workspace,
                     size_t workspace_bytes, float* yg, float* y, void* stream);

/*
 * The expert layer of one transformer block on the residual stream, for decode steps of at
 * most four routed rows (T*k <= 4), in two launches: moe_decode_layer's kernels, of which the
 * first also derives the block's RMSNorm and router logits and the second also adds the
 * residual and prepares the gating sums of the NEXT block (the non-expert work between two
 * expert layers, Sec. 3.3 "Execution"), so that a stack of blocks needs no launch between
 * them.  The gating sums of the rows x[t,:] against a router matrix w_gate [d,E] are
 *     S[t,e] = sum_c x[t,c] * w_gate[c,e]   (e < E),      S[t,E] = sum_c x[t,c]^2
 * kept as `shares` [n_shares][stride] fp32, stride = moe_gate_sums_stride(T, E), S[t,e] at
 * t*(E+1)+e: share b holds the sums over a part of the features c, and the shares are added
 * in order b = 0, 1, ... in a fixed tree (deterministic).  The call computes
 *     scale[t]    = 1 / sqrt(S[t,E] / d + eps)                RMSNorm, unit gain
 *     logits[t,e] = S[t,e] * scale[t]                         written to `logits`
 *     h[t,:]      = x_in[t,:] * scale[t]                      the experts' input rows
 *     routing and expert FFN of the rows h on `logits`, as moe_decode_layer
 *     x_out[t,:]  = x_in[t,:] + y[t,:]
 *     gate_sums_next = the d/16 shares (16 features each) of x_out against w_gate_next
 * With gate_sums NULL, `logits` is an input and h = x_in (no scale).
 *   x_in [T,d] fp32; gate_sums [n_shares][stride] fp32 or NULL, 1 <= n_shares <= 256
 *   logits [T,E] fp32: out, or in when gate_sums is NULL
 *   idx, weights, counts, offsets, perm, inv_perm: as moe_route / moe_permute, all written
 *   workspace >= moe_expert_ffn_workspace(T*k, E, d, f, MOE_F32)
 *   x_out [T,d] fp32 out; may be x_in itself (in place), no other overlap between arguments
 *   w_gate_next [d,E] fp32 or NULL (then gate_sums_next is not written);
 *   gate_sums_next [d/16][stride] fp32 out: pass it, with n_shares = d/16, to the next call
 * MOE_ERR_UNSUPPORTED for fp32 weights, T*k > 4, E > 16, T*(E+1) > 32, d/16 above the number
 * of compute units (or above 32 per wavefront of the first kernel), or a shape the STREAM
 * family does not serve: use the
 * separate calls then.
 */
int moe_decode_block(const moe_weights_t* W, const float* x_in, const float* gate_sums,
                     int n_shares, float eps, float* logits, int T, int k, int32_t* idx,
                     float* weights, int32_t* counts, int32_t* offsets, int32_t* perm,
                     int32_t* inv_perm, void* workspace, size_t workspace_bytes, float* x_out,
                     const float* w_gate_next, float* gate_sums_next, void* stream);
/* HOST query: 1 if moe_decode_block serves these sizes on the current device, else 0. */
int moe_decode_block_supported(int T, int E, int k, int d, int f, moe_dtype_t w_dtype);
/*
 * The gating sums of the first block of a stack: one share (n_shares = 1) with the sums over
 * all d features of the rows x [T,d] against w_gate [d,E]; E <= 16 (MOE_ERR_UNSUPPORTED
 * above).  sums [moe_gate_sums_stride(T, E)] fp32 out, 16-byte aligned.
 */
int moe_gate_sums(const float* x, const float* w_gate, int T, int d, int E, float* sums,
                  void* stream);
/* HOST: floats per share: 32, one 128-byte line (0 for invalid sizes). */
size_t moe_gate_sums_stride(int T, int E);

/*
 * Support steps of the layer-stack workload (non-expert glue the paper keeps
 * on the GPU, Sec. 3.1): RMS normalisation without gain, router logits and the
 * residual add.
 *   moe_rmsnorm:       h[t,:] = x[t,:] / sqrt(mean(x[t,:]^2) + eps)    fp32 [T,d]
 *   moe_router_logits: logits[t,e] = sum_r h[t,r] * w_gate[r,e]        w_gate [d,E] fp32
 *   moe_residual_add:  x[t,:] += y[t,:]                                in place
 *   moe_rmsnorm_router_logits: both of the first two in one launch, any T, E <= 16
 *                      (MOE_ERR_UNSUPPORTED above); logits = (x . w_gate) / rms(x) in fp32,
 *                      i.e. the normalisation is applied after the dot product.
 */
int moe_rmsnorm(const float* x, int T, int d, float eps, float* h, void* stream);
int moe_router_logits(const float* h, const float* w_gate, int T, int d, int E, float* logits,
                      void* stream);
int moe_residual_add(float* x, const float* y, int T, int d, void* stream);
int moe_rmsnorm_router_logits(const float* x, const float* w_gate, int T, int d, int E, float eps,
                              float* h, float* logits, void* stream);

/*
 * Fused front ends for decode-sized batches: the same results as the separate calls, in
 * one launch each (at T = 1 the launch latency of every small kernel is a few percent of
 * the layer).  Both return MOE_ERR_UNSUPPORTED outside their domain; callers then use the
 * separate calls.
 *   moe_route_permute:      moe_route + moe_permute (fp32 x).  T <= 16, E <= 16.
 *   moe_norm_route_permute: moe_rmsnorm + moe_router_logits + moe_route + moe_permute of
 *                           the normalised rows.  T <= 4, E <= 16.  h [T,d] and logits
 *                           [T,E] are outputs; logits = (x . w_gate) / rms(x) in fp32.
 *   moe_combine_residual:   x[t,:] += sum_j weights[t,j] * yg[inv_perm[t*k+j], :]
 *                           (moe_combine + moe_residual_add), any T.
 *   moe_combine_norm_route_permute: the seam between two blocks of a stack in one
 *                           launch: moe_combine_residual of the block that just ran,
 *                             x_out[t,:] = x_in[t,:] + sum_j weights_prev[t,j] *
 *                                          yg_prev[inv_perm_prev[t*k_prev+j], :],
 *                           then moe_norm_route_permute of x_out for the next block.
 *                           Same limits (T <= 4, E <= 16) and the same fp32 arithmetic as
 *                           the two separate calls.  yg_prev may be the unsummed reduction
 *                           parts that moe_expert_ffn_parts leaves: n_parts_prev slabs of
 *                           [T*k_prev, d] floats, added in part order (1: the plain yg; more
 *                           than 4: MOE_ERR_UNSUPPORTED).
 * Aliasing: in the three calls that normalise or gather (all but moe_combine_residual)
 * every workgroup reads the inputs while one writes the outputs, so no output may overlap
 * an input: h, xg (and x_out) must not overlap x (x_in) or yg_prev, and inv_perm / weights
 * must not overlap inv_perm_prev / weights_prev (MOE_ERR_INVALID_ARG otherwise; the caller
 * of the seam call keeps two sets of routing buffers and alternates).  w_gate must be
 * 16-byte aligned.
 */
int moe_route_permute(const float* logits, int T, int E, int k, const float* x, int d,
                      int32_t* idx, float* weights, int32_t* counts, int32_t* offsets,
                      int32_t* perm, int32_t* inv_perm, float* xg, void* stream);
int moe_norm_route_permute(const float* x, const float* w_gate, int T, int d, int E, int k,
                           float eps, float* h, float* logits, int32_t* idx, float* weights,
                           int32_t* counts, int32_t* offsets, int32_t* perm,
                           int32_t* inv_perm, float* xg, void* stream);
int moe_combine_residual(const float* yg, const int32_t* inv_perm, const float* weights, int T,
                         int k, int d, float* x, void* stream);
int moe_combine_norm_route_permute(const float* yg_prev, int n_parts_prev,
                                   const int32_t* inv_perm_prev,
                                   const float* weights_prev, int k_prev, const float* x_in,
                                   float* x_out, const float* w_gate, int T, int d, int E, int k,
                                   float eps, float* h, float* logits, int32_t* idx, float* weights,
                                   int32_t* counts, int32_t* offsets, int32_t* perm,
                                   int32_t* inv_perm, float* xg, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_H_ */
