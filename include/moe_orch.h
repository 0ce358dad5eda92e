/*
 * libmoe_hip -- the paper's own method on top of the expert-layer kernels: execution of a
 * layer whose expert matrices do not all fit in device memory (Fiddler, arXiv 2402.07033,
 * Sec. 3).  Three pieces, each a plain restatement of the paper:
 *
 *   placement      Sec. 3.4: as many experts as the capacity permits are kept in device
 *                  memory, in order of popularity (a profile of how often each expert was
 *                  selected on calibration data), which maximises the expected hit rate.
 *   latency model  Sec. 3.3: the device executes an expert in a time that does not depend
 *                  on its input size, the host in a time proportional to it; a weight
 *                  transfer costs a constant.  The three constants are measured at
 *                  initialisation (moe_orch_calibrate).
 *   Algorithm 1    per expert j with input size s: skip if s == 0; run on the device if its
 *                  weights are there; otherwise run on the device after copying the
 *                  weights if cpu_lat(s) > gpu_lat(s) + transfer_lat, else copy the s
 *                  activation rows to the host and run there (cases (a), (b), (c) of
 *                  Sec. 3.2).
 *
 * The host-side expert execution below is case (c) of the paper, for experts whose weights
 * are NOT in device memory; it is no substitute for the device kernels, and none of the
 * entry points of moe.h ever runs on the host.
 *
 * Conventions as in moe.h (status codes, nothing enqueued on an argument error).  HOST
 * marks host pointers; everything else is a device pointer.
 */
#ifndef MOE_ORCH_H_
#define MOE_ORCH_H_

#include <stddef.h>
#include <stdint.h>

#include "moe.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Where Algorithm 1 sends an expert. */
typedef enum {
    MOE_ORCH_SKIP = 0,          /* no input rows */
    MOE_ORCH_GPU_RESIDENT = 1,  /* Sec. 3.2 case (a) */
    MOE_ORCH_GPU_TRANSFER = 2,  /* case (b): copy the weights to the device, run there */
    MOE_ORCH_CPU = 3            /* case (c): copy the rows to the host, run there */
} moe_orch_decision_t;

/* Sec. 3.3: gpu_lat(s) = gpu_lat_us, cpu_lat(s) = cpu_lat_us_per_row * s,
 * transfer_lat() = transfer_lat_us. */
typedef struct {
    double gpu_lat_us;
    double cpu_lat_us_per_row;
    double transfer_lat_us;
} moe_orch_latency_t;

/*
 * Placement (Sec. 3.4).  popularity [L*E] HOST: non-negative selection counts (or any
 * proportional profile) of expert e of layer l at l*E+e.  The `capacity` most popular
 * experts of the whole model are marked in at_gpu [L*E] HOST out (1 = device memory);
 * among equally popular experts the lower index l*E+e is placed first.
 */
int moe_orch_place(const double* popularity, int L, int E, int capacity, uint8_t* at_gpu);
/* Expected hit rate of a placement under a profile: the share of selections that find
 * their expert in device memory (App. "Expert Popularity").  0 for an all-zero profile. */
double moe_orch_hit_rate(const double* popularity, const uint8_t* at_gpu, int L, int E);

/*
 * Algorithm 1 for one layer.  at_gpu [E] HOST, inp_size [E] HOST, decisions [E] HOST out
 * (moe_orch_decision_t values).
 */
int moe_orch_decide(const uint8_t* at_gpu, const int32_t* inp_size, int E,
                    const moe_orch_latency_t* lat, int32_t* decisions);

/*
 * Host-side expert (case (c)): y = (silu(x . w1) * (x . w3)) . w2 for s rows, bf16 weights
 * widened exactly, fp32 arithmetic.  All pointers HOST: x [s,d] fp32, w1, w3 [d,f] and
 * w2 [f,d] bf16 bit patterns row-major, y [s,d] fp32 out.  Uses the host's cores (OpenMP).
 */
int moe_orch_cpu_expert_ffn(const float* x, int s, const uint16_t* w1, const uint16_t* w3,
                            const uint16_t* w2, int d, int f, float* y);

typedef struct moe_orch_layer moe_orch_layer_t; /* opaque, library-owned */

/*
 * One layer split between device and host memory (initialisation, Sec. 3.3).
 *   w1, w3 [E,d,f], w2 [E,f,d]  HOST bf16 bit patterns, row-major (read during the call)
 *   at_gpu [E] HOST             experts to keep in device memory (packed once, here)
 *   max_rows                    largest T*k a call will pass
 * Experts not at the GPU are copied into pinned host memory (for the weight transfers and
 * the host-side execution); one device staging slot of one expert's size serves case (b).
 * Allocates device and pinned host memory; release with moe_orch_layer_free.
 */
int moe_orch_layer_create(const uint16_t* w1, const uint16_t* w3, const uint16_t* w2, int E, int d,
                          int f, const uint8_t* at_gpu, int max_rows, moe_orch_layer_t** out,
                          void* stream);
int moe_orch_layer_free(moe_orch_layer_t* layer);

/*
 * Measures the three constants of the latency model on this machine (Sec. 3.3: "we also
 * measure the latency to copy weights and execute experts on either the CPU or the GPU"):
 * one expert's transfer + repack, its device execution at 1 and 16 rows (their mean), and
 * the host execution at 1, 2 and 4 rows (least-squares slope through the origin).
 * Synchronises the stream.  Needs at least one expert in host memory
 * (MOE_ERR_UNSUPPORTED otherwise).  workspace as for moe_orch_expert_ffn.
 */
int moe_orch_calibrate(moe_orch_layer_t* layer, void* workspace, size_t workspace_bytes,
                       moe_orch_latency_t* lat, void* stream);

/*
 * The expert FFN of moe_expert_ffn for a split layer: Algorithm 1 decides per expert, then
 * device-resident experts run on the device, the others either after a weight transfer into
 * the staging slot or on the host.  The per-expert input sizes are copied to the host first
 * (the decision is the host's), so the call synchronises the stream once at its start and
 * returns with the remaining work enqueued.
 *   xg [N,d] fp32, offsets [E+1] int32 as moe_permute wrote them, N <= max_rows
 *   workspace >= moe_expert_ffn_workspace(N, 1, d, f, MOE_F32) bytes, 256-byte aligned
 *   yg [N,d] fp32 out
 *   decisions [E] HOST out or NULL: what Algorithm 1 chose
 * One call at a time per layer handle.
 */
int moe_orch_expert_ffn(moe_orch_layer_t* layer, const moe_orch_latency_t* lat, const float* xg,
                        const int32_t* offsets, int N, void* workspace, size_t workspace_bytes,
                        float* yg, int32_t* decisions, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_ORCH_H_ */
