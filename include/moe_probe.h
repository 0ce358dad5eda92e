/*
 * libmoe_hip -- measurement hooks and probes.  Not part of the layer (include/moe.h):
 * they exist so that a benchmark can time the two projection kernels of moe_expert_ffn
 * separately and can measure what the board sustains (the two ceilings the roofline
 * fractions are discussed against).  Same conventions as moe.h: device pointers unless
 * stated, status codes, nothing enqueued on an argument error.
 */
#ifndef MOE_PROBE_H_
#define MOE_PROBE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Measurement hook: when `hip_event` (a hipEvent_t as void*, HOST handle) is
 * non-NULL, every following moe_expert_ffn call records it on its stream
 * between the first projection (x.w1, x.w3, silu*mul) and the second (h.w2),
 * so a caller bracketing the call with its own events can time the two kernels
 * separately.  NULL switches the hook off.  Process-wide (one atomic pointer: the hot path
 * pays one relaxed load per call); callers that time concurrently must serialise.
 */
int moe_set_ffn_mid_event(void* hip_event);

/*
 * Measurement probe (not part of the layer): runs `iters` rounds of a
 * register-resident v_mfma_f32_16x16x32_bf16 loop with no memory traffic on every
 * CU and reports the flop count, so that a caller timing it with events learns the
 * matrix-core rate this board sustains for the given operand bits (the published
 * peak assumes the maximum clock; the board lowers it under load, more so for
 * random operands than for constant ones).
 *   operands  64 KiB of bf16 bit patterns (DEVICE), 16-byte aligned
 *   out       2 * CUs * 256 floats of scratch (DEVICE; 512 * 256 floats suffice)
 *   flops     HOST pointer that receives the flop count of the launch (may be NULL)
 */
int moe_mfma_rate_probe(const void* operands, int iters, float* out, double* flops,
                        void* stream);

/* Measurement probe: one launch of a plain streaming-read kernel (one workgroup of 8 waves
 * per CU, contiguous shares, 16 one-KiB non-temporal requests in flight per wave) - the
 * request structure of the decode kernels without set-up, arithmetic or epilogue; context for
 * the HBM roofline (what fraction of the published 8 TB/s a pure read reaches on this board).
 *   data   buffer to read (DEVICE), 16-byte aligned
 *   bytes  its size; reads floor(bytes / (CUs * 8 * 16 KiB)) * 16 KiB per wave (at least
 *          16 KiB per wave, else MOE_ERR_INVALID_ARG), so slightly less than `bytes`
 *   sink   4 bytes (DEVICE) that keep the loads alive
 */
int moe_hbm_read_probe(const void* data, size_t bytes, unsigned* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_PROBE_H_ */
