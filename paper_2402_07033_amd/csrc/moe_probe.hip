// Measurement probe: a register-resident MFMA loop with no memory traffic in
// it.  It answers one question for the roofline discussion: what rate do the
// matrix cores of THIS board sustain on v_mfma_f32_16x16x32_bf16 when the
// operands are realistic (random) rather than constant?  The published peak
// assumes the maximum clock; under a matrix-core load the board lowers its
// clock, and more so when the operand bits toggle.
#include <atomic>

#include "moe_internal.h"
#include "moe_probe.h"

// Event recorded between the two projections of moe_expert_ffn, or null.
static std::atomic<hipEvent_t> g_mid_event{nullptr};

extern "C" int moe_set_ffn_mid_event(void* hip_event) {
    g_mid_event.store((hipEvent_t)hip_event, std::memory_order_release);
    return MOE_OK;
}

void moe_record_mid_event(hipStream_t s) {
    hipEvent_t ev = g_mid_event.load(std::memory_order_acquire);
    if (ev) (void)hipEventRecord(ev, s);
}

// 4 waves per workgroup, 16 accumulators per wave, operands cycle through 8
// register sets loaded once from `operands` (64 KiB of bf16 bit patterns).
__global__ __launch_bounds__(256) void mfma_rate_kernel(const u32x4_t* __restrict__ operands,
                                                        float* __restrict__ out, int iters) {
    const int lane = threadIdx.x & 63;
    u32x4_t a[8][4], b[8][4];
#pragma unroll
    for (int s = 0; s < 8; s++)
#pragma unroll
        for (int j = 0; j < 4; j++) {
            a[s][j] = operands[((blockIdx.x * 7 + s * 4 + j) & 31) * 64 + lane];
            b[s][j] = operands[((blockIdx.x * 13 + s * 4 + j + 32) & 63) * 64 + lane];
        }
    f32x4_t acc[16];
#pragma unroll
    for (int i = 0; i < 16; i++) acc[i] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; it++) {
#pragma unroll
        for (int s = 0; s < 8; s++)
#pragma unroll
            for (int i = 0; i < 4; i++)
#pragma unroll
                for (int j = 0; j < 4; j++)
                    acc[i * 4 + j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        __builtin_bit_cast(bf16x8_t, a[s][j]), __builtin_bit_cast(bf16x8_t, b[s][i]),
                        acc[i * 4 + j], 0, 0, 0);
    }
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 16; i++) sum += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = sum;
}

extern "C" int moe_mfma_rate_probe(const void* operands, int iters, float* out, double* flops,
                                   void* stream) {
    if (!operands || !out || iters < 1 || iters > (1 << 20) || !moe_aligned16(operands))
        return MOE_ERR_INVALID_ARG;
    const unsigned blocks = (unsigned)(2 * moe_num_cus());
    hipLaunchKernelGGL(mfma_rate_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream,
                       (const u32x4_t*)operands, out, iters);
    if (flops) *flops = (double)blocks * 4.0 * iters * 8.0 * 16.0 * 16384.0;
    return moe_launch_status();
}

// Second probe: what does a plain streaming read get from HBM on this board?  Every
// workgroup (8 waves) reads its contiguous share of `bytes` with fully coalesced
// non-temporal 16-byte-per-lane loads, 16 one-KiB requests in flight per wave - the request
// structure of the decode kernels with the set-up, the arithmetic and the epilogue removed.
#define HBM_PROBE_RING 16
__global__ __launch_bounds__(512) void hbm_read_kernel(const u32x4_t* __restrict__ p,
                                                       unsigned long long loads_per_wave,
                                                       unsigned* __restrict__ sink) {
    const int lane = threadIdx.x & 63;
    const unsigned long long wave_id = (unsigned long long)blockIdx.x * 8 + (threadIdx.x >> 6);
    const u32x4_t* b = p + wave_id * loads_per_wave * 64 + lane;
    u32x4_t acc = {0u, 0u, 0u, 0u};
    u32x4_t buf[HBM_PROBE_RING];
#pragma unroll
    for (int i = 0; i < HBM_PROBE_RING; i++) buf[i] = __builtin_nontemporal_load(b + (size_t)i * 64);
    for (unsigned long long j = HBM_PROBE_RING; j < loads_per_wave; j += HBM_PROBE_RING) {
#pragma unroll
        for (int i = 0; i < HBM_PROBE_RING; i++) {
            acc ^= buf[i];
            buf[i] = __builtin_nontemporal_load(b + (size_t)(j + i) * 64);
        }
    }
#pragma unroll
    for (int i = 0; i < HBM_PROBE_RING; i++) acc ^= buf[i];
    // keeps the loads alive; practically never true
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u) sink[0] = 1u;
}

extern "C" int moe_hbm_read_probe(const void* data, size_t bytes, unsigned* sink, void* stream) {
    if (!data || !sink || !moe_aligned16(data)) return MOE_ERR_INVALID_ARG;
    const unsigned blocks = (unsigned)moe_num_cus();
    // whole rings of one-KiB loads per wave; the rest of the buffer is not read
    const size_t per_wave = bytes / ((size_t)blocks * 8 * 1024 * HBM_PROBE_RING) * HBM_PROBE_RING;
    if (per_wave < HBM_PROBE_RING) return MOE_ERR_INVALID_ARG;
    hipLaunchKernelGGL(hbm_read_kernel, dim3(blocks), dim3(512), 0, (hipStream_t)stream,
                       (const u32x4_t*)data, (unsigned long long)per_wave, sink);
    return moe_launch_status();
}
