// moe_expert_ffn for callers that cannot allocate device memory (code under HIP graph
// capture, tight serving loops, harnesses that forbid hipMalloc): the scratch the kernels
// need lives in a file-scope device array instead of a caller's workspace.
#include <atomic>

#include "moe_internal.h"

// 32 MiB: the decode kernels' scratch (h [N,f] fp32 and the second projection's reduction
// parts [P][N,d] fp32) for every decode-sized call of the shapes at hand -- the Mixtral shape
// needs 120 KiB per routed row.  Every GPU the library runs on holds its own copy until the
// process ends.
#define MOE_NOALLOC_SCRATCH_BYTES ((size_t)32 << 20)
static __device__ __align__(256) unsigned char scratch[MOE_NOALLOC_SCRATCH_BYTES];

// Device address of `scratch` on the current device (each device has its own copy at its own
// address), looked up once per device; null on a HIP error.  Threads that race here ask the
// same question and store the same answer.
static void* noalloc_scratch_ptr() {
    static std::atomic<void*> ptrs[MOE_MAX_DEVICES];
    const int dev = moe_current_device();
    if (dev < 0) return nullptr;
    void* p = ptrs[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return nullptr;
        }
        ptrs[dev].store(p, std::memory_order_release);
    }
    return p;
}

extern "C" {

size_t moe_expert_ffn_noalloc_max_bytes(void) { return MOE_NOALLOC_SCRATCH_BYTES; }

int moe_expert_ffn_noalloc(const moe_weights_t* W, const void* xg, moe_dtype_t act_dtype,
                           const int32_t* offsets, int N, float* yg, void* stream) {
    if (!W || N < 0 || N >= MOE_MAX_N || !offsets) return MOE_ERR_INVALID_ARG;
    if (act_dtype != MOE_F32 && act_dtype != MOE_BF16) return MOE_ERR_INVALID_ARG;
    if (N == 0) return MOE_OK;
    if (!xg || !yg || !moe_aligned16(xg) || !moe_aligned16(yg)) return MOE_ERR_INVALID_ARG;
    if (W->dtype == MOE_F32 && act_dtype != MOE_F32) return MOE_ERR_UNSUPPORTED;
    // scratch of the kernel family that would run (the workspace query of the allocating
    // entry point covers every family at once, which is far more than a decode step needs)
    const int path = W->dtype == MOE_F32 ? MOE_FFN_AUTO : moe_ffn_auto_path(N, W->E, W->d, W->f);
    size_t need;
    if (W->dtype == MOE_F32) need = moe_ffn_f32_workspace(N, W->E, W->d, W->f);
    else if (path == MOE_FFN_STREAM) need = moe_ffn_stream_workspace(N, W->E, W->d, W->f);
    else if (path == MOE_FFN_MID) need = moe_ffn_mid_workspace(N, W->E, W->d, W->f);
    else need = moe_ffn_grouped_workspace(N, W->E, W->d, W->f);
    if (need > MOE_NOALLOC_SCRATCH_BYTES) return MOE_ERR_WORKSPACE;  // beyond the static scratch
    void* ptr = noalloc_scratch_ptr();
    if (!ptr) return MOE_ERR_HIP;
    hipStream_t s = (hipStream_t)stream;
    if (W->dtype == MOE_F32) return moe_ffn_f32_launch(W, (const float*)xg, nullptr, 1, offsets, N, ptr, yg, s);
    if (path == MOE_FFN_STREAM)
        return moe_ffn_stream_launch(W, xg, act_dtype, nullptr, 1, offsets, N, ptr, yg, nullptr, s);
    if (path == MOE_FFN_MID) return moe_ffn_mid_launch(W, xg, act_dtype, nullptr, 1, offsets, N, ptr, yg, s);
    return moe_ffn_grouped_launch(W, xg, act_dtype, nullptr, 1, offsets, N, ptr, yg, s);
}

}  // extern "C"
