// One-time repack of the expert matrices (paper Sec. 3.2: three d x f matrices
// per expert) into the order the matrix-core kernels stream them.
#include <atomic>
#include <new>

#include "moe_internal.h"

int moe_current_device() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return -1;
    }
    return (dev >= 0 && dev < MOE_MAX_DEVICES) ? dev : -1;
}

int moe_num_cus() {
    // 0 = not asked yet; threads that race here store the same value
    static std::atomic<int> cus[MOE_MAX_DEVICES];
    const int dev = moe_current_device();
    if (dev < 0) return 256;
    int n = cus[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            n <= 0) {
            (void)hipGetLastError();
            return 256;
        }
        cus[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

// src: [E][K][C] bf16 row-major (reduction index k, output feature c).
// dst: fragments [E][C/16][nmat][K/32]; this launch fills matrix slot `mat`.
// One thread writes one 16-byte chunk (8 consecutive k of one feature).
__global__ __launch_bounds__(256) void pack_frag_kernel(const uint16_t* __restrict__ src,
                                                        uint4* __restrict__ dst, int E, int K,
                                                        int C, int nmat, int mat) {
    const size_t KS = (size_t)K / 32, NB = (size_t)C / 16;
    const size_t total = (size_t)E * NB * KS * 64;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total;
         i += (size_t)gridDim.x * 256) {
        const int lane = (int)(i & 63);
        size_t fr = i >> 6;  // fragment index within this matrix slot
        const size_t ks = fr % KS;
        fr /= KS;
        const size_t nb = fr % NB;
        const size_t e = fr / NB;
        const size_t c = nb * 16 + (lane & 15);
        const size_t k0 = ks * 32 + 8 * (lane >> 4);
        const uint16_t* s = src + (e * K + k0) * C + c;
        unsigned v[8];
#pragma unroll
        for (int j = 0; j < 8; j++) v[j] = s[(size_t)j * C];
        uint4 o;
        o.x = v[0] | (v[1] << 16);
        o.y = v[2] | (v[3] << 16);
        o.z = v[4] | (v[5] << 16);
        o.w = v[6] | (v[7] << 16);
        const size_t frag = ((e * NB + nb) * nmat + mat) * KS + ks;
        dst[frag * 64 + lane] = o;
    }
}

int moe_weights_pack_impl(const void* w1, const void* w3, const void* w2, int E, int d, int f,
                          moe_dtype_t w_dtype, moe_weights** out, hipStream_t s) {
    moe_weights* W = new (std::nothrow) moe_weights();
    if (!W) return MOE_ERR_HIP;
    W->E = E;
    W->d = d;
    W->f = f;
    W->dtype = w_dtype;
    W->w13 = W->w2 = nullptr;
    W->w1f = W->w3f = W->w2f = nullptr;
    W->bytes = 0;
    if (hipGetDevice(&W->device) != hipSuccess) {
        (void)hipGetLastError();
        delete W;
        return MOE_ERR_HIP;
    }
    const size_t mat_elems = (size_t)E * d * f;
    if (w_dtype == MOE_BF16) {
        if (hipMalloc(&W->w13, mat_elems * 2 * 2) != hipSuccess ||
            hipMalloc(&W->w2, mat_elems * 2) != hipSuccess) {
            (void)hipGetLastError();
            if (W->w13) (void)hipFree(W->w13);
            delete W;
            return MOE_ERR_HIP;
        }
        W->bytes = mat_elems * 2 * 3;
        const unsigned grid = 8192;
        hipLaunchKernelGGL(pack_frag_kernel, dim3(grid), dim3(256), 0, s, (const uint16_t*)w1,
                           (uint4*)W->w13, E, d, f, 2, 0);
        hipLaunchKernelGGL(pack_frag_kernel, dim3(grid), dim3(256), 0, s, (const uint16_t*)w3,
                           (uint4*)W->w13, E, d, f, 2, 1);
        hipLaunchKernelGGL(pack_frag_kernel, dim3(grid), dim3(256), 0, s, (const uint16_t*)w2,
                           (uint4*)W->w2, E, f, d, 1, 0);
        if (moe_launch_status() != MOE_OK) {
            (void)hipFree(W->w13);
            (void)hipFree(W->w2);
            delete W;
            return MOE_ERR_HIP;
        }
    } else {
        void* p[3] = {nullptr, nullptr, nullptr};
        const void* src[3] = {w1, w3, w2};
        for (int i = 0; i < 3; i++) {
            if (hipMalloc(&p[i], mat_elems * 4) != hipSuccess ||
                hipMemcpyAsync(p[i], src[i], mat_elems * 4, hipMemcpyDeviceToDevice, s) !=
                    hipSuccess) {
                (void)hipGetLastError();
                for (int j = 0; j <= i; j++)
                    if (p[j]) (void)hipFree(p[j]);
                delete W;
                return MOE_ERR_HIP;
            }
        }
        W->w1f = (float*)p[0];
        W->w3f = (float*)p[1];
        W->w2f = (float*)p[2];
        W->bytes = mat_elems * 4 * 3;
    }
    *out = W;
    return MOE_OK;
}

// Repack into the buffers of an existing bf16 handle of the same shape (no allocation): the
// staging slot of the split-layer execution.  Sources are device arrays.
int moe_weights_repack_impl(moe_weights* W, const void* w1, const void* w3, const void* w2,
                            hipStream_t s) {
    if (!W || W->dtype != MOE_BF16 || !W->w13 || !W->w2) return MOE_ERR_INVALID_ARG;
    const unsigned grid = 8192;
    hipLaunchKernelGGL(pack_frag_kernel, dim3(grid), dim3(256), 0, s, (const uint16_t*)w1,
                       (uint4*)W->w13, W->E, W->d, W->f, 2, 0);
    hipLaunchKernelGGL(pack_frag_kernel, dim3(grid), dim3(256), 0, s, (const uint16_t*)w3,
                       (uint4*)W->w13, W->E, W->d, W->f, 2, 1);
    hipLaunchKernelGGL(pack_frag_kernel, dim3(grid), dim3(256), 0, s, (const uint16_t*)w2,
                       (uint4*)W->w2, W->E, W->f, W->d, 1, 0);
    return moe_launch_status();
}

int moe_weights_free_impl(moe_weights* W) {
    if (!W) return MOE_OK;
    int rc = MOE_OK;
    // the handle's own device: wait for the kernels that may still read the matrices
    int cur = 0;
    const bool have_cur = hipGetDevice(&cur) == hipSuccess;
    if (have_cur && cur != W->device && hipSetDevice(W->device) != hipSuccess) rc = MOE_ERR_HIP;
    if (hipDeviceSynchronize() != hipSuccess) rc = MOE_ERR_HIP;
    void* p[5] = {W->w13, W->w2, W->w1f, W->w3f, W->w2f};
    for (int i = 0; i < 5; i++)
        if (p[i] && hipFree(p[i]) != hipSuccess) rc = MOE_ERR_HIP;
    if (have_cur && cur != W->device) (void)hipSetDevice(cur);
    if (rc != MOE_OK) (void)hipGetLastError();
    delete W;
    return rc;
}
