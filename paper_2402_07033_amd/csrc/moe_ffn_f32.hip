// fp32 expert FFN (fp32 weights and activations, fp32 FMA): the exact-dtype
// path of the tiny all-fp32 workload.  LDS-tiled, 32 rows x 64 features per
// workgroup, reduction in steps of 16; row tiles never straddle two experts.
#include "moe_internal.h"

#define F32_BM 32
#define F32_BN 64
#define F32_BK 16

// Row tile `tile` of the per-expert segments -> (expert, first row, row count).
__device__ __forceinline__ bool f32_find_tile(const int32_t* __restrict__ offsets, int E, int N,
                                              int tile, int& e_out, int& row0, int& rows) {
    int seen = 0;
    for (int e = 0; e < E; e++) {
        int lo = offsets[e], hi = offsets[e + 1];
        lo = lo < 0 ? 0 : (lo > N ? N : lo);
        hi = hi < lo ? lo : (hi > N ? N : hi);
        const int tiles = (hi - lo + F32_BM - 1) / F32_BM;
        if (tile < seen + tiles) {
            e_out = e;
            row0 = lo + (tile - seen) * F32_BM;
            rows = (hi - row0) < F32_BM ? (hi - row0) : F32_BM;
            return true;
        }
        seen += tiles;
    }
    return false;
}

// UP:   out[i,c] = silu(sum_r act[i,r] wA[e,r,c]) * (sum_r act[i,r] wB[e,r,c])
// !UP:  out[i,c] = sum_r act[i,r] wA[e,r,c]
template <bool UP>
__global__ __launch_bounds__(256) void ffn_f32_kernel(const float* __restrict__ act,
                                                      const int32_t* __restrict__ perm, int perm_k,
                                                      const float* __restrict__ wA,
                                                      const float* __restrict__ wB,
                                                      const int32_t* __restrict__ offsets, int E,
                                                      int N, int K, int C,
                                                      float* __restrict__ out) {
    __shared__ float sX[F32_BK][F32_BM + 1];
    __shared__ float sA[F32_BK][F32_BN];
    __shared__ float sB[UP ? F32_BK : 1][F32_BN];
    int e, row0, rows;
    if (!f32_find_tile(offsets, E, N, blockIdx.y, e, row0, rows)) return;
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;  // 4 features, 2 rows per thread
    const int c0 = blockIdx.x * F32_BN;
    const float* wAe = wA + (size_t)e * K * C;
    const float* wBe = UP ? wB + (size_t)e * K * C : nullptr;
    float accA[2][4] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
    float accB[2][4] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
    for (int k0 = 0; k0 < K; k0 += F32_BK) {
        // activations: 32 rows x 16 k (2 per thread), zero beyond the segment
        for (int i = tid; i < F32_BM * F32_BK; i += 256) {
            const int r = i / F32_BK, kk = i % F32_BK;
            // with perm the batched row i is act[perm[i] / perm_k] (the token array itself)
            float v = 0.f;
            if (r < rows) {
                const int src = perm ? perm[row0 + r] / perm_k : row0 + r;
                v = act[(size_t)src * K + k0 + kk];
            }
            sX[kk][r] = v;
        }
        // weights: 16 k x 64 features (4 per thread)
        for (int i = tid; i < F32_BK * F32_BN; i += 256) {
            const int kk = i / F32_BN, cc = i % F32_BN;
            sA[kk][cc] = wAe[(size_t)(k0 + kk) * C + c0 + cc];
            if (UP) sB[kk][cc] = wBe[(size_t)(k0 + kk) * C + c0 + cc];
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < F32_BK; kk++) {
            const float x0 = sX[kk][ty * 2], x1 = sX[kk][ty * 2 + 1];
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const float a = sA[kk][tx * 4 + j];
                accA[0][j] = fmaf(x0, a, accA[0][j]);
                accA[1][j] = fmaf(x1, a, accA[1][j]);
                if (UP) {
                    const float b = sB[kk][tx * 4 + j];
                    accB[0][j] = fmaf(x0, b, accB[0][j]);
                    accB[1][j] = fmaf(x1, b, accB[1][j]);
                }
            }
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 2; i++) {
        const int r = ty * 2 + i;
        if (r >= rows) continue;
#pragma unroll
        for (int j = 0; j < 4; j++) {
            float v = accA[i][j];
            if (UP) v = v / (1.0f + expf(-v)) * accB[i][j];
            out[(size_t)(row0 + r) * C + c0 + tx * 4 + j] = v;
        }
    }
}

size_t moe_ffn_f32_workspace(int N, int E, int d, int f) {
    (void)E;
    (void)d;
    return (size_t)N * f * sizeof(float);
}

int moe_ffn_f32_launch(const moe_weights* W, const float* xg, const int32_t* perm, int k,
                       const int32_t* offsets, int N, void* ws, float* yg, hipStream_t s) {
    const int max_tiles = N / F32_BM + W->E;  // >= sum_e ceil(M_e / BM)
    if (max_tiles > 65535) return MOE_ERR_UNSUPPORTED;  // gridDim.y limit
    float* h = (float*)ws;
    const unsigned ty = (unsigned)max_tiles;
    hipLaunchKernelGGL(ffn_f32_kernel<true>, dim3((unsigned)(W->f / F32_BN), ty), dim3(256), 0, s,
                       xg, perm, k, (const float*)W->w1f, (const float*)W->w3f, offsets, W->E, N, W->d,
                       W->f, h);
    moe_record_mid_event(s);
    hipLaunchKernelGGL(ffn_f32_kernel<false>, dim3((unsigned)(W->d / F32_BN), ty), dim3(256), 0, s,
                       (const float*)h, (const int32_t*)nullptr, 1, (const float*)W->w2f,
                       (const float*)nullptr, offsets, W->E, N, W->f, W->d, yg);
    return moe_launch_status();
}
