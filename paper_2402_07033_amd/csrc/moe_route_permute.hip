// Gating top-k, per-expert batching and gate-weighted combine for gfx950.
//
// route  : G = next power of two >= E lanes of a wavefront hold one token's
//          logits; k rounds of a butterfly arg-max (value desc, index asc)
//          pick the experts; the softmax over the k winners is fp32.
// permute: a stable counting sort of the T*k slots keyed on the expert.  Ranks
//          come from wavefront ballots (lanes below me with my expert) plus a
//          scan over the waves of a 1024-slot chunk, so the order inside an
//          expert segment is the slot order and the result is unique.
// combine: y[t] = sum_j w[t,j] * yg[inv_perm[t*k+j]], float4 lanes along d.
#include "moe_internal.h"
#include "moe_gate_wave.h"

// ------------------------------------------------------------------ route ----

template <int G>
__global__ __launch_bounds__(256) void route_kernel(const float* __restrict__ logits, int T, int E,
                                                    int k, int32_t* __restrict__ idx,
                                                    float* __restrict__ weights) {
    const int tid = blockIdx.x * 256 + threadIdx.x;
    const int t = tid / G;
    const int gl = tid % G;  // lane inside the token's group = expert id it holds
    const bool live = (t < T);
    float v = -INFINITY;
    int e = 0x7fffffff;
    if (live && gl < E) {
        v = logits[(size_t)t * E + gl];
        e = gl;
    }
    float my_v = 0.f, top_v = 0.f;
    int my_i = 0;
    for (int j = 0; j < k; j++) {
        float bv = v;
        int be = e;
#pragma unroll
        for (int m = 1; m < G; m <<= 1) {
            float ov = __shfl_xor(bv, m, 64);
            int oe = __shfl_xor(be, m, 64);
            if (ov > bv || (ov == bv && oe < be)) {
                bv = ov;
                be = oe;
            }
        }
        if (j == 0) top_v = bv;
        if (gl == j) {
            my_v = bv;
            my_i = be;
        }
        if (e == be) {  // the winner leaves the contest
            v = -INFINITY;
            e = 0x7fffffff;
        }
    }
    float u = (gl < k) ? expf(my_v - top_v) : 0.f;
    float s = u;
#pragma unroll
    for (int m = 1; m < G; m <<= 1) s += __shfl_xor(s, m, 64);
    if (live && gl < k) {
        idx[(size_t)t * k + gl] = my_i;
        weights[(size_t)t * k + gl] = u / s;
    }
}

int moe_route_launch(const float* logits, int T, int E, int k, int32_t* idx, float* weights,
                     hipStream_t s) {
    int G = 1;
    while (G < E) G <<= 1;
    if (G < k) G = 8;  // cannot happen (k <= E); keeps lanes gl < k inside the group
    const int tok_per_block = 256 / G;
    const unsigned grid = (unsigned)((T + tok_per_block - 1) / tok_per_block);
#define ROUTE_CASE(g)                                                                         \
    case g:                                                                                   \
        hipLaunchKernelGGL(route_kernel<g>, dim3(grid), dim3(256), 0, s, logits, T, E, k, idx, \
                           weights);                                                          \
        break;
    switch (G) {
        ROUTE_CASE(1)
        ROUTE_CASE(2)
        ROUTE_CASE(4)
        ROUTE_CASE(8)
        ROUTE_CASE(16)
        ROUTE_CASE(32)
        ROUTE_CASE(64)
        default:
            return MOE_ERR_INVALID_ARG;
    }
#undef ROUTE_CASE
    return moe_launch_status();
}

// ---------------------------------------------------------------- permute ----

#define PERM_THREADS 1024
#define PERM_WAVES (PERM_THREADS / 64)

// Index part of the permute for all N slots, run by ONE workgroup of 1024
// threads (every workgroup of a launch runs it redundantly when N <= 1024, so
// that each can then gather its share of rows without a second launch).
// Outputs are written only when `write` is set.  Returns through LDS: s_off.
__device__ void permute_indices(const int32_t* __restrict__ idx, int N, int E,
                                int32_t* __restrict__ counts, int32_t* __restrict__ offsets,
                                int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm,
                                bool write, int* s_cnt /*[64]*/, int* s_off /*[65]*/,
                                int* s_wave /*[PERM_WAVES][64]*/, int* s_pos /*[1024] or null*/) {
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    if (tid < MOE_MAX_E) s_cnt[tid] = 0;
    __syncthreads();
    for (int p = tid; p < N; p += PERM_THREADS) {
        int e = idx[p];
        e = e < 0 ? 0 : (e >= E ? E - 1 : e);
        atomicAdd(&s_cnt[e], 1);
    }
    __syncthreads();
    if (tid == 0) {
        int run = 0;
        for (int e = 0; e < E; e++) {
            s_off[e] = run;
            run += s_cnt[e];
        }
        s_off[E] = run;
    }
    __syncthreads();
    if (write) {
        if (tid < E) counts[tid] = s_cnt[tid];
        if (tid <= E) offsets[tid] = s_off[tid];
    }
    // s_cnt now becomes the running number of slots already placed per expert.
    __syncthreads();
    if (tid < MOE_MAX_E) s_cnt[tid] = 0;
    __syncthreads();
    const unsigned long long below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    for (int base = 0; base < N; base += PERM_THREADS) {
        const int p = base + tid;
        int e = -1;
        if (p < N) {
            e = idx[p];
            e = e < 0 ? 0 : (e >= E ? E - 1 : e);
        }
        int rank = 0;
        for (int ee = 0; ee < E; ee++) {
            unsigned long long m = __ballot(e == ee);
            if (e == ee) rank = __popcll(m & below);
            if (lane == 0) s_wave[wave * MOE_MAX_E + ee] = __popcll(m);
        }
        __syncthreads();
        if (tid < E) {
            int run = s_cnt[tid];
            for (int w = 0; w < PERM_WAVES; w++) {
                int c = s_wave[w * MOE_MAX_E + tid];
                s_wave[w * MOE_MAX_E + tid] = run;
                run += c;
            }
            s_cnt[tid] = run;
        }
        __syncthreads();
        if (p < N) {
            const int pos = s_off[e] + s_wave[wave * MOE_MAX_E + e] + rank;
            if (write) {
                perm[pos] = p;
                inv_perm[p] = pos;
            }
            if (s_pos) s_pos[p] = pos;
        }
        __syncthreads();
    }
}

// N <= 1024: one launch does everything.  Every workgroup computes the slot
// positions in LDS, workgroup 0 writes the index outputs, and the workgroups
// share the row gather (16-byte chunks, coalesced along d).
__global__ __launch_bounds__(PERM_THREADS) void permute_small_kernel(
    const int32_t* __restrict__ idx, int N, int E, int k, const uint4* __restrict__ x,
    int row_chunks /* 16-byte chunks per row */, int32_t* __restrict__ counts,
    int32_t* __restrict__ offsets, int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm,
    uint4* __restrict__ xg) {
    __shared__ int s_cnt[MOE_MAX_E];
    __shared__ int s_off[MOE_MAX_E + 1];
    __shared__ int s_wave[PERM_WAVES * MOE_MAX_E];
    __shared__ int s_pos[PERM_THREADS];
    permute_indices(idx, N, E, counts, offsets, perm, inv_perm, blockIdx.x == 0, s_cnt, s_off,
                    s_wave, s_pos);
    if (x == nullptr) return;
    __syncthreads();
    for (int p = blockIdx.x; p < N; p += gridDim.x) {
        const uint4* src = x + (size_t)(p / k) * row_chunks;
        uint4* dst = xg + (size_t)s_pos[p] * row_chunks;
        for (int c = threadIdx.x; c < row_chunks; c += PERM_THREADS) dst[c] = src[c];
    }
}

__global__ __launch_bounds__(PERM_THREADS) void permute_index_kernel(
    const int32_t* __restrict__ idx, int N, int E, int32_t* __restrict__ counts,
    int32_t* __restrict__ offsets, int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm) {
    __shared__ int s_cnt[MOE_MAX_E];
    __shared__ int s_off[MOE_MAX_E + 1];
    __shared__ int s_wave[PERM_WAVES * MOE_MAX_E];
    permute_indices(idx, N, E, counts, offsets, perm, inv_perm, true, s_cnt, s_off, s_wave,
                    nullptr);
}

// xg[i,:] = x[perm[i]/k,:]; one workgroup of 256 threads per group of rows.
__global__ __launch_bounds__(256) void gather_rows_kernel(const int32_t* __restrict__ perm, int N,
                                                          int k, const uint4* __restrict__ x,
                                                          int row_chunks,
                                                          uint4* __restrict__ xg) {
    for (int i = blockIdx.x; i < N; i += gridDim.x) {
        const uint4* src = x + (size_t)(perm[i] / k) * row_chunks;
        uint4* dst = xg + (size_t)i * row_chunks;
        for (int c = threadIdx.x; c < row_chunks; c += 256) dst[c] = src[c];
    }
}

int moe_permute_launch(const int32_t* idx, int T, int E, int k, const void* x, int d,
                       moe_dtype_t x_dtype, int32_t* counts, int32_t* offsets, int32_t* perm,
                       int32_t* inv_perm, void* xg, hipStream_t s) {
    const int N = T * k;
    const int row_chunks = (int)(((size_t)d * (x_dtype == MOE_BF16 ? 2 : 4)) / 16);
    if (N <= PERM_THREADS) {
        unsigned grid = 1;
        if (x != nullptr && N > 0) grid = (unsigned)(N < 64 ? N : 64);
        hipLaunchKernelGGL(permute_small_kernel, dim3(grid), dim3(PERM_THREADS), 0, s, idx, N, E, k,
                           (const uint4*)x, row_chunks, counts, offsets, perm, inv_perm,
                           (uint4*)xg);
        return moe_launch_status();
    }
    hipLaunchKernelGGL(permute_index_kernel, dim3(1), dim3(PERM_THREADS), 0, s, idx, N, E, counts,
                       offsets, perm, inv_perm);
    if (moe_launch_status() != MOE_OK) return MOE_ERR_HIP;
    if (x != nullptr) {
        unsigned grid = (unsigned)(N < 8192 ? N : 8192);
        hipLaunchKernelGGL(gather_rows_kernel, dim3(grid), dim3(256), 0, s, perm, N, k,
                           (const uint4*)x, row_chunks, (uint4*)xg);
    }
    return moe_launch_status();
}

// ---------------------------------------------------------------- combine ----

__global__ __launch_bounds__(256) void combine_kernel(const float4* __restrict__ yg,
                                                      const int32_t* __restrict__ inv_perm,
                                                      const float* __restrict__ weights, int T,
                                                      int k, int row_chunks /* d/4 */,
                                                      float4* __restrict__ y) {
    const int t = blockIdx.y;
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (t >= T || c >= row_chunks) return;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int j = 0; j < k; j++) {
        const float w = weights[(size_t)t * k + j];
        const float4 v = yg[(size_t)inv_perm[(size_t)t * k + j] * row_chunks + c];
        acc.x += w * v.x;
        acc.y += w * v.y;
        acc.z += w * v.z;
        acc.w += w * v.w;
    }
    y[(size_t)t * row_chunks + c] = acc;
}

int moe_combine_launch(const float* yg, const int32_t* inv_perm, const float* weights, int T, int k,
                       int d, float* y, hipStream_t s) {
    const int row_chunks = d / 4;
    dim3 grid((unsigned)((row_chunks + 255) / 256), (unsigned)T);
    // gridDim.y is limited to 65535: walk T in slabs
    for (int t0 = 0; t0 < T; t0 += 65535) {
        const int tn = (T - t0) < 65535 ? (T - t0) : 65535;
        grid.y = (unsigned)tn;
        hipLaunchKernelGGL(combine_kernel, grid, dim3(256), 0, s, (const float4*)yg,
                           inv_perm + (size_t)t0 * k, weights + (size_t)t0 * k, tn, k, row_chunks,
                           (float4*)(y + (size_t)t0 * d));
    }
    return moe_launch_status();
}

// ------------------------------------------------- stack support kernels ----

__device__ __forceinline__ float block_sum_256(float v, float* s_red /*[4]*/) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) s_red[threadIdx.x >> 6] = v;
    __syncthreads();
    return s_red[0] + s_red[1] + s_red[2] + s_red[3];
}

__global__ __launch_bounds__(256) void rmsnorm_kernel(const float* __restrict__ x, int d, float eps,
                                                      float* __restrict__ h) {
    __shared__ float s_red[4];
    const float* row = x + (size_t)blockIdx.x * d;
    float ss = 0.f;
    for (int r = threadIdx.x; r < d; r += 256) ss += row[r] * row[r];
    ss = block_sum_256(ss, s_red);
    const float inv = 1.0f / sqrtf(ss / (float)d + eps);
    float* out = h + (size_t)blockIdx.x * d;
    for (int r = threadIdx.x; r < d; r += 256) out[r] = row[r] * inv;
}

// One workgroup per token; thread r-strided partial sums for all E logits.
__global__ __launch_bounds__(256) void router_logits_kernel(const float* __restrict__ h,
                                                            const float* __restrict__ w_gate, int d,
                                                            int E, float* __restrict__ logits) {
    __shared__ float s_red[4];
    const float* row = h + (size_t)blockIdx.x * d;
    for (int e0 = 0; e0 < E; e0 += 8) {
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        const int ne = (E - e0) < 8 ? (E - e0) : 8;
        for (int r = threadIdx.x; r < d; r += 256) {
            const float hv = row[r];
            const float* wr = w_gate + (size_t)r * E + e0;
#pragma unroll
            for (int j = 0; j < 8; j++)
                if (j < ne) acc[j] += hv * wr[j];
        }
#pragma unroll
        for (int j = 0; j < 8; j++) {
            const float tot = block_sum_256(acc[j], s_red);
            if (j < ne && threadIdx.x == 0) logits[(size_t)blockIdx.x * E + e0 + j] = tot;
        }
    }
}

__global__ __launch_bounds__(256) void residual_add_kernel(float4* __restrict__ x,
                                                           const float4* __restrict__ y,
                                                           size_t n4) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (size_t)gridDim.x * 256) {
        float4 a = x[i];
        const float4 b = y[i];
        a.x += b.x;
        a.y += b.y;
        a.z += b.z;
        a.w += b.w;
        x[i] = a;
    }
}

int moe_rmsnorm_launch(const float* x, int T, int d, float eps, float* h, hipStream_t s) {
    hipLaunchKernelGGL(rmsnorm_kernel, dim3((unsigned)T), dim3(256), 0, s, x, d, eps, h);
    return moe_launch_status();
}

int moe_router_logits_launch(const float* h, const float* w_gate, int T, int d, int E,
                             float* logits, hipStream_t s) {
    hipLaunchKernelGGL(router_logits_kernel, dim3((unsigned)T), dim3(256), 0, s, h, w_gate, d, E,
                       logits);
    return moe_launch_status();
}

int moe_residual_add_launch(float* x, const float* y, int T, int d, hipStream_t s) {
    const size_t n4 = (size_t)T * d / 4;
    size_t blocks = (n4 + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(residual_add_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (float4*)x,
                       (const float4*)y, n4);
    return moe_launch_status();
}

// --------------------------------------------- fused gate for decode-sized T ----
// One launch for the whole front end of a decode step (T <= 16 tokens): optional
// RMS normalisation + router logits, top-k routing, per-expert batching and the
// row gather.  Every workgroup recomputes the (tiny) routing state in LDS;
// workgroup 0 writes the index outputs; the workgroups share the row gather.
#define GATE_MAX_T 16       // tokens the fused gate handles
#define GATE_NORM_MAX_T 4   // ... when it also normalises and computes the router logits
#define GATE_MAX_E 16
// Partial sums of one thread for the fused RMSNorm + router: rows r = tid + i * STRIDE.
// TT = tokens handled (compile-time bound on T), UNR = rows whose loads are in flight together.
// The pending combine + residual of the block before (COMB): the row values are
//   x[t,r] + sum_j w_prev[t,j] * yg_prev[pos_prev[t,j], r]
// in the arithmetic of combine_residual_kernel.
struct GatePrev {
    const float* yg;   // [P][N_prev, d] (global): the reduction parts of the block before,
                       // added in part order (P = 1: its plain output)
    const int* pos;    // [T * k] rows of yg (inv_perm of the block before)
    const float* w;    // [T * k] gate weights of the block before
    int k;
    int P;
    size_t pstride;    // floats between two parts
};

#define GATE_MAX_PARTS 4  // reduction parts of the block before that the seam kernel adds

// PMAX: compile-time bound on pv.P; every part's load is issued before the first is used.
template <int TT, int UNR, int KJMAX, int PMAX, int STRIDE = PERM_THREADS>
__device__ __forceinline__ void gate_partial_sums(const float* __restrict__ x,
                                                  const float* __restrict__ w_gate, int T, int d,
                                                  int E, int tid, const GatePrev& pv,
                                                  float (&ss)[GATE_NORM_MAX_T],
                                                  float (&acc)[GATE_NORM_MAX_T][GATE_MAX_E]) {
    constexpr bool COMB = KJMAX > 0;        // KJMAX: compile-time bound on pv.k (0: no combine)
    constexpr int KJ = COMB ? KJMAX : 1;
    const bool vec = (E & 3) == 0;  // rows of w_gate are then 16-byte aligned
    for (int r0 = tid; r0 < d; r0 += UNR * STRIDE) {
        float wr[UNR][GATE_MAX_E], xv[UNR][TT], yv[UNR][TT][KJ][PMAX];
#pragma unroll
        for (int u = 0; u < UNR; u++) {
            const int r = r0 + u * STRIDE;
#pragma unroll
            for (int e = 0; e < GATE_MAX_E; e++) wr[u][e] = 0.f;
#pragma unroll
            for (int t = 0; t < TT; t++) {
                xv[u][t] = 0.f;
#pragma unroll
                for (int j = 0; j < KJ; j++)
#pragma unroll
                    for (int q = 0; q < PMAX; q++) yv[u][t][j][q] = 0.f;
            }
            if (r < d) {
                if (vec) {
#pragma unroll
                    for (int q = 0; q < GATE_MAX_E / 4; q++) {
                        if (4 * q < E) {
                            const float4 v = *(const float4*)(w_gate + (size_t)r * E + 4 * q);
                            wr[u][4 * q] = v.x; wr[u][4 * q + 1] = v.y;
                            wr[u][4 * q + 2] = v.z; wr[u][4 * q + 3] = v.w;
                        }
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < GATE_MAX_E; e++)
                        if (e < E) wr[u][e] = w_gate[(size_t)r * E + e];
                }
#pragma unroll
                for (int t = 0; t < TT; t++) {
                    if (t < T) {
                        xv[u][t] = x[(size_t)t * d + r];
                        if (COMB) {
#pragma unroll
                            for (int j = 0; j < KJ; j++)
                                if (j < pv.k) {
                                    const float* p = pv.yg + (size_t)pv.pos[t * pv.k + j] * d + r;
#pragma unroll
                                    for (int q = 0; q < PMAX; q++)
                                        if (q < pv.P) yv[u][t][j][q] = p[(size_t)q * pv.pstride];
                                }
                        }
                    }
                }
            }
        }
        if (COMB) {
#pragma unroll
            for (int u = 0; u < UNR; u++) {
#pragma unroll
                for (int t = 0; t < TT; t++) {
                    if (t < T) {
                        float a = 0.f;
#pragma unroll
                        for (int j = 0; j < KJ; j++)
                            if (j < pv.k) {
                                float v = yv[u][t][j][0];  // the parts in part order
#pragma unroll
                                for (int q = 1; q < PMAX; q++)
                                    if (q < pv.P) v += yv[u][t][j][q];
                                a += pv.w[t * pv.k + j] * v;
                            }
                        xv[u][t] += a;
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < UNR; u++) {
#pragma unroll
            for (int t = 0; t < TT; t++) {
                ss[t] = fmaf(xv[u][t], xv[u][t], ss[t]);
#pragma unroll
                for (int e = 0; e < GATE_MAX_E; e++) acc[t][e] = fmaf(xv[u][t], wr[u][e], acc[t][e]);
            }
        }
    }
}


template <bool NORM, int KJMAX, int PMAX>
__global__ __launch_bounds__(PERM_THREADS) void gate_small_kernel(
    const float* __restrict__ x, const float* __restrict__ w_gate, const float* __restrict__ logits_in,
    int T, int d, int E, int k, float eps, float* __restrict__ h_out, float* __restrict__ logits_out,
    int32_t* __restrict__ idx, float* __restrict__ weights, int32_t* __restrict__ counts,
    int32_t* __restrict__ offsets, int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm,
    float* __restrict__ xg, const float* __restrict__ yg_prev, int n_parts_prev,
    const int32_t* __restrict__ inv_perm_prev, const float* __restrict__ weights_prev, int k_prev,
    float* __restrict__ x_out) {
    __shared__ int s_ppos[GATE_NORM_MAX_T * MOE_MAX_K];
    __shared__ float s_pw[GATE_NORM_MAX_T * MOE_MAX_K];
    __shared__ int s_cnt[MOE_MAX_E];
    __shared__ int s_off[MOE_MAX_E + 1];
    __shared__ int s_wave[PERM_WAVES * MOE_MAX_E];
    __shared__ int s_pos[GATE_MAX_T * MOE_MAX_K];
    __shared__ int s_idx[GATE_MAX_T * MOE_MAX_K];
    __shared__ float s_logits[GATE_MAX_T * GATE_MAX_E];
    __shared__ float s_inv[GATE_MAX_T];
    __shared__ float s_part[PERM_WAVES][GATE_NORM_MAX_T * (GATE_MAX_E + 1)];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr bool COMB = KJMAX > 0;
    const bool writer = (blockIdx.x == 0);
    // The partial sums read the previous block's positions and weights straight from
    // global memory (uniform addresses), so that their other loads need not wait for a
    // barrier; the LDS copies serve the row phase at the end and are published by the
    // barriers in between.
    GatePrev pv = {yg_prev, inv_perm_prev, weights_prev, k_prev, n_parts_prev,
                   (size_t)T * k_prev * d};
    if (COMB && tid < T * k_prev) {
        s_ppos[tid] = inv_perm_prev[tid];
        s_pw[tid] = weights_prev[tid];
    }

    if (NORM) {
        // T <= GATE_NORM_MAX_T here.  Per thread: rows r = tid, tid+1024, ...; partial sums
        // of x^2 and of x * w_gate[:, e] for every token, reduced over the workgroup.
        float ss[GATE_NORM_MAX_T], acc[GATE_NORM_MAX_T][GATE_MAX_E];
#pragma unroll
        for (int t = 0; t < GATE_NORM_MAX_T; t++) {
            ss[t] = 0.f;
#pragma unroll
            for (int e = 0; e < GATE_MAX_E; e++) acc[t][e] = 0.f;
        }
        // The router matrix is cold in HBM at every layer: all loads of a group of rows
        // are issued before the first use, so a thread pays the memory latency once per
        // group instead of once per row (4 rows per group for one token, else 2).
        if (T == 1)
            gate_partial_sums<1, (KJMAX * PMAX > 2 ? 2 : 4), KJMAX, PMAX>(x, w_gate, T, d, E, tid, pv, ss,
                                                                          acc);
        else
            gate_partial_sums<GATE_NORM_MAX_T, (COMB ? 1 : 2), KJMAX, PMAX>(x, w_gate, T, d, E, tid,
                                                                             pv, ss, acc);
        // wave reduce, then across the 16 waves through LDS
#pragma unroll
        for (int t = 0; t < GATE_NORM_MAX_T; t++) {
            if (t < T) {
#pragma unroll
                for (int m = 32; m >= 1; m >>= 1) ss[t] += __shfl_xor(ss[t], m, 64);
#pragma unroll
                for (int e = 0; e < GATE_MAX_E; e++) {
                    if (e < E) {
#pragma unroll
                        for (int m = 32; m >= 1; m >>= 1) acc[t][e] += __shfl_xor(acc[t][e], m, 64);
                    }
                }
                if (lane == 0) {
                    s_part[wave][t * (GATE_MAX_E + 1) + GATE_MAX_E] = ss[t];
#pragma unroll
                    for (int e = 0; e < GATE_MAX_E; e++)
                        if (e < E) s_part[wave][t * (GATE_MAX_E + 1) + e] = acc[t][e];
                }
            }
        }
        __syncthreads();
        if (tid < T * (GATE_MAX_E + 1)) {
            const int t = tid / (GATE_MAX_E + 1), e = tid % (GATE_MAX_E + 1);
            if (e == GATE_MAX_E || e < E) {
                float v = 0.f;
                for (int w = 0; w < PERM_WAVES; w++) v += s_part[w][t * (GATE_MAX_E + 1) + e];
                if (e == GATE_MAX_E) s_inv[t] = 1.0f / sqrtf(v / (float)d + eps);
                else s_logits[t * GATE_MAX_E + e] = v;
            }
        }
        __syncthreads();
        // logits of the normalised rows: (x . w) * inv
        if (tid < T * GATE_MAX_E) {
            const int t = tid / GATE_MAX_E, e = tid % GATE_MAX_E;
            if (e < E) {
                const float v = s_logits[tid] * s_inv[t];
                s_logits[tid] = v;
                if (writer) logits_out[(size_t)t * E + e] = v;
            }
        }
        __syncthreads();
    } else {
        if (tid < T * GATE_MAX_E) {
            const int t = tid / GATE_MAX_E, e = tid % GATE_MAX_E;
            if (e < E) s_logits[tid] = logits_in[(size_t)t * E + e];
        }
        __syncthreads();
    }

    // ---- top-k routing: 16 lanes per token (E <= 16), same contest as route_kernel ----
    {
        const int t = tid / GATE_MAX_E, gl = tid % GATE_MAX_E;
        const bool live = (t < T);
        float v = -INFINITY;
        int e = 0x7fffffff;
        if (live && gl < E) {
            v = s_logits[t * GATE_MAX_E + gl];
            e = gl;
        }
        float my_v = 0.f, top_v = 0.f;
        int my_i = 0;
        for (int j = 0; j < k; j++) {
            float bv = v;
            int be = e;
#pragma unroll
            for (int m = 1; m < GATE_MAX_E; m <<= 1) {
                const float ov = __shfl_xor(bv, m, 64);
                const int oe = __shfl_xor(be, m, 64);
                if (ov > bv || (ov == bv && oe < be)) {
                    bv = ov;
                    be = oe;
                }
            }
            if (j == 0) top_v = bv;
            if (gl == j) {
                my_v = bv;
                my_i = be;
            }
            if (e == be) {
                v = -INFINITY;
                e = 0x7fffffff;
            }
        }
        const float u = (gl < k) ? expf(my_v - top_v) : 0.f;
        float s = u;
#pragma unroll
        for (int m = 1; m < GATE_MAX_E; m <<= 1) s += __shfl_xor(s, m, 64);
        if (live && gl < k) {
            s_idx[t * k + gl] = my_i;
            if (writer) {
                idx[(size_t)t * k + gl] = my_i;
                weights[(size_t)t * k + gl] = u / s;
            }
        }
    }
    __syncthreads();

    // ---- per-expert batching on the LDS copy of idx, then the row gather ----
    const int N = T * k;
    if (N <= 64) {
        if (wave == 0) permute_indices_wave(s_idx, N, E, counts, offsets, perm, inv_perm, writer, s_pos);
    } else {
        permute_indices(s_idx, N, E, counts, offsets, perm, inv_perm, writer, s_cnt, s_off, s_wave,
                        s_pos);
    }
    __syncthreads();
    const int row_chunks = d / 4;
    // row chunk c of token t, with the pending combine + residual applied
    auto x_chunk = [&](int t, int c) -> float4 {
        float4 r = ((const float4*)(x + (size_t)t * d))[c];
        if (COMB) {
            float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int j = 0; j < k_prev; j++) {
                const float w = s_pw[t * k_prev + j];
                const float4* src = (const float4*)(yg_prev + (size_t)s_ppos[t * k_prev + j] * d) + c;
                float4 pq[PMAX];
#pragma unroll
                for (int q = 0; q < PMAX; q++)
                    if (q < n_parts_prev) pq[q] = src[(size_t)q * (pv.pstride / 4)];
                float4 v = pq[0];
#pragma unroll
                for (int q = 1; q < PMAX; q++)
                    if (q < n_parts_prev) {
                        v.x += pq[q].x; v.y += pq[q].y; v.z += pq[q].z; v.w += pq[q].w;
                    }
                a.x += w * v.x;
                a.y += w * v.y;
                a.z += w * v.z;
                a.w += w * v.w;
            }
            r.x += a.x; r.y += a.y; r.z += a.z; r.w += a.w;
        }
        return r;
    };
    for (int p = blockIdx.x; p < N; p += gridDim.x) {
        const int t = p / k;
        float4* dst = (float4*)(xg + (size_t)s_pos[p] * d);
        const float sc = NORM ? s_inv[t] : 1.0f;
        for (int c = tid; c < row_chunks; c += PERM_THREADS) {
            float4 v = x_chunk(t, c);
            if (NORM) {
                v.x *= sc; v.y *= sc; v.z *= sc; v.w *= sc;
            }
            dst[c] = v;
        }
    }
    if (NORM && writer) {
        for (int t = 0; t < T; t++) {
            const float sc = s_inv[t];
            for (int c = tid; c < row_chunks; c += PERM_THREADS) {
                float4 v = x_chunk(t, c);
                if (COMB) ((float4*)(x_out + (size_t)t * d))[c] = v;
                v.x *= sc; v.y *= sc; v.z *= sc; v.w *= sc;
                ((float4*)(h_out + (size_t)t * d))[c] = v;
            }
        }
    }
}

int moe_gate_small_launch(bool norm, const float* x, const float* w_gate, const float* logits_in,
                          int T, int d, int E, int k, float eps, float* h_out, float* logits_out,
                          int32_t* idx, float* weights, int32_t* counts, int32_t* offsets,
                          int32_t* perm, int32_t* inv_perm, float* xg, const float* yg_prev,
                          int n_parts_prev, const int32_t* inv_perm_prev, const float* weights_prev,
                          int k_prev, float* x_out, hipStream_t s) {
    const int N = T * k;
    const unsigned grid = (unsigned)(N < 32 ? N : 32);
    const bool comb = (yg_prev != nullptr);
    if (comb && !norm) return MOE_ERR_INVALID_ARG;
    if (comb && (n_parts_prev < 1 || n_parts_prev > GATE_MAX_PARTS)) return MOE_ERR_UNSUPPORTED;
#define GATE_LAUNCH(NORM, KJMAX, PMAX)                                                            \
    hipLaunchKernelGGL((gate_small_kernel<NORM, KJMAX, PMAX>), dim3(grid), dim3(PERM_THREADS), 0, \
                       s, x,                                                                      \
                       w_gate, logits_in, T, d, E, k, eps, h_out, logits_out, idx, weights,      \
                       counts, offsets, perm, inv_perm, xg, yg_prev, n_parts_prev,               \
                       inv_perm_prev, weights_prev, k_prev, x_out)
    if (comb && k_prev <= 2 && n_parts_prev == 1) GATE_LAUNCH(true, 2, 1);
    else if (comb && k_prev <= 2) GATE_LAUNCH(true, 2, GATE_MAX_PARTS);
    else if (comb && n_parts_prev == 1) GATE_LAUNCH(true, MOE_MAX_K, 1);
    else if (comb) GATE_LAUNCH(true, MOE_MAX_K, GATE_MAX_PARTS);
    else if (norm) GATE_LAUNCH(true, 0, 1);
    else GATE_LAUNCH(false, 0, 1);
#undef GATE_LAUNCH
    return moe_launch_status();
}

// ------------------------------------------------ combine + residual add ----
__global__ __launch_bounds__(256) void combine_residual_kernel(const float4* __restrict__ yg,
                                                               const int32_t* __restrict__ inv_perm,
                                                               const float* __restrict__ weights,
                                                               int T, int k, int row_chunks,
                                                               float4* __restrict__ x) {
    const int t = blockIdx.y;
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (t >= T || c >= row_chunks) return;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int j = 0; j < k; j++) {
        const float w = weights[(size_t)t * k + j];
        const float4 v = yg[(size_t)inv_perm[(size_t)t * k + j] * row_chunks + c];
        acc.x += w * v.x;
        acc.y += w * v.y;
        acc.z += w * v.z;
        acc.w += w * v.w;
    }
    float4 r = x[(size_t)t * row_chunks + c];
    r.x += acc.x; r.y += acc.y; r.z += acc.z; r.w += acc.w;
    x[(size_t)t * row_chunks + c] = r;
}

int moe_combine_residual_launch(const float* yg, const int32_t* inv_perm, const float* weights, int T,
                                int k, int d, float* x, hipStream_t s) {
    const int row_chunks = d / 4;
    dim3 grid((unsigned)((row_chunks + 255) / 256), 1);
    for (int t0 = 0; t0 < T; t0 += 65535) {
        const int tn = (T - t0) < 65535 ? (T - t0) : 65535;
        grid.y = (unsigned)tn;
        hipLaunchKernelGGL(combine_residual_kernel, grid, dim3(256), 0, s, (const float4*)yg,
                           inv_perm + (size_t)t0 * k, weights + (size_t)t0 * k, tn, k, row_chunks,
                           (float4*)(x + (size_t)t0 * d));
    }
    return moe_launch_status();
}

// ------------------------------------- combine over unsummed reduction parts ----
// The second projection of the decode kernels leaves its reduction parts as slabs
// [P][N,d]; this combine adds them in part order while it weights and gathers:
//   v      = parts[0][pos] + parts[1][pos] + ...          (pos = inv_perm[t*k+j])
//   y[t]   = (RESID ? y[t] : 0) + sum_j w[t,j] * v
// and, when asked, stores v as yg[pos] (every row of yg belongs to exactly one slot).
template <bool RESID>
__global__ __launch_bounds__(256) void combine_parts_kernel(
    const float4* __restrict__ parts, int P, size_t stride4, const int32_t* __restrict__ inv_perm,
    const float* __restrict__ weights, int T, int k, int row_chunks, float4* __restrict__ y,
    float4* __restrict__ yg_out) {
    const int t = blockIdx.y;
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (t >= T || c >= row_chunks) return;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int j = 0; j < k; j++) {
        const float w = weights[(size_t)t * k + j];
        const size_t row = (size_t)inv_perm[(size_t)t * k + j] * row_chunks + c;
        float4 v = parts[row];
        for (int p = 1; p < P; p++) {
            const float4 u = parts[(size_t)p * stride4 + row];
            v.x += u.x; v.y += u.y; v.z += u.z; v.w += u.w;
        }
        if (yg_out) yg_out[row] = v;
        acc.x += w * v.x;
        acc.y += w * v.y;
        acc.z += w * v.z;
        acc.w += w * v.w;
    }
    if (RESID) {
        float4 r = y[(size_t)t * row_chunks + c];
        r.x += acc.x; r.y += acc.y; r.z += acc.z; r.w += acc.w;
        acc = r;
    }
    y[(size_t)t * row_chunks + c] = acc;
}

int moe_combine_parts_launch(const float* parts, int n_parts, size_t part_stride,
                             const int32_t* inv_perm, const float* weights, int T, int k, int d,
                             float* y, bool residual, float* yg_out, hipStream_t s) {
    const int row_chunks = d / 4;
    dim3 grid((unsigned)((row_chunks + 255) / 256), 1);
    for (int t0 = 0; t0 < T; t0 += 65535) {
        const int tn = (T - t0) < 65535 ? (T - t0) : 65535;
        grid.y = (unsigned)tn;
        if (residual)
            hipLaunchKernelGGL(combine_parts_kernel<true>, grid, dim3(256), 0, s, (const float4*)parts,
                               n_parts, part_stride / 4, inv_perm + (size_t)t0 * k,
                               weights + (size_t)t0 * k, tn, k, row_chunks,
                               (float4*)(y + (size_t)t0 * d), (float4*)yg_out);
        else
            hipLaunchKernelGGL(combine_parts_kernel<false>, grid, dim3(256), 0, s, (const float4*)parts,
                               n_parts, part_stride / 4, inv_perm + (size_t)t0 * k,
                               weights + (size_t)t0 * k, tn, k, row_chunks,
                               (float4*)(y + (size_t)t0 * d), (float4*)yg_out);
    }
    return moe_launch_status();
}

// ------------------------------- RMSNorm + router logits for any number of tokens ----
// NL_TOK tokens per workgroup of 1024 threads, so that a row of the router matrix is loaded
// once for NL_TOK tokens; thread-strided partial sums with grouped loads (see
// gate_partial_sums), reduced over the workgroup.  NORM: h = x / rms(x) is written and
// logits = (x . w_gate) / rms(x); else logits = x . w_gate.  E <= GATE_MAX_E.
#define NL_TOK 2
#define NL_THREADS 1024
template <bool NORM>
__global__ __launch_bounds__(NL_THREADS) void norm_logits_kernel(const float* __restrict__ x,
                                                                  const float* __restrict__ w_gate,
                                                                  int T, int d, int E, float eps,
                                                                  float* __restrict__ h,
                                                                  float* __restrict__ logits,
                                                                  float* __restrict__ sums) {
    static_assert(NL_TOK <= GATE_NORM_MAX_T, "gate_partial_sums holds GATE_NORM_MAX_T tokens");
    __shared__ float s_part[NL_THREADS / 64][NL_TOK * (GATE_MAX_E + 1)];
    __shared__ float s_inv[NL_TOK];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t0 = blockIdx.x * NL_TOK;
    const int Tl = (T - t0) < NL_TOK ? (T - t0) : NL_TOK;
    const float* xb = x + (size_t)t0 * d;
    float ss[GATE_NORM_MAX_T], acc[GATE_NORM_MAX_T][GATE_MAX_E];
#pragma unroll
    for (int t = 0; t < NL_TOK; t++) {
        ss[t] = 0.f;
#pragma unroll
        for (int e = 0; e < GATE_MAX_E; e++) acc[t][e] = 0.f;
    }
    const GatePrev none = {nullptr, nullptr, nullptr, 0, 1, 0};
    gate_partial_sums<NL_TOK, 4, 0, 1, NL_THREADS>(xb, w_gate, Tl, d, E, tid, none, ss, acc);
#pragma unroll
    for (int t = 0; t < NL_TOK; t++) {
        if (t < Tl) {
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) ss[t] += __shfl_xor(ss[t], m, 64);
#pragma unroll
            for (int e = 0; e < GATE_MAX_E; e++) {
                if (e < E) {
#pragma unroll
                    for (int m = 32; m >= 1; m >>= 1) acc[t][e] += __shfl_xor(acc[t][e], m, 64);
                }
            }
            if (lane == 0) {
                s_part[wave][t * (GATE_MAX_E + 1) + GATE_MAX_E] = ss[t];
#pragma unroll
                for (int e = 0; e < GATE_MAX_E; e++)
                    if (e < E) s_part[wave][t * (GATE_MAX_E + 1) + e] = acc[t][e];
            }
        }
    }
    __syncthreads();
    if (tid < Tl) {
        float v = 0.f;
        for (int w = 0; w < NL_THREADS / 64; w++) v += s_part[w][tid * (GATE_MAX_E + 1) + GATE_MAX_E];
        s_inv[tid] = NORM ? 1.0f / sqrtf(v / (float)d + eps) : 1.0f;
        if (NORM && sums) sums[(size_t)(t0 + tid) * (E + 1) + E] = v;  // the raw sum of squares
    }
    __syncthreads();
    if (tid < Tl * GATE_MAX_E) {
        const int t = tid / GATE_MAX_E, e = tid % GATE_MAX_E;
        if (e < E) {
            float v = 0.f;
            for (int w = 0; w < NL_THREADS / 64; w++) v += s_part[w][t * (GATE_MAX_E + 1) + e];
            if (logits) logits[(size_t)(t0 + t) * E + e] = NORM ? v * s_inv[t] : v;
            if (NORM && sums) sums[(size_t)(t0 + t) * (E + 1) + e] = v;  // the raw dot product
        }
    }
    if (NORM && h) {
        const int row_chunks = d / 4;
        for (int t = 0; t < Tl; t++) {
            const float sc = s_inv[t];
            const float4* src = (const float4*)(xb + (size_t)t * d);
            float4* dst = (float4*)(h + (size_t)(t0 + t) * d);
            for (int c = tid; c < row_chunks; c += NL_THREADS) {
                float4 v = src[c];
                v.x *= sc; v.y *= sc; v.z *= sc; v.w *= sc;
                dst[c] = v;
            }
        }
    }
}

bool moe_norm_logits_supported(int E) { return E <= GATE_MAX_E; }

// norm: h (if not null) is written too, and sums (if not null) receives the unscaled sums
// [T][E+1]: x . w_gate[:, e] at e, sum(x^2) at E; logits may then be null
int moe_norm_logits_launch(bool norm, const float* x, const float* w_gate, int T, int d, int E,
                           float eps, float* h, float* logits, float* sums, hipStream_t s) {
    const unsigned grid = (unsigned)((T + NL_TOK - 1) / NL_TOK);
    if (norm)
        hipLaunchKernelGGL(norm_logits_kernel<true>, dim3(grid), dim3(NL_THREADS), 0, s, x, w_gate, T,
                           d, E, eps, h, logits, sums);
    else
        hipLaunchKernelGGL(norm_logits_kernel<false>, dim3(grid), dim3(NL_THREADS), 0, s, x, w_gate, T,
                           d, E, eps, h, logits, sums);
    return moe_launch_status();
}
