// Gating and per-expert batching of a decode-sized step by ONE wavefront, without workgroup
// barriers: used where every wave (or every workgroup) of a kernel needs the routing state
// for itself -- the fused front ends in moe_route_permute.hip and the first-projection
// decode kernel that routes in its own prologue (moe_ffn_stream.hip).  Device code only.
#pragma once

#include "moe_internal.h"

#define GATE_WAVE_MAX_E 16   // experts: 16 lanes hold one token's logits
#define GATE_WAVE_MAX_N 64   // slots (tokens x k): one lane per slot

// Top-k contest of the gating function (Sec. 2.1) for the token whose logits sit in a group
// of 16 lanes (lane gl holds expert gl's logit, or -inf / INT_MAX beyond E): k rounds of a
// butterfly arg-max, larger value first, lower expert index among equals.  On return lane
// gl < k of the group holds the gl-th winner (my_i, my_v); top_v is the first winner's logit.
__device__ __forceinline__ void gate_topk16(float v, int e, int gl, int k, float& my_v, int& my_i,
                                            float& top_v) {
    my_v = 0.f;
    top_v = 0.f;
    my_i = 0;
    for (int j = 0; j < k; j++) {
        float bv = v;
        int be = e;
#pragma unroll
        for (int m = 1; m < GATE_WAVE_MAX_E; m <<= 1) {
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
        if (e == be) {  // the winner leaves the contest
            v = -INFINITY;
            e = 0x7fffffff;
        }
    }
}

// One wavefront routes T <= 16 tokens over E <= 16 experts, four tokens per round.  s_idx
// (LDS, [T*k]) receives the expert ids; with `write` the lanes also store idx / weights to
// global memory.  The arithmetic is that of route_kernel: fp32 softmax over the k winners.
__device__ __forceinline__ void gate_route_wave(const float* __restrict__ logits, int T, int E,
                                                int k, int lane, int* s_idx, bool write,
                                                int32_t* __restrict__ idx,
                                                float* __restrict__ weights) {
    const int gl = lane & 15;
    for (int t0 = 0; t0 < T; t0 += 4) {
        const int t = t0 + (lane >> 4);
        const bool live = (t < T);
        float v = -INFINITY;
        int e = 0x7fffffff;
        if (live && gl < E) {
            v = logits[(size_t)t * E + gl];
            e = gl;
        }
        float my_v, top_v;
        int my_i;
        gate_topk16(v, e, gl, k, my_v, my_i, top_v);
        const float u = (gl < k) ? expf(my_v - top_v) : 0.f;
        float s = u;
#pragma unroll
        for (int m = 1; m < GATE_WAVE_MAX_E; m <<= 1) s += __shfl_xor(s, m, 64);
        if (live && gl < k) {
            s_idx[t * k + gl] = my_i;
            if (write) {
                idx[(size_t)t * k + gl] = my_i;
                weights[(size_t)t * k + gl] = u / s;
            }
        }
    }
}

// Per-expert batching (Algorithm 1's inp_size) of N <= 64 slots by one wavefront: lane p
// owns slot p; a ballot per expert gives the expert's count and every lane's rank among the
// lanes of its expert, so the order inside a segment is the slot order.  s_pos[p] receives
// the slot's sorted position.  Returns, in lane e <= E, offsets[e] (lane E: the total).
__device__ __forceinline__ int permute_indices_wave(const int* __restrict__ s_idx, int N, int E,
                                                    int32_t* __restrict__ counts,
                                                    int32_t* __restrict__ offsets,
                                                    int32_t* __restrict__ perm,
                                                    int32_t* __restrict__ inv_perm, bool write,
                                                    int* s_pos) {
    const int lane = threadIdx.x & 63;
    int e = -1;
    if (lane < N) {
        e = s_idx[lane];
        e = e < 0 ? 0 : (e >= E ? E - 1 : e);
    }
    const unsigned long long below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    int run = 0, pos = 0, my_cnt = 0, my_off = 0;
    for (int ee = 0; ee < E; ee++) {
        const unsigned long long m = __ballot(e == ee);
        const int c = __popcll(m);
        if (e == ee) pos = run + __popcll(m & below);
        if (lane == ee) {
            my_cnt = c;
            my_off = run;
        }
        run += c;
    }
    if (lane == E) my_off = run;
    if (lane < N) {
        s_pos[lane] = pos;
        if (write) {
            perm[pos] = lane;
            inv_perm[lane] = pos;
        }
    }
    if (write) {
        if (lane < E) counts[lane] = my_cnt;
        if (lane <= E) offsets[lane] = my_off;
    }
    return my_off;
}
