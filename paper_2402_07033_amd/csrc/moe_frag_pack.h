// Shared by the kernels that work on activations re-laid as B-operand fragments
// (moe_ffn_grouped.hip, moe_ffn_mid.hip): the per-expert block bookkeeping and the pack
// kernel.  Device code only.
#pragma once

#include "moe_internal.h"

// ---- segment bookkeeping: expert e owns blocks [bbase_e, bbase_e + ceil(M_e/16)) ----
struct SegInfo {
    int e;        // expert
    int row0;     // first row of the expert's segment in xg / yg
    int rows;     // rows of the segment
    int bbase;    // first packed block of the segment
};

__device__ __forceinline__ int gg_clamp_off(int v, int lo, int N) {
    return v < lo ? lo : (v > N ? N : v);
}

// Locate packed block `blk` (global block index) -> its segment; false if past the end.
__device__ __forceinline__ bool gg_find_block(const int32_t* __restrict__ offsets, int E, int N,
                                              int blk, SegInfo& si) {
    int bb = 0, prev = 0;
    for (int e = 0; e < E; e++) {
        const int lo = gg_clamp_off(offsets[e], prev, N);
        const int hi = gg_clamp_off(offsets[e + 1], lo, N);
        prev = lo;
        const int nb = (hi - lo + 15) / 16;
        if (blk < bb + nb) {
            si.e = e; si.row0 = lo; si.rows = hi - lo; si.bbase = bb;
            return true;
        }
        bb += nb;
    }
    return false;
}

// ------------------------------------------------------------------- pack ----
// blockIdx.x = packed block: rows [row0 + 16*b, +16) of a segment become d/32 B-operand
// fragments; rows past the segment end are zero.  blockIdx.y splits the block's fragments
// into ranges of GG_PACK_KS reduction steps, so that a launch with few blocks (a few hundred
// rows) still fills the chip.  With `perm` the batched row i is read as xg[perm[i] / k]: xg
// is then the token array itself and the gathered copy is never materialised.
#define GG_PACK_KS 32
template <bool ACT_BF16>
__global__ __launch_bounds__(256) void gg_pack_kernel(const void* __restrict__ xg,
                                                      const int32_t* __restrict__ perm, int k,
                                                      const int32_t* __restrict__ offsets, int E,
                                                      int N, int d, u32x4_t* __restrict__ xp) {
    SegInfo si;
    if (!gg_find_block(offsets, E, N, blockIdx.x, si)) return;
    const int b = blockIdx.x - si.bbase;
    const int KS = d / 32;
    const int ks_lo = blockIdx.y * GG_PACK_KS;
    const int ks_n = (KS - ks_lo) < GG_PACK_KS ? (KS - ks_lo) : GG_PACK_KS;
    // the lane's source row is the same for every fragment of the block
    const int t = threadIdx.x & 15;
    const int r = b * 16 + t;
    int src = si.row0 + r;
    if (perm && r < si.rows) src = perm[si.row0 + r] / k;
    for (int i = threadIdx.x; i < ks_n * 64; i += 256) {
        const int lane = i & 63, ks = ks_lo + (i >> 6);
        const int kq = lane >> 4;
        u32x4_t v = {0u, 0u, 0u, 0u};
        if (r < si.rows) {
            const size_t off = (size_t)src * d + (size_t)ks * 32 + kq * 8;
            if (ACT_BF16) {
                v = *(const u32x4_t*)((const uint16_t*)xg + off);
            } else {
                const float4 v0 = *(const float4*)((const float*)xg + off);
                const float4 v1 = *(const float4*)((const float*)xg + off + 4);
                v[0] = moe_pack_bf16x2(v0.x, v0.y);
                v[1] = moe_pack_bf16x2(v0.z, v0.w);
                v[2] = moe_pack_bf16x2(v1.x, v1.y);
                v[3] = moe_pack_bf16x2(v1.z, v1.w);
            }
        }
        xp[((size_t)blockIdx.x * KS + ks) * 64 + lane] = v;
    }
}

// grid of gg_pack_kernel for `nb` packed blocks of d columns
static inline dim3 gg_pack_grid(size_t nb, int d) {
    return dim3((unsigned)nb, (unsigned)((d / 32 + GG_PACK_KS - 1) / GG_PACK_KS));
}
