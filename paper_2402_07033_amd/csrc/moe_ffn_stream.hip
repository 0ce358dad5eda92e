// Decode-sized expert FFN for gfx950: weight-streaming kernels on the bf16
// matrix cores.
//
// With a handful of rows per expert the layer is bound by the time to read
// each active expert's matrices once (the paper's observation that GPU expert
// latency is set by parameter loading, Sec. 3.1 / Appendix A).  The kernels
// therefore stream every fragment of an active expert exactly once, with
// 16-byte-per-lane fully coalesced loads kept 16 deep per wavefront, and do the
// arithmetic with v_mfma_f32_16x16x32_bf16: the weight fragment is the A
// operand (16 output features x 32 reduction indices), up to 16 token rows of
// the expert form the B operand, fp32 accumulate.  fp32 activations are split
// into bf16 high and low parts and multiplied separately, which keeps them to
// ~2^-16 relative; the matrix cores are otherwise idle here.
//
// Work decomposition (both projections): a unit is (row tile of <=16 rows of
// one expert, reduction part, block of 16 output features).  The W waves of a
// workgroup split the unit's reduction range; their partial 16x16 tiles meet
// in LDS.  Each wave keeps its slice of the activations in registers across
// all consecutive units of the same (tile, part), so activations are read once
// per workgroup, and the units are dealt to the workgroups in contiguous,
// equal ranges so that every workgroup streams the same number of bytes.
//   up   (x.w1, x.w3 -> silu*mul -> h): one part (the nonlinearity needs the
//        full sum), 8 waves x d/256 reduction steps.
//   down (h.w2 -> yg): the long reduction over f is cut into P parts; every part stores
//        its partial sums into its own slab [part][N][d] and a small kernel (or the
//        consumer: the gate-weighted combine) adds the slabs in part order, so the result
//        does not depend on the order in which workgroups finish.
//   down, one to four routed rows (stream_down_small_kernel): the rows of h fit in LDS, one
//        workgroup per block of 16 output features takes the block's whole reduction, and the
//        gate-weighted combine happens in its epilogue: no slabs, nothing left to add.
// The first-projection kernel can also run the gating function and the per-expert batching
// of a decode step (T <= 16 tokens, at most 64 slots) in its own prologue, every wave for
// itself, and then reads the activations straight from the token rows: one launch less and
// no gathered copy (moe_decode_layer).  For a stack of transformer blocks (moe_decode_block)
// it further derives the block's RMSNorm scale and router logits from shares of the gating
// sums that the small-row kernel of the block before left behind, together with the
// residual add: two launches per block and none between blocks.
#include <atomic>

#include "moe_internal.h"
#include "moe_gate_wave.h"

#define ST_MAX_TILES 128
#define ST_MAX_WAVES 8

struct StreamArgs {
    const u32x4_t* wfrag;  // fragment-ordered weights
    const void* act;       // [N,K] fp32 or bf16
    const int32_t* row_perm;  // or null; else row i of the activations is act[row_perm[i] / row_k]
    int row_k;
    const int32_t* offsets;
    float* out;       // up: h [N,C]; down: yg [N,C] (P == 1) or the slabs [P][N][C]
    size_t part_stride;  // floats between two slabs of `out` (0 when P == 1)
    int E, N, K, C;
    int NB;  // C / 16
    int KS;  // K / 32
    int P;   // reduction parts per unit row
    int W;   // waves per workgroup
    // gating in the prologue (GATE instantiations only): act = x [T,K], offsets unused
    const float* logits;  // [T,E]
    int T, k;
    int32_t* idx;         // [T,k]   written by workgroup 0
    float* weights;       // [T,k]
    int32_t* counts;      // [E]
    int32_t* offsets_out; // [E+1]
    int32_t* perm;        // [T*k]
    int32_t* inv_perm;    // [T*k]
    float* xg;            // [T*k,K] gathered rows, or null (the kernel itself does not need them)
    // or, instead of logits: the shares of the RMSNorm and router sums of the token rows,
    // [n_shares][gate_stride] with (t, e) at t*(E+1)+e = sum_c x[t,c]*w_gate[c,e] and
    // (t, E) = sum_c x[t,c]^2 over the share's features.  Every wave adds the shares in
    // order, derives 1/rms and the logits, and reads the rows scaled by 1/rms.
    const float* gate_sums;
    int n_shares, gate_stride;
    float eps;
    float* logits_out;    // [T,E] or null: the logits derived from the shares (workgroup 0)
};

#define GS_MAX_ITEMS 32                    // T * (E + 1) of the shares, at most
#define GS_WAVE_ROWS 32                    // shares one wave adds

// Adds the shares [row0, row1) (at most GS_WAVE_ROWS) for one wave with few instructions (the
// first weight request of the kernel waits for this): lane r copies row r into LDS, then lane
// `it` adds column `it` in row order.  s_rows: GS_WAVE_ROWS x GS_MAX_ITEMS floats of this
// wave; s_out[it] receives the totals.
__device__ __forceinline__ void gate_add_shares(const float* __restrict__ sums, int row0, int row1,
                                                int stride, int items, int lane, float* s_rows,
                                                float* s_out) {
    const int nrows = row1 - row0;
    if (lane < nrows) {
        // a share is a whole 128-byte line: all of it is copied, whatever `items`
        const float4* src = (const float4*)(sums + (size_t)(row0 + lane) * stride);
        float4* dst = (float4*)(s_rows + lane * GS_MAX_ITEMS);
        const float4 v0 = src[0], v1 = src[1], v2 = src[2], v3 = src[3], v4 = src[4], v5 = src[5],
                     v6 = src[6], v7 = src[7];
        dst[0] = v0; dst[1] = v1; dst[2] = v2; dst[3] = v3;
        dst[4] = v4; dst[5] = v5; dst[6] = v6; dst[7] = v7;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (lane < items) {
        float v = 0.f;
        for (int r = 0; r < nrows; r++) v += s_rows[r * GS_MAX_ITEMS + lane];
        s_out[lane] = v;
    }
}

// rowmap (LDS, or null): source row of sorted row i -- the kernels that route in their own
// prologue read the token rows directly.
template <int KSW, bool ACT_BF16>
__device__ __forceinline__ void stream_load_act(bf16x8_t (&act)[KSW][ACT_BF16 ? 1 : 2],
                                                const void* actp, int K, int row0, int rows,
                                                int ks0, int lane, const int* rowmap,
                                                const int32_t* perm, int perm_k,
                                                const float* row_scale) {
#pragma clang fp contract(off)
    const int t = lane & 15, kq = lane >> 4;
    int src_row = row0 + t;
    if (rowmap && t < rows) src_row = rowmap[row0 + t];
    if (perm && t < rows) src_row = perm[row0 + t] / perm_k;
    float sc = 1.0f;
    if (!ACT_BF16 && row_scale && t < rows) sc = row_scale[src_row];
#pragma unroll
    for (int s = 0; s < KSW; s++) {
        const size_t off = (size_t)src_row * K + (size_t)(ks0 + s) * 32 + kq * 8;
        if (ACT_BF16) {
            u32x4_t v = {0u, 0u, 0u, 0u};
            if (t < rows) v = *(const u32x4_t*)((const uint16_t*)actp + off);
            act[s][0] = __builtin_bit_cast(bf16x8_t, v);
        } else {
            float x[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            if (t < rows) {
                const float4 v0 = *(const float4*)((const float*)actp + off);
                const float4 v1 = *(const float4*)((const float*)actp + off + 4);
                x[0] = v0.x; x[1] = v0.y; x[2] = v0.z; x[3] = v0.w;
                x[4] = v1.x; x[5] = v1.y; x[6] = v1.z; x[7] = v1.w;
            }
            // the scale is applied here, outside the branch of the loads and without a branch
            // of its own: a use of the loaded values inside it would make every step wait for
            // its own loads before the next step's are issued (sc is 1 without a scale: exact).
            // The product is rounded to fp32 before the split below uses it, as if the scaled
            // row had been stored (hence no contraction in this function).
#pragma unroll
            for (int j = 0; j < 8; j++) x[j] *= sc;
            unsigned hi[8], lo[8];
#pragma unroll
            for (int j = 0; j < 8; j++) {
                hi[j] = moe_bf16_rne(x[j]);
                lo[j] = moe_bf16_rne(x[j] - moe_bf16_to_f32(hi[j]));
            }
            u32x4_t vh = {hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16), hi[4] | (hi[5] << 16),
                          hi[6] | (hi[7] << 16)};
            u32x4_t vl = {lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16), lo[4] | (lo[5] << 16),
                          lo[6] | (lo[7] << 16)};
            act[s][0] = __builtin_bit_cast(bf16x8_t, vh);
            act[s][ACT_BF16 ? 0 : 1] = __builtin_bit_cast(bf16x8_t, vl);
        }
    }
}

// Row tiles of the routed rows, built by every wave for itself: lane e takes expert e's
// row range, a wave scan numbers the tiles, and the lane writes its experts' tiles into the
// wave's own copy of the list in LDS.  No workgroup barrier and no serial walk: the list is
// ready one global-load latency after the kernel starts.  Returns the number of tiles.
// lo, hi: lane e's row range [offsets[e], offsets[e+1]) (anything for lanes >= E).
template <int TR, int MAXT>
__device__ __forceinline__ int stream_tile_list(int lo, int hi, int E, int N, int lane, int* te,
                                                int* tr0, int* trn) {
    if (lane >= E) lo = hi = 0;
    lo = lo < 0 ? 0 : (lo > N ? N : lo);
    hi = hi < lo ? lo : (hi > N ? N : hi);
    const int nt = (hi - lo + TR - 1) / TR;
    int incl = nt;
#pragma unroll
    for (int dlt = 1; dlt < 64; dlt <<= 1) {
        const int v = __shfl_up(incl, dlt, 64);
        if (lane >= dlt) incl += v;
    }
    const int first = incl - nt;
    for (int i = 0; i < nt; i++) {
        const int ti = first + i;
        if (ti < MAXT) {
            const int r = lo + i * TR;
            te[ti] = lane;
            tr0[ti] = r;
            trn[ti] = (hi - r) < TR ? (hi - r) : TR;
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    const int total = __shfl(incl, 63, 64);
    return __builtin_amdgcn_readfirstlane(total < MAXT ? total : MAXT);
}

constexpr int stream_ring_depth(int nl) {
    int r = nl < 16 ? nl : 16;
    while (nl % r) --r;
    return r;
}

template <int KSW, int NMAT, bool ACT_BF16, bool GATE>
__global__ __launch_bounds__(512) void stream_kernel(StreamArgs a) {
    static_assert(!GATE || (NMAT == 2 && !ACT_BF16), "gating runs in the first projection on fp32 rows");
    constexpr int TERMS = ACT_BF16 ? 1 : 2;
    constexpr int NL = KSW * NMAT;         // fragment loads per unit per wave
    // Loads kept in flight per wave: the largest divisor of NL up to 16.  Load j of a unit
    // sits in ring slot j % R, and the next unit's load j is requested into the slot of this
    // unit's load j + NL - R; the two agree only when R divides NL.
    constexpr int R = stream_ring_depth(NL);
    static_assert(R >= 1 && R <= 16 && NL % R == 0, "the ring depth must divide the loads per unit");
    __shared__ int s_tiles[ST_MAX_WAVES][3][ST_MAX_TILES];  // per wave: expert, first row, rows
    __shared__ f32x4_t s_red[2][ST_MAX_WAVES][NMAT][64];
    static_assert(!GATE || sizeof(f32x4_t) * 2 * NMAT * 64 >= sizeof(float) * GS_WAVE_ROWS * GS_MAX_ITEMS,
                  "an eighth of s_red holds a wave's rows of the shares");
    // per wave (GATE): expert id of every slot, its sorted position, source token of every
    // sorted row
    __shared__ int s_gate[GATE ? ST_MAX_WAVES : 1][3][GATE_WAVE_MAX_N];
    // per wave (GATE, shares given): the summed shares, 1/rms per token, the logits
    __shared__ float s_gsum[GATE ? ST_MAX_WAVES : 1][3][64];
    __shared__ float s_gpart[GATE ? ST_MAX_WAVES : 1][GS_MAX_ITEMS];  // the waves' parts of the shares

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    int* s_te = s_tiles[wave][0];
    int* s_tr0 = s_tiles[wave][1];
    int* s_trn = s_tiles[wave][2];
    int lo = 0, hi = 0;
    const int* rowmap = nullptr;
    const float* row_scale = nullptr;  // [T] in LDS: token row t is multiplied by it first
    if (GATE) {
        // gating function and per-expert batching (Sec. 3.3 "Execution"; Algorithm 1's
        // inp_size), every wave for itself: no workgroup barrier before the first weight
        // request.  Wave 0 of workgroup 0 writes the index outputs.
        int* s_idx = s_gate[wave][0];
        int* s_pos = s_gate[wave][1];
        int* s_src = s_gate[wave][2];
        const bool writer = (blockIdx.x == 0 && wave == 0);
        const float* lg = a.logits;
        if (a.gate_sums) {
            float* s_sum = s_gsum[wave][0];
            float* s_inv = s_gsum[wave][1];
            float* s_lg = s_gsum[wave][2];
            // every wave adds its part of the shares (each share is then loaded once per
            // workgroup), the waves' parts are added in wave order by every wave for itself
            const int items = a.T * (a.E + 1);
            const int per_w = (a.n_shares + a.W - 1) / a.W;
            const int row0 = wave * per_w;
            const int row1 = (row0 + per_w) < a.n_shares ? (row0 + per_w) : a.n_shares;
            // (the reduction buffer is idle until the first unit is finished)
            gate_add_shares(a.gate_sums, row0, row1, a.gate_stride, items, lane,
                            (float*)s_red + wave * (GS_WAVE_ROWS * GS_MAX_ITEMS), s_gpart[wave]);
            __syncthreads();
            if (lane < items) {
                float v = s_gpart[0][lane];
                for (int w = 1; w < a.W; w++) v += s_gpart[w][lane];
                s_sum[lane] = v;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            if (lane < a.T) s_inv[lane] = 1.0f / sqrtf(s_sum[lane * (a.E + 1) + a.E] / (float)a.K + a.eps);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            if (lane < a.T * a.E) {
                const int tok = lane / a.E, ex = lane % a.E;
                const float v = s_sum[tok * (a.E + 1) + ex] * s_inv[tok];
                s_lg[lane] = v;
                if (writer && a.logits_out) a.logits_out[lane] = v;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            lg = s_lg;
            row_scale = s_inv;
        }
        gate_route_wave(lg, a.T, a.E, a.k, lane, s_idx, writer, a.idx, a.weights);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const int off = permute_indices_wave(s_idx, a.N, a.E, a.counts, a.offsets_out, a.perm,
                                             a.inv_perm, writer, s_pos);
        if (lane < a.N) s_src[s_pos[lane]] = lane / a.k;
        lo = off;
        hi = __shfl_down(off, 1, 64);
        rowmap = s_src;
    } else if (lane < a.E) {
        lo = a.offsets[lane];
        hi = a.offsets[lane + 1];
    }
    // The gathered rows, when the caller wants them, are written last: stores pending next
    // to loads would turn the waits for the first loads into waits for everything.
    auto write_xg = [&]() {
        if (GATE && a.xg) {
            const int chunks = a.K / 4;
            for (int i = blockIdx.x; i < a.N; i += gridDim.x) {
                const float4* src = (const float4*)((const float*)a.act + (size_t)rowmap[i] * a.K);
                float4* dst = (float4*)(a.xg + (size_t)i * a.K);
                for (int c = tid; c < chunks; c += blockDim.x) dst[c] = src[c];
            }
        }
    };
    const int n_tiles = stream_tile_list<16, ST_MAX_TILES>(lo, hi, a.E, a.N, lane, s_te, s_tr0, s_trn);
    // units of this workgroup: an equal share of tiles x parts x column blocks (the product
    // stays below 2^31, host check)
    const unsigned total = (unsigned)n_tiles * (unsigned)a.P * (unsigned)a.NB;
    const unsigned per = total / gridDim.x, rem = total % gridDim.x;
    const unsigned u_begin = per * blockIdx.x + rem * blockIdx.x / gridDim.x;
    const unsigned u_end = per * (blockIdx.x + 1) + rem * (blockIdx.x + 1) / gridDim.x;
    if (u_begin >= u_end) {  // uniform over the workgroup
        write_xg();
        return;
    }

    const int wave_ks = wave * KSW;  // this wave's first reduction step inside a part
    const int part_ks = a.W * KSW;   // reduction steps per part
    // fragment index of load 0 of unit u for this wave
    auto frag_base = [&](unsigned u, int& tile, int& part, int& nb) -> size_t {
        nb = (int)(u % (unsigned)a.NB);
        const unsigned tp = u / (unsigned)a.NB;
        part = (int)(tp % (unsigned)a.P);
        tile = (int)(tp / (unsigned)a.P);
        const int e = s_te[tile];
        return (((size_t)e * a.NB + nb) * NMAT) * a.KS + (size_t)part * part_ks + wave_ks;
    };
    auto ld = [&](size_t fb, int i) -> u32x4_t {
        const int mat = i / KSW, s = i % KSW;
        return __builtin_nontemporal_load(a.wfrag + ((fb + (size_t)mat * a.KS + s) * 64 + lane));
    };

    int tile, part, nb;
    size_t fb = frag_base(u_begin, tile, part, nb);
    u32x4_t buf[R];
#pragma unroll
    for (int i = 0; i < R; i++) buf[i] = ld(fb, i);

    bf16x8_t act[KSW][TERMS];
    int cur_tile = -1, cur_part = -1;
    int it = 0;
    for (unsigned u = u_begin; u < u_end; ++u, ++it) {
        const int row0 = s_tr0[tile], rows = s_trn[tile];
        if (tile != cur_tile || part != cur_part) {
            stream_load_act<KSW, ACT_BF16>(act, a.act, a.K, row0, rows, part * part_ks + wave_ks,
                                           lane, rowmap, a.row_perm, a.row_k, row_scale);
            cur_tile = tile;
            cur_part = part;
        }
        const bool has_next = (u + 1 < u_end);
        int ntile = tile, npart = part, nnb = nb;
        size_t fb_next = fb;
        if (has_next) fb_next = frag_base(u + 1, ntile, npart, nnb);

        f32x4_t acc[NMAT][TERMS];
#pragma unroll
        for (int m = 0; m < NMAT; m++)
#pragma unroll
            for (int t = 0; t < TERMS; t++) acc[m][t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < NL; i++) {
            const int mat = i / KSW, s = i % KSW;
            const bf16x8_t wf = __builtin_bit_cast(bf16x8_t, buf[i % R]);
#pragma unroll
            for (int t = 0; t < TERMS; t++)
                acc[mat][t] =
                    __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, act[s][t], acc[mat][t], 0, 0, 0);
            const int j = i + R;
            if (j < NL) {
                buf[i % R] = ld(fb, j);
            } else if (has_next) {
                buf[i % R] = ld(fb_next, j - NL);
            }
        }
#pragma unroll
        for (int m = 0; m < NMAT; m++) {
            f32x4_t v = acc[m][0];
            if (TERMS == 2) v += acc[m][TERMS - 1];
            s_red[it & 1][wave][m][lane] = v;
        }
        __syncthreads();
        if (wave == it % a.W) {  // the waves take turns at the epilogue
            f32x4_t sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
            for (int w = 0; w < a.W; w++) {
                sa += s_red[it & 1][w][0][lane];
                if (NMAT == 2) sb += s_red[it & 1][w][NMAT - 1][lane];
            }
            const int t = lane & 15;
            if (t < rows) {
                float* dst = a.out + (size_t)part * a.part_stride + (size_t)(row0 + t) * a.C +
                             nb * 16 + 4 * (lane >> 4);
                if (NMAT == 2) {
                    float4 h;
                    h.x = sa[0] / (1.0f + __expf(-sa[0])) * sb[0];
                    h.y = sa[1] / (1.0f + __expf(-sa[1])) * sb[1];
                    h.z = sa[2] / (1.0f + __expf(-sa[2])) * sb[2];
                    h.w = sa[3] / (1.0f + __expf(-sa[3])) * sb[3];
                    *(float4*)dst = h;
                } else {
                    *(float4*)dst = make_float4(sa[0], sa[1], sa[2], sa[3]);
                }
            }
        }
        fb = fb_next;
        tile = ntile;
        part = npart;
        nb = nnb;
    }
    write_xg();
}

// yg = slab 0 + slab 1 + ... in that order (the second projection's reduction parts).
__global__ __launch_bounds__(256) void stream_reduce_kernel(const float4* __restrict__ part,
                                                            size_t n4, int P,
                                                            float4* __restrict__ yg) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (size_t)gridDim.x * 256) {
        float4 s = part[i];
        for (int p = 1; p < P; p++) {
            const float4 v = part[(size_t)p * n4 + i];
            s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
        }
        yg[i] = s;
    }
}

// ---------------------------------------------------------------------------------------
// Second projection for one to four routed rows (one or two tokens' worth: the single-batch
// decode step of Sec. 4.1, scenario (a)): one workgroup per block of 16 output features
// streams that block's whole reduction for every row, so the sum over f is finished inside
// the workgroup -- no slabs, no second pass -- and the gate-weighted combine of the rows
// (Sec. 3.2: the layer's output is the gate-weighted sum of the selected experts' outputs)
// is done on the spot.  The rows of h, split into bf16 high and low halves, sit in LDS; a
// wave owns one row and a contiguous share of its reduction steps and keeps 16 fragment
// loads in flight.  The sums are added in a fixed order: the result is deterministic.
#define SM_MAX_ROWS 4
#define SM_WAVES 8
#ifndef SM_RING
#define SM_RING 16
#endif
#define SM_STAGE_ITERS 8   // h groups (of 8 floats) per thread, at most

struct SmallDownArgs {
    const u32x4_t* wfrag;     // w2 fragments [E][NB][KS]
    const float* h;           // [N,K] fp32
    const int32_t* offsets;   // [E+1]
    const int32_t* inv_perm;  // [T*k], or null: no combine
    const float* weights;     // [T,k]
    float* y;                 // [T,C] out (with inv_perm)
    float* yg;                // [N,C] out, or null
    int E, N, K, C, NB, KS, T, k;
    // BLOCK instantiation: y = x_in + combine (the block's residual add), and, with
    // w_gate_next, this workgroup's share of the next block's RMSNorm and router sums
    const float* x_in;         // [T,C]
    const float* w_gate_next;  // [C,E] fp32 or null
    float* sums_next;          // [NB][gate_stride] out: see StreamArgs::gate_sums
    int gate_stride;
};

#define SM_MAX_E 16                      // experts the BLOCK epilogue handles
#define SM_ITEMS_MAX GS_MAX_ITEMS        // (token, expert or sum of squares) pairs
#define SM_EXTRA_FLOATS (16 * SM_MAX_E + 4 * SM_ITEMS_MAX)

// BLOCK: the transformer block's residual add and the next block's gating inputs in this
// kernel's epilogue.  Every workgroup owns 16 features of the output rows: it adds the
// residual and writes its 16 features' share of sum(y^2) and of y . w_gate_next; the next
// block's first kernel adds the shares in workgroup order (deterministic).  No workgroup
// waits for another and nothing is counted.
template <bool BLOCK>
__global__ __launch_bounds__(64 * SM_WAVES) void stream_down_small_kernel(SmallDownArgs a) {
    extern __shared__ __align__(16) unsigned char sm_raw[];
    // [N*KS*4] groups of {hi 16 B, lo 16 B}, then 32 B of zeros, then the waves' partial tiles
    u32x4_t* s_h = (u32x4_t*)sm_raw;
    const int n_groups = a.N * a.KS * 4;
    u32x4_t* s_zero = s_h + 2 * (size_t)n_groups;
    f32x4_t* s_red = (f32x4_t*)(s_zero + 2);
    // BLOCK: this workgroup's 16 rows of w_gate_next, the four lanes' shares, the totals
    float* s_wg = (float*)(s_red + SM_WAVES * 64);
    float* s_fin = s_wg + 16 * SM_MAX_E;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nb = blockIdx.x;
    const bool gate_next = BLOCK && a.w_gate_next != nullptr;

    // h first (its loads are the oldest, so the wait for them does not include the weights)
    float4 hv[SM_STAGE_ITERS][2];
#pragma unroll
    for (int i = 0; i < SM_STAGE_ITERS; i++) {
        const int g = tid + i * 64 * SM_WAVES;
        if (g < n_groups) {
            hv[i][0] = *(const float4*)(a.h + (size_t)g * 8);
            hv[i][1] = *(const float4*)(a.h + (size_t)g * 8 + 4);
        }
    }
    float wgv = 0.f;
    if (gate_next && tid < 16 * a.E) wgv = a.w_gate_next[(size_t)nb * 16 * a.E + tid];

    // this wave's row and share of its reduction steps
    const int wpr = SM_WAVES / a.N;  // waves per row
    const int r = wave / wpr, sub = wave % wpr;
    const int chunk = (a.KS + wpr - 1) / wpr;
    int ks0 = sub * chunk, S = 0;
    int e = 0;
    if (r < a.N) {
        const int ks1 = (ks0 + chunk) < a.KS ? (ks0 + chunk) : a.KS;
        S = ks1 > ks0 ? ks1 - ks0 : 0;
        int lo = 0, hi = 0;
        if (lane < a.E) {
            lo = a.offsets[lane];
            hi = a.offsets[lane + 1];
        }
        const unsigned long long m = __ballot(lane < a.E && lo <= r && r < hi);
        if (m == 0ull) S = 0;  // offsets that do not cover the row: nothing is read
        e = __builtin_amdgcn_readfirstlane(m ? (int)__builtin_ctzll(m) : 0);
    }
    S = __builtin_amdgcn_readfirstlane(S);
    const u32x4_t* wsrc = a.wfrag + (((size_t)e * a.NB + nb) * a.KS + ks0) * 64 + lane;
    u32x4_t buf[SM_RING];
    if (S > 0) {
#pragma unroll
        for (int i = 0; i < SM_RING; i++) {
            const int st = i < S ? i : S - 1;
            buf[i] = __builtin_nontemporal_load(wsrc + (size_t)st * 64);
        }
    }

    // stage h: bf16 high and low halves, in the matrix cores' operand order
#pragma unroll
    for (int i = 0; i < SM_STAGE_ITERS; i++) {
        const int g = tid + i * 64 * SM_WAVES;
        if (g < n_groups) {
            const float x[8] = {hv[i][0].x, hv[i][0].y, hv[i][0].z, hv[i][0].w,
                                hv[i][1].x, hv[i][1].y, hv[i][1].z, hv[i][1].w};
            unsigned hi[8], lo[8];
#pragma unroll
            for (int j = 0; j < 8; j++) {
                hi[j] = moe_bf16_rne(x[j]);
                lo[j] = moe_bf16_rne(x[j] - moe_bf16_to_f32(hi[j]));
            }
            s_h[2 * g] = u32x4_t{hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16), hi[4] | (hi[5] << 16),
                                 hi[6] | (hi[7] << 16)};
            s_h[2 * g + 1] = u32x4_t{lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16),
                                     lo[4] | (lo[5] << 16), lo[6] | (lo[7] << 16)};
        }
    }
    if (tid < 2) s_zero[tid] = u32x4_t{0u, 0u, 0u, 0u};
    if (gate_next && tid < 16 * a.E) s_wg[tid] = wgv;
    __syncthreads();

    // B operand: column 0 carries the row, the other 15 columns are zero
    const int t = lane & 15, kq = lane >> 4;
    const u32x4_t* bsrc = (t == 0) ? s_h + 2 * (((size_t)r * a.KS + ks0) * 4 + kq) : s_zero;
    const int bstep = (t == 0) ? 8 : 0;  // u32x4 per reduction step
    f32x4_t acc_hi = {0.f, 0.f, 0.f, 0.f}, acc_lo = {0.f, 0.f, 0.f, 0.f};
    for (int base = 0; base < S; base += SM_RING) {
#pragma unroll
        for (int i = 0; i < SM_RING; i++) {
            const int st = base + i;
            if (st < S) {
                const bf16x8_t wf = __builtin_bit_cast(bf16x8_t, buf[i]);
                const bf16x8_t bh = __builtin_bit_cast(bf16x8_t, bsrc[(size_t)st * bstep]);
                const bf16x8_t bl = __builtin_bit_cast(bf16x8_t, bsrc[(size_t)st * bstep + 1]);
                acc_hi = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, bh, acc_hi, 0, 0, 0);
                acc_lo = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, bl, acc_lo, 0, 0, 0);
                if (st + SM_RING < S)
                    buf[i] = __builtin_nontemporal_load(wsrc + (size_t)(st + SM_RING) * 64);
            }
        }
    }
    s_red[wave * 64 + lane] = acc_hi + acc_lo;
    __syncthreads();

    // lanes 0, 16, 32, 48 of wave 0 hold features 4*kq .. 4*kq+3 of column 0
    const int items = a.T * (a.E + 1);  // BLOCK: (token, expert) sums and (token, sum of squares)
    if (wave == 0) {
        if (t == 0) {
            auto row_sum = [&](int row) -> float4 {
                f32x4_t v = s_red[(row * wpr) * 64 + lane];
                for (int w = 1; w < wpr; w++) v += s_red[(row * wpr + w) * 64 + lane];
                return make_float4(v[0], v[1], v[2], v[3]);
            };
            const size_t col = (size_t)nb * 16 + 4 * kq;
            if (a.yg)
                for (int row = 0; row < a.N; row++)
                    *(float4*)(a.yg + (size_t)row * a.C + col) = row_sum(row);
            if (a.inv_perm) {
                for (int tok = 0; tok < a.T; tok++) {
                    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
                    for (int j = 0; j < a.k; j++) {
                        const float w = a.weights[tok * a.k + j];
                        int row = a.inv_perm[tok * a.k + j];
                        row = row < 0 ? 0 : (row >= a.N ? a.N - 1 : row);
                        const float4 v = row_sum(row);
                        acc.x += w * v.x;
                        acc.y += w * v.y;
                        acc.z += w * v.z;
                        acc.w += w * v.w;
                    }
                    if (BLOCK) {
                        float4 xr = *(const float4*)(a.x_in + (size_t)tok * a.C + col);
                        xr.x += acc.x; xr.y += acc.y; xr.z += acc.z; xr.w += acc.w;
                        acc = xr;
                    }
                    *(float4*)(a.y + (size_t)tok * a.C + col) = acc;
                    if (gate_next) {
                        // this lane's four features' share of the token's sums
                        const float xv[4] = {acc.x, acc.y, acc.z, acc.w};
                        float* fin = s_fin + kq * SM_ITEMS_MAX + tok * (a.E + 1);
                        float ss = 0.f;
#pragma unroll
                        for (int i = 0; i < 4; i++) ss = fmaf(xv[i], xv[i], ss);
                        fin[a.E] = ss;
                        for (int ex = 0; ex < a.E; ex++) {
                            float d = 0.f;
#pragma unroll
                            for (int i = 0; i < 4; i++) d = fmaf(xv[i], s_wg[(4 * kq + i) * a.E + ex], d);
                            fin[ex] = d;
                        }
                    }
                }
            }
        }
        if (gate_next) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            for (int it = lane; it < items; it += 64) {
                float v = s_fin[it];
#pragma unroll
                for (int q = 1; q < 4; q++) v += s_fin[q * SM_ITEMS_MAX + it];
                a.sums_next[(size_t)nb * a.gate_stride + it] = v;
            }
        }
    }
}

static size_t small_down_lds(int N, int KS) {
    return (size_t)N * KS * 4 * 32 + 32 + (size_t)SM_WAVES * 64 * sizeof(f32x4_t) +
           SM_EXTRA_FLOATS * sizeof(float);
}

// The small-row kernel serves a call when its rows fit in LDS and one workgroup per feature
// block fills the chip no worse than one round of it.
static bool small_down_ok(int N, int d, int f) {
    if (N < 1 || N > SM_MAX_ROWS) return false;
    const int KS = f / 32, NB = d / 16;
    if (f % 32 || d % 16) return false;
    if ((long long)N * KS * 4 > (long long)SM_STAGE_ITERS * 64 * SM_WAVES) return false;
    if (small_down_lds(N, KS) > 160 * 1024) return false;
    return NB <= moe_num_cus();
}

// What the BLOCK instantiation needs beyond the plain kernel's arguments.
struct SmallBlock {
    const float* x_in;
    const float* w_gate_next;
    float* sums_next;
    int gate_stride;
};

static int small_down_launch(const moe_weights* W, const float* h, const int32_t* offsets, int N,
                             const int32_t* inv_perm, const float* weights, int T, int k, float* y,
                             float* yg, const SmallBlock* blk, hipStream_t s) {
    SmallDownArgs a = {};
    a.wfrag = (const u32x4_t*)W->w2;
    a.h = h;
    a.offsets = offsets;
    a.inv_perm = inv_perm;
    a.weights = weights;
    a.y = y;
    a.yg = yg;
    a.E = W->E; a.N = N; a.K = W->f; a.C = W->d; a.NB = W->d / 16; a.KS = W->f / 32;
    a.T = T; a.k = k;
    if (blk) {
        a.x_in = blk->x_in;
        a.w_gate_next = blk->w_gate_next;
        a.sums_next = blk->sums_next;
        a.gate_stride = blk->gate_stride;
    }
    const size_t lds = small_down_lds(N, a.KS);
    static std::atomic<bool> attr_set[MOE_MAX_DEVICES];
    const int dev = moe_current_device();
    if (dev < 0) return MOE_ERR_HIP;
    if (!attr_set[dev].load(std::memory_order_relaxed)) {
        MOE_HIP_TRY(hipFuncSetAttribute((const void*)stream_down_small_kernel<false>,
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        MOE_HIP_TRY(hipFuncSetAttribute((const void*)stream_down_small_kernel<true>,
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        attr_set[dev].store(true, std::memory_order_relaxed);
    }
    if (blk)
        hipLaunchKernelGGL(stream_down_small_kernel<true>, dim3((unsigned)a.NB), dim3(64 * SM_WAVES),
                           lds, s, a);
    else
        hipLaunchKernelGGL(stream_down_small_kernel<false>, dim3((unsigned)a.NB), dim3(64 * SM_WAVES),
                           lds, s, a);
    return moe_launch_status();
}

// Split a reduction of KS steps (of 32) into P parts x W waves x KSW steps.
static bool stream_pick(int KS, bool allow_parts, int& W, int& KSW, int& P) {
    int best = -1;
    const int ksws[6] = {16, 10, 8, 4, 2, 1};
    for (int i = 0; i < 6; i++)
        for (int w = ST_MAX_WAVES; w >= 1; w--) {
            const int span = w * ksws[i];
            if (KS % span) continue;
            const int p = KS / span;
            if (!allow_parts && p != 1) continue;
            const int score = span * 16 + w;
            if (score > best) {
                best = score;
                W = w;
                KSW = ksws[i];
                P = p;
            }
        }
    return best >= 0;
}

struct StreamPlan {
    int Wu, KSWu;      // first projection: waves, reduction steps per wave (one part)
    int Wd, KSWd, Pd;  // second projection: waves, steps per wave, reduction parts
};

static bool stream_plan(int d, int f, StreamPlan& pl) {
    int Pu;
    return stream_pick(d / 32, false, pl.Wu, pl.KSWu, Pu) &&
           stream_pick(f / 32, true, pl.Wd, pl.KSWd, pl.Pd);
}

bool moe_ffn_stream_supported(int d, int f) {
    StreamPlan pl;
    return stream_plan(d, f, pl);
}

static inline size_t st_align256(size_t v) { return (v + 255) & ~(size_t)255; }

// h [N,f] fp32, then the second projection's slabs [Pd][N,d] fp32
size_t moe_ffn_stream_workspace(int N, int E, int d, int f) {
    (void)E;
    StreamPlan pl;
    size_t need = st_align256((size_t)N * f * sizeof(float));
    if (stream_plan(d, f, pl)) need += (size_t)pl.Pd * N * d * sizeof(float);
    return need;
}

// Launches the instantiation for KSW with as many workgroups per CU as fit (kernels with
// short per-wave reductions use few registers; several resident workgroups then keep
// enough loads in flight per CU).  The work ranges are equal whatever the grid size.
template <int NMAT, bool ACT_BF16, bool GATE>
static int stream_dispatch(int KSW, int waves, hipStream_t s, const StreamArgs& a) {
    const void* fn = nullptr;
    int slot = 0;
    switch (KSW) {
        case 1: fn = (const void*)stream_kernel<1, NMAT, ACT_BF16, GATE>; slot = 0; break;
        case 2: fn = (const void*)stream_kernel<2, NMAT, ACT_BF16, GATE>; slot = 1; break;
        case 4: fn = (const void*)stream_kernel<4, NMAT, ACT_BF16, GATE>; slot = 2; break;
        case 8: fn = (const void*)stream_kernel<8, NMAT, ACT_BF16, GATE>; slot = 3; break;
        case 16: fn = (const void*)stream_kernel<16, NMAT, ACT_BF16, GATE>; slot = 4; break;
        case 10: fn = (const void*)stream_kernel<10, NMAT, ACT_BF16, GATE>; slot = 5; break;
        default: return MOE_ERR_UNSUPPORTED;
    }
    // per device and instantiation: 0 = not asked yet.  Threads that race here ask the
    // same question and store the same answer.
    static std::atomic<int> occ_cache[MOE_MAX_DEVICES][6][ST_MAX_WAVES + 1];
    const int dev = moe_current_device();
    if (dev < 0) return MOE_ERR_HIP;
    int occ = occ_cache[dev][slot][waves].load(std::memory_order_relaxed);
    if (occ == 0) {
        MOE_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, fn, 64 * waves, 0));
        occ = occ < 1 ? 1 : (occ > 4 ? 4 : occ);
        occ_cache[dev][slot][waves].store(occ, std::memory_order_relaxed);
    }
    StreamArgs args = a;
    void* params[1] = {(void*)&args};
    MOE_HIP_TRY(hipLaunchKernel(fn, dim3((unsigned)(moe_num_cus() * occ)), dim3(64 * waves), params,
                                0, s));
    return moe_launch_status();
}

static bool stream_shape_ok(const StreamPlan& pl, int N, int E, int d, int f) {
    if (N / 16 + E > ST_MAX_TILES) return false;
    // unit numbers (tiles x parts x column blocks) are 32-bit in the kernels
    return (long long)ST_MAX_TILES * pl.Pd * ((d > f ? d : f) / 16) < (1ll << 31);
}

static StreamArgs stream_args_up(const moe_weights* W, const StreamPlan& pl, const void* act,
                                 const int32_t* offsets, int N, float* h) {
    StreamArgs up = {};
    up.wfrag = (const u32x4_t*)W->w13;
    up.act = act;
    up.offsets = offsets;
    up.out = h;
    up.part_stride = 0;
    up.E = W->E; up.N = N; up.K = W->d; up.C = W->f;
    up.NB = W->f / 16; up.KS = W->d / 32; up.P = 1; up.W = pl.Wu;
    return up;
}

// out: yg itself when there is one part, else the slabs
static StreamArgs stream_args_down(const moe_weights* W, const StreamPlan& pl, const float* h,
                                   const int32_t* offsets, int N, float* out) {
    StreamArgs dn = {};
    dn.wfrag = (const u32x4_t*)W->w2;
    dn.act = h;
    dn.offsets = offsets;
    dn.out = out;
    dn.part_stride = pl.Pd > 1 ? (size_t)N * W->d : 0;
    dn.E = W->E; dn.N = N; dn.K = W->f; dn.C = W->d;
    dn.NB = W->d / 16; dn.KS = W->f / 32; dn.P = pl.Pd; dn.W = pl.Wd;
    return dn;
}

int moe_ffn_stream_parts(int N, int d, int f) {
    StreamPlan pl;
    if (!stream_plan(d, f, pl)) return 0;
    return small_down_ok(N, d, f) ? 1 : pl.Pd;
}

// n_parts == null: `out` is yg [N,d]; the slabs of a split reduction go to the workspace and
// are added by a third launch.  Else `out` holds moe_ffn_stream_parts(N, d, f) slabs [N,d]
// that are left for the caller to add, and *n_parts receives their number.
int moe_ffn_stream_launch(const moe_weights* W, const void* xg, moe_dtype_t act_dtype,
                          const int32_t* perm, int k, const int32_t* offsets, int N, void* ws,
                          float* out, int* n_parts, hipStream_t s) {
    const int d = W->d, f = W->f, E = W->E;
    StreamPlan pl;
    if (!stream_plan(d, f, pl) || !stream_shape_ok(pl, N, E, d, f)) return MOE_ERR_UNSUPPORTED;
    float* h = (float*)ws;
    float* slabs = n_parts ? out
                           : (float*)((unsigned char*)ws + st_align256((size_t)N * f * sizeof(float)));
    StreamArgs up = stream_args_up(W, pl, xg, offsets, N, h);
    up.row_perm = perm;
    up.row_k = k;
    int rc = (act_dtype == MOE_BF16) ? stream_dispatch<2, true, false>(pl.KSWu, pl.Wu, s, up)
                                     : stream_dispatch<2, false, false>(pl.KSWu, pl.Wu, s, up);
    if (rc != MOE_OK) return rc;
    moe_record_mid_event(s);
    if (small_down_ok(N, d, f)) {
        if (n_parts) *n_parts = 1;
        return small_down_launch(W, h, offsets, N, nullptr, nullptr, 0, 0, nullptr, out, nullptr, s);
    }
    const StreamArgs dn = stream_args_down(W, pl, h, offsets, N, pl.Pd > 1 ? slabs : out);
    rc = stream_dispatch<1, false, false>(pl.KSWd, pl.Wd, s, dn);
    if (n_parts) *n_parts = pl.Pd;
    if (rc != MOE_OK || pl.Pd == 1 || n_parts) return rc;
    const size_t n4 = (size_t)N * d / 4;
    size_t blocks = (n4 + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(stream_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, s,
                       (const float4*)slabs, n4, pl.Pd, (float4*)out);
    return moe_launch_status();
}

bool moe_ffn_stream_decode_supported(int T, int E, int k, int d, int f) {
    StreamPlan pl;
    return T >= 1 && T <= 16 && E <= GATE_WAVE_MAX_E && T * k <= GATE_WAVE_MAX_N &&
           stream_plan(d, f, pl) && stream_shape_ok(pl, T * k, E, d, f);
}

// Both projections of a decode step with the gating function and the per-expert batching in
// the first kernel's prologue.  With one to four routed rows the second kernel also does the
// gate-weighted combine: y (and yg, if not null) are written and *n_parts is 0.  Otherwise
// the second projection's result stays in *n_parts slabs of [T*k, d] floats at *parts,
// *part_stride floats apart, for the caller's combine to add.
int moe_ffn_stream_decode_launch(const moe_weights* W, const float* x, const float* logits, int T,
                                 int k, int32_t* idx, float* weights, int32_t* counts,
                                 int32_t* offsets, int32_t* perm, int32_t* inv_perm, float* xg,
                                 void* ws, float* y, float* yg, const float** parts, int* n_parts,
                                 size_t* part_stride, hipStream_t s) {
    const int d = W->d, f = W->f, E = W->E, N = T * k;
    StreamPlan pl;
    if (!moe_ffn_stream_decode_supported(T, E, k, d, f) || !stream_plan(d, f, pl))
        return MOE_ERR_UNSUPPORTED;
    float* h = (float*)ws;
    float* slabs = (float*)((unsigned char*)ws + st_align256((size_t)N * f * sizeof(float)));
    StreamArgs up = stream_args_up(W, pl, x, nullptr, N, h);
    up.logits = logits;
    up.T = T;
    up.k = k;
    up.idx = idx;
    up.weights = weights;
    up.counts = counts;
    up.offsets_out = offsets;
    up.perm = perm;
    up.inv_perm = inv_perm;
    up.xg = xg;
    int rc = stream_dispatch<2, false, true>(pl.KSWu, pl.Wu, s, up);
    if (rc != MOE_OK) return rc;
    moe_record_mid_event(s);
    if (small_down_ok(N, d, f)) {
        *parts = nullptr;
        *n_parts = 0;
        *part_stride = 0;
        return small_down_launch(W, h, offsets, N, inv_perm, weights, T, k, y, yg, nullptr, s);
    }
    StreamArgs dn = stream_args_down(W, pl, h, offsets, N, slabs);
    dn.part_stride = (size_t)N * d;
    rc = stream_dispatch<1, false, false>(pl.KSWd, pl.Wd, s, dn);
    *parts = slabs;
    *n_parts = pl.Pd;
    *part_stride = (size_t)N * d;
    return rc;
}

bool moe_ffn_stream_block_supported(int T, int E, int k, int d, int f) {
    // (a wave of the first kernel adds at most GS_WAVE_ROWS shares of GS_MAX_ITEMS sums)
    StreamPlan pl;
    return moe_ffn_stream_decode_supported(T, E, k, d, f) && stream_plan(d, f, pl) &&
           E <= SM_MAX_E && T * (E + 1) <= GS_MAX_ITEMS && T * E <= 64 &&
           d / 16 <= GS_WAVE_ROWS * pl.Wu && small_down_ok(T * k, d, f);
}

// A share is one 128-byte line: the workgroups that write neighbouring shares sit on different
// XCDs, and a line written from two L2s is written back in pieces.
int moe_ffn_stream_gate_stride(int T, int E) {
    (void)T;
    (void)E;
    return GS_MAX_ITEMS;
}

// One transformer block's expert layer on the residual stream in two launches: the first
// projection derives the gating inputs from the shares (or takes the logits as given), routes
// in its prologue and reads the token rows; the second finishes with the combine, the
// residual add and the shares of the next block's gating sums.
int moe_ffn_stream_block_launch(const moe_weights* W, const float* x_in, const float* gate_sums,
                                int n_shares, float eps, float* logits, int T, int k, int32_t* idx,
                                float* weights, int32_t* counts, int32_t* offsets, int32_t* perm,
                                int32_t* inv_perm, void* ws, float* x_out, const float* w_gate_next,
                                float* gate_sums_next, hipStream_t s) {
    const int d = W->d, f = W->f, E = W->E, N = T * k;
    StreamPlan pl;
    if (!moe_ffn_stream_block_supported(T, E, k, d, f) || !stream_plan(d, f, pl))
        return MOE_ERR_UNSUPPORTED;
    if (gate_sums && (n_shares < 1 || n_shares > GS_WAVE_ROWS * pl.Wu)) return MOE_ERR_INVALID_ARG;
    float* h = (float*)ws;
    SmallBlock blk = {};
    blk.x_in = x_in;
    blk.w_gate_next = w_gate_next;
    blk.sums_next = gate_sums_next;
    blk.gate_stride = moe_ffn_stream_gate_stride(T, E);
    StreamArgs up = stream_args_up(W, pl, x_in, nullptr, N, h);
    up.logits = logits;
    up.T = T;
    up.k = k;
    up.idx = idx;
    up.weights = weights;
    up.counts = counts;
    up.offsets_out = offsets;
    up.perm = perm;
    up.inv_perm = inv_perm;
    if (gate_sums) {
        up.gate_sums = gate_sums;
        up.n_shares = n_shares;
        up.gate_stride = blk.gate_stride;
        up.eps = eps;
        up.logits_out = logits;
    }
    int rc = stream_dispatch<2, false, true>(pl.KSWu, pl.Wu, s, up);
    if (rc != MOE_OK) return rc;
    moe_record_mid_event(s);
    return small_down_launch(W, h, offsets, N, inv_perm, weights, T, k, x_out, nullptr, &blk, s);
}
