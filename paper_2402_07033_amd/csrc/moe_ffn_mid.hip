// Expert FFN for tens to a few hundred rows per expert on gfx950: weight-streaming
// grouped GEMM on the bf16 matrix cores.
//
// In this range every expert's matrices are read about once per launch, so the layer is
// bound by the weight stream from HBM (the paper's observation that expert latency on the
// GPU is set by parameter loading, Sec. 3.1 / Appendix A), but there are too many rows to
// keep them in registers as the decode kernels do, and too few to fill the 256-row tiles
// of the prefill kernel.  Here a workgroup of 8 waves owns (up to 192 rows of one expert)
// x (16 weight fragment rows); wave w owns fragment rows 2w, 2w+1 for ALL row blocks:
//   * its two rows are adjacent in the packed layout, so the wave streams one contiguous
//     run of fragments, 8..16 one-KiB loads in flight at all times (like the decode
//     kernels: 128 KiB per CU, enough to saturate HBM);
//   * the rows' B fragments (packed by gg_pack_kernel) are staged through LDS in chunks of
//     4 reduction steps, double buffered, by direct-to-LDS loads, and shared by the 8 waves;
//   * per step a wave reads the RBT row-block fragments from LDS and issues 2 x RBT MFMAs;
//     the body is instantiated for RBT = 4, 8, 12 row blocks and chosen per unit (longer
//     experts take several row tiles of 192 rows);
//   * two waves per SIMD (<= 96 accumulator registers each), so the matrix cores of one wave
//     run while the other waits for memory.
//   up   : unit = (row tile, 16 fragment rows = 8 h-column blocks x (w1,w3)), full reduction,
//          SiLU*mul in registers, h written as bf16 B-operand fragments for the second GEMM
//   down : unit = (row tile, 16 fragment rows = 256 features), yg fp32
// The (unit, 4-step chunk) sequence of a launch, feature tile fastest, is cut into equal
// contiguous shares, one per persistent workgroup, so that every workgroup streams the same
// number of weight bytes whatever the unit count (896 first-projection units of the Mixtral
// shape at 8 x 128 rows are 3.5 per CU; the 128 second-projection units half a unit per CU).
// A workgroup that covers only a piece of a unit's reduction stores its partial sums and
// mid_fixup_kernel adds the pieces of the unit in workgroup order (deterministic, no
// atomics) and finishes it.
#include <atomic>

#include "moe_internal.h"
#include "moe_frag_pack.h"

#define MD_WAVES 8
#define MD_THREADS (64 * MD_WAVES)
#define MD_KC 4          // reduction steps per LDS chunk
#define MD_MAX_RB 12     // row blocks (of 16 rows) per row tile (192 rows)
#define MD_BD 2          // LDS reads of B fragments kept ahead of the matrix instructions
#define MD_MAX_PIECES 512 // workgroups of the GEMM launch (pieces a unit can have)
#define MD_MAX_TILES 192 // row tiles per launch (N / 192 + E)

struct MidArgs {
    const u32x4_t* wfrag;  // packed weights (w13 or w2)
    const u32x4_t* bfrag;  // packed activations (xp or hp)
    const int32_t* offsets;
    void* out;        // up: hp fragments (bf16); down: yg [N,d] fp32
    float* part;      // partial tiles of split units: [workgroup][2][16*MD_MAX_RB][256] fp32
    int E, N;
    int KS;      // reduction steps of 32
    int FR;      // weight fragment rows per expert (up: 2*f/16, down: d/16)
    int NT;      // feature tiles = FR / 16
    int KS_out;  // up: f/32 (fragment columns of hp)
    int C;       // down: d (row length of yg)
};

#define MD_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))

template <int V>
struct MdInt {
    static constexpr int value = V;
};

// One unit of work for one wave.  RBT = row blocks computed (>= the tile's nblk, multiple
// of 4); `wsrc` = this wave's first weight fragment of the unit's reduction range (+ lane),
// its second row follows KS fragments later; `bsrc` = the tile's first packed block at the
// start of the reduction range (+ lane); KP = reduction steps of the unit (multiple of 4).
template <bool UP, int RBT>
__device__ __forceinline__ void mid_unit(const MidArgs& a, u32x4_t* lds, const u32x4_t* wsrc,
                                         const u32x4_t* bsrc, int KP, int nblk, int wave, int lane,
                                         int e_row0, int e_rows, int bbase_blk, int blk0, int ft,
                                         bool whole, size_t slot) {
    constexpr int NQ = RBT * MD_KC / MD_WAVES;  // direct-to-LDS requests per wave and chunk
    const int NCH = KP / MD_KC;
    f32x4_t acc[RBT][2];
#pragma unroll
    for (int i = 0; i < RBT; i++) {
        acc[i][0] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        acc[i][1] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    }
    u32x4_t wbuf[2][MD_KC][2];  // [chunk parity][step][row]

    // stage chunk c of the tile's B fragments: fragment q = (block q / 4, step q % 4);
    // blocks past the tile's last one repeat it (their products are never stored)
    auto issue_b = [&](int c) {
#pragma unroll
        for (int n = 0; n < NQ; n++) {
            const int q = wave + MD_WAVES * n;
            int i = q / MD_KC;
            const int s = q % MD_KC;
            const int dst = ((c & 1) * MD_MAX_RB + i) * MD_KC + s;
            i = i < nblk ? i : nblk - 1;
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)(bsrc + ((size_t)i * a.KS + c * MD_KC + s) * 64),
                (__attribute__((address_space(3))) void*)(lds + (size_t)dst * 64), 16, 0, 0);
        }
    };
    auto load_w = [&](int c, int s, int m) -> u32x4_t {
        return __builtin_nontemporal_load(wsrc + ((size_t)m * a.KS + c * MD_KC + s) * 64);
    };

    // prologue: weights of chunk 0, B of chunk 0, weights of chunk 1 -- the same order of
    // requests the loop body leaves behind (weights c, B c, weights c+1), so that the
    // compiler's own count of requests in flight is exact at the loop head
#pragma unroll
    for (int s = 0; s < MD_KC; s++) {
        wbuf[0][s][0] = load_w(0, s, 0);
        wbuf[0][s][1] = load_w(0, s, 1);
    }
    issue_b(0);
    if (NCH > 1) {
#pragma unroll
        for (int s = 0; s < MD_KC; s++) {
            wbuf[1][s][0] = load_w(1, s, 0);
            wbuf[1][s][1] = load_w(1, s, 1);
        }
    }

    // FULL: chunks c+1 and c+2 exist (the steady state: no conditions, so that the compiler
    // keeps exact counts of the requests in flight); else the tail of the unit.
    auto chunk = [&](auto par, auto full, int c) {
        constexpr int PAR = decltype(par)::value;
        constexpr bool FULL = decltype(full)::value != 0;
        const bool has1 = FULL || (c + 1 < NCH), has2 = FULL || (c + 2 < NCH);
        // Requests retire in order.  Needed now: this wave's share of chunk c's B fragments
        // and the weights of chunk c; the only younger requests are the 8 weight loads of
        // chunk c+1, when there is one.
        if (has1) MD_WAIT_VMCNT(2 * MD_KC);
        else MD_WAIT_VMCNT(0);
        // publishes chunk c's buffer; every wave has finished reading the other one (chunk c-1)
        __builtin_amdgcn_s_barrier();
        if (has1) issue_b(c + 1);
#if MD_BD > 0
        // the chunk's MD_KC x RBT (step, row block) products in one sequence, the B fragment
        // of product j+MD_BD read from LDS while product j runs on the matrix cores
        constexpr int NJ = MD_KC * RBT;
        const u32x4_t* pb = lds + (size_t)(PAR * MD_MAX_RB) * MD_KC * 64 + lane;
        auto read_b = [&](const int j) -> bf16x8_t {
            return __builtin_bit_cast(bf16x8_t, pb[(size_t)((j % RBT) * MD_KC + j / RBT) * 64]);
        };
        bf16x8_t bq[MD_BD + 1];
#pragma unroll
        for (int j = 0; j < MD_BD; j++) bq[j] = read_b(j);
#pragma unroll
        for (int j = 0; j < NJ; j++) {
            const int s = j / RBT, i = j % RBT;
            if (j + MD_BD < NJ) bq[(j + MD_BD) % (MD_BD + 1)] = read_b(j + MD_BD);
            const bf16x8_t b = bq[j % (MD_BD + 1)];
            acc[i][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                __builtin_bit_cast(bf16x8_t, wbuf[PAR][s][0]), b, acc[i][0], 0, 0, 0);
            acc[i][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                __builtin_bit_cast(bf16x8_t, wbuf[PAR][s][1]), b, acc[i][1], 0, 0, 0);
            if (has2 && i == RBT - 1) {
                wbuf[PAR][s][0] = load_w(c + 2, s, 0);
                wbuf[PAR][s][1] = load_w(c + 2, s, 1);
            }
        }
#else
#pragma unroll
        for (int s = 0; s < MD_KC; s++) {
            const bf16x8_t w0 = __builtin_bit_cast(bf16x8_t, wbuf[PAR][s][0]);
            const bf16x8_t w1 = __builtin_bit_cast(bf16x8_t, wbuf[PAR][s][1]);
            const u32x4_t* pb = lds + ((size_t)(PAR * MD_MAX_RB) * MD_KC + s) * 64 + lane;
#pragma unroll
            for (int i = 0; i < RBT; i++) {
                const bf16x8_t b = __builtin_bit_cast(bf16x8_t, pb[(size_t)i * MD_KC * 64]);
                acc[i][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w0, b, acc[i][0], 0, 0, 0);
                acc[i][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w1, b, acc[i][1], 0, 0, 0);
            }
            if (has2) {
                wbuf[PAR][s][0] = load_w(c + 2, s, 0);
                wbuf[PAR][s][1] = load_w(c + 2, s, 1);
            }
        }
#endif
    };
    int c = 0;
    for (; c + 3 < NCH; c += 2) {
        chunk(MdInt<0>{}, MdInt<1>{}, c);
        chunk(MdInt<1>{}, MdInt<1>{}, c + 1);
    }
    for (; c < NCH; c += 2) {
        chunk(MdInt<0>{}, MdInt<0>{}, c);
        if (c + 1 < NCH) chunk(MdInt<1>{}, MdInt<0>{}, c + 1);
    }
    // the next unit's prologue overwrites buffer 0: wait until every wave has left the loop
    __builtin_amdgcn_s_barrier();

    // ---- epilogue: D lane l holds rows 4*(l/16)+r (features) x column l%16 (token) ----
    const int t = lane & 15, fq = lane >> 4;
    if (!whole) {
        // a piece of a unit's reduction: raw partial sums [row][16 fragment rows x 16] to this
        // workgroup's scratch slot; mid_fixup_kernel adds the pieces of the unit
        float* p0 = a.part + (slot * (16 * MD_MAX_RB) + t) * 256 + (2 * wave) * 16 + 4 * fq;
#pragma unroll
        for (int i = 0; i < RBT; i++) {
            if (i >= nblk) continue;
#pragma unroll
            for (int m = 0; m < 2; m++)
                *(float4*)(p0 + (size_t)i * 16 * 256 + m * 16) =
                    make_float4(acc[i][m][0], acc[i][m][1], acc[i][m][2], acc[i][m][3]);
        }
    } else if (UP) {
        // fragment rows 2*wave (w1) and 2*wave+1 (w3) of the same 16 h-columns
        const int colblk = ft * 8 + wave;
        const int ks_o = colblk >> 1;
        const int lane_o = ((colblk & 1) * 2 + (fq >> 1)) * 16 + t;
#pragma unroll
        for (int i = 0; i < RBT; i++) {
            if (i >= nblk) continue;
            float hv[4];
#pragma unroll
            for (int r = 0; r < 4; r++)
                hv[r] = acc[i][0][r] / (1.0f + __expf(-acc[i][0][r])) * acc[i][1][r];
            uint2 pk;
            pk.x = moe_pack_bf16x2(hv[0], hv[1]);
            pk.y = moe_pack_bf16x2(hv[2], hv[3]);
            *(uint2*)((unsigned char*)a.out +
                      (((size_t)(bbase_blk + blk0 + i) * a.KS_out + ks_o) * 64 + lane_o) * 16 +
                      (fq & 1) * 8) = pk;
        }
    } else {
#pragma unroll
        for (int i = 0; i < RBT; i++) {
            if (i >= nblk) continue;
            const int r_in_seg = (blk0 + i) * 16 + t;
            if (r_in_seg >= e_rows) continue;
            float* row = (float*)a.out + (size_t)(e_row0 + r_in_seg) * a.C + (ft * 16 + 2 * wave) * 16 + 4 * fq;
#pragma unroll
            for (int m = 0; m < 2; m++)
                *(float4*)(row + m * 16) =
                    make_float4(acc[i][m][0], acc[i][m][1], acc[i][m][2], acc[i][m][3]);
        }
    }
}

// The launch's work is the sequence of (unit, chunk) pairs, unit = (row tile, feature tile),
// chunk = MD_KC reduction steps; workgroup b of `grid` takes the pairs [cut(b), cut(b+1)), so
// every workgroup streams the same number of weight bytes whatever the number of units.
__device__ __forceinline__ long long mid_cut(long long G, int b, int grid) { return G * b / grid; }

// Scratch slot of workgroup b's piece of unit u (or -1 if b finishes u alone / has no part
// of it): its first unit's piece takes slot 0, its last unit's piece the next free one.
__device__ __forceinline__ int mid_piece_slot(long long G, int NCH, int grid, int b, long long u) {
    const long long gb = mid_cut(G, b, grid), ge = mid_cut(G, b + 1, grid);
    const long long u_lo = u * NCH, u_hi = u_lo + NCH;
    if (ge <= u_lo || gb >= u_hi || gb >= ge) return -1;
    if (gb <= u_lo && ge >= u_hi) return -1;  // whole unit
    const long long u_first = gb / NCH;
    if (u == u_first) return 2 * b;
    const bool head_partial = !((gb % NCH) == 0 && ge >= (u_first + 1) * NCH);
    return 2 * b + (head_partial ? 1 : 0);
}

// Row tiles of the launch (<= MD_MAX_RB blocks of one expert each), listed in LDS by thread 0.
__device__ __forceinline__ void mid_tile_list(const int32_t* __restrict__ offsets, int E, int N,
                                              int* s_offs, int* s_te, int* s_blk0, int* s_nblk,
                                              int* s_row0, int* s_rows, int* s_bbase, int* s_nt) {
    const int tid = threadIdx.x;
    if (tid <= E) s_offs[tid] = offsets[tid];
    __syncthreads();
    if (tid == 0) {
        int n = 0, bb = 0, prev = 0;
        for (int e = 0; e < E; e++) {
            const int lo = gg_clamp_off(s_offs[e], prev, N);
            const int hi = gg_clamp_off(s_offs[e + 1], lo, N);
            prev = lo;
            const int nb = (hi - lo + 15) / 16;
            s_row0[e] = lo; s_rows[e] = hi - lo; s_bbase[e] = bb;
            for (int b0 = 0; b0 < nb && n < MD_MAX_TILES; b0 += MD_MAX_RB) {
                s_te[n] = e;
                s_blk0[n] = b0;
                s_nblk[n] = (nb - b0) < MD_MAX_RB ? (nb - b0) : MD_MAX_RB;
                n++;
            }
            bb += nb;
        }
        *s_nt = n;
    }
    __syncthreads();
}

template <bool UP>
__global__ __launch_bounds__(MD_THREADS) void mid_kernel(MidArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    u32x4_t* lds = (u32x4_t*)smem;  // [2 buffers][MD_MAX_RB blocks][MD_KC steps][64 lanes]
    __shared__ int s_te[MD_MAX_TILES], s_blk0[MD_MAX_TILES], s_nblk[MD_MAX_TILES];
    __shared__ int s_row0[MOE_MAX_E], s_rows[MOE_MAX_E], s_bbase[MOE_MAX_E];
    __shared__ int s_offs[MOE_MAX_E + 1];
    __shared__ int s_nt;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    mid_tile_list(a.offsets, a.E, a.N, s_offs, s_te, s_blk0, s_nblk, s_row0, s_rows, s_bbase, &s_nt);
    // unit index = row tile * NT + feature tile
    const int NCH = a.KS / MD_KC;
    const long long G = (long long)s_nt * a.NT * NCH;
    const long long g_end = mid_cut(G, blockIdx.x + 1, gridDim.x);
    int piece = 0;
    for (long long g = mid_cut(G, blockIdx.x, gridDim.x); g < g_end;) {
        const long long u = g / NCH;
        const int c0 = (int)(g % NCH);
        const int nch = (int)((g_end - g) < (NCH - c0) ? (g_end - g) : (NCH - c0));
        const bool whole = (nch == NCH);
        const int ft = (int)(u % a.NT);
        const int tile = (int)(u / a.NT);
        const int e = s_te[tile], blk0 = s_blk0[tile], nblk = s_nblk[tile];
        const int k0 = c0 * MD_KC, KP = nch * MD_KC;
        const u32x4_t* wsrc =
            a.wfrag + (((size_t)e * a.FR + (size_t)ft * 16 + 2 * wave) * a.KS + k0) * 64 + lane;
        const u32x4_t* bsrc = a.bfrag + ((size_t)(s_bbase[e] + blk0) * a.KS + k0) * 64 + lane;
        const int row0 = s_row0[e], rows = s_rows[e], bbase = s_bbase[e];
        const size_t slot = (size_t)blockIdx.x * 2 + piece;
        if (!whole) piece++;
        if (nblk <= 4)
            mid_unit<UP, 4>(a, lds, wsrc, bsrc, KP, nblk, wave, lane, row0, rows, bbase, blk0, ft, whole, slot);
        else if (nblk <= 8)
            mid_unit<UP, 8>(a, lds, wsrc, bsrc, KP, nblk, wave, lane, row0, rows, bbase, blk0, ft, whole, slot);
        else
            mid_unit<UP, 12>(a, lds, wsrc, bsrc, KP, nblk, wave, lane, row0, rows, bbase, blk0, ft, whole, slot);
        g += nch;
    }
}

// Units whose reduction was shared by several workgroups: adds their pieces in workgroup
// order (deterministic), then writes yg (second projection) or applies SiLU*mul and writes
// the h fragments (first).  One workgroup per unit; `grid` = the GEMM launch's workgroup
// count (<= MD_MAX_PIECES).
template <bool UP>
__global__ __launch_bounds__(256) void mid_fixup_kernel(MidArgs a, int grid) {
    __shared__ int s_te[MD_MAX_TILES], s_blk0[MD_MAX_TILES], s_nblk[MD_MAX_TILES];
    __shared__ int s_row0[MOE_MAX_E], s_rows[MOE_MAX_E], s_bbase[MOE_MAX_E];
    __shared__ int s_offs[MOE_MAX_E + 1];
    __shared__ int s_nt;
    mid_tile_list(a.offsets, a.E, a.N, s_offs, s_te, s_blk0, s_nblk, s_row0, s_rows, s_bbase, &s_nt);
    const long long u = blockIdx.x;
    const int tile = (int)(u / a.NT), ft = (int)(u % a.NT);
    if (tile >= s_nt) return;
    const int NCH = a.KS / MD_KC;
    const long long G = (long long)s_nt * a.NT * NCH;
    // workgroups that hold the unit's first and last chunk
    const long long g_lo = u * NCH, g_hi = g_lo + NCH - 1;
    int b_lo = (int)(g_lo * grid / G), b_hi = (int)(g_hi * grid / G);
    while (b_lo > 0 && mid_cut(G, b_lo, grid) > g_lo) b_lo--;
    while (b_lo + 1 < grid && mid_cut(G, b_lo + 1, grid) <= g_lo) b_lo++;
    while (b_hi > 0 && mid_cut(G, b_hi, grid) > g_hi) b_hi--;
    while (b_hi + 1 < grid && mid_cut(G, b_hi + 1, grid) <= g_hi) b_hi++;
    if (b_lo == b_hi) return;  // one workgroup did the whole unit and wrote the result itself
    // the pieces' scratch slots, in workgroup order (a unit has at most `grid` pieces)
    __shared__ int s_slot[MD_MAX_PIECES];
    const int nb = (b_hi - b_lo + 1) < MD_MAX_PIECES ? (b_hi - b_lo + 1) : MD_MAX_PIECES;
    for (int i = threadIdx.x; i < nb; i += 256) s_slot[i] = mid_piece_slot(G, NCH, grid, b_lo + i, u);
    __syncthreads();
    const int e = s_te[tile];
    const int first = s_blk0[tile] * 16;  // first row of the tile in its segment
    // second projection: the tile's real rows; first: every row of its blocks
    int rows = 16 * s_nblk[tile];
    if (!UP && s_rows[e] - first < rows) rows = s_rows[e] - first;
    if (UP) {
        // item = (row, block of 16 h-columns cb, feature quad fq): a = x.w1 from fragment row
        // 2cb, b = x.w3 from fragment row 2cb+1, four columns each
        for (int idx = threadIdx.x; idx < rows * 32; idx += 256) {
            const int row = idx >> 5, cb = (idx >> 2) & 7, fq = idx & 3;
            float4 sa = make_float4(0.f, 0.f, 0.f, 0.f), sb = sa;
            for (int i = 0; i < nb; i++) {
                if (s_slot[i] < 0) continue;
                const float* src = a.part + ((size_t)s_slot[i] * (16 * MD_MAX_RB) + row) * 256 + (2 * cb) * 16 + 4 * fq;
                const float4 va = *(const float4*)src, vb = *(const float4*)(src + 16);
                sa.x += va.x; sa.y += va.y; sa.z += va.z; sa.w += va.w;
                sb.x += vb.x; sb.y += vb.y; sb.z += vb.z; sb.w += vb.w;
            }
            const float av[4] = {sa.x, sa.y, sa.z, sa.w}, bv[4] = {sb.x, sb.y, sb.z, sb.w};
            float hv[4];
#pragma unroll
            for (int q = 0; q < 4; q++) hv[q] = av[q] / (1.0f + __expf(-av[q])) * bv[q];
            const int blk = s_blk0[tile] + (row >> 4), t = row & 15;
            const int colblk = ft * 8 + cb;
            const int ks_o = colblk >> 1;
            const int lane_o = ((colblk & 1) * 2 + (fq >> 1)) * 16 + t;
            uint2 pk;
            pk.x = moe_pack_bf16x2(hv[0], hv[1]);
            pk.y = moe_pack_bf16x2(hv[2], hv[3]);
            *(uint2*)((unsigned char*)a.out +
                      (((size_t)(s_bbase[e] + blk) * a.KS_out + ks_o) * 64 + lane_o) * 16 +
                      (fq & 1) * 8) = pk;
        }
    } else {
        for (int idx = threadIdx.x; idx < rows * 64; idx += 256) {
            const int row = idx >> 6, c4 = idx & 63;
            float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int i = 0; i < nb; i++) {
                if (s_slot[i] < 0) continue;
                const float4 v = *(const float4*)(a.part + ((size_t)s_slot[i] * (16 * MD_MAX_RB) + row) * 256 + c4 * 4);
                sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
            }
            *(float4*)((float*)a.out + (size_t)(s_row0[e] + first + row) * a.C + ft * 256 + c4 * 4) = sum;
        }
    }
}

// ---------------------------------------------------------------- host side ----
static inline size_t md_align256(size_t v) { return (v + 255) & ~(size_t)255; }
static inline size_t md_max_blocks(int N, int E) { return (size_t)N / 16 + E; }

bool moe_ffn_mid_supported(int N, int E, int d, int f) {
    // 16 fragment rows per unit in both projections; reductions in chunks of 4 steps
    if (f % 128 != 0 || d % 256 != 0 || d % (32 * MD_KC) != 0 || f % (32 * MD_KC) != 0) return false;
    if (moe_num_cus() > MD_MAX_PIECES) return false;
    return (size_t)N / (16 * MD_MAX_RB) + E <= MD_MAX_TILES;
}

static inline size_t md_max_tiles(int N, int E) { return (size_t)N / (16 * MD_MAX_RB) + E; }

// scratch for the pieces of split units: 2 slots of (16*MD_MAX_RB) x 256 fp32 per workgroup
static inline size_t md_part_bytes() {
    return (size_t)moe_num_cus() * 2 * (16 * MD_MAX_RB) * 256 * sizeof(float);
}

size_t moe_ffn_mid_workspace(int N, int E, int d, int f) {
    const size_t nb = md_max_blocks(N, E);
    return md_align256(nb * 16 * d * 2) + md_align256(nb * 16 * f * 2) + md_part_bytes();
}

int moe_ffn_mid_launch(const moe_weights* W, const void* xg, moe_dtype_t act_dtype,
                       const int32_t* perm, int k, const int32_t* offsets, int N, void* ws,
                       float* yg, hipStream_t s) {
    const int d = W->d, f = W->f, E = W->E;
    if (!moe_ffn_mid_supported(N, E, d, f)) return MOE_ERR_UNSUPPORTED;
    const size_t nb = md_max_blocks(N, E);
    u32x4_t* xp = (u32x4_t*)ws;
    u32x4_t* hp = (u32x4_t*)((unsigned char*)ws + md_align256(nb * 16 * d * 2));
    const size_t lds_bytes = (size_t)2 * MD_MAX_RB * MD_KC * MOE_FRAG_BYTES;  // 96 KiB
    const unsigned grid = (unsigned)moe_num_cus();

    // once per device; threads that race here set the same attributes
    static std::atomic<int> attr_set[MOE_MAX_DEVICES];
    const int dev = moe_current_device();
    if (dev < 0) return MOE_ERR_HIP;
    if (!attr_set[dev].load(std::memory_order_acquire)) {
        MOE_HIP_TRY(hipFuncSetAttribute((const void*)mid_kernel<true>,
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes));
        MOE_HIP_TRY(hipFuncSetAttribute((const void*)mid_kernel<false>,
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes));
        attr_set[dev].store(1, std::memory_order_release);
    }

    if (act_dtype == MOE_BF16)
        hipLaunchKernelGGL(gg_pack_kernel<true>, gg_pack_grid(nb, d), dim3(256), 0, s, xg, perm, k,
                           offsets, E, N, d, xp);
    else
        hipLaunchKernelGGL(gg_pack_kernel<false>, gg_pack_grid(nb, d), dim3(256), 0, s, xg, perm, k,
                           offsets, E, N, d, xp);

    float* part = (float*)((unsigned char*)ws + md_align256(nb * 16 * d * 2) + md_align256(nb * 16 * f * 2));
    const unsigned max_units_per_nt = (unsigned)md_max_tiles(N, E);

    MidArgs up;
    up.wfrag = (const u32x4_t*)W->w13;
    up.bfrag = xp;
    up.offsets = offsets;
    up.out = hp;
    up.part = part;
    up.E = E; up.N = N;
    up.KS = d / 32;
    up.FR = 2 * (f / 16);
    up.NT = up.FR / 16;
    up.KS_out = f / 32;
    up.C = 0;
    hipLaunchKernelGGL(mid_kernel<true>, dim3(grid), dim3(MD_THREADS), lds_bytes, s, up);
    hipLaunchKernelGGL(mid_fixup_kernel<true>, dim3(max_units_per_nt * up.NT), dim3(256), 0, s, up,
                       (int)grid);
    moe_record_mid_event(s);

    MidArgs dn;
    dn.wfrag = (const u32x4_t*)W->w2;
    dn.bfrag = hp;
    dn.offsets = offsets;
    dn.out = yg;
    dn.part = part;
    dn.E = E; dn.N = N;
    dn.KS = f / 32;
    dn.FR = d / 16;
    dn.NT = dn.FR / 16;
    dn.KS_out = 0;
    dn.C = d;
    hipLaunchKernelGGL(mid_kernel<false>, dim3(grid), dim3(MD_THREADS), lds_bytes, s, dn);
    hipLaunchKernelGGL(mid_fixup_kernel<false>, dim3(max_units_per_nt * dn.NT), dim3(256), 0, s, dn,
                       (int)grid);
    return moe_launch_status();
}
