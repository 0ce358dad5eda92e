// Prefill-sized expert FFN for gfx950: grouped GEMM on the bf16 matrix cores.
//
// Both operands of v_mfma_f32_16x16x32_bf16 are kept in fragment order (see
// moe_internal.h): the packed weights are the A operand (16 output features x
// 32 reduction indices), and the activations are first re-laid into B-operand
// fragments (32 reduction indices x 16 token rows) per expert segment, padded
// with zero rows to a multiple of 16, so that no tile straddles two experts
// and the GEMM main loop has no bounds checks.  A fragment is 1 KiB: one
// wavefront moves it with a single coalesced 16-byte-per-lane access, and the
// LDS copy is read back conflict-free (lane l reads bytes 16l..16l+15).
//
//   pack  : xg [N,d] (fp32 or bf16) -> xp fragments [block][d/32]
//   up    : per (token tile of 256 rows, 128 h-columns): a = x.w1, b = x.w3,
//           h = silu(a)*b written as bf16 straight into B-operand fragments
//           hp [block][f/32] for the second GEMM
//   down  : per (token tile of 256 rows, 256 output features): yg = h.w2, fp32
//
// Workgroup: 8 waves as 2 (token halves of 128 rows) x 4 (groups of 4 weight
// fragment rows = 64 features); each wave owns a 128 x 64 accumulator tile
// (32 MFMA tiles, 128 registers).  The reduction advances 64 indices per
// stage; stages are double-buffered in LDS (2 x 64 KiB).
//
// The grid covers the worst case number of token tiles (N/256 + E); a
// workgroup finds its expert from the device-side offsets and leaves if its
// tile does not exist, so the host never learns the per-expert sizes.
#include "moe_internal.h"

#define GG_TILE_BLOCKS 16  // 16-row blocks per token tile (256 rows)
#define GG_FROWS 16        // weight fragment rows per workgroup tile (256 features)
#define GG_THREADS 512
#define GG_NS 4              // LDS stages in flight
#define GG_LOADS_PER_WAVE 4  // fragments each wave brings in per stage (32 / 8 waves)

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

// Locate token tile `tt` (tiles of GG_TILE_BLOCKS blocks, per expert).
__device__ __forceinline__ bool gg_find_tile(const int32_t* __restrict__ offsets, int E, int N,
                                             int tt, SegInfo& si, int& tile_in_seg) {
    int bb = 0, tiles = 0, prev = 0;
    for (int e = 0; e < E; e++) {
        const int lo = gg_clamp_off(offsets[e], prev, N);
        const int hi = gg_clamp_off(offsets[e + 1], lo, N);
        prev = lo;
        const int nb = (hi - lo + 15) / 16;
        const int nt = (nb + GG_TILE_BLOCKS - 1) / GG_TILE_BLOCKS;
        if (tt < tiles + nt) {
            si.e = e; si.row0 = lo; si.rows = hi - lo; si.bbase = bb;
            tile_in_seg = tt - tiles;
            return true;
        }
        bb += nb;
        tiles += nt;
    }
    return false;
}

// ------------------------------------------------------------------- pack ----
// One workgroup per packed block: rows [row0 + 16*b, +16) of a segment become
// d/32 B-operand fragments; rows past the segment end are zero.
template <bool ACT_BF16>
__global__ __launch_bounds__(256) void gg_pack_kernel(const void* __restrict__ xg,
                                                      const int32_t* __restrict__ offsets, int E,
                                                      int N, int d, u32x4_t* __restrict__ xp) {
    SegInfo si;
    if (!gg_find_block(offsets, E, N, blockIdx.x, si)) return;
    const int b = blockIdx.x - si.bbase;
    const int KS = d / 32;
    for (int i = threadIdx.x; i < KS * 64; i += 256) {
        const int lane = i & 63, ks = i >> 6;
        const int t = lane & 15, kq = lane >> 4;
        const int r = b * 16 + t;
        u32x4_t v = {0u, 0u, 0u, 0u};
        if (r < si.rows) {
            const size_t off = (size_t)(si.row0 + r) * d + (size_t)ks * 32 + kq * 8;
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

// ------------------------------------------------------------------- GEMM ----
struct GroupedArgs {
    const u32x4_t* wfrag;  // A operand: packed weights (w13 or w2)
    const u32x4_t* bfrag;  // B operand: packed activations (xp or hp)
    const int32_t* offsets;
    void* out;  // up: hp fragments (bf16); down: yg [N,d] fp32
    int E, N;
    int KS;      // reduction steps of 32
    int FR;      // weight fragment rows per expert (up: 2*f/16, down: d/16)
    int NT;      // workgroup tiles along the features = FR / GG_FROWS
    int KS_out;  // up: f/32 (fragment columns of hp); down: unused
    int C;       // down: d (row length of yg)
};

// s_waitcnt with only the vector-memory counter constrained (gfx9 encoding:
// vmcnt = bits 3:0 and 15:14, expcnt 6:4 = 7 and lgkmcnt 11:8 = 15 left open).
#define GG_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))
#define GG_WAIT_LGKM0() __builtin_amdgcn_s_waitcnt(0xC07F)

// Wait until at most `batches` of this wave's stage loads (GG_LOADS_PER_WAVE each) are in flight.
__device__ __forceinline__ void gg_wait_batches(int batches) {
    if (batches >= 3) GG_WAIT_VMCNT(3 * GG_LOADS_PER_WAVE);
    else if (batches == 2) GG_WAIT_VMCNT(2 * GG_LOADS_PER_WAVE);
    else if (batches == 1) GG_WAIT_VMCNT(1 * GG_LOADS_PER_WAVE);
    else GG_WAIT_VMCNT(0);
}

// Logical tile index -> (expert segment, tile inside the segment, feature tile).
// Logical order: expert, then feature tile, then token tile (fastest), so that
// workgroups with neighbouring indices share the same weight tile.
__device__ __forceinline__ bool gg_find_logical(const int32_t* __restrict__ offsets, int E, int N,
                                                int NT, int xcd, int slot, SegInfo& si,
                                                int& tile_in_seg, int& nt) {
    int total = 0, prev = 0;
    for (int e = 0; e < E; e++) {
        const int lo = gg_clamp_off(offsets[e], prev, N);
        const int hi = gg_clamp_off(offsets[e + 1], lo, N);
        prev = lo;
        total += ((hi - lo + 16 * GG_TILE_BLOCKS - 1) / (16 * GG_TILE_BLOCKS)) * NT;
    }
    // Workgroup ids are dealt round-robin to the 8 XCDs (one L2 each): give every XCD
    // one contiguous eighth of the logical order.
    const int per_xcd = (total + 7) / 8;
    if (slot >= per_xcd) return false;
    const int L = xcd * per_xcd + slot;
    if (L >= total) return false;
    int base = 0, bb = 0;
    prev = 0;
    for (int e = 0; e < E; e++) {
        const int lo = gg_clamp_off(offsets[e], prev, N);
        const int hi = gg_clamp_off(offsets[e + 1], lo, N);
        prev = lo;
        const int nb = (hi - lo + 15) / 16;
        const int tiles = (nb + GG_TILE_BLOCKS - 1) / GG_TILE_BLOCKS;
        if (L < base + tiles * NT) {
            const int r = L - base;
            nt = r / tiles;
            tile_in_seg = r % tiles;
            si.e = e; si.row0 = lo; si.rows = hi - lo; si.bbase = bb;
            return true;
        }
        base += tiles * NT;
        bb += nb;
    }
    return false;
}

// Grouped GEMM tile: 256 token rows x 16 weight fragment rows, 8 waves.
//
// The reduction advances one MFMA step (32 indices) per stage; a stage is 16 A
// fragments (weights) + 16 B fragments (token blocks) = 32 KiB, brought into a
// ring of GG_NS stages in LDS by direct-to-LDS loads (each wave instruction
// moves one whole fragment; no registers, no LDS store instructions).
//
// The two waves that share a SIMD (wave w and w+4; they own the two token
// halves) run half a period apart: while one reads its 12 fragments of stage
// k from LDS, the other issues the 32 MFMAs of the stage it read before, and
// a workgroup barrier separates the half-periods.  Time slot t: group 0 reads
// stage k at t = 2k and multiplies at t = 2k+1; group 1 reads at 2k+1 and
// multiplies at 2k+2.  Stage j's LDS buffer is free again from slot 2j+2, and
// that is when every wave issues its share of stage j+GG_NS.
template <bool UP>
__global__ __launch_bounds__(GG_THREADS) void gg_gemm_kernel(GroupedArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    u32x4_t* lds = (u32x4_t*)smem;  // [GG_NS stages][32 fragments][64 lanes]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    SegInfo si;
    int tis, nt;
    if (!gg_find_logical(a.offsets, a.E, a.N, a.NT, blockIdx.x & 7, blockIdx.x >> 3, si, tis, nt))
        return;
    const int seg_blocks = (si.rows + 15) / 16;
    const int blk0 = tis * GG_TILE_BLOCKS;  // first block of this tile inside the segment
    const int nblk = (seg_blocks - blk0) < GG_TILE_BLOCKS ? (seg_blocks - blk0) : GG_TILE_BLOCKS;

    // The ping-pong groups must pair the two waves that share a SIMD.  Read the SIMD
    // each wave actually landed on (HW_ID bits 5:4): the first wave on a SIMD joins
    // group 0, the second group 1.  If the placement is not 2 waves per SIMD, fall back
    // to halves by wave index (still correct, only less overlap).
    __shared__ int s_simd[8];
    if (lane == 0) s_simd[wave] = (int)__builtin_amdgcn_s_getreg((1 << 11) | (4 << 6) | 4);
    __syncthreads();
    int wt = wave >> 2;  // token half: blocks [8*wt, 8*wt+8); also the ping-pong group
    int wn = wave & 3;   // fragment rows [4*wn, 4*wn+4)
    {
        int grp[8], cnt0 = 0, cnt1 = 0;
        bool ok = true;
#pragma unroll
        for (int w = 0; w < 8; w++) {
            int rank = 0;
#pragma unroll
            for (int v = 0; v < 8; v++)
                if (v < w && s_simd[v] == s_simd[w]) rank++;
            grp[w] = rank;
            if (rank == 0) cnt0++;
            else if (rank == 1) cnt1++;
            else ok = false;
        }
        if (ok && cnt0 == 4 && cnt1 == 4) {
            int g = 0, n = 0;
#pragma unroll
            for (int w = 0; w < 8; w++)
                if (w == wave) g = grp[w];
#pragma unroll
            for (int w = 0; w < 8; w++)
                if (w < wave && grp[w] == g) n++;
            wt = g;
            wn = n;
        }
    }
    const int my_blocks = (nblk - 8 * wt) < 0 ? 0 : ((nblk - 8 * wt) > 8 ? 8 : (nblk - 8 * wt));

    // loader role: wave w moves fragments 4w..4w+3 of the 32 in a stage
    // (q < 16: A fragment row q; q >= 16: B block q-16, clamped to an existing block so
    // that every wave always issues the same number of loads).
    const u32x4_t* src[GG_LOADS_PER_WAVE];
#pragma unroll
    for (int i = 0; i < GG_LOADS_PER_WAVE; i++) {
        const int q = wave * GG_LOADS_PER_WAVE + i;
        if (q < 16) {
            src[i] = a.wfrag + (((size_t)si.e * a.FR + (size_t)nt * GG_FROWS + q) * a.KS) * 64 + lane;
        } else {
            int blk = q - 16;
            blk = blk < nblk ? blk : nblk - 1;
            src[i] = a.bfrag + (((size_t)(si.bbase + blk0 + blk)) * a.KS) * 64 + lane;
        }
    }
    auto issue_stage = [&](int j) {
        const int buf = j % GG_NS;
#pragma unroll
        for (int i = 0; i < GG_LOADS_PER_WAVE; i++) {
            const int q = wave * GG_LOADS_PER_WAVE + i;
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)(src[i] + (size_t)j * 64),
                (__attribute__((address_space(3))) void*)(lds + (buf * 32 + q) * 64), 16, 0, 0);
        }
    };

    f32x4_t acc[8][4];
#pragma unroll
    for (int i = 0; i < 8; i++)
#pragma unroll
        for (int j = 0; j < 4; j++) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    bf16x8_t af[4], bfr[8];
    auto read_frags = [&](int k) {
        const int buf = k % GG_NS;
#pragma unroll
        for (int j = 0; j < 4; j++)
            af[j] = __builtin_bit_cast(bf16x8_t, lds[(buf * 32 + 4 * wn + j) * 64 + lane]);
#pragma unroll
        for (int i = 0; i < 8; i++)
            if (i < my_blocks)
                bfr[i] = __builtin_bit_cast(bf16x8_t, lds[(buf * 32 + 16 + 8 * wt + i) * 64 + lane]);
        GG_WAIT_LGKM0();
    };
    auto mma_range = [&](int i0, int i1) {
#pragma unroll
        for (int i = 0; i < 8; i++)
            if (i >= i0 && i < i1 && i < my_blocks) {
#pragma unroll
                for (int j = 0; j < 4; j++)
                    acc[i][j] =
                        __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[j], bfr[i], acc[i][j], 0, 0, 0);
            }
    };
    auto mma = [&]() { mma_range(0, 8); };

    const int KT = a.KS;
    for (int j = 0; j < GG_NS && j < KT; j++) issue_stage(j);
    gg_wait_batches((KT - 1) < (GG_NS - 1) ? (KT - 1) : (GG_NS - 1));
    __builtin_amdgcn_s_barrier();
    if (wt == 0) {
        for (int k = 0; k < KT; k++) {
            // slot 2k: read stage k (and refill the buffer stage k-1 has left)
            if (k >= 1 && k + GG_NS - 1 < KT) issue_stage(k + GG_NS - 1);
            read_frags(k);
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            // slot 2k+1: multiply stage k; before leaving, stage k+1 must have landed
            mma();
            __builtin_amdgcn_sched_barrier(0);
            if (k + 1 < KT) gg_wait_batches((KT - 2 - k) < (GG_NS - 2) ? (KT - 2 - k) : (GG_NS - 2));
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
        }
    } else {
        __builtin_amdgcn_s_barrier();  // slot 0: idle
        for (int k = 0; k < KT; k++) {
            // slot 2k+1: read stage k; before leaving, stage k+1 must have landed
            read_frags(k);
            if (k + 1 < KT) gg_wait_batches((KT - 2 - k) < (GG_NS - 2) ? (KT - 2 - k) : (GG_NS - 2));
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            // slot 2k+2: stage k's buffer is free: refill it, then multiply stage k
            mma_range(0, 2);
            if (k + GG_NS < KT) issue_stage(k + GG_NS);
            mma_range(2, 8);
            __builtin_amdgcn_sched_barrier(0);
            if (k + 1 < KT) __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // ---- epilogue ----
    const int t = lane & 15, fq = lane >> 4;  // token in block, feature quad
#pragma unroll
    for (int i = 0; i < 8; i++) {
        if (i >= my_blocks) continue;
        const int blk = blk0 + 8 * wt + i;  // block inside the segment
        if (UP) {
            // fragment rows 4*wn+j: j even = w1 rows, j odd = w3 rows of the same 16 columns.
#pragma unroll
            for (int jj = 0; jj < 2; jj++) {
                const f32x4_t av = acc[i][2 * jj], bv = acc[i][2 * jj + 1];
                float hv[4];
#pragma unroll
                for (int r = 0; r < 4; r++) hv[r] = av[r] / (1.0f + __expf(-av[r])) * bv[r];
                // h column c = colblk*16 + 4*fq + r, colblk = global 16-column block
                const int colblk = nt * (GG_FROWS / 2) + 2 * wn + jj;
                const int ks_o = colblk >> 1;
                const int lane_o = ((colblk & 1) * 2 + (fq >> 1)) * 16 + t;
                uint2 pk;
                pk.x = moe_pack_bf16x2(hv[0], hv[1]);
                pk.y = moe_pack_bf16x2(hv[2], hv[3]);
                unsigned char* dst = (unsigned char*)a.out +
                                     (((size_t)(si.bbase + blk) * a.KS_out + ks_o) * 64 + lane_o) * 16 +
                                     (fq & 1) * 8;
                *(uint2*)dst = pk;
            }
        } else {
            const int r_in_seg = blk * 16 + t;
            if (r_in_seg < si.rows) {
                float* row = (float*)a.out + (size_t)(si.row0 + r_in_seg) * a.C;
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    const int feat = (nt * GG_FROWS + 4 * wn + j) * 16 + 4 * fq;
                    *(float4*)(row + feat) =
                        make_float4(acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]);
                }
            }
        }
    }
}

// ---------------------------------------------------------------- host side ----
static inline size_t gg_align256(size_t v) { return (v + 255) & ~(size_t)255; }
static inline size_t gg_max_blocks(int N, int E) { return (size_t)N / 16 + E; }

size_t moe_ffn_grouped_workspace(int N, int E, int d, int f) {
    const size_t nb = gg_max_blocks(N, E);
    return gg_align256(nb * 16 * d * 2) + gg_align256(nb * 16 * f * 2);
}

int moe_ffn_grouped_launch(const moe_weights* W, const void* xg, moe_dtype_t act_dtype,
                           const int32_t* offsets, int N, void* ws, float* yg, hipStream_t s) {
    const int d = W->d, f = W->f, E = W->E;
    // up tile = 16 fragment rows = 8 column blocks x (w1,w3): f % 128 == 0;
    // down tile = 256 features: d % 256 == 0; stages of 64: d % 64 == 0, f % 64 == 0.
    if (f % 128 != 0 || d % 256 != 0) return MOE_ERR_UNSUPPORTED;
    const size_t nb = gg_max_blocks(N, E);
    u32x4_t* xp = (u32x4_t*)ws;
    u32x4_t* hp = (u32x4_t*)((unsigned char*)ws + gg_align256(nb * 16 * d * 2));
    const int max_tiles = N / (16 * GG_TILE_BLOCKS) + E;
    const size_t lds_bytes = GG_NS * 32 * MOE_FRAG_BYTES;

    static bool attr_set = false;
    if (!attr_set) {
        MOE_HIP_TRY(hipFuncSetAttribute((const void*)gg_gemm_kernel<true>,
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes));
        MOE_HIP_TRY(hipFuncSetAttribute((const void*)gg_gemm_kernel<false>,
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes));
        attr_set = true;
    }

    if (act_dtype == MOE_BF16)
        hipLaunchKernelGGL(gg_pack_kernel<true>, dim3((unsigned)nb), dim3(256), 0, s, xg, offsets, E,
                           N, d, xp);
    else
        hipLaunchKernelGGL(gg_pack_kernel<false>, dim3((unsigned)nb), dim3(256), 0, s, xg, offsets,
                           E, N, d, xp);

    GroupedArgs up;
    up.wfrag = (const u32x4_t*)W->w13;
    up.bfrag = xp;
    up.offsets = offsets;
    up.out = hp;
    up.E = E; up.N = N;
    up.KS = d / 32;
    up.FR = 2 * (f / 16);
    up.NT = up.FR / GG_FROWS;
    up.KS_out = f / 32;
    up.C = 0;
    hipLaunchKernelGGL(gg_gemm_kernel<true>, dim3((unsigned)((up.NT * max_tiles + 7) / 8 * 8)), dim3(GG_THREADS),
                       lds_bytes, s, up);
    moe_record_mid_event(s);

    GroupedArgs dn;
    dn.wfrag = (const u32x4_t*)W->w2;
    dn.bfrag = hp;
    dn.offsets = offsets;
    dn.out = yg;
    dn.E = E; dn.N = N;
    dn.KS = f / 32;
    dn.FR = d / 16;
    dn.NT = dn.FR / GG_FROWS;
    dn.KS_out = 0;
    dn.C = d;
    hipLaunchKernelGGL(gg_gemm_kernel<false>, dim3((unsigned)((dn.NT * max_tiles + 7) / 8 * 8)), dim3(GG_THREADS),
                       lds_bytes, s, dn);
    return moe_launch_status();
}
