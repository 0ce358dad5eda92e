// Prefill-sized expert FFN for gfx950: grouped GEMM on the bf16 matrix cores.
//
// Both operands of v_mfma_f32_16x16x32_bf16 are kept in fragment order (see
// moe_internal.h): the packed weights are the A operand (16 output features x
// 32 reduction indices), and the activations are first re-laid into B-operand
// fragments (32 reduction indices x 16 token rows) per expert segment, padded
// with zero rows to a multiple of 16, so that no tile straddles two experts
// and the GEMM main loop has no bounds checks.  A fragment is 1 KiB: one
// wavefront moves it with a single coalesced 16-byte-per-lane access.
//
//   pack  : xg [N,d] (fp32 or bf16) -> xp fragments [block][d/32]
//   up    : per (token tile of 256 rows, 128 h-columns): a = x.w1, b = x.w3,
//           h = silu(a)*b written as bf16 straight into B-operand fragments
//           hp [block][f/32] for the second GEMM
//   down  : per (token tile of 256 rows, 256 output features): yg = h.w2, fp32
//
// GEMM kernel (measured figures behind it: one 256 x 256 x 32 step = 1024 matrix-core
// clocks per SIMD; four waves read ~140 B/clk from LDS and pull ~60 B/clk of L2-resident
// data per CU, more with more waves; the operand stream of this tile is 31 B/clk at the
// full matrix rate, 29 % of which misses L2):
//   * workgroup tile 256 tokens x 16 weight fragment rows, 4 waves, one per
//     SIMD; wave w owns fragment rows 4w..4w+3 for ALL 16 token blocks:
//     64 MFMA tiles = 256 accumulator registers (pinned to the accumulation
//     register file through the inline-asm constraint).
//   * weights (A) never touch LDS: each wave streams its own 4 fragments per
//     step straight from global memory into a 4-deep register ring (the
//     packed layout makes these 1 KiB coalesced loads with no redundancy
//     between waves).
//   * token fragments (B) are shared by the 4 waves through an 8-stage LDS ring
//     filled by direct-to-LDS loads (no staging registers, no LDS stores);
//     every wave reads the 16 B fragments of the next step while it issues the
//     64 MFMAs of the current one (single register set, refilled in place right
//     after its last use).  LDS traffic per step: 64 KiB reads + 16 KiB writes.
//   * the vector-memory requests (4 direct-to-LDS + 4 weight loads per wave
//     and step) and the 16 LDS reads are spread between the MFMAs, one barrier
//     per step publishes the next stage.
//   * the workgroup is persistent (one per CU) and the load stream runs across
//     tile boundaries: while the last steps of a tile are multiplied, the first
//     stages of the next tile are already being requested.
//   * tiles are walked in an order that keeps a weight tile on one XCD (one L2):
//     expert, then feature tile, then token tile, one contiguous eighth of that
//     order per XCD.
#include <atomic>

#include "moe_internal.h"
#include "moe_frag_pack.h"

// Tile shapes (token blocks of 16 rows x weight fragment rows of 16 features per workgroup;
// a wave owns all token blocks x FRW = fragment rows / 4; at most 64 MFMA tiles per wave):
//   16 x 16 (256 tokens x 256 features): the default;
//   12 x 16 (192 tokens x 256 features): 97..256 rows per expert on average, where a quarter
//           of the default tile's matrix work would be padding (measured 2-4 % faster);
//    8 x 32 (128 tokens x 512 features): experts with up to ~128 rows, where the default
//           tile is half empty -- twice the weight bytes per step, no padded matrix work.
#define GG_THREADS 256
#ifndef GG_NS
#define GG_NS 8            // LDS stages of B fragments (one KiB per token block each)
#endif
// The weight fragments of step k are requested GG_LA steps earlier into a register ring that
// is named statically, so the step loop is unrolled GG_U times (GG_LA < GG_U, reduction %
// GG_U == 0; GG_LA <= GG_NS - 3, see the waits in the step).  Deeper rings (8 / 5 with 8
// stages, 8 / 7 with 10 stages on the 192-row tile) measured no faster.
#ifndef GG_U
#define GG_U 4
#endif
#ifndef GG_LA
#define GG_LA 3
#endif
#ifndef GG_WIDE_MAX_ROWS
#define GG_WIDE_MAX_ROWS 96  // mean rows per expert up to which the 128 x 512 tile is used
#endif
#ifndef GG_R192_MAX_ROWS
#define GG_R192_MAX_ROWS 256  // ... and up to which the 192 x 256 tile is used
#endif

// ------------------------------------------------------------------- GEMM ----
struct GroupedArgs {
    const u32x4_t* wfrag;  // A operand: packed weights (w13 or w2)
    const u32x4_t* bfrag;  // B operand: packed activations (xp or hp)
    const int32_t* offsets;
    void* out;  // up: hp fragments (bf16); down: yg [N,d] fp32
    int E, N;
    int KS;      // reduction steps of 32
    int FR;      // weight fragment rows per expert (up: 2*f/16, down: d/16)
    int TB;      // token blocks (of 16 rows) per tile: 16 or 8
    int FROWS;   // weight fragment rows per tile: 16 or 32
    int NT;      // workgroup tiles along the features = FR / FROWS
    int KS_out;  // up: f/32 (fragment columns of hp); down: unused
    int C;       // down: d (row length of yg)
    int split;   // deal the left-over tiles of each XCD in pieces of their reduction
    float* part; // split: partial tiles [8 XCDs][workgroups per XCD][2][16*TB][16*FROWS] fp32
};

// s_waitcnt with only one counter constrained (gfx9 encoding: vmcnt = bits 3:0 and
// 15:14, expcnt = 6:4, lgkmcnt = 11:8; all-ones = no wait).
#define GG_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))
#define GG_WAIT_LGKM(n) __builtin_amdgcn_s_waitcnt(0xC07F | ((n) << 8))

struct TileInfo {
    SegInfo si;
    int tis;   // token tile inside the segment
    int nt;    // feature tile
    int blk0;  // first block of the tile inside the segment
    int nblk;  // blocks of the tile that exist (1..TB)
    // the part of the tile's reduction this unit of work covers (whole tile: 0, KS)
    int k_lo, klen;
    bool partial;
    int piece;  // 0 or 1: which of this workgroup's two partial-tile slots it writes
};

// Logical tiles of a launch: NT * sum_e ceil(M_e / (16 * TB)), in the order expert, then
// feature tile, then token tile (fastest), so that neighbouring indices share a weight tile.
// The experts' segments are decoded once per workgroup into a table in LDS
// (entry e: expert e; entries >= E hold no tiles).  A tile index is then decoded with LDS
// reads and a ballot -- no global memory access, and in particular no wait on the vector
// memory counter, which would also cover the operand loads in flight for the next tile.
#define GG_SEG_LO 0     // first row
#define GG_SEG_ROWS 1   // rows
#define GG_SEG_NB 2     // 16-row blocks
#define GG_SEG_TILES 3  // token tiles
#define GG_SEG_BASE 4   // first logical tile index
#define GG_SEG_BB 5     // first packed block
#define GG_SEG_FIELDS 6

// One wave fills the table (lane e: expert e); returns the number of logical tiles.
__device__ __forceinline__ int gg_seg_table(const int32_t* __restrict__ offsets, int E, int N,
                                            int NT, int TB, int lane, int (*tab)[64], bool write) {
    // offsets that do not ascend or leave [0, N] are clamped, as in the pack kernel:
    // lo_e = clamp(offsets[e], lo_{e-1}, N) = min(N, running max of offsets[0..e], at least 0);
    // hi_e = clamp(offsets[e+1], lo_e, N)
    const int o0 = (lane < E) ? offsets[lane] : 0, o1 = (lane < E) ? offsets[lane + 1] : 0;
    int run = o0 < 0 ? 0 : o0;
#pragma unroll
    for (int dlt = 1; dlt < 64; dlt <<= 1) {
        const int v = __shfl_up(run, dlt, 64);
        if (lane >= dlt) run = run > v ? run : v;
    }
    int lo = run > N ? N : run;
    int hi = o1 < lo ? lo : (o1 > N ? N : o1);
    if (lane >= E) {
        lo = 0;
        hi = 0;
    }
    const int rows = hi - lo, nb = (rows + 15) / 16, tiles = (nb + TB - 1) / TB;
    int inc_t = tiles * NT, inc_b = nb;
#pragma unroll
    for (int dlt = 1; dlt < 64; dlt <<= 1) {
        const int vt = __shfl_up(inc_t, dlt, 64), vb = __shfl_up(inc_b, dlt, 64);
        if (lane >= dlt) {
            inc_t += vt;
            inc_b += vb;
        }
    }
    if (write) {
        tab[GG_SEG_LO][lane] = lo;
        tab[GG_SEG_ROWS][lane] = rows;
        tab[GG_SEG_NB][lane] = nb;
        tab[GG_SEG_TILES][lane] = tiles;
        tab[GG_SEG_BASE][lane] = inc_t - tiles * NT;
        tab[GG_SEG_BB][lane] = inc_b - nb;
    }
    return __builtin_amdgcn_readlane(inc_t, 63);
}

// Logical tile index -> tile, from the table.
__device__ __forceinline__ bool gg_decode_tile_tab(const int (*tab)[64], int lane, int NT, int TB,
                                                   int L, TileInfo& ti) {
    const int my_tiles = tab[GG_SEG_TILES][lane], my_base = tab[GG_SEG_BASE][lane];
    const unsigned long long m = __ballot(my_tiles > 0 && L >= my_base && L < my_base + my_tiles * NT);
    if (m == 0ull) return false;
    const int e = __builtin_amdgcn_readfirstlane((int)__builtin_ctzll(m));
    const int tiles = __builtin_amdgcn_readfirstlane(tab[GG_SEG_TILES][e]);
    const int nb = __builtin_amdgcn_readfirstlane(tab[GG_SEG_NB][e]);
    const int r = L - __builtin_amdgcn_readfirstlane(tab[GG_SEG_BASE][e]);
    ti.nt = r / tiles;
    ti.tis = r % tiles;
    ti.si.e = e;
    ti.si.row0 = __builtin_amdgcn_readfirstlane(tab[GG_SEG_LO][e]);
    ti.si.rows = __builtin_amdgcn_readfirstlane(tab[GG_SEG_ROWS][e]);
    ti.si.bbase = __builtin_amdgcn_readfirstlane(tab[GG_SEG_BB][e]);
    ti.blk0 = ti.tis * TB;
    ti.nblk = (nb - ti.blk0) < TB ? (nb - ti.blk0) : TB;
    ti.k_lo = 0;
    ti.klen = 0;  // filled in by the caller
    ti.partial = false;
    ti.piece = 0;
    return true;
}

// Cut points of the left-over tiles' joint reduction (S = R tiles x KS steps) for the
// workgroups of one XCD: workgroup j covers [cut(j), cut(j+1)).  Pieces are multiples of
// `unit` steps (KS is one too) and no piece is shorter than the smallest multiple of `unit`
// that covers the `ns` LDS stages of the kernel's pipeline.
__device__ __forceinline__ int gg_piece_cut(int j, int S, int KS, int wgs, int unit, int ns) {
    const int minp = (ns + unit - 1) / unit * unit;
    int per = ((S + wgs - 1) / wgs + unit - 1) / unit * unit;
    per = per < 32 ? 32 : per;
    const int c = j * per;
    if (c >= S) return S;
    const int r = c % KS;
    if (r < minp) return c - r;
    if (KS - r < minp) return c + (KS - r);
    return c;
}

// Weight fragment load.  ANT: non-temporal - when nearly every expert has a single token
// tile its weights are read once and should not push the token fragments (re-read by every
// feature tile) out of L2.  Measured, 8 layers of the Mixtral shape, balanced routing:
// 128 x 512 tile T=256 5.16 -> 4.65 ms, T=384 5.44 -> 4.88; 192 x 256 tile T=512 5.44 -> 5.22
// but T=1024 8.10 -> 9.17 (experts with two tiles then re-read their weights from HBM
// instead of L2), hence the rule in gg_weights_read_once.
template <bool ANT>
__device__ __forceinline__ u32x4_t gg_ld_a(const u32x4_t* p) {
    return ANT ? __builtin_nontemporal_load(p) : *p;
}

// The lane number, recomputed where it is used and invisible to the optimiser (which would
// otherwise share it with the copy made at kernel start and keep that alive, or derive
// per-lane addresses from it ahead of the main loop).
__device__ __forceinline__ int gg_lane_opaque() {
    int l;
    asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(l));
    return l;
}

// MFMA with the accumulator pinned to the accumulation registers: 256 of them
// are live per wave, and left to itself the register allocator shuffles them
// through the vector registers inside the loop.
__device__ __forceinline__ void gg_mfma(f32x4_t& c, const u32x4_t& a, const bf16x8_t& b) {
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
}

// Global source pointers of one tile for this wave (all wave-uniform).
template <int FRW, int NBQ>
struct TileSrc {
    const u32x4_t* a[FRW];  // this wave's weight fragment rows (start of the reduction)
    const u32x4_t* b[NBQ];  // the token blocks this wave requests into LDS
};

template <int FRW, int NBQ>
__device__ __forceinline__ void gg_tile_src(const GroupedArgs& a, const TileInfo& ti, int wave,
                                            TileSrc<FRW, NBQ>& ts) {
#pragma unroll
    for (int j = 0; j < FRW; j++)
        ts.a[j] = a.wfrag +
                  (((size_t)ti.si.e * a.FR + (size_t)ti.nt * (4 * FRW) + FRW * wave + j) * a.KS + ti.k_lo) * 64;
#pragma unroll
    for (int i = 0; i < NBQ; i++) {
        int blk = NBQ * wave + i;
        blk = blk < ti.nblk ? blk : ti.nblk - 1;  // clamp: every wave always issues NBQ requests
        ts.b[i] = a.bfrag + (((size_t)(ti.si.bbase + ti.blk0 + blk)) * a.KS + ti.k_lo) * 64;
    }
}

// MODE: which units of work a launch covers: 0 = whole tiles and pieces (second projection:
// one epilogue serves both), 1 = whole tiles only, 2 = pieces only (the first projection
// takes two launches, because an epilogue with both the SiLU*mul body and the raw store of
// partial sums makes the compiler spill ~150 accumulators per tile).
// NBW x FRW: token blocks of the tile x fragment rows of a wave (16 x 4 or 8 x 8).
template <bool UP, int NBW, int FRW, int MODE, int U, int LA, int NS, bool ANT>
__device__ __forceinline__ void gg_gemm_body(const GroupedArgs& a) {
    static_assert(NBW * FRW <= 64 && NBW % 4 == 0, "at most 64 MFMA tiles (256 accumulators) per wave");
    static_assert(LA < U && LA <= NS - 3, "ring and stage depths, see the waits in the step");
    constexpr int FROWS = 4 * FRW;     // fragment rows of the workgroup tile
    constexpr int NBQ = NBW / 4;       // token blocks each wave requests into LDS per step
    constexpr int VREQ = FRW + NBQ;    // vector-memory requests per wave and step
    extern __shared__ __align__(16) unsigned char smem[];
    u32x4_t* lds = (u32x4_t*)smem;  // [NS stages][NBW fragments][64 lanes]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // fragment rows [FRW*wave, +FRW)
    const unsigned voff = (unsigned)lane * 16u;                  // byte offset inside a fragment

    // This workgroup's units of work.  The logical tiles of XCD x are x*per_xcd ... ; the
    // 32 workgroups of an XCD take them round-robin (slot = id/8, id/8 + wgs, ...).  When
    // the tile count is not a multiple of the workgroup count the last round would leave
    // most CUs idle (576 second-projection tiles over 256 CUs = 2.25 rounds), so the
    // left-over tiles are cut along the reduction instead, in equal pieces for all
    // workgroups; every piece stores its partial sums into scratch and gg_fixup_kernel adds
    // the pieces of a tile in a fixed order (then applies SiLU*mul, first projection).
    __shared__ int s_seg[GG_SEG_FIELDS][64];
    const int total = gg_seg_table(a.offsets, a.E, a.N, a.NT, NBW, lane, s_seg, wave == 0);
    __syncthreads();
    const int per_xcd = (total + 7) / 8;
    const int xcd = blockIdx.x & 7;
    const int wgs = gridDim.x >> 3;
    const int me = blockIdx.x >> 3;
    int chunk = total - xcd * per_xcd;
    chunk = chunk < 0 ? 0 : (chunk > per_xcd ? per_xcd : chunk);  // tiles of this XCD
    const bool split = a.split && (chunk % wgs) != 0;
    const int n_full = split ? chunk / wgs : (chunk - me + wgs - 1) / wgs;  // whole tiles I own
    // pieces of the left-over tiles (slots n_full*wgs ... chunk-1) for this workgroup
    // (plain scalars, no arrays: an array indexed at run time would live in scratch memory, and
    // every read of it would wait on the counter of the operand loads in flight)
    int pc_tile0 = 0, pc_lo0 = 0, pc_len0 = 0, pc_tile1 = 0, pc_len1 = 0, n_pieces = 0;
    if (split) {
        const int R = chunk - n_full * wgs;
        const int S = R * a.KS;
        const int c0 = gg_piece_cut(me, S, a.KS, wgs, U, NS), c1 = gg_piece_cut(me + 1, S, a.KS, wgs, U, NS);
        if (c0 < c1) {
            const int rA = c0 / a.KS;
            const int endA = c1 < (rA + 1) * a.KS ? c1 : (rA + 1) * a.KS;
            pc_tile0 = rA; pc_lo0 = c0 - rA * a.KS; pc_len0 = endA - c0;
            n_pieces = 1;
            if (c1 > endA) {
                pc_tile1 = rA + 1; pc_len1 = c1 - endA;  // starts at step 0 of its tile
                n_pieces = 2;
            }
        }
    }
    // uniform values, pinned to scalar registers (the compiler otherwise keeps them in a table
    // in scratch memory for the selection below)
    pc_tile0 = __builtin_amdgcn_readfirstlane(pc_tile0);
    pc_lo0 = __builtin_amdgcn_readfirstlane(pc_lo0);
    pc_len0 = __builtin_amdgcn_readfirstlane(pc_len0);
    pc_tile1 = __builtin_amdgcn_readfirstlane(pc_tile1);
    pc_len1 = __builtin_amdgcn_readfirstlane(pc_len1);
    n_pieces = __builtin_amdgcn_readfirstlane(n_pieces);
    const int n_units = (MODE == 1) ? n_full : n_full + n_pieces;
    auto unit_at = [&](int n, TileInfo& ti) -> bool {
        if (n >= n_units) return false;
        int sl, lo = 0, len = a.KS;
        if (n < n_full) {
            sl = me + n * wgs;
        } else {
            // first or second piece, selected by arithmetic (a two-way choice on n is turned
            // into a table in scratch memory by the compiler)
            const int first = (n == n_full) ? 1 : 0;
            sl = n_full * wgs + pc_tile1 + first * (pc_tile0 - pc_tile1);
            lo = first * pc_lo0;
            len = pc_len1 + first * (pc_len0 - pc_len1);
        }
        // (the lane number is recomputed here, opaquely, so that no address derived from it
        // has to stay in a register through the main loop; see the epilogue)
        const int lane_d = gg_lane_opaque();
        if (!gg_decode_tile_tab(s_seg, lane_d, a.NT, NBW, xcd * per_xcd + sl, ti)) return false;
        ti.k_lo = lo;
        ti.klen = len;
        ti.partial = (n >= n_full);  // pieces always go through scratch and the fix-up
        ti.piece = n < n_full ? 0 : n - n_full;
        return true;
    };

    int unit = (MODE == 2) ? n_full : 0;
    TileInfo cur, nxt;
    if (!unit_at(unit, cur)) return;
    bool has_next = unit_at(unit + 1, nxt);
    TileSrc<FRW, NBQ> scur, snxt;
    gg_tile_src(a, cur, wave, scur);
    if (has_next) gg_tile_src(a, nxt, wave, snxt); else snxt = scur;
    int KT = cur.klen;  // steps of the current unit: a multiple of U, >= NS

    // look-ahead sources: reduction step j of the current tile, or j-KT of the next one
    auto b_src = [&](int i, int j) -> const char* {
        const u32x4_t* p = (j < KT) ? scur.b[i] + (size_t)j * 64 : snxt.b[i] + (size_t)(j - KT) * 64;
        return (const char*)p + voff;
    };
    auto a_src = [&](int jr, int j) -> const u32x4_t* {
        const u32x4_t* p = (j < KT) ? scur.a[jr] + (size_t)j * 64 : snxt.a[jr] + (size_t)(j - KT) * 64;
        return (const u32x4_t*)((const char*)p + voff);
    };
    // g = running step count of this workgroup (never reset): LDS stage g % NS
    auto issue_b = [&](int i, int j, unsigned gstage) {
        __builtin_amdgcn_global_load_lds(
            (const __attribute__((address_space(1))) void*)b_src(i, j),
            (__attribute__((address_space(3))) void*)(lds + ((gstage % NS) * NBW + NBQ * wave + i) * 64),
            16, 0, 0);
    };

    f32x4_t acc[NBW][FRW];
    u32x4_t areg[U][FRW];
    bf16x8_t breg[NBW];

    // ---- prologue of the first tile: request stages 0..NS-2 and A of steps 0..PA-2 ----
    for (int j = 0; j < NS - 1; j++)
#pragma unroll
        for (int i = 0; i < NBQ; i++) issue_b(i, j, j);
#pragma unroll
    for (int s = 0; s < LA; s++)
#pragma unroll
        for (int j = 0; j < FRW; j++) areg[s][j] = gg_ld_a<ANT>(a_src(j, s));
    GG_WAIT_VMCNT(0);
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int i = 0; i < NBW; i++) breg[i] = __builtin_bit_cast(bf16x8_t, lds[i * 64 + lane]);
    GG_WAIT_LGKM(0);

    unsigned g = 0;  // running step count (unsigned: g % NS is a mask for the 8-stage ring)
    for (;;) {
#pragma unroll
        for (int i = 0; i < NBW; i++)
#pragma unroll
            for (int j = 0; j < FRW; j++) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        // the compiler cannot see the MFMAs below: cover the register write -> matrix read hazard
        asm volatile("s_nop 7" ::: "memory");

        // One reduction step.  Ac: weight fragments of this step; An: ring slot that
        // receives the fragments of step k+LA.  fast: every look-ahead lies inside
        // the current tile, so there is nothing to decide (compile-time after inlining).
        auto step = [&](int k, u32x4_t(&Ac)[FRW], u32x4_t(&An)[FRW], const bool fast) {
            // The look-ahead requests carry no condition: behind the workgroup's last unit they
            // re-read the first steps of that unit (snxt == scur then), into stages and
            // registers that nothing reads any more.  With conditions the compiler cannot
            // count the loads in flight and waits for all of them before the weights' use.
            constexpr bool la_b = true, la_a = true, more = true;
            // The weights of step k were requested LA steps ago, after that step's requests
            // for stage k+NS-1-LA; requests retire in order, so with at most the last
            // LA-1 steps' worth still in flight they have arrived, and so have the stages
            // requested before them (LA <= NS-3: up to stage k+2).
            GG_WAIT_VMCNT((LA - 1) * VREQ);
            // One barrier per TWO steps: at an even step every wave has waited for its
            // shares of stages k+1 and k+2 (see above), so both are published here; and the
            // buffers refilled during steps k and k+1 (stages k-1 and k) were last read
            // before this barrier.
            if (more && (k & 1) == 0) __builtin_amdgcn_s_barrier();
            const u32x4_t* pb = lds + ((g + 1) % NS) * NBW * 64 + lane;
            // request number v of this step: 0..NBQ-1 = this wave's blocks of stage k+NS-1
            // (straight into LDS), NBQ.. = its FRW weight fragments of step k+LA
            auto issue = [&](const int v) {
                    if (v < NBQ) {
                        if (fast) {
                            __builtin_amdgcn_global_load_lds(
                                (const __attribute__((address_space(1))) void*)(
                                    (const char*)(scur.b[v] + (size_t)(k + NS - 1) * 64) + voff),
                                (__attribute__((address_space(3))) void*)(
                                    lds + (((g + NS - 1) % NS) * NBW + NBQ * wave + v) * 64),
                                16, 0, 0);
                        } else if (la_b) {
                            issue_b(v, k + NS - 1, g + NS - 1);
                        }
                    } else {
                        if (fast)
                            An[v - NBQ] = gg_ld_a<ANT>((const u32x4_t*)((const char*)(scur.a[v - NBQ] +
                                                            (size_t)(k + LA) * 64) + voff));
                        else if (la_a)
                            An[v - NBQ] = gg_ld_a<ANT>(a_src(v - NBQ, k + LA));
                    }
            };
#pragma unroll
            for (int i = 0; i < NBW; i++) {
                // the vector-memory requests are spread evenly over the blocks (one per
                // 8 MFMAs for 16 x 4), so that the requests of the four waves never
                // queue up in front of the matrix instructions
#pragma unroll
                for (int v = (i * VREQ + NBW - 1) / NBW; v < ((i + 1) * VREQ + NBW - 1) / NBW; v++)
                    issue(v);
                // LDS reads return in order: with at most NBW-2 younger ones in flight,
                // breg[i] and breg[i+1] (refilled one step ago) have arrived
                if ((i & 1) == 0) GG_WAIT_LGKM(NBW - 2);
#pragma unroll
                for (int j = 0; j < FRW; j++) gg_mfma(acc[i][j], Ac[j], breg[i]);
                if (more) breg[i] = __builtin_bit_cast(bf16x8_t, pb[i * 64]);
            }
            g++;
        };
        // steps whose look-aheads (k+NS-1 at most) stay inside this tile: no conditions
        const int k_fast = ((KT - NS + 1) / U) * U;
        int k = 0;
        for (; k < k_fast; k += U) {
#pragma unroll
            for (int u = 0; u < U; u++) step(k + u, areg[u], areg[(u + LA) % U], true);
        }
        for (; k < KT; k += U) {
#pragma unroll
            for (int u = 0; u < U; u++) step(k + u, areg[u], areg[(u + LA) % U], false);
        }

        // ---- epilogue of the current tile (the next tile's loads are in flight) ----
        // the compiler cannot see the MFMAs: cover the matrix-core write -> read hazard
        asm volatile("s_nop 15\n s_nop 15" ::: "memory");
        // The epilogue's per-lane addresses are derived from a copy of the lane number that the
        // compiler cannot trace back to the one above: it would otherwise compute them before
        // the main loop and keep them in registers through it -- registers the loop does not
        // have (the reload of a spilled one is a scratch load, and the wait for it also covers
        // every store of the epilogue and every operand load of the next tile).
        const int lane_e = gg_lane_opaque();
        const int t = lane_e & 15, fq = lane_e >> 4;  // token in block, feature quad
        // a piece's partial sums: [16*NBW rows][16*FROWS columns] fp32 in this workgroup's slot
        float* slot = a.part + (((size_t)xcd * wgs + me) * 2 + cur.piece) * (256 * 256) +
                      (size_t)t * (16 * FROWS) + (FRW * wave) * 16 + 4 * fq;
        if (UP && MODE == 2) {
            // piece of a tile: raw partial sums to scratch; the fix-up kernel adds the
            // pieces and applies SiLU*mul
#pragma unroll
            for (int i = 0; i < NBW; i++) {
                if (i >= cur.nblk) continue;
#pragma unroll
                for (int j = 0; j < FRW; j++)
                    *(float4*)(slot + (size_t)i * 16 * (16 * FROWS) + j * 16) =
                        make_float4(acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]);
            }
        } else if (UP) {
#pragma unroll
            for (int i = 0; i < NBW; i++) {
                if (i >= cur.nblk) continue;
                const int blk = cur.blk0 + i;  // block inside the segment
                // fragment rows FRW*wave+j: j even = w1 rows, j odd = w3 rows of the same columns
#pragma unroll
                for (int jj = 0; jj < FRW / 2; jj++) {
                    const f32x4_t av = acc[i][2 * jj], bv = acc[i][2 * jj + 1];
                    float hv[4];
#pragma unroll
                    for (int r = 0; r < 4; r++) hv[r] = av[r] / (1.0f + __expf(-av[r])) * bv[r];
                    const int colblk = cur.nt * (FROWS / 2) + (FRW / 2) * wave + jj;  // 16 h-columns
                    const int ks_o = colblk >> 1;
                    const int lane_o = ((colblk & 1) * 2 + (fq >> 1)) * 16 + t;
                    uint2 pk;
                    pk.x = moe_pack_bf16x2(hv[0], hv[1]);
                    pk.y = moe_pack_bf16x2(hv[2], hv[3]);
                    unsigned char* dst =
                        (unsigned char*)a.out +
                        (((size_t)(cur.si.bbase + blk) * a.KS_out + ks_o) * 64 + lane_o) * 16 +
                        (fq & 1) * 8;
                    *(uint2*)dst = pk;
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < NBW; i++) {
                if (i >= cur.nblk) continue;
                const int blk = cur.blk0 + i;  // block inside the segment
                // whole tiles go to yg; pieces of a tile to this workgroup's scratch slot
                // (same code, only the destination differs)
                const int r_in_seg = blk * 16 + t;
                if (r_in_seg < cur.si.rows) {
                    float* row = cur.partial ? slot + (size_t)i * 16 * (16 * FROWS)
                                             : (float*)a.out + (size_t)(cur.si.row0 + r_in_seg) * a.C +
                                                   (cur.nt * FROWS + FRW * wave) * 16 + 4 * fq;
#pragma unroll
                    for (int j = 0; j < FRW; j++)
                        *(float4*)(row + j * 16) =
                            make_float4(acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]);
                }
            }
        }
        if (!has_next) {
            // the unconditional look-ahead of the last steps is still in flight (some of it on
            // its way into LDS): it must land before the workgroup gives its LDS back
            GG_WAIT_VMCNT(0);
            break;
        }
        // advance: next becomes current; look one unit further ahead
        unit++;
        cur = nxt;
        scur = snxt;
        KT = cur.klen;
        has_next = unit_at(unit + 1, nxt);
        if (has_next) gg_tile_src(a, nxt, wave, snxt);
        GG_WAIT_LGKM(0);  // scalar loads of the decode must not sit in the LDS read counter
    }
}

// Are the weights of (nearly) every expert read by a single token tile?  Then they are
// streamed.  The rule: token tiles beyond the first of an expert make up at most 15 % of all
// token tiles (measured crossover: 11 % wins 8 %, 20 % loses 4 %, 50 % loses 13 %).
__device__ __forceinline__ bool gg_weights_read_once(const int32_t* __restrict__ offsets, int E,
                                                     int N, int TB) {
    int tiles = 0, active = 0, prev = 0;
    for (int e = 0; e < E; e++) {
        const int lo = gg_clamp_off(offsets[e], prev, N);
        const int hi = gg_clamp_off(offsets[e + 1], lo, N);
        prev = lo;
        tiles += (hi - lo + 16 * TB - 1) / (16 * TB);
        active += (hi > lo) ? 1 : 0;
    }
    return (tiles - active) * 100 <= 15 * tiles;
}

// The two load flavours are two copies of the whole persistent loop: nothing is live across
// the choice (a choice per tile inside one loop made the compiler spill the accumulators).
template <bool UP, int NBW, int FRW, int MODE, int U, int LA, int NS>
__global__ __launch_bounds__(GG_THREADS) void gg_gemm_kernel(GroupedArgs a) {
    // (the 256-token tile is chosen above 256 rows per expert, where the rule never holds)
    if (NBW < 16 && gg_weights_read_once(a.offsets, a.E, a.N, NBW))
        gg_gemm_body<UP, NBW, FRW, MODE, U, LA, NS, true>(a);
    else
        gg_gemm_body<UP, NBW, FRW, MODE, U, LA, NS, false>(a);
}

// Adds the pieces of every left-over tile in the order of the workgroups that produced them
// (deterministic), then writes yg (second projection) or applies SiLU*mul and writes the h
// fragments (first projection).  blockIdx.x = (XCD, left-over tile), blockIdx.y = group of
// 16 rows of the tile; every workgroup recomputes the cut points the GEMM workgroups used.
// FROWS = fragment rows of the tile shape (16 or 32); a.TB = its token blocks.
#define GG_FIX_ROWS 16
template <bool UP, int FROWS>
__global__ __launch_bounds__(256) void gg_fixup_kernel(GroupedArgs a, int wgs, int unit, int ns) {
    __shared__ int s_slot[64];
    __shared__ int s_n;
    constexpr int RS = 16 * FROWS;  // floats per row of a partial tile
    const int xcd = blockIdx.x / wgs, r = blockIdx.x % wgs;
    // the segment table as in the GEMM: one parallel read of the offsets and two wave scans
    // instead of a walk over the experts with one memory round trip each (most workgroups of
    // this grid find nothing to do and should find out quickly)
    __shared__ int s_seg[GG_SEG_FIELDS][64];
    const int lane = threadIdx.x & 63;
    const int total = gg_seg_table(a.offsets, a.E, a.N, a.NT, a.TB, lane, s_seg, threadIdx.x < 64);
    const int per_xcd = (total + 7) / 8;
    int chunk = total - xcd * per_xcd;
    chunk = chunk < 0 ? 0 : (chunk > per_xcd ? per_xcd : chunk);
    if (chunk % wgs == 0) return;   // (uniform over the workgroup, as the returns below)
    const int n_full = chunk / wgs;
    const int R = chunk - n_full * wgs;
    if (r >= R) return;
    __syncthreads();
    TileInfo ti;
    if (!gg_decode_tile_tab(s_seg, lane, a.NT, a.TB, xcd * per_xcd + n_full * wgs + r, ti)) return;
    // second projection: the tile's real rows; first: every row of its blocks (h is kept in
    // whole 16-row fragments, padding rows included)
    const int tile_max = 16 * a.TB;
    const int tile_rows = UP ? ti.nblk * 16
                             : ((ti.si.rows - ti.blk0 * 16) < tile_max ? (ti.si.rows - ti.blk0 * 16)
                                                                       : tile_max);
    const int row_lo = blockIdx.y * GG_FIX_ROWS;
    if (row_lo >= tile_rows) return;
    // lane j of the first wave looks at workgroup j's cut: it holds at most one piece of
    // this tile; a ballot keeps the pieces in workgroup order (wgs <= 64)
    if (threadIdx.x < 64) {
        const int j = threadIdx.x;
        const int S = R * a.KS;
        int slot = -1;
        if (j < wgs) {
            const int c0 = gg_piece_cut(j, S, a.KS, wgs, unit, ns),
                      c1 = gg_piece_cut(j + 1, S, a.KS, wgs, unit, ns);
            if (c0 < c1) {
                const int rA = c0 / a.KS;
                const int endA = c1 < (rA + 1) * a.KS ? c1 : (rA + 1) * a.KS;
                if (rA == r) slot = (xcd * wgs + j) * 2 + 0;
                else if (c1 > endA && rA + 1 == r) slot = (xcd * wgs + j) * 2 + 1;
            }
        }
        const unsigned long long m = __ballot(slot >= 0);
        const unsigned long long below = (j == 0) ? 0ull : (~0ull >> (64 - j));
        if (slot >= 0) s_slot[__popcll(m & below)] = slot;
        if (j == 0) s_n = __popcll(m);
    }
    __syncthreads();
    const int n = s_n;
    const int rows = (tile_rows - row_lo) < GG_FIX_ROWS ? (tile_rows - row_lo) : GG_FIX_ROWS;
    if (UP) {
        // item = (row, block of 16 h-columns cb, feature quad fq): a = x.w1 from fragment
        // row 2cb, b = x.w3 from fragment row 2cb+1, four columns each
        constexpr int PER_ROW = (FROWS / 2) * 4;
        constexpr int IT = GG_FIX_ROWS * PER_ROW / 256;
        float4 sa[IT], sb[IT];
        const float* src[IT];
#pragma unroll
        for (int it = 0; it < IT; it++) {
            const int idx = it * 256 + threadIdx.x;
            const int rr = (idx / PER_ROW) < rows ? (idx / PER_ROW) : 0;
            const int cb = (idx >> 2) % (FROWS / 2), fq = idx & 3;
            src[it] = a.part + (size_t)(row_lo + rr) * RS + (2 * cb) * 16 + 4 * fq;
            sa[it] = make_float4(0.f, 0.f, 0.f, 0.f);
            sb[it] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
        for (int p = 0; p < n; p++) {
            const size_t base = (size_t)s_slot[p] * 256 * 256;
            float4 va[IT], vb[IT];
#pragma unroll
            for (int it = 0; it < IT; it++) {
                va[it] = *(const float4*)(src[it] + base);
                vb[it] = *(const float4*)(src[it] + base + 16);
            }
#pragma unroll
            for (int it = 0; it < IT; it++) {
                sa[it].x += va[it].x; sa[it].y += va[it].y; sa[it].z += va[it].z; sa[it].w += va[it].w;
                sb[it].x += vb[it].x; sb[it].y += vb[it].y; sb[it].z += vb[it].z; sb[it].w += vb[it].w;
            }
        }
#pragma unroll
        for (int it = 0; it < IT; it++) {
            const int idx = it * 256 + threadIdx.x;
            if ((idx / PER_ROW) >= rows) continue;
            const int row = row_lo + idx / PER_ROW, cb = (idx >> 2) % (FROWS / 2), fq = idx & 3;
            const float av[4] = {sa[it].x, sa[it].y, sa[it].z, sa[it].w};
            const float bv[4] = {sb[it].x, sb[it].y, sb[it].z, sb[it].w};
            float hv[4];
#pragma unroll
            for (int q = 0; q < 4; q++) hv[q] = av[q] / (1.0f + __expf(-av[q])) * bv[q];
            // same fragment address as the first projection's own epilogue
            const int blk = ti.blk0 + (row >> 4), t = row & 15;
            const int colblk = ti.nt * (FROWS / 2) + cb;
            const int ks_o = colblk >> 1;
            const int lane_o = ((colblk & 1) * 2 + (fq >> 1)) * 16 + t;
            uint2 pk;
            pk.x = moe_pack_bf16x2(hv[0], hv[1]);
            pk.y = moe_pack_bf16x2(hv[2], hv[3]);
            *(uint2*)((unsigned char*)a.out +
                      (((size_t)(ti.si.bbase + blk) * a.KS_out + ks_o) * 64 + lane_o) * 16 +
                      (fq & 1) * 8) = pk;
        }
    } else {
        constexpr int PER_ROW = RS / 4;                      // float4 per row
        constexpr int IT = GG_FIX_ROWS * PER_ROW / 256;      // float4 per thread
        float4 sum[IT];
        const float* src[IT];
#pragma unroll
        for (int it = 0; it < IT; it++) {
            const int idx = it * 256 + threadIdx.x;
            // rows past the end of the tile read row 0 of the group instead (never stored)
            const int row = row_lo + ((idx / PER_ROW) < rows ? (idx / PER_ROW) : 0);
            src[it] = a.part + (size_t)row * RS + (idx % PER_ROW) * 4;
            sum[it] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
        for (int p = 0; p < n; p++) {
            const size_t base = (size_t)s_slot[p] * 256 * 256;
            float4 v[IT];
#pragma unroll
            for (int it = 0; it < IT; it++) v[it] = *(const float4*)(src[it] + base);
#pragma unroll
            for (int it = 0; it < IT; it++) {
                sum[it].x += v[it].x; sum[it].y += v[it].y; sum[it].z += v[it].z; sum[it].w += v[it].w;
            }
        }
#pragma unroll
        for (int it = 0; it < IT; it++) {
            const int idx = it * 256 + threadIdx.x;
            if ((idx / PER_ROW) < rows)
                *(float4*)((float*)a.out +
                           (size_t)(ti.si.row0 + ti.blk0 * 16 + row_lo + idx / PER_ROW) * a.C +
                           ti.nt * FROWS * 16 + (idx % PER_ROW) * 4) = sum[it];
        }
    }
}

// ---------------------------------------------------------------- host side ----
static inline size_t gg_align256(size_t v) { return (v + 255) & ~(size_t)255; }
static inline size_t gg_max_blocks(int N, int E) { return (size_t)N / 16 + E; }

// scratch for the partial tiles of the second projection: 2 slots of 256 x 256 fp32 per
// persistent workgroup (one workgroup per CU, rounded up to a multiple of 8)
static inline size_t gg_part_bytes() {
    return (size_t)((moe_num_cus() + 7) / 8 * 8) * 2 * 256 * 256 * sizeof(float);
}

size_t moe_ffn_grouped_workspace(int N, int E, int d, int f) {
    const size_t nb = gg_max_blocks(N, E);
    return gg_align256(nb * 16 * d * 2) + gg_align256(nb * 16 * f * 2) + gg_part_bytes();
}

// Kernel variants by rows per expert (see the tile shapes at the top of the file): token
// blocks and fragment rows of the tile, unroll / weight look-ahead / LDS stages of the loop.
enum GgVariant { GG_STD = 0, GG_WIDE = 1, GG_R192 = 2, GG_NVARIANTS = 3 };
struct GgShape { int tb, frows, u, la, ns; };
static GgShape gg_shape(GgVariant v) {
    switch (v) {
        case GG_WIDE: return {8, 32, GG_U, GG_LA, GG_NS};
        case GG_R192: return {12, 16, GG_U, GG_LA, GG_NS};
        default: return {16, 16, GG_U, GG_LA, GG_NS};
    }
}

template <bool UP, int MODE>
static const void* gg_kernel_ptr(GgVariant v) {
    switch (v) {
        case GG_WIDE: return (const void*)gg_gemm_kernel<UP, 8, 8, MODE, GG_U, GG_LA, GG_NS>;
        case GG_R192: return (const void*)gg_gemm_kernel<UP, 12, 4, MODE, GG_U, GG_LA, GG_NS>;
        default: return (const void*)gg_gemm_kernel<UP, 16, 4, MODE, GG_U, GG_LA, GG_NS>;
    }
}

// One projection: the persistent GEMM (whole tiles; for the first projection the pieces of
// the left-over tiles are a second launch) and the fix-up of the pieces.
template <bool UP>
static int gg_launch_projection(GroupedArgs& a, GgVariant v, unsigned pgrid, hipStream_t s) {
    const GgShape sh = gg_shape(v);
    a.TB = sh.tb;
    a.FROWS = sh.frows;
    if (a.FR % a.FROWS != 0) return MOE_ERR_UNSUPPORTED;
    a.NT = a.FR / a.FROWS;
    // pieces of >= 32 steps go to scratch and a fix-up kernel adds them; it lists the pieces
    // of a tile with one wave, hence at most 64 workgroups per XCD
    a.split = (a.KS >= 64 && pgrid / 8 <= 64) ? 1 : 0;
    void* params[1] = {(void*)&a};
    const size_t lds_bytes = (size_t)sh.ns * a.TB * MOE_FRAG_BYTES;
    if (UP) {
        MOE_HIP_TRY(hipLaunchKernel(gg_kernel_ptr<true, 1>(v), dim3(pgrid), dim3(GG_THREADS), params,
                                    lds_bytes, s));
        if (a.split)
            MOE_HIP_TRY(hipLaunchKernel(gg_kernel_ptr<true, 2>(v), dim3(pgrid), dim3(GG_THREADS),
                                        params, lds_bytes, s));
    } else {
        MOE_HIP_TRY(hipLaunchKernel(gg_kernel_ptr<false, 0>(v), dim3(pgrid), dim3(GG_THREADS), params,
                                    lds_bytes, s));
    }
    if (a.split) {
        const dim3 fgrid(pgrid, (unsigned)a.TB);
        if (a.FROWS == 32)
            hipLaunchKernelGGL((gg_fixup_kernel<UP, 32>), fgrid, dim3(256), 0, s, a, (int)(pgrid / 8),
                               sh.u, sh.ns);
        else
            hipLaunchKernelGGL((gg_fixup_kernel<UP, 16>), fgrid, dim3(256), 0, s, a, (int)(pgrid / 8),
                               sh.u, sh.ns);
    }
    return MOE_OK;
}

// Variant of each projection by the mean number of rows per expert (the host never sees the
// real counts): up to GG_WIDE_MAX_ROWS the 128-token x 512-feature tile (needs f % 256 == 0
// for the first projection, d % 512 == 0 for the second; each falls back on its own), up to
// GG_R192_MAX_ROWS the 192-token x 256-feature one, above that 256 x 256.
static bool gg_choose(int N, int E, int d, int f, GgVariant& vu, GgVariant& vd) {
    // up tile = 16 fragment rows = 8 column blocks x (w1,w3): f % 128 == 0;
    // down tile = 256 features: d % 256 == 0; both give reductions of >= 8 steps, step
    // counts that are multiples of 4.
    if (f % 128 != 0 || d % 256 != 0) return false;
    const long long mean_rows = ((long long)N + E - 1) / E;
    vu = vd = GG_STD;
    if (mean_rows <= GG_WIDE_MAX_ROWS) {
        if (f % 256 == 0) vu = GG_WIDE;
        if (d % 512 == 0) vd = GG_WIDE;
    } else if (mean_rows <= GG_R192_MAX_ROWS) {
        vu = vd = GG_R192;
    }
    // the step loop is unrolled u times and looks ns-1 steps ahead: a variant whose loop does
    // not fit a reduction gives way to the standard one
    auto fits = [&](GgVariant v, int ks) {
        const GgShape sh = gg_shape(v);
        return ks % sh.u == 0 && ks >= sh.ns;
    };
    if (!fits(vu, d / 32)) vu = GG_STD;
    if (!fits(vd, f / 32)) vd = GG_STD;
    return fits(vu, d / 32) && fits(vd, f / 32);
}

int moe_ffn_grouped_plan(int N, int E, int d, int f, moe_ffn_plan_t* plan) {
    GgVariant vu, vd;
    if (!gg_choose(N, E, d, f, vu, vd)) return MOE_ERR_UNSUPPORTED;
    const GgShape su = gg_shape(vu), sd = gg_shape(vd);
    plan->up_tile_rows = 16 * su.tb;
    plan->up_tile_features = 16 * su.frows;
    plan->down_tile_rows = 16 * sd.tb;
    plan->down_tile_features = 16 * sd.frows;
    return MOE_OK;
}

int moe_ffn_grouped_launch(const moe_weights* W, const void* xg, moe_dtype_t act_dtype,
                           const int32_t* perm, int k, const int32_t* offsets, int N, void* ws,
                           float* yg, hipStream_t s) {
    const int d = W->d, f = W->f, E = W->E;
    GgVariant vu, vd;
    if (!gg_choose(N, E, d, f, vu, vd)) return MOE_ERR_UNSUPPORTED;
    const size_t nb = gg_max_blocks(N, E);
    u32x4_t* xp = (u32x4_t*)ws;
    u32x4_t* hp = (u32x4_t*)((unsigned char*)ws + gg_align256(nb * 16 * d * 2));
    const unsigned pgrid = (unsigned)((moe_num_cus() + 7) / 8 * 8);  // persistent: one per CU

    // once per device; threads that race here set the same attributes
    static std::atomic<int> attr_set[MOE_MAX_DEVICES];
    const int dev = moe_current_device();
    if (dev < 0) return MOE_ERR_HIP;
    if (!attr_set[dev].load(std::memory_order_acquire)) {
        for (int v = 0; v < GG_NVARIANTS; v++) {
            const GgShape sh = gg_shape((GgVariant)v);
            const void* all[3] = {gg_kernel_ptr<true, 1>((GgVariant)v), gg_kernel_ptr<true, 2>((GgVariant)v),
                                  gg_kernel_ptr<false, 0>((GgVariant)v)};
            for (int i = 0; i < 3; i++)
                MOE_HIP_TRY(hipFuncSetAttribute(all[i], hipFuncAttributeMaxDynamicSharedMemorySize,
                                                (int)((size_t)sh.ns * sh.tb * MOE_FRAG_BYTES)));
        }
        attr_set[dev].store(1, std::memory_order_release);
    }

    if (act_dtype == MOE_BF16)
        hipLaunchKernelGGL(gg_pack_kernel<true>, gg_pack_grid(nb, d), dim3(256), 0, s, xg, perm, k,
                           offsets, E, N, d, xp);
    else
        hipLaunchKernelGGL(gg_pack_kernel<false>, gg_pack_grid(nb, d), dim3(256), 0, s, xg, perm, k,
                           offsets, E, N, d, xp);

    // scratch of the pieces of left-over tiles, behind the two fragment buffers
    float* part = (float*)((unsigned char*)ws + gg_align256(nb * 16 * d * 2) +
                           gg_align256(nb * 16 * f * 2));

    GroupedArgs up;
    up.wfrag = (const u32x4_t*)W->w13;
    up.bfrag = xp;
    up.offsets = offsets;
    up.out = hp;
    up.E = E; up.N = N;
    up.KS = d / 32;
    up.FR = 2 * (f / 16);
    up.KS_out = f / 32;
    up.C = 0;
    up.part = part;
    int rc = gg_launch_projection<true>(up, vu, pgrid, s);
    if (rc != MOE_OK) return rc;
    moe_record_mid_event(s);

    GroupedArgs dn;
    dn.wfrag = (const u32x4_t*)W->w2;
    dn.bfrag = hp;
    dn.offsets = offsets;
    dn.out = yg;
    dn.E = E; dn.N = N;
    dn.KS = f / 32;
    dn.FR = d / 16;
    dn.KS_out = 0;
    dn.C = d;
    dn.part = part;
    rc = gg_launch_projection<false>(dn, vd, pgrid, s);
    if (rc != MOE_OK) return rc;
    return moe_launch_status();
}
