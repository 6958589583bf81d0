// Small-batch fused decode (2 <= M <= 16 tokens per launch) on the matrix cores:
// V2 codebooks, 4-, 3- or 2-bit indices, K a multiple of 128.  The weights are
// read from HBM once for all tokens.  (Kernel template; instantiated per bit
// width in xfp_decode_batch.hip, xfp_decode_batch3.hip and xfp_decode_batch2.hip.)  Rows of up to 8192 columns are one launch; longer
// rows (up to 32768) are cut into slices of at most 8192 columns, grid y =
// slice, whose fp32 partial sums a second kernel adds in slice order.
//
// Work unit: a workgroup of 8 waves walks tiles of 16 output rows; wave w owns
// NL consecutive 128-weight groups of every row (its K slice), so its share of
// the activations stays in VGPRs for the whole kernel as ready-made MFMA B
// operands.  v_mfma_f32_16x16x32_f16 contracts 32 k per issue:
//     A (16 rows x 32 k)   dequantised weights, lane (i, q) supplies 8 consecutive k of row i;
//     B (32 k x 16 tokens) activations, lane (m, q) supplies the same 8 k of token m;
//     D (16 x 16 fp32)     partial y of the wave's K slice.
//
// Index stream.  Adjacent lanes of the A operand are different ROWS, which is
// the worst case for a load (64 lanes, 64 cache lines).  So the loads use
// another mapping: lane l reads row l / 4 of the tile, chunk l % 4 (32 weights:
// 16 bytes at 4 bits, 12 at 3, 8 at 2) of a group, i.e. every quad of lanes reads
// 64 (48, 32) contiguous bytes, every byte of the stream exactly once.  What a
// lane got is four pieces d of 8 weights each (a dword at 4 bits; at 3 bits the
// 96 bits are first cut into four 24-bit pieces with three funnel shifts, at 2
// bits the two dwords into halves), which are then
// transposed IN REGISTERS to the operand layout by
// exchanging lane-index bits with register-index bits:
//     v_permlane32_swap, v_permlane16_swap   lane bits 5, 4  <->  register bits 1, 0
//     quad-permute DPP + select              lane bits 1, 0  <->  register bits 1, 0
// after which lane (i, q) holds, in register b, piece q of chunk b of tile row
// pi(i) = 4 (i % 4) + i / 4.  The row permutation costs nothing: the tables and
// the epilogue simply use pi.  12 to 20 VALU operations per 32 weights, no LDS
// (the same permutation through ds_bpermute_b32 measured no faster: the LDS
// pipe, busy with the lookups, is the scarcer resource).
// The registers of a group are reloaded for the workgroup's next tile as soon
// as they are transposed, so one tile of index words is always in flight.
//
// Dequantisation is one LDS lookup per PAIR of weights: a per-row table maps an
// index pair (a byte at 4 bits, 6 bits at 3, 4 at 2) to two fp16 values, the packed form
// the A operand wants.  Entry e of slot s lives at byte e*256 + s*4; slot =
// buffer*32 + i + 16*(q & 1), i.e. every row's table is stored twice so that
// the 32 lanes the LDS serves per clock hit 32 different banks, and the tables
// of the next tile are built (other buffer) while this one is decoded.  A
// lookup address is ONE v_perm_b32 at 4 bits (index byte -> address byte 1), a
// bit-field extract and a shift-or at 3 and 2 bits.
//
// V2a (MODE 1): a group's codebook is the library entry its id names, so the
// tables are per library entry, not per row: L pair tables (entry e of library
// entry l at byte (l * entries + e) * 4) are built once per workgroup, and every
// lane carries the table base of its row's current group (ids of the next tile
// are requested as those of this one are consumed).  Lookups of the 64 lanes
// then fall on banks at random, as in the streaming kernel.
//
// Per tile, the 8 partial D blocks meet in LDS and are summed in a fixed order
// (deterministic, no atomics) by 256 threads, which also add the CSR outlier
// products of the tile.  One thread per outlier entry computes its 16
// products: row pointers come through the scalar cache, col/val through
// bounds-checked buffer loads one tile ahead, and the 16 tokens' activations at
// that column come as ONE 32-byte read from a k-major (transposed) copy of x.
// Gathering them from the row-major x instead costs 16 cache lines per entry.
// That copy, and a second one in the order the B operands are loaded, are
// written by a tiny kernel launched in front of the decode kernel on the same
// stream (xfp_decode_batch.hip).
#pragma once
#include "xfp_device.h"

#include <atomic>
#include <type_traits>

namespace xfp {
namespace {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) uint32_t lds_u32_t;
typedef __attribute__((address_space(3))) const uint32_t lds_cu32_t;
typedef __attribute__((address_space(3))) float lds_f32_t;
typedef __attribute__((address_space(3))) float4_t lds_f4_t;
typedef __attribute__((address_space(4))) const int32_t const_i32_t;   // uniform reads go through the scalar cache

constexpr int kTile = 16;                  // rows per tile = tokens per launch
constexpr int kProdCap = 448;              // outlier entries of a tile whose products are kept in LDS
constexpr int kProdPad = 32;               // entries the epilogue may read past the cap (masked)
constexpr int kRd = 8;                     // product reads per lane issued unconditionally (4 * kRd entries per row)
static_assert(4 * kRd <= kProdPad, "unmasked reads stay inside the buffer");

// W waves per workgroup, each owning 1/W of K.
template <int BITS, int MODE, int W>
struct BatchLds {
    // V2: [pair entries][2 buffers x 32 slots] dwords; V2a: [L][pair entries] dwords, at most 64 KB
    static constexpr int kTabBytes = MODE == 1 ? 64 * 1024 : (1 << (2 * BITS)) * 256;
    static constexpr int kRedOne = W * 256 * 4;                       // partial D blocks of a tile
    static constexpr int kProdOne = (kProdCap + kProdPad) * 16 * 4;
    static constexpr int kRed = kTabBytes;
    static constexpr int kProd = kRed + 2 * kRedOne;
    static constexpr int kTotal = kProd + 2 * kProdOne;               // 140 KB at 4 bits, 92 KB at 3, 80 KB at 2 (W = 8)
};

struct BatchArgs {
    DecodeArgs a;
    const uint4 *xt;      // [K][16 tokens] fp16
    const uint4 *xb;      // [K / 8][16 tokens][8 k] fp16
    int M;
    int y_f32;
};

// NL: groups per wave per tile (K <= NL * 8 * 128).  RAGGED: K < NL * 8 * 128,
// some waves own groups past the end of the row.  SPLIT: a.K is the length of a
// slice of the rows (NL * 8 groups), workgroup y decodes slice y, whose last one
// may be shorter (so SPLIT implies RAGGED), folds an equal share of each tile's
// outlier entries and writes fp32 to its own plane y + blockIdx.y * z_stride.
template <int BITS, int MODE, int W, int NL, bool RAGGED, bool SPLIT>
__global__ __launch_bounds__(W * kWave) void decode_batch_kernel(BatchArgs ta)
{
    static_assert(MODE == 0 || MODE == 1, "V2 or V2a");
    constexpr uint32_t ENT = 1u << (2 * BITS);             // entries of a pair table
    static_assert(BITS >= 2 && BITS <= 4, "pair tables of 16, 64 or 256 entries");
    static_assert(!SPLIT || RAGGED, "the last slice may be short");
    using L = BatchLds<BITS, MODE, W>;
    constexpr int CW = BITS;                               // dwords of a lane's chunk of 32 weights
    constexpr int kRed = L::kRed, kRedOne = L::kRedOne, kProd = L::kProd, kProdOne = L::kProdOne;
    constexpr int RPW = kTile / W;                         // rows a wave finishes in the epilogue (2 or 1)
    constexpr int NS = 4 * NL;                             // MFMA steps per tile per wave
    extern __shared__ __align__(16) unsigned char smem[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    const DecodeArgs &a = ta.a;
    const int M = ta.M;

    const uint32_t tid = threadIdx.x, lane = tid & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t i = lane & 15, q = lane >> 4;           // operand layout: A row / token, k block
    const uint32_t la = lane >> 2, lb = lane & 3;          // load layout: tile row, chunk of a group
    const uint32_t N = a.N, K = a.K;
    const uint32_t zg = SPLIT ? blockIdx.y * (K / kGroup) : 0u;                    // first group of this slice
    const uint32_t G = SPLIT ? min(K / kGroup, a.row_words / (4 * CW) - zg) : K / kGroup;  // groups of this slice
    const uint32_t wpr = SPLIT ? a.row_words : K / 32 * CW;    // dwords per row
    const uint32_t Gtot = wpr / (4 * CW);                  // groups of a full row
    const uint32_t ntiles = (N + kTile - 1) / kTile;
    const uint32_t tstep = gridDim.x;
    const_i32_t *rp = (const_i32_t *)(uintptr_t)a.rp;
    if (lds0 & 0xFFFFu) return;                            // the lookup addresses assume the tables at LDS offset 0

    const uint32_t g0 = wave * NL;                         // first group of this wave's K slice

    // ---------------------------------------------------------------- loaders
    // Index words of group g0 + c of a tile: this lane's 16 bytes sit at a per-tile
    // base plus a compile-time offset (RAGGED: groups past the end of the row read
    // the last group again).  A tile that does not exist reads the matrix's first row.
    typedef uint32_t chunk_t __attribute__((ext_vector_type(CW), aligned(4)));   // 3-bit chunks are 12-byte aligned
    uint32_t iw[NL][CW];
    auto tile_base = [&](uint32_t tile, bool on) {
        const uint32_t row = min(tile * kTile + la, N - 1);
        return a.idx + (on ? (size_t)row * wpr : 0) + (size_t)((zg + g0) * 4 + lb) * CW;
    };
    auto load_group = [&](int c, const uint32_t *base) {
        const uint32_t *p = RAGGED ? base + 4 * CW * ((int32_t)min(g0 + c, G - 1) - (int32_t)g0) : base + 4 * CW * c;
        const chunk_t v = __builtin_nontemporal_load(reinterpret_cast<const chunk_t *>(p));   // read once: keep L2 for x
#pragma unroll
        for (int d = 0; d < CW; ++d) iw[c][d] = v[d];
    };
    // CSR bookkeeping of a tile, all wave-uniform (scalar loads): the entry range
    // of the tile and of the rows this wave finishes (w, and w + 8 when W = 8).
    struct TileRp { int32_t base, end, lo[RPW], hi[RPW]; };
    auto load_rp = [&](uint32_t tile) {
        const uint32_t n0 = tile * kTile;
        TileRp r;
        r.base = rp[min(n0, N)];
        r.end = rp[min(n0 + kTile, N)];
        if constexpr (SPLIT) {
            // every slice sees all of x, so the tile's entries are dealt to the slices by
            // position, an equal share each, whatever their columns
            const uint32_t cnt = (uint32_t)(r.end - r.base), S = gridDim.y, z = blockIdx.y;
            r.end = r.base + (int32_t)(cnt * (z + 1) / S);
            r.base += (int32_t)(cnt * z / S);
        }
#pragma unroll
        for (int h = 0; h < RPW; ++h) {
            r.lo[h] = rp[min(n0 + wave + W * h, N)];
            r.hi[h] = rp[min(n0 + wave + W * h + 1, N)];
            if constexpr (SPLIT) {
                r.lo[h] = min(max(r.lo[h], r.base), r.end);
                r.hi[h] = min(max(r.hi[h], r.base), r.end);
            }
        }
        return r;
    };
    // Outlier entry `tid` of a tile: col and val through bounds-checked buffer loads
    // (entries past the end of the tile read as zero).
    auto load_col = [&](const TileRp &r, uint32_t &col) {
        __amdgpu_buffer_rsrc_t rc = __builtin_amdgcn_make_buffer_rsrc((void *)(a.col + r.base), 0, (r.end - r.base) * 4, 0x00020000);
        col = __builtin_amdgcn_raw_buffer_load_b32(rc, tid * 4, 0, 0);
    };
    auto load_val = [&](const TileRp &r, uint32_t &val) {
        __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc((void *)(a.val + r.base), 0, (r.end - r.base) * 2, 0x00020000);
        val = __builtin_amdgcn_raw_buffer_load_b16(rv, tid * 2, 0, 0);
    };
    // V2a: library ids of the groups g0 .. g0 + NL of this lane's operand row.
    uint32_t gidr[NL];
    auto gid_base = [&](uint32_t tile, bool on) {
        const uint32_t row = min(tile * kTile + 4 * (i & 3) + (i >> 2), N - 1);
        return a.gid + (on ? (size_t)row * Gtot : 0) + zg + g0;
    };
    auto load_gid = [&](int c, const uint8_t *base) {
        gidr[c] = base[RAGGED ? (int32_t)min(g0 + c, G - 1) - (int32_t)g0 : c];
    };
    // Table builder role of this thread: slot tid % 32 (operand row i = slot % 16,
    // i.e. tile row pi(i)) and role tid / 32 = 4 rb + ra.  Two register sets of
    // codebook values, one per tile parity, so that a tile's codebook can be
    // requested a whole pass before its tables are built.
    //   4 bits: the 16 entries whose first index is 4 ra + u and second index
    //           4 rb + v (u, v = 0..3): 4 + 4 codebook values, two 8-byte loads;
    //   3 bits: the 4 entries whose first index is 4 (ra & 1) + u and second index
    //           2 rb + ra / 2: 4 + 1 codebook values (cbh.x holds the one, low half);
    //   2 bits: the entry (first index ra, second index rb): cbl.x and cbh.x, low halves.
    static_assert(W == 8, "32 slots x 16 builder roles = 512 threads");
    constexpr int NB = (1 << (2 * BITS)) / 16;             // table entries a thread writes per tile
    const uint32_t tb_slot = tid & 31, tb_ra = (tid >> 5) & 3, tb_rb = tid >> 7;
    const uint32_t tb_row = 4 * (tb_slot & 3) + ((tb_slot & 15) >> 2);
    const uint32_t tb_i1 = 2 * tb_rb + (tb_ra >> 1);       // 3 bits: second index of this role
    uint2 cbl[2], cbh[2];
    auto load_codebook = [&](int set, uint32_t tile) {
        const uint16_t *p = a.cb + (size_t)min(tile * kTile + tb_row, N - 1) * (1 << BITS);
        if constexpr (BITS == 4) {
            cbl[set] = *reinterpret_cast<const uint2 *>(p + 4 * tb_ra);
            cbh[set] = *reinterpret_cast<const uint2 *>(p + 4 * tb_rb);
        } else if constexpr (BITS == 3) {
            cbl[set] = *reinterpret_cast<const uint2 *>(p + 4 * (tb_ra & 1));
            cbh[set].x = p[tb_i1];
            cbh[set].y = 0u;
        } else {
            cbl[set] = make_uint2(p[tb_ra], 0u);
            cbh[set] = make_uint2(p[tb_rb], 0u);
        }
    };
    auto build_step = [&](uint32_t buf, int set, int j) {
        if constexpr (BITS == 4) {                         // j = 4 v + u
            const int u = j & 3, v = j >> 2;
            const uint32_t base = lds0 + (4 * tb_ra + 64 * tb_rb) * 256 + (buf * 32 + tb_slot) * 4;
            const uint32_t lw = u < 2 ? cbl[set].x : cbl[set].y, hw = v < 2 ? cbh[set].x : cbh[set].y;
            const uint32_t lo = (u & 1) ? lw >> 16 : lw & 0xFFFFu;
            const uint32_t hi = (v & 1) ? hw & 0xFFFF0000u : hw << 16;
            *(lds_u32_t *)(uintptr_t)(base + (u + 16 * v) * 256) = lo | hi;
        } else if constexpr (BITS == 3) {                  // j = u
            const uint32_t base = lds0 + (4 * (tb_ra & 1) + 8 * tb_i1) * 256 + (buf * 32 + tb_slot) * 4;
            const uint32_t lw = j < 2 ? cbl[set].x : cbl[set].y;
            const uint32_t lo = (j & 1) ? lw >> 16 : lw & 0xFFFFu;
            *(lds_u32_t *)(uintptr_t)(base + j * 256) = lo | (cbh[set].x << 16);
        } else {
            const uint32_t base = lds0 + (tb_ra + 4 * tb_rb) * 256 + (buf * 32 + tb_slot) * 4;
            *(lds_u32_t *)(uintptr_t)base = cbl[set].x | (cbh[set].x << 16);
        }
    };

    uint32_t t = blockIdx.x;
    if (t >= ntiles) return;

    // ---------------------------------------------------------------- prologue
    // Codebooks first (they gate the tables), then per group its activations (L2
    // hits) followed by its index words (HBM): vector loads return in order and a
    // CU only tracks about a tile's worth of outstanding loads, so this order lets
    // the first MFMA steps start while the later groups are still streaming in.
    TileRp rp_c = load_rp(t);
    const bool have1 = t + tstep < ntiles;
    TileRp rp_n = load_rp(have1 ? t + tstep : t);
    // Every workgroup reads the whole operand-ordered copy of x, all in the same
    // order, so every line would be a (merged) miss for all of them.  The L2 is
    // per XCD and workgroups are dealt to the 8 XCDs round-robin: wave w of the
    // j-th workgroup of an XCD touches KB number 8 j + w of the copy first, so
    // that each XCD has all of it in its L2 after one miss latency.
    uint4 warm;
    {
        const uint32_t kib = ((blockIdx.x >> 3) * W + wave) % (G * (kGroup * kTile * 2 / 1024));
        warm = ta.xb[(size_t)(zg * (kGroup * kTile * 2 / 1024) + kib) * 64 + lane];
    }
    if constexpr (MODE == 0) load_codebook(0, t);
    // a1: B operands.  Step s = 4 c + b contracts, in k block q, piece q of chunk b
    // of group g0 + c.
    uint32_t xr[NS][4];
    {
        const uint32_t *b0 = tile_base(t, true);
#pragma unroll
        for (int c = 0; c < NL; ++c) {
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int s = 4 * c + b;
                const uint32_t g = g0 + c;
                const uint32_t kb = (zg + min(g, G - 1)) * (kGroup / 8) + b * 4 + q;  // k block of this lane
                const uint4 v = ta.xb[(size_t)kb * kTile + i];
                const bool on = !RAGGED || g < G;
                xr[s][0] = on ? v.x : 0u; xr[s][1] = on ? v.y : 0u; xr[s][2] = on ? v.z : 0u; xr[s][3] = on ? v.w : 0u;
            }
            load_group(c, b0);
        }
    }
    if constexpr (MODE == 1) {
        const uint8_t *gb0 = gid_base(t, true);
#pragma unroll
        for (int c = 0; c < NL; ++c) load_gid(c, gb0);
    }
    asm volatile("" :: "v"(warm.x), "v"(warm.y), "v"(warm.z), "v"(warm.w));
    // a2: tables of the first tile.
    if constexpr (MODE == 0) {
#pragma unroll
        for (int j = 0; j < NB; ++j) build_step(0, 0, j);
        load_codebook(1, have1 ? t + tstep : t);
    } else {
        // the library's pair tables, once: entry e = (second index, first index) of library entry l
        const uint32_t total = a.L * ENT;
#pragma unroll 4
        for (uint32_t e = tid; e < total; e += W * kWave) {
            const uint16_t *cbk = a.cb + (size_t)(e / ENT) * (1u << BITS);
            const uint32_t lo = cbk[e & ((1u << BITS) - 1u)], hi = cbk[(e % ENT) >> BITS];
            *(lds_u32_t *)(uintptr_t)(lds0 + e * 4) = lo | (hi << 16);
        }
    }
    uint32_t ocol = 0, oval = 0;
    load_col(rp_c, ocol);
    load_val(rp_c, oval);
    lds_barrier();
    const uint32_t bank4 = (((q & 1) << 4) | i) * 4;       // this lane's private bank


    // ---------------------------------------------------------------- one tile
    // P = parity of the tile within this workgroup's sequence: table buffer,
    // codebook registers, reduction and product buffers.  Only the MFMA loop and
    // one barrier are on a wave's critical path; everything else a tile needs is
    // spread over the steps of a loop, where its VALU and LDS instructions fill
    // the slots the lookups leave open.  Vector loads return in the order they
    // were issued, so every load is issued BEFORE the index words that will be
    // consumed ahead of it, and its consumer never waits for younger index words:
    //   before step 0 : gather x at this tile's outlier columns (col came a pass ago);
    //   step 1        : request col of the next tile and the codebook of the tile after;
    //   steps NS/4 .. : the table of the NEXT tile, a few entries per step (other buffer);
    //   late          : outlier products of this tile -> LDS (the gather is older
    //                   than every index word of this tile), request val of the
    //                   next tile; then cross-wave sum, outlier fold and store of
    //                   the PREVIOUS tile (its partial sums and products sit in
    //                   the other parity's buffers, complete since the barrier
    //                   that ended its pass).
    constexpr int BPS = (NB + NS - 1) / NS;                // table entries written per step
    constexpr int BUILD_STEPS = (NB + BPS - 1) / BPS;      // steps that write table entries
    constexpr int BUILD_FROM = NS >= 2 * BUILD_STEPS ? NS / 4 : 0;
    constexpr int AHEAD_STEP = NS >= 8 ? 1 : 0;
    constexpr int PROD_STEP = NS >= 16 ? NS - 4 : NS - 1;
    constexpr int EPI_STEP = NS >= 16 ? NS - 2 : NS - 1;

    // ---- a8: cross-wave sum, outlier fold, store (fixed order) ----
    // output (row, token m) is summed by the 4 lanes of a quad: lane j takes waves
    // j, j+4, ... and entries lo+j, lo+j+4, ...; a wave finishes row w (and w + 8).
    struct Epi { float part[RPW][W / 4], pv[RPW][kRd]; int32_t lo[RPW], hi[RPW], hf[RPW]; };
    const uint32_t sub = lane & 3, em = lane >> 2;
    auto epi_read = [&](auto Ptag, const TileRp &r, Epi &e) {
        constexpr int P = decltype(Ptag)::value;
        const int32_t ob = r.base;
        const uint32_t pbase = lds0 + kProd + P * kProdOne;
        const uint32_t rbase = lds0 + kRed + P * kRedOne;
#pragma unroll
        for (int h = 0; h < RPW; ++h) {
            const uint32_t o = (wave + W * h) * 16 + em;
#pragma unroll
            for (int j = 0; j < W / 4; ++j)
                e.part[h][j] = *(lds_f32_t *)(uintptr_t)(rbase + (sub + 4 * j) * 1024 + o * 4);
            e.lo[h] = r.lo[h] - ob;
            e.hf[h] = r.hi[h] - ob;
            e.hi[h] = min(e.hf[h], (int32_t)kProdCap);
            // reads past the row's entries stay inside the padded buffer and are masked
            const uint32_t eb = pbase + (uint32_t)(min(e.lo[h], (int32_t)kProdCap) + (int32_t)sub) * 64 + em * 4;
#pragma unroll
            for (int j = 0; j < kRd; ++j) e.pv[h][j] = *(lds_f32_t *)(uintptr_t)(eb + j * 256);
        }
    };
    auto epi_sum = [&](auto Ptag, const TileRp &r, uint32_t n0, const Epi &e) {
        constexpr int P = decltype(Ptag)::value;
        const int32_t ob = r.base;
        const uint32_t pbase = lds0 + kProd + P * kProdOne;
        const uint16_t *xrow = a.x + (size_t)min(em, (uint32_t)M - 1) * a.x_stride;
#pragma unroll
        for (int h = 0; h < RPW; ++h) {
            const uint32_t n = n0 + wave + W * h;
            float s = e.part[h][0];
#pragma unroll
            for (int j = 1; j < W / 4; ++j) s += e.part[h][j];
            const int32_t nv = e.hi[h] - e.lo[h] - (int32_t)sub;       // entry 4 j of this lane is valid iff 4 j < nv
#pragma unroll
            for (int j = 0; j < kRd; ++j) s += 4 * j < nv ? e.pv[h][j] : 0.f;
            // both rare paths hang on wave-uniform conditions, so that skipping them costs a scalar branch each
            if (e.hi[h] - e.lo[h] > 4 * kRd)                                                              // long rows
                for (int32_t en = e.lo[h] + (int32_t)sub + 4 * kRd; en < e.hi[h]; en += 4)
                    s += *(lds_f32_t *)(uintptr_t)(pbase + en * 64 + em * 4);
            if (e.hf[h] > (int32_t)kProdCap)                                                              // > kProdCap per tile
                for (int32_t en = max(e.lo[h], (int32_t)kProdCap) + (int32_t)sub; en < e.hf[h]; en += 4)
                    s = fmaf(half_bits_to_float(a.val[ob + en]), x_bits_to_float(xrow[a.col[ob + en]], a.x_bf16 != 0), s);
            s = dpp_add<0xB1>(s);                          // quad_perm [1,0,3,2]
            s = dpp_add<0x4E>(s);                          // quad_perm [2,3,0,1]
            if (sub == 0 && n < N && em < (uint32_t)M) {
                const int64_t oo = (int64_t)em * a.y_stride + n;
                if constexpr (SPLIT) static_cast<float *>(a.y)[(int64_t)blockIdx.y * a.z_stride + oo] = s;
                else store_out(a.y, oo, s, ta.y_f32 != 0, a.y_bf16 != 0);
            }
        }
    };

    TileRp rp_p = rp_c;                                    // previous tile (none yet)
    uint32_t n0_p = 0;
    bool have_prev = false;

    auto tile_pass = [&](auto Ptag, uint32_t tile) {
        constexpr int P = decltype(Ptag)::value;
        using Prev = std::integral_constant<int, P ^ 1>;
        const uint32_t t1 = tile + tstep, t2 = tile + 2 * tstep;
        const bool have_next = t1 < ntiles, have2 = t2 < ntiles;
        const TileRp rp_f = load_rp(have2 ? t2 : tile);    // two tiles ahead (scalar cache)
        const uint32_t *nbase = tile_base(t1, have_next);
        const uint8_t *ngid = MODE == 1 ? gid_base(t1, have_next) : nullptr;

        // ---- a3-a6: transpose, depack, pair lookup, MFMA; lookups run two steps ahead ----
        float4_t acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
        const uint32_t sel = bank4 + P * 128;
        uint32_t pw[2][4];                                 // transposed pieces of the current and the next group
        uint32_t gtab[2];                                  // V2a: table base of the current and the next group
        constexpr int LA = 2;                              // steps the lookups run ahead of the MFMAs
        static_assert(LA >= 1 && LA <= 3, "a group is transposed while the previous one is still being looked up");
        uint32_t av[LA + 1][4];
        auto transpose_group = [&](int c) {
            uint32_t (&v)[4] = pw[c & 1];
            if constexpr (BITS == 4) {
                v[0] = iw[c][0]; v[1] = iw[c][1]; v[2] = iw[c][2]; v[3] = iw[c][3];
            } else if constexpr (BITS == 3) {              // piece d = bits [24 d, 24 d + 24) of the 96; bits above 24 are ignored
                v[0] = iw[c][0];
                v[1] = __builtin_amdgcn_alignbit(iw[c][1], iw[c][0], 24);
                v[2] = __builtin_amdgcn_alignbit(iw[c][2], iw[c][1], 16);
                v[3] = iw[c][2] >> 8;
            } else {                                       // piece d = 16 bits; bits above 16 are ignored
                v[0] = iw[c][0]; v[1] = iw[c][0] >> 16; v[2] = iw[c][1]; v[3] = iw[c][1] >> 16;
            }
            to_operand_layout(v);
            load_group(c, nbase);                          // the registers are free: next tile's words
            if constexpr (MODE == 1) {
                gtab[c & 1] = gidr[c] * (ENT * 4);
                load_gid(c, ngid);
            }
        };
        auto lookup = [&](int s, uint32_t (&v)[4]) {
            const uint32_t w = pw[(s / 4) & 1][s & 3];
            if constexpr (MODE == 1) {
                const uint32_t gb = gtab[(s / 4) & 1];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    v[j] = *(lds_cu32_t *)(uintptr_t)((((w >> (2 * BITS * j)) & (ENT - 1u)) << 2) | gb);
            } else if constexpr (BITS == 4) {
                v[0] = *(lds_cu32_t *)(uintptr_t)__builtin_amdgcn_perm(w, sel, 0x0c0c0400u);
                v[1] = *(lds_cu32_t *)(uintptr_t)__builtin_amdgcn_perm(w, sel, 0x0c0c0500u);
                v[2] = *(lds_cu32_t *)(uintptr_t)__builtin_amdgcn_perm(w, sel, 0x0c0c0600u);
                v[3] = *(lds_cu32_t *)(uintptr_t)__builtin_amdgcn_perm(w, sel, 0x0c0c0700u);
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    v[j] = *(lds_cu32_t *)(uintptr_t)((((w >> (2 * BITS * j)) & ((1u << (2 * BITS)) - 1u)) << 8) | sel);
            }
        };
        // a7: outlier products of the first kProdCap entries -> LDS
        uint4 ox0 = make_uint4(0u, 0u, 0u, 0u), ox1 = ox0;     // x at this thread's outlier column
        auto products = [&]() {
            if (W * kWave <= kProdCap || tid < (uint32_t)kProdCap) {
                const float v = half_bits_to_float((uint16_t)oval);
                const uint32_t xw[8] = {ox0.x, ox0.y, ox0.z, ox0.w, ox1.x, ox1.y, ox1.z, ox1.w};
                float p[16];
#pragma unroll
                for (int m = 0; m < 16; ++m)
                    p[m] = v * half_bits_to_float((uint16_t)(m & 1 ? xw[m / 2] >> 16 : xw[m / 2] & 0xFFFFu));
                lds_f4_t *dst = (lds_f4_t *)(uintptr_t)(lds0 + kProd + P * kProdOne + tid * 64);
#pragma unroll
                for (int g = 0; g < 4; ++g) dst[g] = float4_t{p[4 * g], p[4 * g + 1], p[4 * g + 2], p[4 * g + 3]};
            }
            load_val(rp_n, oval);                          // next tile's values
        };
        ox0 = ta.xt[(size_t)ocol * 2];
        ox1 = ta.xt[(size_t)ocol * 2 + 1];
        transpose_group(0);
#pragma unroll
        for (int s = 0; s < LA && s < NS; ++s) lookup(s, av[s]);
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            // group c + 1 must be transposed before the lookup of its first step, 4 (c + 1), is issued
            if ((s + LA) % 4 == 3 && (s + LA) / 4 + 1 < NL) transpose_group((s + LA) / 4 + 1);
            if (s + LA < NS) lookup(s + LA, av[(s + LA) % (LA + 1)]);
            __builtin_amdgcn_sched_barrier(0);
            const uint32_t (&cur)[4] = av[s % (LA + 1)];
            half8_t af = __builtin_bit_cast(half8_t, u32x4_t{cur[0], cur[1], cur[2], cur[3]});
            half8_t bf = __builtin_bit_cast(half8_t, u32x4_t{xr[s][0], xr[s][1], xr[s][2], xr[s][3]});
            if (!RAGGED || g0 + s / 4 < G) {
                if (s & 1) acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(af, bf, acc1, 0, 0, 0);
                else acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(af, bf, acc0, 0, 0, 0);
            }
            if (s == AHEAD_STEP) {
                load_col(rp_n, ocol);                      // next tile's columns
                if constexpr (MODE == 0) load_codebook(P, have2 ? t2 : tile);   // two tiles ahead: this parity's registers are free
            }
            if (MODE == 0 && s >= BUILD_FROM && s < BUILD_FROM + BUILD_STEPS) {
#pragma unroll
                for (int j = (s - BUILD_FROM) * BPS; j < (s - BUILD_FROM + 1) * BPS && j < NB; ++j) build_step(P ^ 1, P ^ 1, j);
            }
            if (s == PROD_STEP) products();
            if (s == EPI_STEP && have_prev) {
                Epi ep;
                epi_read(Prev{}, rp_p, ep);
                epi_sum(Prev{}, rp_p, n0_p, ep);
            }
            __builtin_amdgcn_sched_barrier(0);
        }

        // ---- partial D of this wave -> LDS, indexed by tile row ----
        {
            const float4_t d = acc0 + acc1;                // lane (m, q'), register r: operand row 4q' + r = tile row 4r + q'
            const uint32_t rb = lds0 + kRed + P * kRedOne + wave * 1024;
#pragma unroll
            for (int r = 0; r < 4; ++r) *(lds_f32_t *)(uintptr_t)(rb + ((4 * r + q) * 16 + i) * 4) = d[r];
        }
        lds_barrier();
        rp_p = rp_c;
        n0_p = tile * kTile;
        have_prev = true;
        rp_c = rp_n;
        rp_n = rp_f;
    };
    auto last_epilogue = [&](auto Ptag) {
        Epi ep;
        epi_read(Ptag, rp_p, ep);
        epi_sum(Ptag, rp_p, n0_p, ep);
    };

    for (;;) {
        tile_pass(std::integral_constant<int, 0>{}, t);
        t += tstep;
        if (t >= ntiles) { last_epilogue(std::integral_constant<int, 0>{}); break; }
        tile_pass(std::integral_constant<int, 1>{}, t);
        t += tstep;
        if (t >= ntiles) { last_epilogue(std::integral_constant<int, 1>{}); break; }
    }
}

int device_cus()
{
    static std::atomic<int> cus{0};
    int c = cus.load(std::memory_order_relaxed);
    if (c == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return 256;
        c = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
        cus.store(c, std::memory_order_relaxed);
    }
    return c;
}

// Groups per wave per slice of a long row: S = ceil(G / 64) slices, each
// ceil(G / S) groups rounded up to a multiple of 8 (one group more or less per
// wave), the last one shorter.  0 if the row is not split.
inline int batch_split_nl(uint32_t K)
{
    const uint32_t G = K / kGroup;
    if (G <= 64) return 0;
    const uint32_t S = (G + 63) / 64;
    return (int)(((G + S - 1) / S + 7) / 8);
}

// a.K: columns of a full row; xt, xb: the two re-laid copies of x.  SPLIT: slices
// of NL * W groups, a.y an fp32 plane buffer [slices][M][N].
template <int BITS, int MODE, int W, int NL, bool RAGGED, bool SPLIT = false>
hipError_t launch_batch_t(const DecodeArgs &a, int M, bool y_f32, const void *xt, const void *xb, hipStream_t s)
{
    constexpr int kBatchLds = BatchLds<BITS, MODE, W>::kTotal;
    auto kern = decode_batch_kernel<BITS, MODE, W, NL, RAGGED, SPLIT>;
    static std::atomic<int> configured[kMaxDevices];       // per device; idempotent attribute, benign race
    const int dev = current_device();
    if (dev < 0) return hipErrorInvalidDevice;
    if (!configured[dev].load(std::memory_order_relaxed)) {
        hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kBatchLds);
        if (err != hipSuccess) return err;
        configured[dev].store(1, std::memory_order_relaxed);
    }
    BatchArgs ta;
    ta.a = a;
    ta.M = M;
    ta.y_f32 = (int)y_f32;
    ta.xt = static_cast<const uint4 *>(xt);
    ta.xb = static_cast<const uint4 *>(xb);
    const uint32_t ntiles = (a.N + kTile - 1) / kTile;
    uint32_t wgs = (uint32_t)device_cus(), slices = 1;
    if constexpr (SPLIT) {
        constexpr uint32_t GS = NL * W;                    // groups per slice
        slices = (a.K / kGroup + GS - 1) / GS;
        ta.a.row_words = a.K / 32 * BITS;
        ta.a.K = GS * kGroup;
        ta.a.y_stride = a.N;
        ta.a.z_stride = (int64_t)M * a.N;
        wgs = wgs / slices > 0 ? wgs / slices : 1;         // one workgroup per CU over all slices
    }
    hipLaunchKernelGGL(kern, dim3(ntiles < wgs ? ntiles : wgs, slices), dim3(W * kWave), kBatchLds, s, ta);
    return hipGetLastError();
}

template <int BITS, int MODE, int NL>
hipError_t launch_batch_n(const DecodeArgs &a, int M, bool y_f32, const void *xt, const void *xb, hipStream_t s)
{
    if (a.K / kGroup == (uint32_t)NL * 8) return launch_batch_t<BITS, MODE, 8, NL, false>(a, M, y_f32, xt, xb, s);
    return launch_batch_t<BITS, MODE, 8, NL, true>(a, M, y_f32, xt, xb, s);
}

// One launch of up to 16 tokens for one bit width.  Eight waves share a tile of
// 16 rows: with 16 waves (128 registers each) the compiler spills the in-flight
// index words and the kernel runs at half the speed.  part: an fp32 scratch plane
// for the partial sums of a row cut into slices (K > 8192), unused otherwise.
template <int BITS, int MODE = 0>
hipError_t launch_batch_bits(const DecodeArgs &a, int M, bool y_f32, float *part, const void *xt, const void *xb,
                             hipStream_t s)
{
    const int nl = batch_split_nl(a.K);
    if (nl == 0) {
        switch ((a.K / kGroup + 7) / 8) {
        case 1: return launch_batch_n<BITS, MODE, 1>(a, M, y_f32, xt, xb, s);
        case 2: return launch_batch_n<BITS, MODE, 2>(a, M, y_f32, xt, xb, s);
        case 3: return launch_batch_n<BITS, MODE, 3>(a, M, y_f32, xt, xb, s);
        case 4: return launch_batch_n<BITS, MODE, 4>(a, M, y_f32, xt, xb, s);
        case 5: return launch_batch_n<BITS, MODE, 5>(a, M, y_f32, xt, xb, s);
        case 6: return launch_batch_n<BITS, MODE, 6>(a, M, y_f32, xt, xb, s);
        case 7: return launch_batch_n<BITS, MODE, 7>(a, M, y_f32, xt, xb, s);
        case 8: return launch_batch_n<BITS, MODE, 8>(a, M, y_f32, xt, xb, s);
        default: return hipErrorInvalidValue;
        }
    }
    if (!part) return hipErrorInvalidValue;
    hipError_t err = hipSuccess;
    DecodeArgs c = a;
    c.y = part;
    switch (nl) {
    case 5: err = launch_batch_t<BITS, MODE, 8, 5, true, true>(c, M, true, xt, xb, s); break;
    case 6: err = launch_batch_t<BITS, MODE, 8, 6, true, true>(c, M, true, xt, xb, s); break;
    case 7: err = launch_batch_t<BITS, MODE, 8, 7, true, true>(c, M, true, xt, xb, s); break;
    case 8: err = launch_batch_t<BITS, MODE, 8, 8, true, true>(c, M, true, xt, xb, s); break;
    default: return hipErrorInvalidValue;
    }
    if (err != hipSuccess) return err;
    const uint32_t slices = (a.K / kGroup + (uint32_t)nl * 8 - 1) / ((uint32_t)nl * 8);
    return launch_splitk_sum(part, slices, a.N, M, a.y, a.y_stride, y_f32, a.y_bf16 != 0, s);
}

}  // namespace
}  // namespace xfp
