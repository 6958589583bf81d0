// Wide form of the batched decode on the matrix cores: up to 64 tokens per pass
// over the weights (V2 codebooks or a V2a library, 2-, 3- or 4-bit indices): the batched variant
// of the fused kernel for M >= 16 (paper section 5), same four fused steps.
//
// Why: the 16-token kernel keeps its tokens' activations in registers as B
// operands (128 of a wave's 256 registers), so more than 16 tokens mean another
// pass over the weights, and every pass pays the whole dequantisation again: it
// is bound by the lookups and the instruction issue, not by HBM.  Here the roles
// are swapped: what stays on chip is the DEQUANTISED weight operand of a step,
// used for every token, and the activations stream past it.
//
// Work unit: a workgroup of 8 waves owns a tile of 32 output rows (two MFMA row
// blocks of 16) and up to 16 T tokens (T = 1..4 chunks of 16).  Wave w takes the
// 128-weight groups w, w + 8, ... of the rows (any number of groups: no slices).
// A step contracts 32 k:
//     A (16 rows x 32 k)   dequantised weights of one row block: 4 pair lookups per lane;
//     B (32 k x 16 tokens) activations of one chunk: one 16-byte load per lane from the
//                          operand-ordered copy of x (1 KB contiguous per wave, L2 hits);
//     D (16 x 16 fp32)     one accumulator per (row block, chunk): 2 T of them.
// 2 T v_mfma_f32_16x16x32_f16 per 8 lookups: by instruction count the matrix
// cores, not the lookups, set the pace at T = 4 (measured, the kernel mostly
// waits: a wave's loads complete in issue order, so its B operands, L2 hits,
// queue behind its index words, HBM misses).  A 32-row tile halves the B traffic of a 16-row one
// (every B operand meets two A operands); the B operands live in a ring of a few
// steps, requested that many steps ahead.
//
// Index words: coalesced loads (lane l reads row l / 4, chunk l % 4 of a group:
// every quad 64 contiguous bytes), transposed in registers to the operand layout
// (to_operand_layout: operand row i = tile row 4 (i % 4) + i / 4), the next
// group's words requested as soon as this group's are transposed.
// Pair tables: entry e of slot s at LDS byte e * 256 + s * 4, slot = 32 * row block
// + 16 * (q & 1) + i, every row's table twice, so that the 32 lanes the LDS serves
// per clock hit 32 banks; a lookup address is one v_perm_b32.  Built once per
// workgroup (one tile per workgroup).  V2a: the library's tables instead, entry e
// of library entry l at byte (l * 4^BITS + e) * 4, shared by all rows.
//
// Epilogue: after a barrier the 8 partial D blocks go to LDS planes that reuse the
// table region, [wave][token][row].  Outliers: wave w owns tile rows 4 w .. 4 w + 3;
// lane (e, o) takes entries e, e + 8, ... of a row and the token octet o: the eight
// tokens' activations at an entry's column are ONE 16-byte read from a k-major
// copy of x (a wave instruction covers 8 entries x 64 tokens: the vector-memory
// path, which the B operands keep busy, sees few instructions), a lane sums its
// entries in order, the eight lanes of an octet are added in a fixed tree and the
// sums go to a ninth plane.  512 threads then add the nine planes in plane order
// and store.  No atomics: every sum has a fixed order.
#include "xfp_device.h"

#include <atomic>
#include <type_traits>

namespace xfp {
namespace {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x3_t __attribute__((ext_vector_type(3)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) uint32_t lds_u32_t;
typedef __attribute__((address_space(3))) const uint32_t lds_cu32_t;
typedef __attribute__((address_space(3))) float lds_f32_t;
typedef __attribute__((address_space(4))) const int32_t const_i32_t;   // uniform reads go through the scalar cache

constexpr int kWideRows = 32;              // rows of a tile: two MFMA row blocks
constexpr int kWideWaves = 8;
constexpr int kWideThreads = kWideWaves * kWave;
constexpr int kTokStride = 33;             // floats between two tokens of a plane (32 rows + 1: spreads the banks)

constexpr int kWideLibTab = 64 * 1024;     // V2a: the library's pair tables, L * 4^BITS dwords at most

template <int BITS, int T, int MODE>
struct WideLds {
    // pair tables: V2 [4^BITS entries][64 slots] dwords; V2a [L][4^BITS entries] dwords
    static constexpr int kTab = MODE != 0 ? kWideLibTab : (1 << (2 * BITS)) * 256;
    static constexpr int kPlane = 16 * T * kTokStride * 4;             // [16 T tokens][33] floats
    static constexpr int kOut = kWideWaves * kPlane > kTab ? kWideWaves * kPlane : kTab;   // the outlier plane: behind both
    static constexpr int kTotal = kOut + kPlane;                       // 76 032 bytes at T = 4; 4 bits, T = 1: 67 648
    // MODE 2: behind it the tile's scales and mid-points, one dword (scale | mid << 16) per (group, row), 128 G bytes
    static constexpr int kAff = kTotal;
};

// Where a group's four pieces per row block live: at 4 bits they are the index words themselves (in place), else
// registers of their own.
__device__ __forceinline__ uint32_t (&pieces_of(uint32_t (&words)[2][4], uint32_t (&)[1][4]))[2][4] { return words; }
template <int CW>
__device__ __forceinline__ uint32_t (&pieces_of(uint32_t (&)[2][CW], uint32_t (&own)[2][4]))[2][4] { return own; }

struct WideArgs {
    DecodeArgs a;
    const uint16_t *xt;    // [K][16 T tokens] fp16
    const uint16_t *xb;    // [T][K / 8][16 tokens][8 k] fp16
    const float *sx;       // MODE 2: [K / 128][16 tokens] sums of a token's activations over a group
    int M;
    int y_f32;
};

// MODE 0: V2, a codebook per row.  MODE 1: V2a, a library of a.L codebooks and an id per (row, group); the
// library's pair tables are shared by all rows, so their lookups meet in the banks at random.  MODE 2: V2a with a
// scale and a mid-point per group (T = 1 only): W = entry * scale + mid, evaluated exactly by linearity: a group's
// four steps accumulate into a block of their own, D_g, and the row's result takes scale * D_g + mid * (the
// token's activation sum over the group, precomputed by the re-layout kernel) in fp32.
template <int BITS, int T, int MODE>
__global__ __launch_bounds__(kWideThreads) __attribute__((amdgpu_waves_per_eu(4, 4)))
void decode_wide_kernel(WideArgs ta)
{
    static_assert(BITS >= 2 && BITS <= 4, "pair tables of 16, 64 or 256 entries");
    static_assert(MODE >= 0 && MODE <= 2, "V2, V2a, V2a with a scale and a mid-point per group");
    static_assert(MODE != 2 || T == 1, "scale and mid-point: 16 tokens per launch");
    constexpr bool LIB = MODE != 0, AFF = MODE == 2;
    using L = WideLds<BITS, T, MODE>;
    constexpr int CW = BITS;                               // dwords of a lane's chunk of 32 weights
    constexpr uint32_t ENT = 1u << (2 * BITS);             // entries of a pair table
    constexpr int NSLOT = T <= 2 ? 4 : 2;                  // steps of B operands in flight
    constexpr int D = T == 4 ? 2 : T == 3 ? 4 : T == 2 ? 5 : MODE == 2 ? 4 : 6;   // groups of index words in flight (what the registers allow)
    constexpr uint32_t MP = 16 * T;                        // tokens of the re-laid copies
    extern __shared__ __align__(16) unsigned char smem[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    if (lds0 & 0xFFFFu) return;                            // the lookup addresses assume the tables at LDS offset 0
    const DecodeArgs &a = ta.a;

    const uint32_t tid = threadIdx.x, lane = tid & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t i = lane & 15, q = lane >> 4;           // operand layout: A row / token, k block
    const uint32_t la = lane >> 2, lb = lane & 3;          // load layout: row of a row block, chunk of a group
    const uint32_t N = a.N, K = a.K;
    const uint32_t G = K / kGroup, wpr = K / 32 * CW;      // groups, dwords of a row
    const uint32_t n0 = blockIdx.x * kWideRows;
    const uint32_t rows_here = min((uint32_t)kWideRows, N - n0);
    const_i32_t *rp = (const_i32_t *)(uintptr_t)a.rp;

    // ---------------------------------------------------------------- loads, oldest consumer first
    // table builder role: slot tid % 64 (row block, copy, operand row), part tid / 64 (0..7) builds ENT / 8 entries:
    //   4 bits: the 32 entries whose second index is 2 part or 2 part + 1 (16 + 2 codebook values);
    //   3 bits: the 8 entries whose second index is part (8 + 1 values);
    //   2 bits: the 2 entries (first index 2 (part & 1) + {0, 1}, second index part / 2).
    const uint32_t slot = tid & 63, part = tid >> 6;
    const uint32_t trow = (slot >> 5) * 16 + 4 * (slot & 3) + ((slot & 15) >> 2);
    const uint16_t *cbr = a.cb + (size_t)min(n0 + trow, N - 1) * (1u << BITS);
    uint4 c0 = make_uint4(0u, 0u, 0u, 0u), c1 = c0;
    uint32_t chi = 0;
    if constexpr (LIB) {
        // V2a: the tables come from the library; nothing per row
    } else if constexpr (BITS == 4) {
        c0 = *reinterpret_cast<const uint4 *>(cbr);
        c1 = *reinterpret_cast<const uint4 *>(cbr + 8);
        chi = reinterpret_cast<const uint32_t *>(cbr)[part];
    } else if constexpr (BITS == 3) {
        c0 = *reinterpret_cast<const uint4 *>(cbr);
        chi = cbr[part];
    } else {
        c0.x = reinterpret_cast<const uint32_t *>(cbr)[part & 1];
        chi = cbr[part >> 1];
    }
    // the wave's outlier run: tile rows 4 wave .. 4 wave + 3
    int32_t oe[5];
#pragma unroll
    for (int r = 0; r < 5; ++r) oe[r] = rp[min(n0 + 4 * wave + r, N)];

    __amdgpu_buffer_rsrc_t ri = __builtin_amdgcn_make_buffer_rsrc((void *)(a.idx + (size_t)n0 * wpr), 0, rows_here * wpr * 4, 0x00020000);
    __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void *)ta.xb, 0, T * K * 32, 0x00020000);
    const uint32_t ioff0 = la * (wpr * 4) + lb * (4 * CW), ioff1 = ioff0 + 16 * (wpr * 4);
    // Index words: a ring of D groups per wave, i.e. D x 2 KB (4 bits) in flight: a CU needs about 64 KB on the
    // way to keep HBM busy, and a group is consumed faster the fewer tokens there are.  A lane's chunk of 32
    // weights is 16, 12 or 8 bytes; the quad reads 64, 48 or 32 contiguous bytes.
    uint32_t iw[D][2][CW];
    // V2a: the library ids of a group travel with its index words.  Lane (i, q) fetches the id of its operand row
    // (row 4 (i % 4) + i / 4 of a block) in row block q % 2, one byte load per group; a row swap hands every lane
    // both blocks' ids when the group is decoded.  Rows past the end read id 0.
    uint32_t gidw[LIB ? D : 1];
    __amdgpu_buffer_rsrc_t rg = __builtin_amdgcn_make_buffer_rsrc((void *)(LIB ? a.gid + (size_t)n0 * G : nullptr), 0,
                                                                  LIB ? rows_here * G : 0u, 0x00020000);
    const uint32_t goff = (16 * (q & 1) + 4 * (i & 3) + (i >> 2)) * G;
    auto load_ids = [&](uint32_t &id, uint32_t g) { id = __builtin_amdgcn_raw_buffer_load_b8(rg, goff, g, 0); };
    auto load_group = [&](uint32_t (&w)[2][CW], uint32_t g) {  // rows past the end of the matrix read zeros
        // plain loads: two neighbouring groups of a row share a 128-byte line and are fetched by different waves at
        // different times; with the non-temporal hint the line often left L2 in between (4 % slower)
        const uint32_t so = g * (16 * CW);
        if constexpr (BITS == 4) {
            const u32x4_t v0 = __builtin_amdgcn_raw_buffer_load_b128(ri, ioff0, so, 0);
            const u32x4_t v1 = __builtin_amdgcn_raw_buffer_load_b128(ri, ioff1, so, 0);
            w[0][0] = v0.x; w[0][1] = v0.y; w[0][2] = v0.z; w[0][3] = v0.w;
            w[1][0] = v1.x; w[1][1] = v1.y; w[1][2] = v1.z; w[1][3] = v1.w;
        } else if constexpr (BITS == 3) {
            const u32x3_t v0 = __builtin_amdgcn_raw_buffer_load_b96(ri, ioff0, so, 0);
            const u32x3_t v1 = __builtin_amdgcn_raw_buffer_load_b96(ri, ioff1, so, 0);
            w[0][0] = v0.x; w[0][1] = v0.y; w[0][2] = v0.z;
            w[1][0] = v1.x; w[1][1] = v1.y; w[1][2] = v1.z;
        } else {
            const u32x2_t v0 = __builtin_amdgcn_raw_buffer_load_b64(ri, ioff0, so, 0);
            const u32x2_t v1 = __builtin_amdgcn_raw_buffer_load_b64(ri, ioff1, so, 0);
            w[0][0] = v0.x; w[0][1] = v0.y;
            w[1][0] = v1.x; w[1][1] = v1.y;
        }
    };
    // B operands of step b of group g, all chunks: lane (token i, k block q) reads 16 bytes, the wave 1 KB
    uint32_t xr[NSLOT][T][4];
    auto load_b = [&](int sl, uint32_t g, int b) {
#pragma unroll
        for (int c = 0; c < T; ++c) {
            const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(rx, lane * 16, (uint32_t)c * (K * 32) + (g * 16 + b * 4) * 256, 0);
            xr[sl][c][0] = v.x; xr[sl][c][1] = v.y; xr[sl][c][2] = v.z; xr[sl][c][3] = v.w;
        }
    };
    __builtin_amdgcn_sched_barrier(0);

    // ---------------------------------------------------------------- a7, first half: the wave's outlier entries
    // The whole outlier term is computed HERE, in front of the first barrier, where a wave otherwise only waits
    // (for its codebook, for the other waves' table parts); its result goes to a plane of its own outside the
    // table region and is picked up by the final sum.
    // Lane (e8, o8) = (lane / OP, lane % OP) takes entries e8, e8 + EP, ... of each of the wave's four rows and the
    // eight tokens 8 o8 .. 8 o8 + 7, where OP is the number of token octets rounded up to a power of two (2, 4 or 8)
    // and EP = 64 / OP the entries one wave instruction covers (32, 16 or 8).  The run's first 128 (column, value)
    // pairs are fetched with lane = entry, four load instructions per wave (a CU keeps only about 64 vector-memory instructions in flight, and at
    // this point every wave of the chip wants its codebook), and dealt to their lanes through the LDS crossbar.
    constexpr int OP = T == 1 ? 2 : T == 2 ? 4 : 8, EP = 64 / OP;
    constexpr int JP = 32 / EP;                            // EP JP = 32 entries of a row without a loop
    constexpr int RB = JP == 4 ? 2 : 4;                    // rows whose gathers are issued together
    const uint32_t e8 = lane / OP, o8 = lane % OP;
    uint32_t run[2];                                       // column | value << 16 of run entries lane, 64 + lane
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int32_t e = oe[0] + 64 * h + (int32_t)lane;
        run[h] = e < oe[4] ? (uint32_t)a.col[e] | ((uint32_t)a.val[e] << 16) : 0u;
    }
    __builtin_amdgcn_sched_barrier(0);
    if (wave < G) {
        if constexpr (LIB) load_ids(gidw[0], wave);
        load_group(iw[0], wave);
#pragma unroll
        for (int b = 0; b < NSLOT; ++b) load_b(b, wave, b);
    }
    __builtin_amdgcn_sched_barrier(0);

    // MODE 2: the tile's scales and mid-points -> LDS, element (group g, tile row 16 rb + 4 r + q) at dword
    // ((2 g + rb) * 4 + q) * 4 + r, so that lane (i, q) reads the four rows of its accumulator registers in a row
    // block with one 16-byte read.  Rows past the end of the matrix: scale 0, mid 0.
    if constexpr (AFF) {
        for (uint32_t e = tid; e < 32u * G; e += kWideThreads) {
            const uint32_t row = e / G, g = e - row * G;
            uint32_t v = 0u;
            if (row < rows_here)
                v = (uint32_t)a.gscale[(size_t)(n0 + row) * G + g] | ((uint32_t)a.gmid[(size_t)(n0 + row) * G + g] << 16);
            const uint32_t rb = row >> 4, r = (row & 15) >> 2, qq = row & 3;
            *(lds_u32_t *)(uintptr_t)(lds0 + L::kAff + ((((2 * g + rb) * 4 + qq) * 4 + r) * 4)) = v;
        }
    }
    // ---------------------------------------------------------------- a2: the tile's pair tables
    if constexpr (LIB) {
        // item = (library entry l, second index hi): the 2^BITS consecutive entries (first index 0.., hi) of l's
        // table, entry e = hi * 2^BITS + first index of library entry l at byte (l * 4^BITS + e) * 4
        constexpr uint32_t E1 = 1u << BITS;
        for (uint32_t item = tid; item < (a.L << BITS); item += kWideThreads) {
            const uint16_t *cbk = a.cb + (size_t)(item >> BITS) * E1;
            const uint32_t hiv = (uint32_t)cbk[item & (E1 - 1u)] << 16;
            uint32_t lw[E1 / 2];
            if constexpr (BITS == 4) {
                const uint4 v0 = *reinterpret_cast<const uint4 *>(cbk), v1 = *reinterpret_cast<const uint4 *>(cbk + 8);
                lw[0] = v0.x; lw[1] = v0.y; lw[2] = v0.z; lw[3] = v0.w; lw[4] = v1.x; lw[5] = v1.y; lw[6] = v1.z; lw[7] = v1.w;
            } else if constexpr (BITS == 3) {
                const uint4 v0 = *reinterpret_cast<const uint4 *>(cbk);
                lw[0] = v0.x; lw[1] = v0.y; lw[2] = v0.z; lw[3] = v0.w;
            } else {
                const uint2 v0 = *reinterpret_cast<const uint2 *>(cbk);
                lw[0] = v0.x; lw[1] = v0.y;
            }
            const uint32_t base = lds0 + item * (E1 * 4);
#pragma unroll
            for (uint32_t j = 0; j < E1; j += 4) {
                u32x4_t o;
                o.x = (lw[j / 2] & 0xFFFFu) | hiv; o.y = (lw[j / 2] >> 16) | hiv;
                o.z = (lw[j / 2 + 1] & 0xFFFFu) | hiv; o.w = (lw[j / 2 + 1] >> 16) | hiv;
                *(__attribute__((address_space(3))) u32x4_t *)(uintptr_t)(base + j * 4) = o;
            }
        }
    } else {
        const uint32_t clo[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
        constexpr int EPT = (int)ENT / 8;                  // entries per thread: 32, 8, 2
        const uint32_t base = lds0 + part * (EPT * 256) + slot * 4;
#pragma unroll
        for (int j = 0; j < EPT; ++j) {                    // entry part * EPT + j = first index + 2^BITS * second index
            const int lo = BITS == 2 ? j : j % (1 << BITS);                // within this thread's codebook words
            const uint32_t lw = clo[lo / 2];
            const uint32_t lov = (lo & 1) ? lw >> 16 : lw & 0xFFFFu;
            const uint32_t hiv = (BITS == 4 && j >= 16) ? chi & 0xFFFF0000u : chi << 16;
            *(lds_u32_t *)(uintptr_t)(base + j * 256) = lov | hiv;
        }
    }
    __builtin_amdgcn_sched_barrier(0);

    // ---------------------------------------------------------------- a7, second half: gather, multiply, reduce
    // One 16-byte read per lane fetches the eight tokens' activations at the entry's column from the k-major
    // copy (a wave instruction covers EP entries x all tokens); a lane sums its entries of a row in entry order,
    // the EP lanes of a token octet are then added in a fixed tree, and lanes 0 .. OP - 1 write the row's sums to
    // the ninth plane.
    auto outlier_term = [&]() {
        constexpr uint32_t OCT = 2 * T;                    // token octets of the copies
        const uint4 *xt4 = reinterpret_cast<const uint4 *>(ta.xt) + min(o8, OCT - 1);
        constexpr uint32_t kNone = 0x8000u;                // no entry: bit 15, which no column has (K <= 32768), and value 0
        auto gather = [&](uint32_t ent) {
            uint4 g = make_uint4(0u, 0u, 0u, 0u);
            if (!(ent & kNone)) g = xt4[(size_t)(ent & 0x7FFFu) * OCT];
            return g;
        };
        auto mac8 = [&](float (&acc8)[8], uint32_t ent, const uint4 &g) {
            const float v = half_bits_to_float((uint16_t)(ent >> 16));     // no entry: value 0 times zeros
            const uint32_t w[4] = {g.x, g.y, g.z, g.w};
#pragma unroll
            for (int t = 0; t < 8; ++t)
                acc8[t] = fmaf(v, half_bits_to_float((uint16_t)(t & 1 ? w[t / 2] >> 16 : w[t / 2] & 0xFFFFu)), acc8[t]);
        };
        // entry EP j + e8 of row r, as (column | value << 16): from the run registers when it is among the run's
        // first 128, else from memory
        uint32_t pent[4][JP];
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int j = 0; j < JP; ++j) {
                const int32_t e = oe[r] + EP * j + (int32_t)e8;
                const uint32_t pos = (uint32_t)(e - oe[0]);
                const uint32_t v0 = (uint32_t)__builtin_amdgcn_ds_bpermute((int)((pos & 63u) * 4u), (int)run[0]);
                const uint32_t v1 = (uint32_t)__builtin_amdgcn_ds_bpermute((int)((pos & 63u) * 4u), (int)run[1]);
                uint32_t ent = pos < 64u ? v0 : v1;
                if (pos >= 128u && e < oe[r + 1]) ent = (uint32_t)a.col[e] | ((uint32_t)a.val[e] << 16);
                pent[r][j] = e < oe[r + 1] ? ent : kNone;
            }
        const uint32_t ob = lds0 + L::kOut + (8 * o8 * kTokStride + 4 * wave) * 4;
#pragma unroll
        for (int h = 0; h < 4 / RB; ++h) {                 // RB rows at a time: RB JP gathers in flight
            uint4 gx[RB][JP];
#pragma unroll
            for (int r = 0; r < RB; ++r)
#pragma unroll
                for (int j = 0; j < JP; ++j) gx[r][j] = gather(pent[RB * h + r][j]);
#pragma unroll
            for (int r = 0; r < RB; ++r) {
                const int row = RB * h + r;
                float s8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int j = 0; j < JP; ++j) mac8(s8, pent[row][j], gx[r][j]);
                // rows with more than 32 entries (wave-uniform loop)
                for (int32_t e0 = oe[row] + EP * JP; e0 < oe[row + 1]; e0 += EP) {
                    const int32_t e = e0 + (int32_t)e8;
                    const uint32_t ent = e < oe[row + 1] ? (uint32_t)a.col[e] | ((uint32_t)a.val[e] << 16) : kNone;
                    mac8(s8, ent, gather(ent));
                }
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    // over the EP entry lanes (those with the same lane % OP), VALU only: rotations inside the
                    // row of 16 lanes, then the two row swaps (both copies of x go in, the two results are the
                    // lane's own half and its partner's)
                    float x = s8[t];
                    if constexpr (OP <= 2) x = dpp_add<0x122>(x);          // row_ror:2
                    if constexpr (OP <= 4) x = dpp_add<0x124>(x);          // row_ror:4
                    x = dpp_add<0x128>(x);                                 // row_ror:8
                    const uint32_t xb16 = __builtin_bit_cast(uint32_t, x);
                    const auto p16 = __builtin_amdgcn_permlane16_swap(xb16, xb16, false, false);
                    x = __builtin_bit_cast(float, (uint32_t)p16[0]) + __builtin_bit_cast(float, (uint32_t)p16[1]);
                    const uint32_t xb32 = __builtin_bit_cast(uint32_t, x);
                    const auto p32 = __builtin_amdgcn_permlane32_swap(xb32, xb32, false, false);
                    x = __builtin_bit_cast(float, (uint32_t)p32[0]) + __builtin_bit_cast(float, (uint32_t)p32[1]);
                    if (e8 == 0 && o8 < OCT) *(lds_f32_t *)(uintptr_t)(ob + (t * kTokStride + row) * 4) = x;
                }
            }
        }
    };
    outlier_term();
    __builtin_amdgcn_sched_barrier(0);
    // the rest of the ring of index words (their registers were the outlier term's until here)
#pragma unroll
    for (int d = 1; d < D; ++d)
        if (wave + d * kWideWaves < G) {
            if constexpr (LIB) load_ids(gidw[d], wave + d * kWideWaves);
            load_group(iw[d], wave + d * kWideWaves);
        }
    lds_barrier();

    // ---------------------------------------------------------------- a3-a6: the wave's groups
    float4_t acc[2][T];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int c = 0; c < T; ++c) acc[rb][c] = float4_t{0.f, 0.f, 0.f, 0.f};
    const uint32_t sel = (((q & 1) << 4) | i) * 4;         // this lane's bank in a row block's 32 slots
    // one group: its index words sit in ring slot d, which is refilled with the group D turns ahead once the last
    // lookup address has been formed from it
    auto group_body = [&](auto dtag, uint32_t g) {
        constexpr int d = decltype(dtag)::value;
        // four pieces of 8 weights per row block (a dword at 4 bits, 24 bits at 3, 16 at 2; bits above a piece
        // are ignored), then the transposition to the operand layout.  At 4 bits the pieces ARE the index words:
        // they are transposed in place and the slot is refilled once its last lookup address is formed; at 3 and
        // 2 bits the pieces are registers of their own and the slot is refilled at once.
        uint32_t pw_own[BITS == 4 ? 1 : 2][4];
        uint32_t (&pw)[2][4] = pieces_of(iw[d], pw_own);
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            if constexpr (BITS == 3) {
                const uint32_t (&w)[CW] = iw[d][rb];
                pw[rb][0] = w[0];
                pw[rb][1] = __builtin_amdgcn_alignbit(w[1], w[0], 24);
                pw[rb][2] = __builtin_amdgcn_alignbit(w[2], w[1], 16);
                pw[rb][3] = w[2] >> 8;
            } else if constexpr (BITS == 2) {
                const uint32_t (&w)[CW] = iw[d][rb];
                pw[rb][0] = w[0]; pw[rb][1] = w[0] >> 16; pw[rb][2] = w[1]; pw[rb][3] = w[1] >> 16;
            }
            to_operand_layout(pw[rb]);
        }
        constexpr int REFILL_STEP = BITS == 4 ? 2 : 0;
        const bool more = g + kWideWaves < G;
        uint32_t gtab[2] = {0u, 0u};                       // V2a: byte offset of the group's table for either row block
        if constexpr (LIB) {
            // lanes 0..15 and 32..47 hold block 0's ids, the others block 1's: the swap gives every lane both
            const auto both = __builtin_amdgcn_permlane16_swap(gidw[d], gidw[d], false, false);
            gtab[0] = (uint32_t)both[0] * (ENT * 4);
            gtab[1] = (uint32_t)both[1] * (ENT * 4);
        }
        uint32_t av[2][2][4];
        auto lookup = [&](int b, uint32_t (&v)[2][4]) {
#pragma unroll
            for (int rb = 0; rb < 2; ++rb) {
                const uint32_t w = pw[rb][b];
                if constexpr (LIB) {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        v[rb][j] = *(lds_cu32_t *)(uintptr_t)((((w >> (2 * BITS * j)) & (ENT - 1u)) << 2) | gtab[rb]);
                } else if constexpr (BITS == 4) {
                    v[rb][0] = *(lds_cu32_t *)(uintptr_t)(__builtin_amdgcn_perm(w, sel, 0x0c0c0400u) + rb * 128);
                    v[rb][1] = *(lds_cu32_t *)(uintptr_t)(__builtin_amdgcn_perm(w, sel, 0x0c0c0500u) + rb * 128);
                    v[rb][2] = *(lds_cu32_t *)(uintptr_t)(__builtin_amdgcn_perm(w, sel, 0x0c0c0600u) + rb * 128);
                    v[rb][3] = *(lds_cu32_t *)(uintptr_t)(__builtin_amdgcn_perm(w, sel, 0x0c0c0700u) + rb * 128);
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        v[rb][j] = *(lds_cu32_t *)(uintptr_t)(((((w >> (2 * BITS * j)) & (ENT - 1u)) << 8) | sel) + rb * 128);
                }
            }
        };
        // MODE 2: the group's own block, its scales and mid-points (requested now, used after the fourth step) and
        // the token's activation sum over the group
        float4_t dg[2] = {float4_t{0.f, 0.f, 0.f, 0.f}, float4_t{0.f, 0.f, 0.f, 0.f}};
        u32x4_t sm[2] = {u32x4_t{0u, 0u, 0u, 0u}, u32x4_t{0u, 0u, 0u, 0u}};
        float sxg = 0.f;
        if constexpr (AFF) {
            typedef __attribute__((address_space(3))) const u32x4_t lds_cu4_t;
#pragma unroll
            for (int rb = 0; rb < 2; ++rb) sm[rb] = *(lds_cu4_t *)(uintptr_t)(lds0 + L::kAff + (((2 * g + rb) * 4 + q) * 16));
            sxg = ta.sx[g * 16 + i];
        }
        lookup(0, av[0]);
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            if (b < 3) lookup(b + 1, av[(b + 1) & 1]);
            if (b == REFILL_STEP && g + D * kWideWaves < G) {
                if constexpr (LIB) load_ids(gidw[d], g + D * kWideWaves);
                load_group(iw[d], g + D * kWideWaves);
            }
            __builtin_amdgcn_sched_barrier(0);
            const uint32_t (&cur)[2][4] = av[b & 1];
#pragma unroll
            for (int c = 0; c < T; ++c) {
                const uint32_t (&xv)[4] = xr[b % NSLOT][c];
                const half8_t bf = __builtin_bit_cast(half8_t, u32x4_t{xv[0], xv[1], xv[2], xv[3]});
#pragma unroll
                for (int rb = 0; rb < 2; ++rb) {
                    const half8_t af = __builtin_bit_cast(half8_t, u32x4_t{cur[rb][0], cur[rb][1], cur[rb][2], cur[rb][3]});
                    if constexpr (AFF) dg[rb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(af, bf, dg[rb], 0, 0, 0);
                    else acc[rb][c] = __builtin_amdgcn_mfma_f32_16x16x32_f16(af, bf, acc[rb][c], 0, 0, 0);
                }
            }
            // the ring slot is free: the B operands NSLOT steps ahead
            if (b + NSLOT < 4) load_b(b % NSLOT, g, b + NSLOT);
            else if (more) load_b(b % NSLOT, g + kWideWaves, b + NSLOT - 4);
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (AFF) {
            // register r of a block is its row 4 r + q: scale * D_g + mid * (sum of the token's activations)
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float sc = half_bits_to_float((uint16_t)(sm[rb][r] & 0xFFFFu)), md = half_bits_to_float((uint16_t)(sm[rb][r] >> 16));
                    acc[rb][0][r] = fmaf(md, sxg, fmaf(sc, dg[rb][r], acc[rb][0][r]));
                }
        }
    };
    for (uint32_t g = wave; g < G; g += D * kWideWaves) {
#define XFP_WIDE_STAGE(d)                                                                                  \
        if constexpr (d < D) {                                                                             \
            if (d == 0 || g + d * kWideWaves < G) group_body(std::integral_constant<int, d>{}, g + d * kWideWaves); \
        }
        XFP_WIDE_STAGE(0) XFP_WIDE_STAGE(1) XFP_WIDE_STAGE(2) XFP_WIDE_STAGE(3) XFP_WIDE_STAGE(4) XFP_WIDE_STAGE(5)
#undef XFP_WIDE_STAGE
    }

    // ---------------------------------------------------------------- a8: partial sums -> planes (the tables are dead)
    lds_barrier();
    {
        const uint32_t pb = lds0 + wave * L::kPlane;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int c = 0; c < T; ++c)
#pragma unroll
                for (int r = 0; r < 4; ++r)    // lane (token i, q), register r: operand row 4 q + r = row 4 r + q of the block
                    *(lds_f32_t *)(uintptr_t)(pb + ((c * 16 + i) * kTokStride + rb * 16 + 4 * r + q) * 4) = acc[rb][c][r];
    }

    lds_barrier();

    // ---------------------------------------------------------------- sum of the nine planes, store
    {
        const uint32_t t = tid >> 3, r0 = (tid & 7) * 4;   // token, first of four rows
        if (t < MP) {
            float s[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int w = 0; w < kWideWaves; ++w)
#pragma unroll
                for (int r = 0; r < 4; ++r) s[r] += *(lds_f32_t *)(uintptr_t)(lds0 + w * L::kPlane + (t * kTokStride + r0 + r) * 4);
#pragma unroll
            for (int r = 0; r < 4; ++r) s[r] += *(lds_f32_t *)(uintptr_t)(lds0 + L::kOut + (t * kTokStride + r0 + r) * 4);
            if (t < (uint32_t)ta.M) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (n0 + r0 + r < N) store_out(a.y, (int64_t)t * a.y_stride + n0 + r0 + r, s[r], ta.y_f32 != 0, a.y_bf16 != 0);
            }
        }
    }
}

// blocks [0, K T / 128): xt, one thread per (k, token octet); the rest: xb, one thread per (chunk, k block, token).
// Tokens >= M are zero in both; bf16 activations are converted to fp16 on the way.
// sx (may be null): [K / 128][16] sums of a token's activations (as fp16 values) over a group, in fp32, k ascending:
// the blocks behind the other two, one thread per (group, token), T = 1 only.
__global__ __launch_bounds__(256) void relayout_x_wide_kernel(const uint16_t *x, int64_t ldx, int M, uint32_t K, int T,
                                                              int bf16, uint16_t *xt, uint16_t *xb, float *sx)
{
    const uint32_t nb_t = (K * 2 * (uint32_t)T + 255) / 256;
    const uint32_t nb_b = (K / 8 * 16 * (uint32_t)T + 255) / 256;
    if (blockIdx.x >= nb_t + nb_b) {
        const uint32_t id = (blockIdx.x - nb_t - nb_b) * 256 + threadIdx.x;   // = group * 16 + token
        if (id >= K / kGroup * 16) return;
        const uint32_t g = id >> 4, m = id & 15;
        float s0 = 0.f, s1 = 0.f;
        if ((int)m < M) {
            const uint4 *p = reinterpret_cast<const uint4 *>(x + (size_t)m * ldx + (size_t)g * kGroup);
            const half2_t ones = __builtin_bit_cast(half2_t, 0x3C003C00u);
#pragma unroll 4
            for (int j = 0; j < kGroup / 8; ++j) {
                uint4 v = p[j];
                if (bf16) v = make_uint4(bf16x2_to_f16x2(v.x), bf16x2_to_f16x2(v.y), bf16x2_to_f16x2(v.z), bf16x2_to_f16x2(v.w));
                s0 = dot2(as_half2(v.x), ones, s0); s1 = dot2(as_half2(v.y), ones, s1);
                s0 = dot2(as_half2(v.z), ones, s0); s1 = dot2(as_half2(v.w), ones, s1);
            }
        }
        sx[id] = s0 + s1;
        return;
    }
    if (blockIdx.x < nb_t) {
        const uint32_t id = blockIdx.x * 256 + threadIdx.x;               // = k * 2 T + octet
        if (id >= K * 2 * (uint32_t)T) return;
        const uint32_t k = id / (2 * (uint32_t)T), c = id - k * (2 * (uint32_t)T);
        uint32_t v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int m = 8 * (int)c + 2 * j;
            const uint32_t lo = m < M ? x[(size_t)m * ldx + k] : 0u;
            const uint32_t hi = m + 1 < M ? x[(size_t)(m + 1) * ldx + k] : 0u;
            v[j] = lo | (hi << 16);
            if (bf16) v[j] = bf16x2_to_f16x2(v[j]);
        }
        reinterpret_cast<uint4 *>(xt)[id] = make_uint4(v[0], v[1], v[2], v[3]);
    } else {
        const uint32_t id = (blockIdx.x - nb_t) * 256 + threadIdx.x;      // = (chunk * K / 8 + k block) * 16 + token of the chunk
        const uint32_t per = K / 8 * 16;
        if (id >= per * (uint32_t)T) return;
        const uint32_t c = id / per, rem = id - c * per, kb = rem >> 4, m = c * 16 + (rem & 15);
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if ((int)m < M) v = *reinterpret_cast<const uint4 *>(x + (size_t)m * ldx + (size_t)kb * 8);
        if (bf16) v = make_uint4(bf16x2_to_f16x2(v.x), bf16x2_to_f16x2(v.y), bf16x2_to_f16x2(v.z), bf16x2_to_f16x2(v.w));
        reinterpret_cast<uint4 *>(xb)[id] = v;
    }
}

template <int BITS, int T, int MODE>
hipError_t launch_wide_t(const WideArgs &ta, hipStream_t s)
{
    // MODE 2: plus the tile's scales and mid-points, 128 bytes per group (the attribute is set for the longest row)
    constexpr int kLdsMax = WideLds<BITS, T, MODE>::kTotal + (MODE == 2 ? kXtMaxK : 0);
    const int kLds = WideLds<BITS, T, MODE>::kTotal + (MODE == 2 ? (int)(ta.a.K / kGroup) * 128 : 0);
    auto kern = decode_wide_kernel<BITS, T, MODE>;
    static std::atomic<int> configured[kMaxDevices];       // per device; idempotent attribute, benign race
    const int dev = current_device();
    if (dev < 0) return hipErrorInvalidDevice;
    if (!configured[dev].load(std::memory_order_relaxed)) {
        hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, kLdsMax);
        if (err != hipSuccess) return err;
        configured[dev].store(1, std::memory_order_relaxed);
    }
    hipLaunchKernelGGL(kern, dim3((ta.a.N + kWideRows - 1) / kWideRows), dim3(kWideThreads), kLds, s, ta);
    return hipGetLastError();
}

template <int BITS, int MODE>
hipError_t launch_wide_b(const WideArgs &ta, int T, hipStream_t s)
{
    switch (T) {
    case 1: return launch_wide_t<BITS, 1, MODE>(ta, s);
    case 2: return launch_wide_t<BITS, 2, MODE>(ta, s);
    case 3: return launch_wide_t<BITS, 3, MODE>(ta, s);
    default: return launch_wide_t<BITS, 4, MODE>(ta, s);
    }
}

}  // namespace

// V2 and V2a (library tables within 64 KB) at 2 to 4 bits, up to 64 tokens whose re-laid copies fit the workspace
// (16 ceil(M / 16) K halves each).
// mode: 0 V2, 1 V2a, 2 V2a with a scale and a mid-point per group (16 tokens per launch).
bool wide_supports(int bits, int mode, uint32_t L, uint32_t N, uint32_t K, int M, uint64_t copy_cap)
{
    if (!(bits >= 2 && bits <= 4 && M >= 1 && M <= 64 && K % kGroup == 0 && K >= kGroup && N >= 1)) return false;
    if (!(mode == 0 || ((mode == 1 || mode == 2) && L >= 1 && ((uint64_t)L << (2 * bits)) * 4 <= (uint64_t)kWideLibTab))) return false;
    if (mode == 2 && (M > 16 || K > (uint32_t)kXtMaxK)) return false;
    return (uint64_t)K * 16u * (uint64_t)((M + 15) / 16) <= copy_cap && (uint64_t)K * 32u * 4u <= 0xFFFFFFFFull;
}

// M <= 64 tokens in one pass over the weights.  xc: the workspace's re-laid activation copies, written by a
// small kernel in front of the decode kernel (launches on one stream may share them).
// sx: MODE 2 only, room for 16 K / 128 floats (a scratch plane of the workspace).
hipError_t launch_decode_wide(int bits, int mode, const DecodeArgs &a, int M, bool y_f32, XCopies *xc, float *sx, hipStream_t s)
{
    if (!xc || bits < 2 || bits > 4 || M < 1 || M > 64 || mode < 0 || mode > 2) return hipErrorInvalidValue;
    if (mode == 2 && (!sx || M > 16 || !a.gscale || !a.gmid)) return hipErrorInvalidValue;
    const int T = (M + 15) / 16;
    const uint32_t nb = (a.K * 2 * (uint32_t)T + 255) / 256 + (a.K / 8 * 16 * (uint32_t)T + 255) / 256 +
                        (mode == 2 ? (a.K / kGroup * 16 + 255) / 256 : 0u);
    hipLaunchKernelGGL(relayout_x_wide_kernel, dim3(nb), dim3(256), 0, s, a.x, a.x_stride, M, a.K, T, (int)a.x_bf16, xc->xt, xc->xb,
                       mode == 2 ? sx : nullptr);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    WideArgs ta;
    ta.a = a;
    ta.xt = xc->xt;
    ta.xb = xc->xb;
    ta.sx = mode == 2 ? sx : nullptr;
    ta.M = M;
    ta.y_f32 = (int)y_f32;
    if (mode == 2)
        return bits == 4 ? launch_wide_t<4, 1, 2>(ta, s) : bits == 3 ? launch_wide_t<3, 1, 2>(ta, s) : launch_wide_t<2, 1, 2>(ta, s);
    if (mode == 1) return bits == 4 ? launch_wide_b<4, 1>(ta, T, s) : bits == 3 ? launch_wide_b<3, 1>(ta, T, s) : launch_wide_b<2, 1>(ta, T, s);
    return bits == 4 ? launch_wide_b<4, 0>(ta, T, s) : bits == 3 ? launch_wide_b<3, 0>(ta, T, s) : launch_wide_b<2, 0>(ta, T, s);
}

}  // namespace xfp
