// Streaming fused decode kernel, M = 1 per slot, V2 (one codebook per output
// channel) and V2a (a library of codebooks plus one id per 128-weight group).
// This is the fast path for the shapes decode actually sees.
//
// Work unit: one wave owns a run of output rows.  V2: a workgroup is a single
// wave, so nothing ever waits at a barrier and every LDS address is a
// compile-time constant that folds into the lookups' offset field.  V2a: a
// workgroup is four waves that share the library's tables (one barrier after
// they are built, none afterwards).  Design points, all for gfx950:
//  - The activation row lives in VGPRs, not LDS: lane l always decodes the
//    same k range of every row (32 consecutive k per 2048-wide chunk), so its
//    32 activations per chunk are loaded once per wave and reused for every
//    row.  This is the paper's activation-row caching (section 5) moved one
//    level closer to the ALUs; it leaves the LDS pipe to the codebook lookups.
//  - Index words are streamed with one 16-byte (4-bit), 12-byte (3-bit) or
//    8-byte (2-bit) load per lane per chunk; a wave issues the loads of a
//    whole batch of rows before it touches any of them, and no load is
//    conditional (out-of-range rows and lanes read a clamped address).
//  - Codebook lookups go to LDS, through a pair table (two indices -> two
//    fp16 in one dword) built per row (V2) or per library codebook (V2a, once
//    per workgroup): one lookup and one v_dot2_f32_f16 serve two weights, and
//    the address of an entry is one SDWA shift of an index byte (4-/2-bit) or a
//    shift and a mask (3-bit).  V2a: the group's library id picks the table
//    per lane; it is OR-ed into the lookup address.  The lookups of 64 lanes
//    into one row's table are random and collide on the 32 banks (5.5 clocks
//    per wave instruction against 2.6 conflict-free): this, not HBM, is what
//    bounds the 4-bit kernel once the data is flowing.
//  - Lookups are software-pipelined in groups of eight: the addresses and LDS
//    reads of group t+1 are issued before the multiply-accumulates of group t.
//  - fp32 accumulation in a fixed order, DPP reduction, no atomics: results
//    are run-to-run deterministic.
//  - The CSR outliers of a batch of rows are contiguous; they are fetched with
//    one bounds-checked buffer load per lane while the index stream is still
//    in flight and folded into the owning row's sum before the reduction.
//  - Variants (compile-time, one translation unit each): split-K for rows
//    longer than a wave holds in registers, and a gate/up form that pairs each
//    gate row with its up row in a batch and stores SiLU(gate) * up.
#pragma once
#include "xfp_device.h"

#include <type_traits>

namespace xfp {
namespace {

typedef __attribute__((address_space(3))) const uint16_t lds_u16_t;
typedef __attribute__((address_space(3))) const uint32_t lds_u32_t;
typedef __attribute__((address_space(3))) uint32_t lds_u32_w_t;

#define XFP_SDWA_BYTE(op, dst, amount, src, J)                                                   \
    asm(op " %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_" #J     \
        : "=v"(dst) : "v"(amount), "v"(src))

// (byte j of m) << amount and (byte j of m) >> amount in one VALU op each.
// j must be a compile-time constant after unrolling.
__device__ __forceinline__ uint32_t byte_shl(uint32_t m, int j, uint32_t amount)
{
    uint32_t r;
    switch (j) {
    case 0: XFP_SDWA_BYTE("v_lshlrev_b32_sdwa", r, amount, m, 0); break;
    case 1: XFP_SDWA_BYTE("v_lshlrev_b32_sdwa", r, amount, m, 1); break;
    case 2: XFP_SDWA_BYTE("v_lshlrev_b32_sdwa", r, amount, m, 2); break;
    default: XFP_SDWA_BYTE("v_lshlrev_b32_sdwa", r, amount, m, 3); break;
    }
    return r;
}
__device__ __forceinline__ uint32_t byte_shr(uint32_t m, int j, uint32_t amount)
{
    uint32_t r;
    switch (j) {
    case 0: XFP_SDWA_BYTE("v_lshrrev_b32_sdwa", r, amount, m, 0); break;
    case 1: XFP_SDWA_BYTE("v_lshrrev_b32_sdwa", r, amount, m, 1); break;
    case 2: XFP_SDWA_BYTE("v_lshrrev_b32_sdwa", r, amount, m, 2); break;
    default: XFP_SDWA_BYTE("v_lshrrev_b32_sdwa", r, amount, m, 3); break;
    }
    return r;
}

// Geometry of the per-row LDS table for each bit width.  A pair table maps two
// adjacent indices (4, 6 or 8 stream bits) to two fp16 values in one dword.
template <int BITS>
struct TableFmt {
    static constexpr int kEntries = 1 << BITS;
    static constexpr int kRowBytes = 4 << (2 * BITS);          // 64, 256, 1024
    static constexpr int kRawBytes = 2 * kEntries;             // 8, 16, 32: the codebook itself
    static constexpr int kGroupsPerLaneLoad = 2;               // groups of 8 lookups (16 pairs = 32 weights)
};

// Eight lookups of one lane-load: compute LDS addresses and issue the reads.
//   tb    LDS byte address of the table (wave-uniform, folds into the offset field)
//   bias  per-lane table selector added on top of tb when BIASED: the number of
//         tables to skip (row of a multi-row chunk, or the all-zero table for
//         lanes past the end of a short row).  It is OR-ed into the index bytes
//         (4-/2-bit) or the address (3-bit), which costs no extra instruction.
//         WIDE: the selector may exceed 15 (a V2a library id); for 2-bit indices
//         it is then OR-ed into the address instead of the index bytes.
template <int BITS, bool BIASED, bool WIDE = false>
__device__ __forceinline__ void issue_group(const LaneWords<BITS> &lw, int g, uint32_t tb, uint32_t bias,
                                            uint32_t (&v)[8], uint32_t k2)
{
    if constexpr (BITS == 4) {
        // an index byte (two indices) selects one dword of the row's 256-entry pair table
        const uint32_t ab = BIASED ? bias * TableFmt<4>::kRowBytes : 0u;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t a = byte_shl(lw.w[2 * g + (i >> 2)], i & 3, k2);   // byte * 4
            v[i] = *(lds_u32_t *)(uintptr_t)(tb + (BIASED ? (a | ab) : a));
        }
    } else if constexpr (BITS == 3) {
        const uint32_t ab = BIASED ? bias * TableFmt<3>::kRowBytes : 0u;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int bit = 6 * (g * 8 + i), word = bit / 32, sh = bit % 32;   // pair = 6 stream bits
            uint32_t t;
            if (sh + 6 <= 32) t = sh >= 2 ? lw.w[word] >> (sh - 2) : lw.w[word] << (2 - sh);
            else t = __builtin_amdgcn_alignbit(lw.w[(word + 1) % 3], lw.w[word], sh - 2);
            const uint32_t a = BIASED ? ((t & 0xFCu) | ab) : (t & 0xFCu);      // pair index * 4
            v[i] = *(lds_u32_t *)(uintptr_t)(tb + a);
        }
    } else {
        const uint32_t w = lw.w[g];
        uint32_t m0, m1;
        const uint32_t ab = (BIASED && WIDE) ? bias * TableFmt<2>::kRowBytes : 0u;
        if constexpr (BIASED) {
            const uint32_t bb = WIDE ? 0u : bias * 0x10101010u;
            m0 = (w & 0x0F0F0F0Fu) | bb;
            m1 = ((w >> 4) & 0x0F0F0F0Fu) | bb;
        } else {
            m0 = w & 0x0F0F0F0Fu;
            m1 = w & 0xF0F0F0F0u;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t a0 = byte_shl(m0, j, k2);                             // nibble (= pair) * 4
            uint32_t a1 = BIASED ? byte_shl(m1, j, k2) : byte_shr(m1, j, k2);
            if constexpr (BIASED && WIDE) { a0 |= ab; a1 |= ab; }
            v[2 * j] = *(lds_u32_t *)(uintptr_t)(tb + a0);
            v[2 * j + 1] = *(lds_u32_t *)(uintptr_t)(tb + a1);
        }
    }
}

// Multiply-accumulate the eight looked-up values of group g against the
// matching activations xw[0..15] of the lane-load.
template <int BITS>
__device__ __forceinline__ void consume_group(int g, const uint32_t (&v)[8], const uint32_t *xw, float (&acc)[4])
{
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i & 3] = dot2(as_half2(v[i]), as_half2(xw[g * 8 + i]), acc[i & 3]);
}

// NCH : 2048-wide chunks per row (RPC == 1), K <= NCH * 2048
// RPC : rows per chunk (K == 2048 / RPC exactly) for short rows; then NCH == 1
// TAIL: K is not a multiple of 2048 (RPC == 1): lanes past the row's end in the
//       last chunk read a clamped address, zero activations and the zero table
// MODE: 0 V2 (a codebook per row); 1 V2a (a library, an id per group); 2 V2a with a scale and a mid-point per
// group (W = entry * scale + mid, paper section 3.4 as read in the descriptor's documentation)
constexpr int stream_waves(int mode) { return mode == 0 ? 1 : 4; }   // waves per workgroup
// waves a launch aims for at most (measured: V2 is fastest with about 16 single-wave
// workgroups per CU, V2a with about 2 four-wave workgroups)
constexpr uint32_t stream_max_waves(int mode) { return mode == 0 ? 6144 : 3072; }

// U: row groups a wave decodes at once (all their loads are issued before the
// first is touched).  The launcher picks the smallest U that lets every wave
// finish its rows in ONE batch, so that nothing is loaded late.
// AFF: the kernel also holds a scale and a mid-point per lane-load and the lane's activation sums.
template <int BITS, int NCH, int RPC, int U_, bool AFF = false>
struct StreamCfg {
    static constexpr int kUnroll = U_;
    static constexpr int kBatchRows = kUnroll * RPC;           // rows a wave decodes at once
    static constexpr int kLanesPerRow = kWave / RPC;
    static constexpr int kTableBytes = (kBatchRows + 1) * TableFmt<BITS>::kRowBytes;   // + zero table
    static constexpr int kRawBytes = kBatchRows * TableFmt<BITS>::kRawBytes;
    // registers: 16 per chunk for x, BITS per lane-load in flight, ~60 working
    static constexpr int kRegs = 16 * NCH + BITS * NCH * kUnroll + 60 + (AFF ? 2 * NCH * kUnroll + NCH + 4 : 0);
    static constexpr int kWavesPerSimd = kRegs <= 128 ? 4 : (kRegs <= 168 ? 3 : 2);
    // largest U the registers allow (x: 16 per chunk; index words: BITS per chunk and row group)
    static constexpr bool kFits = BITS * NCH * kUnroll <= 64 && kRegs <= 250;
};

// LDS byte address of a static array of BYTES bytes (one per instantiation).
template <int BYTES>
__device__ __forceinline__ uint32_t static_lds()
{
    __shared__ __align__(16) unsigned char buf[BYTES];
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)buf;
}

// VAR: 0 plain; 1 split-K (grid z = slice of K, fp32 partial sums); 2 gate/up
// rows paired in a batch and SiLU(gate) * up applied in the store.  Compile-time,
// because every instruction in front of the first loads is on the critical path
// of a call this short.
template <int BITS, int NCH, int RPC, bool TAIL, int MODE, int UNROLL, int VAR>
__global__ __launch_bounds__(stream_waves(MODE) * kWave, (StreamCfg<BITS, NCH, RPC, UNROLL, MODE == 2>::kWavesPerSimd))
void decode_stream_kernel(DecodeArgs a, int y_f32)
{
    constexpr bool SPLIT = VAR == 1, FUSED = VAR == 2;
    constexpr bool LIB = MODE != 0, AFF = MODE == 2;
    static_assert(!AFF || (VAR == 0 && RPC == 1), "scale and mid-point: plain variant, rows of 2048 columns and more");
    constexpr int kStreamWaves = stream_waves(MODE), kStreamThreads = kStreamWaves * kWave;
    using Cfg = StreamCfg<BITS, NCH, RPC, UNROLL, AFF>;
    using Fmt = TableFmt<BITS>;
    constexpr int U = Cfg::kUnroll, B = Cfg::kBatchRows, LPR = Cfg::kLanesPerRow;
    constexpr int ENT = Fmt::kEntries, GPL = Fmt::kGroupsPerLaneLoad;
    // V2: the wave's tables, a static array.  V2a: the library's tables fill the
    // dynamic segment, which starts at LDS address 0 because this instantiation
    // has no static LDS; a constant base keeps the lookups free of address adds.
    uint32_t lds_base = 0u;
    if constexpr (MODE == 0) {
        lds_base = static_lds<Cfg::kTableBytes + Cfg::kRawBytes + 16>();
    } else {
        extern __shared__ __align__(16) unsigned char lds_dyn[];
        if ((uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)lds_dyn != 0u) return;
    }
    const uint32_t lds0 = lds_base;

    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t wv = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const uint32_t seg = RPC > 1 ? lane / LPR : 0u;            // which row of a chunk this lane is in
    const uint32_t lis = RPC > 1 ? lane % LPR : lane;          // lane within its row
    const uint32_t slot = blockIdx.y;
    const uint32_t e = a.eids ? (uint32_t)a.eids[slot] : 0u;
    const uint32_t N = a.N, K = a.K;
    // split-K: this workgroup decodes columns [z K, (z + 1) K) of every row; only
    // slice 0 folds the outliers (their columns index the whole activation row)
    const uint32_t z = SPLIT ? blockIdx.z : 0u;
    const uint32_t wpr = SPLIT ? a.row_words : K / 32 * BITS;          // dwords of a full row
    const uint32_t G = SPLIT ? a.gid_row : K / kGroup;                 // library ids of a full row
    const uint32_t *idx = a.idx + (size_t)e * N * wpr + (size_t)z * (K / 32 * BITS);
    const uint32_t *cbw = reinterpret_cast<const uint32_t *>(a.cb) + (size_t)e * (MODE == 0 ? N : a.L) * (ENT / 2);
    const uint8_t *gid = LIB ? a.gid + (size_t)e * N * G + (size_t)z * (K / kGroup) : nullptr;
    const uint16_t *gsp = AFF ? a.gscale + (size_t)e * N * G : nullptr, *gmp = AFF ? a.gmid + (size_t)e * N * G : nullptr;
    const int32_t *rp = a.rp + (size_t)e * N;
    const uint16_t *x = a.x + (int64_t)slot * a.x_stride + (size_t)z * K;
    const bool with_outliers = !SPLIT || z == 0;

    const bool live_last = !TAIL || ((NCH - 1) * kWave + lis) * kLaneWeights < K;
    const uint32_t unit_last = live_last ? (NCH - 1) * kWave + lis : 0u;

    // Rows of this wave.  A wave past the end of the matrix still runs the
    // prologue (every address below is clamped into the matrix) and leaves
    // before the row loop.
    const uint32_t row_begin = (blockIdx.x * kStreamWaves + wv) * a.rows_per_block;
    const uint32_t row_end = min(N, row_begin + a.rows_per_block);
    // Fused SiLU(gate) * up: a batch is B / 2 gate rows followed by their B / 2 up
    // rows, so that both sums of an output meet in one lane.  Batch row r of the
    // batch that starts at virtual row rb is matrix row arow(rb, r); its CSR
    // boundaries sit in lanes bl(r), bl(r) + 1 of rpv.
    const uint32_t FI = FUSED ? a.fuse_half : 0u;
    auto arow = [&](uint32_t rb, uint32_t r) -> uint32_t {
        return FI ? (r < (uint32_t)B / 2 ? rb / 2 + r : FI + rb / 2 + (r - B / 2)) : rb + r;
    };
    auto bl = [&](uint32_t r) -> uint32_t { return FI ? (r < (uint32_t)B / 2 ? r : 32 + r - B / 2) : r; };
    auto rp_lane = [&](uint32_t rb) -> int32_t {
        if (!with_outliers) return 0;
        if (FI) return rp[min((lane < 32 ? rb / 2 : FI + rb / 2) + (lane & 31), N)];
        return rp[min(rb + lane, N)];
    };
    const uint32_t cb_last = (FI ? N : min(N, max(row_end, 1u))) * (ENT / 2) - 1;   // last valid codebook dword
    auto cb_word = [&](uint32_t rb, uint32_t li) -> uint32_t {             // dword li of the batch's codebooks
        return min(arow(rb, li / (ENT / 2)) * (ENT / 2) + li % (ENT / 2), cb_last);
    };
    const uint32_t k2 = 2;                                     // SDWA shift amount, kept in a VGPR
    constexpr int CBW = (B * (ENT / 2) + kWave - 1) / kWave;   // codebook dwords per lane per batch

    // a3: the index words (and V2a library ids) of one batch of rows; rows past
    // the end are clamped to the last row and never stored.
    LaneWords<BITS> lw[U][NCH];
    uint32_t lib[LIB ? U : 1][LIB ? NCH : 1];
    uint32_t gsc[AFF ? U : 1][AFF ? NCH : 1], gmd[AFF ? U : 1][AFF ? NCH : 1];   // fp16 scale and mid-point of the lane-load's group
    auto load_batch = [&](uint32_t rb) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t row = min(arow(rb, u * RPC + seg), N - 1);
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                const uint32_t unit = c == NCH - 1 ? unit_last : c * kWave + lis;
                lw[u][c] = load_lane_words<BITS>(idx + (size_t)row * wpr + (size_t)unit * BITS);
                if constexpr (LIB) lib[u][c] = gid[(size_t)row * G + unit / (kGroup / kLaneWeights)];
                if constexpr (AFF) {
                    gsc[u][c] = gsp[(size_t)row * G + unit / (kGroup / kLaneWeights)];
                    gmd[u][c] = gmp[(size_t)row * G + unit / (kGroup / kLaneWeights)];
                }
            }
        }
    };

    // Vector loads complete in issue order, so the order below is the order in
    // which their consumers can start: row pointers (they gate the outlier
    // loads), codebooks (they gate the first lookup), activations, index words.
    // Lanes 0..B hold rp[rb + lane]: the CSR boundaries of the batch.
    int32_t rpv = rp_lane(row_begin);
    uint32_t cbv[CBW];
    if constexpr (MODE == 0) {
#pragma unroll
        for (int i = 0; i < CBW; ++i) cbv[i] = cbw[cb_word(row_begin, i * kWave + lane)];
    }
    // V2a: this thread's share of the library, requested ahead of everything that
    // streams (loads return in issue order, and the tables gate the first lookup).
    // Item j = (codebook l = j / ENT, second index hi = j % ENT) builds the ENT
    // pair entries (lo, hi), lo = 0 .. ENT-1, which are contiguous in table l; it
    // needs codebook l (ENT / 2 dwords) and its entry hi.
    constexpr int CW = ENT / 2;
    // The items of a library of up to 32 codebooks (j = tid, tid + threads, ...: PRE per thread) are
    // loaded here, in front of everything that streams: a load inside the build loop is a full memory
    // round trip in front of the barrier, for every wave of the workgroup (it cost workload 3 0.85 of
    // its 5.5 us while the all-zero table's items still went through such a load).
    constexpr int PRE = (32 * ENT + kStreamThreads - 1) / kStreamThreads < 4 ? (32 * ENT + kStreamThreads - 1) / kStreamThreads : 4;
    uint32_t libw[LIB ? PRE : 1][LIB ? CW : 1], libhi[LIB ? PRE : 1];
    if constexpr (LIB) {
#pragma unroll
        for (int p = 0; p < PRE; ++p) {
            const uint32_t j = threadIdx.x + p * kStreamThreads;
            const uint32_t l = min(j / ENT, a.L - 1), hi = j % ENT;
#pragma unroll
            for (int d = 0; d < CW; ++d) libw[p][d] = cbw[l * CW + d];
            libhi[p] = reinterpret_cast<const uint16_t *>(cbw)[l * ENT + hi];
        }
    }
    __builtin_amdgcn_sched_barrier(0);

    // a1: this lane's activations, once per wave.
    uint32_t xr[NCH][16];
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const uint32_t unit = c == NCH - 1 ? unit_last : c * kWave + lis;   // 32-weight unit in the row
        const uint4 *xp = reinterpret_cast<const uint4 *>(x + (size_t)unit * kLaneWeights);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint4 v = xp[i];
            xr[c][4 * i] = v.x; xr[c][4 * i + 1] = v.y; xr[c][4 * i + 2] = v.z; xr[c][4 * i + 3] = v.w;
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    load_batch(row_begin);
    __builtin_amdgcn_sched_barrier(0);

    if constexpr (LIB) {
        // a2 (V2a): the library's pair tables, once per workgroup, while the first
        // loads are in flight.  Table l sits at l * kRowBytes; table L is all zero
        // (lanes past the end of a short row).  One barrier: nothing is staged.
        const uint32_t L = a.L, items = (L + 1) * ENT;
        auto build_item = [&](uint32_t j, const uint32_t (&w)[CW], uint32_t hv) {
            const uint32_t l = j / ENT, hi = j % ENT;
            const uint32_t keep = l < L ? 0xFFFFFFFFu : 0u, hs = hv << 16;       // table L: all zero
            const uint32_t dst = lds0 + l * Fmt::kRowBytes + hi * ENT * 4;
#pragma unroll
            for (int c4 = 0; c4 < ENT / 4; ++c4) {
                uint32_t v[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int lo = 4 * c4 + k;
                    v[k] = (((lo & 1) ? w[lo / 2] >> 16 : w[lo / 2] & 0xFFFFu) | hs) & keep;
                }
                typedef uint32_t u4 __attribute__((ext_vector_type(4)));
                *(__attribute__((address_space(3))) u4 *)(uintptr_t)(dst + c4 * 16) = u4{v[0], v[1], v[2], v[3]};
            }
        };
#pragma unroll
        for (int p = 0; p < PRE; ++p) {
            const uint32_t j = threadIdx.x + p * kStreamThreads;
            if (j < items) build_item(j, libw[p], libhi[p]);
        }
        for (uint32_t j = threadIdx.x + PRE * kStreamThreads; j < items; j += kStreamThreads) {
            uint32_t w[CW], hv = 0u;                           // larger libraries: loaded here
#pragma unroll
            for (int d = 0; d < CW; ++d) w[d] = 0u;
            if (j / ENT < L) {                                 // (the all-zero table needs no load)
#pragma unroll
                for (int d = 0; d < CW; ++d) w[d] = cbw[(j / ENT) * CW + d];
                hv = reinterpret_cast<const uint16_t *>(cbw)[j];
            }
            build_item(j, w, hv);
        }
        __syncthreads();
    } else if constexpr (TAIL) {
        // the all-zero table that lanes past the end of the row look up
#pragma unroll
        for (int i = lane; i < Fmt::kRowBytes / 4; i += kWave)
            *(lds_u32_w_t *)(uintptr_t)(lds_base + B * Fmt::kRowBytes + i * 4) = 0u;
    }
    if (row_begin >= N) return;
    // bf16 activations: converted in place, once per wave (they were requested ahead
    // of the index words, so this waits for nothing that streams)
    const bool xbf = a.x_bf16 != 0;
    if (xbf) {
#pragma unroll
        for (int c = 0; c < NCH; ++c)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                // one register at a time: left to itself the compiler converts all of them at once and
                // pays for the temporaries with the occupancy of the fp16 path too
                asm volatile("" : "+v"(xr[c][i]));
                xr[c][i] = bf16x2_to_f16x2(xr[c][i]);
                asm volatile("" : "+v"(xr[c][i]));
            }
    }

    // Scale and mid-point per group: a lane-load lies inside one group, so its share of the row sum is
    // scale * (sum of x * entry over its 32 weights) + mid * (sum of its 32 activations); the second sum does
    // not depend on the row and is formed once (zero for lanes past the end of a short row).
    float sx[AFF ? NCH : 1] = {};
    if constexpr (AFF) {
        const half2_t ones = __builtin_bit_cast(half2_t, 0x3C003C00u);
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            float t0 = 0.f, t1 = 0.f;
#pragma unroll
            for (int i = 0; i < 16; i += 2) {
                t0 = dot2(as_half2(xr[c][i]), ones, t0);
                t1 = dot2(as_half2(xr[c][i + 1]), ones, t1);
            }
            sx[c] = (TAIL && c == NCH - 1 && !live_last) ? 0.f : t0 + t1;
        }
    }

    // One batch of rows.  FIRST: its index words were loaded in the prologue.
    auto pass = [&](auto first, uint32_t rb) {
        if constexpr (!decltype(first)::value) {
            load_batch(rb);
            __builtin_amdgcn_sched_barrier(0);
        }
        // a7 (issue): the CSR entries of the batch are contiguous.  Each lane
        // takes one entry per row group through a bounds-checked buffer load
        // (offsets past the end read as zero): no loop, no branch.
        // (Fused gate/up batches hold two contiguous runs of rows: lanes 0..31 take
        // the gate rows' entries, lanes 32..63 the up rows', with masked loads.)
        const int32_t ob0 = __builtin_amdgcn_readlane(rpv, 0);       // entry range of the batch
        const int32_t ob1 = __builtin_amdgcn_readlane(rpv, B);
        __amdgpu_buffer_rsrc_t rc = __builtin_amdgcn_make_buffer_rsrc(
            (void *)(a.col + ob0), 0, (ob1 - ob0) * 4, 0x00020000);
        __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc(
            (void *)(a.val + ob0), 0, (ob1 - ob0) * 2, 0x00020000);
        constexpr int OV = RPC > 1 ? U : 1;
        int32_t olo[RPC > 1 ? 1 : U], ohi[RPC > 1 ? 1 : U];   // RPC == 1: entry range of every row (uniform)
        int32_t oj[OV], oj1[OV];             // this lane's entry and the end of its range
        uint32_t ocol[OV], oval[OV];
        if constexpr (RPC == 1) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                olo[u] = __builtin_amdgcn_readlane(rpv, bl(u));
                ohi[u] = __builtin_amdgcn_readlane(rpv, bl(u) + 1);
            }
            if (!FI) {
                oj[0] = ob0 + (int32_t)lane;
                oj1[0] = ob1;
                ocol[0] = __builtin_amdgcn_raw_buffer_load_b32(rc, lane * 4, 0, 0);
                oval[0] = __builtin_amdgcn_raw_buffer_load_b16(rv, lane * 2, 0, 0);
            } else {
                const int32_t g0 = ob0, g1 = __builtin_amdgcn_readlane(rpv, B / 2);
                const int32_t u0 = __builtin_amdgcn_readlane(rpv, 32), u1 = __builtin_amdgcn_readlane(rpv, 32 + B / 2);
                oj[0] = (lane < 32 ? g0 : u0) + (int32_t)(lane & 31);
                oj1[0] = lane < 32 ? g1 : u1;
                const bool on = oj[0] < oj1[0];
                ocol[0] = on ? (uint32_t)a.col[oj[0]] : 0u;
                oval[0] = on ? (uint32_t)a.val[oj[0]] : 0u;
            }
        } else {
            olo[0] = ohi[0] = 0;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t b = bl(u * RPC + seg);
                const int32_t r0 = __shfl(rpv, b);
                oj1[u] = __shfl(rpv, b + 1);
                oj[u] = r0 + (int32_t)lis;
                if (!FI) {
                    ocol[u] = __builtin_amdgcn_raw_buffer_load_b32(rc, (oj[u] - ob0) * 4, 0, 0);
                    oval[u] = __builtin_amdgcn_raw_buffer_load_b16(rv, (oj[u] - ob0) * 2, 0, 0);
                } else {
                    const bool on = oj[u] < oj1[u];
                    ocol[u] = on ? (uint32_t)a.col[oj[u]] : 0u;
                    oval[u] = on ? (uint32_t)a.val[oj[u]] : 0u;
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);

        // a2 (V2): codebooks of the batch -> LDS tables.
        if constexpr (MODE == 0) {
            __builtin_amdgcn_wave_barrier();
            const uint32_t raw_base = lds_base + Cfg::kTableBytes;
#pragma unroll
            for (int i = 0; i < CBW; ++i)
                if (CBW * kWave == B * (ENT / 2) || i * kWave + lane < B * (ENT / 2))
                    *(lds_u32_w_t *)(uintptr_t)(raw_base + (i * kWave + lane) * 4) = cbv[i];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            // entry e = (first index) | (second index) << BITS; this lane builds e = lane, lane+64, ...
            constexpr int PE = 1 << (2 * BITS);                // pair entries per row (16, 64 or 256)
            constexpr int PR = PE >= kWave ? PE / kWave : 1;
            if constexpr (BITS == 4 && NCH <= 4) {
                // 256 entries: this lane builds the four consecutive entries 4 lane .. 4 lane + 3 (second index
                // lane / 4, first indices 4 (lane % 4) ..): one 8-byte and one 2-byte read, one 16-byte write per row
                // instead of five reads and four writes (measured: 1 % on 8192x4096, 8 % on split-K slices, which
                // rebuild every row's table; with more than four chunks of x in registers it is slower)
                typedef uint32_t u2 __attribute__((ext_vector_type(2)));
                typedef uint32_t u4 __attribute__((ext_vector_type(4)));
                typedef __attribute__((address_space(3))) const u2 lds_u2_t;
#pragma unroll
                for (int r = 0; r < B; ++r) {
                    const u2 w = *(lds_u2_t *)(uintptr_t)(raw_base + r * Fmt::kRawBytes + (lane & 3) * 8);
                    const uint32_t hs = (uint32_t)*(lds_u16_t *)(uintptr_t)(raw_base + r * Fmt::kRawBytes + (lane >> 2) * 2) << 16;
                    *(__attribute__((address_space(3))) u4 *)(uintptr_t)(lds_base + r * Fmt::kRowBytes + lane * 16) =
                        u4{(w.x & 0xFFFFu) | hs, (w.x >> 16) | hs, (w.y & 0xFFFFu) | hs, (w.y >> 16) | hs};
                }
            } else if (PE >= kWave || lane < PE) {
#pragma unroll
                for (int r = 0; r < B; ++r) {
                    // 64 is a multiple of the codebook size, so the first index of every
                    // entry this lane builds is the same
                    const uint32_t lo = *(lds_u16_t *)(uintptr_t)(raw_base + r * Fmt::kRawBytes + (lane & (ENT - 1)) * 2);
#pragma unroll
                    for (int p = 0; p < PR; ++p) {
                        const uint32_t e = lane + p * kWave;
                        const uint32_t hi = *(lds_u16_t *)(uintptr_t)(raw_base + r * Fmt::kRawBytes + (e >> BITS) * 2);
                        *(lds_u32_w_t *)(uintptr_t)(lds_base + r * Fmt::kRowBytes + e * 4) = lo | (hi << 16);
                    }
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
        // next batch's row pointers and codebooks: issued now, consumed next pass
        if (rb + B < row_end) {
            rpv = rp_lane(rb + B);
            if constexpr (MODE == 0) {
#pragma unroll
                for (int i = 0; i < CBW; ++i)
                    cbv[i] = cbw[cb_word(rb + B, i * kWave + lane)];
            }
        }
        __builtin_amdgcn_sched_barrier(0);

        // Keep the activations as packed fp16 pairs: without this the compiler
        // hoists their fp32 conversions out of the loop and doubles the registers.
#pragma unroll
        for (int c = 0; c < NCH; ++c)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                if (TAIL && c == NCH - 1) xr[c][i] = live_last ? xr[c][i] : 0u;
                asm volatile("" : "+v"(xr[c][i]));
            }

        // a4-a6: depack, gather, multiply-accumulate, software-pipelined over
        // groups of eight lookups: task t = (row u, chunk c, group g).
        float sum[U];
        uint16_t oxv[OV];
        {
            constexpr int TPR = NCH * GPL;                     // tasks per row
            constexpr int NT = U * TPR;
            uint32_t val[2][8];
            float acc[4] = {0.f, 0.f, 0.f, 0.f};
            float tot = 0.f;                                   // AFF: the row's sum of scaled lane-load sums
            auto issue = [&](int t, uint32_t (&v)[8]) {
                const int u = t / TPR, c = (t % TPR) / GPL, g = t % GPL;
                const uint32_t tb = lds_base + u * RPC * Fmt::kRowBytes;
                if constexpr (LIB) {
                    const uint32_t dead = TAIL && c == NCH - 1 && !live_last;
                    issue_group<BITS, true, true>(lw[u][c], g, lds_base, dead ? a.L : lib[u][c], v, k2);
                } else if (RPC > 1)
                    issue_group<BITS, true>(lw[u][c], g, tb, seg, v, k2);
                else if (TAIL && c == NCH - 1)
                    issue_group<BITS, true>(lw[u][c], g, tb, live_last ? 0u : (uint32_t)(B - u), v, k2);
                else
                    issue_group<BITS, false>(lw[u][c], g, tb, 0u, v, k2);
            };
            issue(0, val[0]);
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const int u = t / TPR, c = (t % TPR) / GPL, g = t % GPL;
                if (t + 1 < NT) issue(t + 1, val[(t + 1) & 1]);
                if (t == 3 * NT / 4) {
                    // a7 (gather): x at the outlier columns.  col was requested after the index
                    // words and loads return in order, so this waits for the whole batch: late
                    // enough that little is left to wait for, early enough that the last quarter
                    // of the multiply-accumulates covers part of the gather's latency
#pragma unroll
                    for (int v = 0; v < OV; ++v) oxv[v] = x[ocol[v]];
                }
                __builtin_amdgcn_sched_barrier(0);
                consume_group<BITS>(g, val[t & 1], xr[c], acc);
                if constexpr (AFF) {
                    if (g == GPL - 1) {                        // lane-load finished: its group's scale and mid-point
                        const bool dead = TAIL && c == NCH - 1 && !live_last;      // (its terms are zero: keep them so)
                        const float sc = dead ? 0.f : half_bits_to_float((uint16_t)gsc[u][c]);
                        const float md = dead ? 0.f : half_bits_to_float((uint16_t)gmd[u][c]);
                        tot = fmaf(sc, (acc[0] + acc[1]) + (acc[2] + acc[3]), tot);
                        tot = fmaf(md, sx[c], tot);
                        acc[0] = acc[1] = acc[2] = acc[3] = 0.f;
                    }
                    if (t % TPR == TPR - 1) {                  // row finished
                        sum[u] = tot;
                        tot = 0.f;
                    }
                } else if (t % TPR == TPR - 1) {               // row finished
                    sum[u] = (acc[0] + acc[1]) + (acc[2] + acc[3]);
                    acc[0] = acc[1] = acc[2] = acc[3] = 0.f;
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }

        // a7 (fold): add each outlier product to the row that owns the entry.
        {
            if constexpr (RPC == 1) {
                const float p = half_bits_to_float((uint16_t)oval[0]) * x_bits_to_float(oxv[0], xbf);
#pragma unroll
                for (int u = 0; u < U; ++u) sum[u] += (oj[0] >= olo[u] && oj[0] < ohi[u]) ? p : 0.f;
                const int32_t ostep = FI ? 32 : kWave;
                for (int32_t jj = oj[0] + ostep; jj < oj1[0]; jj += ostep) {     // more entries than lanes: rare
                    const float q = half_bits_to_float(a.val[jj]) * x_bits_to_float(x[a.col[jj]], xbf);
#pragma unroll
                    for (int u = 0; u < U; ++u) sum[u] += (jj >= olo[u] && jj < ohi[u]) ? q : 0.f;
                }
            } else {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const float p = half_bits_to_float((uint16_t)oval[u]) * x_bits_to_float(oxv[u], xbf);
                    sum[u] += oj[u] < oj1[u] ? p : 0.f;
                    for (int32_t jj = oj[u] + LPR; jj < oj1[u]; jj += LPR)         // > LPR entries: rare
                        sum[u] = fmaf(half_bits_to_float(a.val[jj]), x_bits_to_float(x[a.col[jj]], xbf), sum[u]);
                }
            }
        }
        // a8: reduce and store.
        if (FI) {
            // gate row u and its up row u + U / 2 end in the same lane: h = SiLU(g) * u in fp32
            if constexpr (U % 2 == 0) {
#pragma unroll
                for (int u = 0; u < U / 2; ++u) {
                    const uint32_t j = rb / 2 + u * RPC + seg;
                    const float g = segment_sum<LPR>(sum[u]), up = segment_sum<LPR>(sum[u + U / 2]);
                    const float h = g / (1.0f + __expf(-g)) * up;
                    if (lis == 0 && j < row_end / 2) {
                        const int64_t o = (int64_t)slot * a.y_stride + j;
                        store_out(a.y, o, h, y_f32 != 0, a.y_bf16 != 0);
                    }
                }
            }
            return;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t row = rb + u * RPC + seg;
            float t = segment_sum<LPR>(sum[u]);
            if (lis == 0 && row < row_end) {
                const int64_t o = (int64_t)z * a.z_stride + (int64_t)slot * a.y_stride + row;
                store_out(a.y, o, t, y_f32 != 0, a.y_bf16 != 0);
            }
        }
    };

    pass(std::true_type{}, row_begin);
    for (uint32_t rb = row_begin + B; rb < row_end; rb += B) pass(std::false_type{}, rb);
}

// rows per wave: a multiple of the batch, sized so that the grid is a few
// thousand waves (about 16 per CU) when the problem is large enough.
template <int VAR, int BITS, int NCH, int RPC, bool TAIL, int MODE, int UNROLL>
static hipError_t launch_stream_u(DecodeArgs a, int slots, bool y_f32, hipStream_t s)
{
    using Cfg = StreamCfg<BITS, NCH, RPC, UNROLL, MODE == 2>;
    using Fmt = TableFmt<BITS>;
    if constexpr (!Cfg::kFits) {
        return hipErrorInvalidValue;
    } else {
        constexpr int B = Cfg::kBatchRows;
        constexpr int kStreamWaves = stream_waves(MODE), kStreamThreads = kStreamWaves * kWave;
        const uint32_t S = VAR == 1 ? a.k_slices : 1u;
        const uint64_t total_rows = (uint64_t)a.N * slots * S;
        uint32_t rpw = B;
        while ((total_rows + rpw - 1) / rpw > stream_max_waves(MODE) && rpw < 64 * B) rpw += B;
        a.rows_per_block = rpw;
        const uint32_t waves = (a.N + rpw - 1) / rpw;
        const size_t smem = MODE == 0 ? 0 : (size_t)(a.L + 1) * Fmt::kRowBytes;
        auto kern = decode_stream_kernel<BITS, NCH, RPC, TAIL, MODE, UNROLL, VAR>;
        if (smem > 48 * 1024) {
            hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
            if (err != hipSuccess) return err;
        }
        dim3 grid((waves + kStreamWaves - 1) / kStreamWaves, slots, S);
        hipLaunchKernelGGL(kern, grid, dim3(kStreamThreads), smem, s, a, (int)y_f32);
        return hipGetLastError();
    }
}

// Smallest batch (1, 2 or 4 row groups) with which every wave has ONE batch,
// i.e. all of a wave's loads are issued up front; the largest the registers
// allow when even that leaves more than the target number of waves.
template <int VAR, int BITS, int NCH, int RPC, bool TAIL, int MODE>
static hipError_t launch_stream_t(const DecodeArgs &a, int slots, bool y_f32, hipStream_t s)
{
    const uint64_t groups = ((uint64_t)a.N * slots * (VAR == 1 ? a.k_slices : 1u) + RPC - 1) / RPC;
    constexpr uint32_t W = stream_max_waves(MODE);
    constexpr bool f2 = StreamCfg<BITS, NCH, RPC, 2, MODE == 2>::kFits, f4 = StreamCfg<BITS, NCH, RPC, 4, MODE == 2>::kFits;
    if (VAR == 2 && !f2) return hipErrorInvalidValue;       // gate and up rows pair up inside an even batch
    if (VAR != 2 && (groups <= W || !f2)) return launch_stream_u<VAR, BITS, NCH, RPC, TAIL, MODE, 1>(a, slots, y_f32, s);
    if (groups <= 2 * W || !f4) return launch_stream_u<VAR, BITS, NCH, RPC, TAIL, MODE, 2>(a, slots, y_f32, s);
    return launch_stream_u<VAR, BITS, NCH, RPC, TAIL, MODE, 4>(a, slots, y_f32, s);
}

template <int VAR, int BITS, int NCH, int RPC, bool TAIL>
static hipError_t launch_stream_m(const DecodeArgs &a, int mode, int slots, bool y_f32, hipStream_t s)
{
    if (mode == 0) return launch_stream_t<VAR, BITS, NCH, RPC, TAIL, 0>(a, slots, y_f32, s);
    return launch_stream_t<VAR, BITS, NCH, RPC, TAIL, 1>(a, slots, y_f32, s);
}

template <int VAR, int BITS, int NCH>
static hipError_t launch_stream_n(const DecodeArgs &a, int mode, int slots, bool y_f32, hipStream_t s)
{
    if (a.K % 2048 == 0) return launch_stream_m<VAR, BITS, NCH, 1, false>(a, mode, slots, y_f32, s);
    return launch_stream_m<VAR, BITS, NCH, 1, true>(a, mode, slots, y_f32, s);
}

template <int VAR, int BITS>
static hipError_t launch_stream_b(const DecodeArgs &a, int mode, int slots, bool y_f32, hipStream_t s)
{
    const uint32_t K = a.K;
    if (K == 1024) return launch_stream_m<VAR, BITS, 1, 2, false>(a, mode, slots, y_f32, s);
    if (K == 512) return launch_stream_m<VAR, BITS, 1, 4, false>(a, mode, slots, y_f32, s);
    switch ((K + 2047) / 2048) {
    case 1: return launch_stream_n<VAR, BITS, 1>(a, mode, slots, y_f32, s);
    case 2: return launch_stream_n<VAR, BITS, 2>(a, mode, slots, y_f32, s);
    case 3: return launch_stream_n<VAR, BITS, 3>(a, mode, slots, y_f32, s);
    case 4: return launch_stream_n<VAR, BITS, 4>(a, mode, slots, y_f32, s);
    case 5: return launch_stream_n<VAR, BITS, 5>(a, mode, slots, y_f32, s);
    case 6: return launch_stream_n<VAR, BITS, 6>(a, mode, slots, y_f32, s);
    case 7: return launch_stream_n<VAR, BITS, 7>(a, mode, slots, y_f32, s);
    default: return launch_stream_n<VAR, BITS, 8>(a, mode, slots, y_f32, s);
    }
}

// V2a with a scale and a mid-point per group (MODE 2): the plain variant, one row per pass of a lane's units; rows
// shorter than 2048 columns take the short-row (TAIL) form.
template <int BITS, int NCH>
static hipError_t launch_stream_aff_n(const DecodeArgs &a, int slots, bool y_f32, hipStream_t s)
{
    if (a.K % 2048 == 0) return launch_stream_t<0, BITS, NCH, 1, false, 2>(a, slots, y_f32, s);
    return launch_stream_t<0, BITS, NCH, 1, true, 2>(a, slots, y_f32, s);
}

template <int BITS>
static hipError_t launch_stream_aff_b(const DecodeArgs &a, int slots, bool y_f32, hipStream_t s)
{
    switch ((a.K + 2047) / 2048) {
    case 1: return launch_stream_aff_n<BITS, 1>(a, slots, y_f32, s);
    case 2: return launch_stream_aff_n<BITS, 2>(a, slots, y_f32, s);
    case 3: return launch_stream_aff_n<BITS, 3>(a, slots, y_f32, s);
    case 4: return launch_stream_aff_n<BITS, 4>(a, slots, y_f32, s);
    case 5: return launch_stream_aff_n<BITS, 5>(a, slots, y_f32, s);
    case 6: return launch_stream_aff_n<BITS, 6>(a, slots, y_f32, s);
    case 7: return launch_stream_aff_n<BITS, 7>(a, slots, y_f32, s);
    default: return launch_stream_aff_n<BITS, 8>(a, slots, y_f32, s);
    }
}

static hipError_t launch_stream_aff(int bits, bool y_f32, const DecodeArgs &a, int slots, hipStream_t s)
{
    switch (bits) {
    case 2: return launch_stream_aff_b<2>(a, slots, y_f32, s);
    case 3: return launch_stream_aff_b<3>(a, slots, y_f32, s);
    default: return launch_stream_aff_b<4>(a, slots, y_f32, s);
    }
}

// One variant of the kernel for all bit widths: each of the three small
// translation units instantiates exactly one, so that they compile in parallel.
template <int VAR>
static hipError_t launch_stream_variant(int bits, int mode, bool y_f32, const DecodeArgs &a, int slots, hipStream_t s)
{
    switch (bits) {
    case 2: return launch_stream_b<VAR, 2>(a, mode, slots, y_f32, s);
    case 3: return launch_stream_b<VAR, 3>(a, mode, slots, y_f32, s);
    default: return launch_stream_b<VAR, 4>(a, mode, slots, y_f32, s);
    }
}

}  // namespace
}  // namespace xfp
