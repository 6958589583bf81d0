// Tile form of the fused decode for M = 1 per slot, V2 codebooks: rows across
// lanes, one pair table per LANE, conflict-free lookups.
//
// Why: the streaming kernel gives a wave ONE row at a time, so its 64 lanes look
// up random entries of one 1 KB pair table and collide on the 32 LDS banks
// (5.5 clocks per wave instruction against 2.65 conflict-free); on every matrix
// that is not tiny the LDS pipe, not HBM, bounds it.  Here a workgroup owns a
// tile of 32 output rows and every lane works on a row of its own, whose pair
// table lives in that lane's private bank:
//     entry e of tile row r at LDS byte e * 256 + r * 4,
// so the 32 lanes the LDS serves per clock hit 32 different banks whatever their
// indices are, and a lookup address is ONE v_perm_b32 (index byte -> address
// byte 1, the lane's row * 4 in byte 0).
//
// Work split: wave w of the workgroup takes the slabs w, w + W, ... of the tile;
// a slab is 32 rows x 2 groups of 128 weights: lanes 0..31 decode group 2s of
// rows 0..31, lanes 32..63 group 2s + 1 of the same rows (lanes l and l + 32 share
// a bank and are served in different passes).  The partial sums of the W waves
// meet in LDS and are added in a fixed order; no atomics.
//
// Index words are loaded coalesced, not lane-shaped: load j of a slab gives lane
// 4a + b chunk b (32 weights, 16 bytes at 4 bits) of unit 16j + a, a unit being
// one (row, group) of the slab, so every quad of lanes reads 64 contiguous bytes
// and every byte of the stream is read once.  A 4 x 4 transposition between the
// two low lane bits and the load index (two stages of v_cndmask_b32 with a
// quad-permute DPP source, 32 VALU operations per 8192 weights) then leaves each
// lane with the 16 dwords of ITS unit.
//
// Activations: all 32 lanes of a half-wave need the same activation pair at the
// same time.  Each lane loads 16 bytes of its group's 256 (one load per slab per
// lane), and the multiply-accumulate reads the pair it needs from the lane that
// holds it with a DPP row broadcast inside the instruction:
//     v_dot2c_f32_f16_dpp acc, x, w  row_newbcast:n
// (pair p of a group sits in register p % 4 of lane p / 4 of every row of 16
// lanes).  No LDS traffic, no extra instruction, 4 registers per slab.
//
// Per pair of weights: one v_perm_b32, one ds_read_b32, one v_dot2c_f32_f16.
#include "xfp_device.h"

#include <atomic>

namespace xfp {
namespace {

typedef __attribute__((address_space(3))) const uint32_t lds_cu32_t;
typedef __attribute__((address_space(3))) uint32_t lds_u32_t;
typedef __attribute__((address_space(3))) float lds_f32_t;
typedef __attribute__((address_space(4))) const int32_t const_i32_t;   // uniform reads go through the scalar cache

constexpr int kTileRows = 32;

template <int BITS, int W>
struct TileLds {
    static constexpr int kPairs = 1 << (2 * BITS);             // entries of a pair table
    static constexpr int kTab = kPairs * 256;                  // 64 KB at 4 bits
    static constexpr int kRed = kTab;                          // W x 64 partial sums
    static constexpr int kProd = kRed + W * kWave * 4;         // one outlier product per thread
    static constexpr int kTotal = kProd + W * kWave * 4;
};

#define XFP_DOT2C_BCAST(acc, x, w, n)                                                                \
    asm volatile("v_dot2c_f32_f16_dpp %0, %1, %2 row_newbcast:" #n " row_mask:0xf bank_mask:0xf"       \
                 : "+v"(acc) : "v"(x), "v"(w))

// acc[i] += dot2(pair i of lane N of this row of 16 lanes, w[i]) for the four pairs of one index dword
template <int N>
__device__ __forceinline__ void mac_dword(float (&acc)[4], const uint32_t (&x)[4], const uint32_t (&w)[4])
{
#define XFP_MAC4(n)                                                                                  \
    XFP_DOT2C_BCAST(acc[0], x[0], w[0], n); XFP_DOT2C_BCAST(acc[1], x[1], w[1], n);                   \
    XFP_DOT2C_BCAST(acc[2], x[2], w[2], n); XFP_DOT2C_BCAST(acc[3], x[3], w[3], n)
    if constexpr (N == 0) { XFP_MAC4(0); } else if constexpr (N == 1) { XFP_MAC4(1); }
    else if constexpr (N == 2) { XFP_MAC4(2); } else if constexpr (N == 3) { XFP_MAC4(3); }
    else if constexpr (N == 4) { XFP_MAC4(4); } else if constexpr (N == 5) { XFP_MAC4(5); }
    else if constexpr (N == 6) { XFP_MAC4(6); } else if constexpr (N == 7) { XFP_MAC4(7); }
    else if constexpr (N == 8) { XFP_MAC4(8); } else if constexpr (N == 9) { XFP_MAC4(9); }
    else if constexpr (N == 10) { XFP_MAC4(10); } else if constexpr (N == 11) { XFP_MAC4(11); }
    else if constexpr (N == 12) { XFP_MAC4(12); } else if constexpr (N == 13) { XFP_MAC4(13); }
    else if constexpr (N == 14) { XFP_MAC4(14); } else { XFP_MAC4(15); }
#undef XFP_MAC4
}

template <int M>
struct StepTag { static constexpr int value = M; };

// BITS = 4.  W: waves per workgroup (4, 8 or 16).  XBF: the activations are bf16 (compile-time: as a run-time
// choice the compiler turns the conversion into selects and every fp16 call pays its 40 instructions per slab).
template <int BITS, int W, bool XBF>
__global__ __launch_bounds__(W * kWave) void decode_tile_kernel(DecodeArgs a, int y_f32)
{
    static_assert(BITS == 4, "4-bit indices: a chunk of 32 weights is 16 bytes, an index byte is a pair");
    using L = TileLds<BITS, W>;
    constexpr int T = W * kWave;
    constexpr int ENT = 1 << BITS;
    constexpr int PARTS = T / kTileRows;                       // table builders per row
    constexpr int EPT = L::kPairs / PARTS;                     // entries a thread builds (8, 16 or 32)
    extern __shared__ __align__(16) unsigned char smem[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;

    const uint32_t tid = threadIdx.x, lane = tid & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t slot = blockIdx.y;
    const uint32_t e = a.eids ? (uint32_t)a.eids[slot] : 0u;
    const uint32_t N = a.N, K = a.K;
    const uint32_t n0 = blockIdx.x * kTileRows;
    const uint32_t wpr = K / 32 * BITS;                        // dwords of a row
    const uint32_t G = K / kGroup, S = (G + 1) / 2;            // groups, slabs of a row
    const uint32_t *idx = a.idx + (size_t)e * N * wpr;
    const uint16_t *cb = a.cb + (size_t)e * N * ENT;
    const int32_t *rp = a.rp + (size_t)e * N;
    const uint16_t *x = a.x + (int64_t)slot * a.x_stride;
    constexpr bool xbf = XBF;

    // ---------------------------------------------------------------- loads, in the order their consumers run
    // (vector loads return in issue order).  The tile's entry range first: it gates the outlier loads.
    const int32_t obv = rp[min(n0, N)], oev = rp[min(n0 + kTileRows, N)];
    // table builder role: tile row tid % 32, part tid / 32 builds entries [part * EPT, (part + 1) * EPT)
    const uint32_t trow = tid & 31, part = tid >> 5;
    const uint16_t *cbr = cb + (size_t)min(n0 + trow, N - 1) * ENT;
    uint32_t clo[EPT >= 16 ? 8 : 4];                           // first indices of this part: 16 (8) codebook values
    uint32_t chi;                                              // second index (indices): one (two) codebook values
    if constexpr (EPT == 8) {
        const uint4 v = *reinterpret_cast<const uint4 *>(cbr + 8 * (part & 1));
        clo[0] = v.x; clo[1] = v.y; clo[2] = v.z; clo[3] = v.w;
        chi = cbr[part >> 1];
    } else {
        const uint4 v0 = *reinterpret_cast<const uint4 *>(cbr), v1 = *reinterpret_cast<const uint4 *>(cbr + 8);
        clo[0] = v0.x; clo[1] = v0.y; clo[2] = v0.z; clo[3] = v0.w;
        clo[4] = v1.x; clo[5] = v1.y; clo[6] = v1.z; clo[7] = v1.w;
        if constexpr (EPT == 16) chi = cbr[part];
        else chi = reinterpret_cast<const uint32_t *>(cbr)[part];          // EPT == 32: second indices 2 part, 2 part + 1
    }
    // final sums: thread 4 r + q (r < 32) adds a quarter of row r's terms
    const uint32_t rr = min(tid >> 2, (uint32_t)kTileRows - 1), rq = tid & 3;
    const int32_t rlo = rp[min(n0 + rr, N)], rhi = rp[min(n0 + rr + 1, N)];

    // This lane's unit of a slab: tile row urow, group ugrp of the slab's two.  Load j of a slab: lane
    // 4a + b reads chunk b of the unit (row (a & 7) + 8j, group a >> 3); after the transposition lane 4a + b
    // holds the unit (row (a & 7) + 8b, group a >> 3).  Index words and activations come through buffer
    // loads: a per-lane offset that never changes plus a scalar offset per slab, no address arithmetic in
    // the loop; a group past the end of the row (second group of the last slab when the row has an odd
    // number of groups) reads zeros for the activations and whatever follows for the indices.
    const uint32_t la = lane >> 2, lb = lane & 3;
    const uint32_t ugrp = la >> 3, urow = (la & 7) + 8 * lb;
    const uint32_t sel = urow * 4;                             // byte 0 of every lookup address: the lane's bank
    const uint32_t rows_here = min((uint32_t)kTileRows, N - n0);
    constexpr uint32_t kUnitBytes = kGroup * BITS / 8;         // index bytes of one row's group
    __amdgpu_buffer_rsrc_t ri = __builtin_amdgcn_make_buffer_rsrc((void *)(idx + (size_t)n0 * wpr), 0, rows_here * wpr * 4, 0x00020000);
    __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void *)x, 0, K * 2, 0x00020000);
    uint32_t ioff[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
        ioff[j] = min((la & 7) + 8 * j, rows_here - 1) * (wpr * 4) + ugrp * kUnitBytes + lb * (kUnitBytes / 4);
    const uint32_t xoff = ugrp * (kGroup * 2) + (lane & 15) * 16;
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    struct SlabRegs { uint32_t iw[4][BITS], xw[4]; };
    SlabRegs ra;                                               // the slab in flight (measured: a second one in flight, or the next
                                                               // one requested before this one is touched, is 4 to 10 % slower)
    auto load_slab = [&](SlabRegs &R, uint32_t s) {
        const u32x4 xv4 = __builtin_amdgcn_raw_buffer_load_b128(rx, xoff, s * (2 * kGroup * 2), 0);
        R.xw[0] = xv4.x; R.xw[1] = xv4.y; R.xw[2] = xv4.z; R.xw[3] = xv4.w;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const u32x4 v4 = __builtin_amdgcn_raw_buffer_load_b128(ri, ioff[j], s * (2 * kUnitBytes), 2);   // read once: non-temporal
            R.iw[j][0] = v4.x; R.iw[j][1] = v4.y; R.iw[j][2] = v4.z; R.iw[j][3] = v4.w;
        }
    };
    uint32_t s = wave;
    __builtin_amdgcn_sched_barrier(0);
    // outlier entry ob + tid: column and value through bounds-checked buffer loads (past the end: zero)
    const int32_t ob = __builtin_amdgcn_readfirstlane(obv), oe = __builtin_amdgcn_readfirstlane(oev);
    __amdgpu_buffer_rsrc_t rc = __builtin_amdgcn_make_buffer_rsrc((void *)(a.col + ob), 0, (oe - ob) * 4, 0x00020000);
    __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc((void *)(a.val + ob), 0, (oe - ob) * 2, 0x00020000);
    const uint32_t ocol = __builtin_amdgcn_raw_buffer_load_b32(rc, tid * 4, 0, 0);
    const uint32_t oval = __builtin_amdgcn_raw_buffer_load_b16(rv, tid * 2, 0, 0);
    __builtin_amdgcn_sched_barrier(0);

    // ---------------------------------------------------------------- a2: the tile's pair tables
    {
        const uint32_t base = lds0 + part * (EPT * 256) + trow * 4;
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
            const int lo = j % 16;                             // first index within this part's range
            const uint32_t lw = clo[lo / 2];
            const uint32_t lov = (lo & 1) ? lw >> 16 : lw & 0xFFFFu;
            uint32_t hiv;
            if constexpr (EPT == 32) hiv = j < 16 ? chi << 16 : chi & 0xFFFF0000u;
            else hiv = chi << 16;
            *(lds_u32_t *)(uintptr_t)(base + j * 256) = lov | hiv;
        }
    }
    // The index words are requested only now, behind the codebooks' arrival: requested at the start they
    // queue in front of the later waves' codebook loads, every table is late and with it every wave
    // (workload 2: 7.5 us against 6.6 us this way).
    __builtin_amdgcn_sched_barrier(0);
    if (s < S) load_slab(ra, s);
    __builtin_amdgcn_sched_barrier(0);
    lds_barrier();

    // ---------------------------------------------------------------- a3-a6: the wave's slabs
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    uint16_t oxv = 0;
    bool gathered = false;
    auto process = [&](SlabRegs &R, uint32_t s) {
        // transpose: afterwards v[4c + d] is dword d of chunk c of this lane's unit
        uint32_t v[16], xv[4];
#pragma unroll
        for (int d = 0; d < BITS; ++d) {
            uint32_t t0 = R.iw[0][d], t1 = R.iw[1][d], t2 = R.iw[2][d], t3 = R.iw[3][d];
            lane_reg_exchange<1>(t0, t2, t1, t3);
            lane_reg_exchange<0>(t0, t1, t2, t3);
            v[0 + d] = t0; v[4 + d] = t1; v[8 + d] = t2; v[12 + d] = t3;
        }
        const bool dead = 2 * s + ugrp >= G;                   // second group of the last slab when G is odd
#pragma unroll
        for (int i = 0; i < 4; ++i) xv[i] = R.xw[i];
        if constexpr (XBF) {
#pragma unroll
            for (int i = 0; i < 4; ++i) xv[i] = bf16x2_to_f16x2(xv[i]);
        }
        if (s + W < S) load_slab(R, s + W);                    // the registers are free: next slab
        __builtin_amdgcn_sched_barrier(0);
        float sacc[4] = {0.f, 0.f, 0.f, 0.f};
        // lookups run LA dwords (4 LA pairs) ahead of the multiply-accumulates
        constexpr int LA = 4;
        uint32_t val[LA + 1][4];
        auto lookup = [&](int m, uint32_t (&o)[4]) {
            o[0] = *(lds_cu32_t *)(uintptr_t)__builtin_amdgcn_perm(v[m], sel, 0x0c0c0400u);
            o[1] = *(lds_cu32_t *)(uintptr_t)__builtin_amdgcn_perm(v[m], sel, 0x0c0c0500u);
            o[2] = *(lds_cu32_t *)(uintptr_t)__builtin_amdgcn_perm(v[m], sel, 0x0c0c0600u);
            o[3] = *(lds_cu32_t *)(uintptr_t)__builtin_amdgcn_perm(v[m], sel, 0x0c0c0700u);
        };
#pragma unroll
        for (int m = 0; m < LA; ++m) lookup(m, val[m]);
        asm volatile("s_nop 1");                               // a DPP read wants two wait states after a vector write of its source
        auto step = [&](auto tag) {
            constexpr int m = decltype(tag)::value;
            if constexpr (m + LA < 16) lookup(m + LA, val[(m + LA) % (LA + 1)]);
            __builtin_amdgcn_sched_barrier(0);
            mac_dword<m>(sacc, xv, val[m % (LA + 1)]);
            __builtin_amdgcn_sched_barrier(0);
        };
        step(StepTag<0>{}); step(StepTag<1>{}); step(StepTag<2>{}); step(StepTag<3>{});
        step(StepTag<4>{}); step(StepTag<5>{}); step(StepTag<6>{}); step(StepTag<7>{});
        if (!gathered) {
            // a7 (gather): the activation at this thread's outlier column.  The column was requested behind the
            // first slab's index words and has had half a slab's arithmetic to arrive; the gather's own round
            // trip runs under the other half.
            oxv = x[ocol];
            gathered = true;
        }
        step(StepTag<8>{}); step(StepTag<9>{}); step(StepTag<10>{}); step(StepTag<11>{});
        step(StepTag<12>{}); step(StepTag<13>{}); step(StepTag<14>{}); step(StepTag<15>{});
        // a lane past the end of the row decoded real indices against zero activations; its products are dropped
        // outright, so that an infinite codebook entry cannot turn them into NaN
        if (G & 1) {
#pragma unroll
            for (int i = 0; i < 4; ++i) sacc[i] = dead ? 0.f : sacc[i];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] += sacc[i];
    };
    for (; s < S; s += W) process(ra, s);
    if (!gathered) oxv = x[ocol];                              // a wave without a slab (more waves than slabs)
    *(lds_f32_t *)(uintptr_t)(lds0 + L::kRed + tid * 4) = (acc[0] + acc[1]) + (acc[2] + acc[3]);

    // ---------------------------------------------------------------- a7: one outlier product per thread
    {
        const float p = half_bits_to_float((uint16_t)oval) * x_bits_to_float(oxv, xbf);
        *(lds_f32_t *)(uintptr_t)(lds0 + L::kProd + tid * 4) = p;
    }
    lds_barrier();
    // More entries in the tile than threads (long rows, dense outliers): every thread takes further entries,
    // T at a time, and the products go where the tables were (every wave is past its lookups).
    constexpr int kProdMore = L::kTab / 4;                     // products the table region takes
    const int32_t cnt = oe - ob;
    if (cnt > T) {
        constexpr int RU = 4;                                  // rounds in flight
        for (int32_t r0 = T; r0 < min(cnt, T + kProdMore); r0 += RU * T) {
            uint32_t c[RU], vv[RU];
            uint16_t xg[RU];
#pragma unroll
            for (int r = 0; r < RU; ++r) {
                c[r] = __builtin_amdgcn_raw_buffer_load_b32(rc, (r0 + r * T + tid) * 4, 0, 0);
                vv[r] = __builtin_amdgcn_raw_buffer_load_b16(rv, (r0 + r * T + tid) * 2, 0, 0);
            }
#pragma unroll
            for (int r = 0; r < RU; ++r) xg[r] = x[c[r]];
#pragma unroll
            for (int r = 0; r < RU; ++r) {
                const int32_t j = r0 + r * T + (int32_t)tid - T;
                if (j < kProdMore)
                    *(lds_f32_t *)(uintptr_t)(lds0 + j * 4) = half_bits_to_float((uint16_t)vv[r]) * x_bits_to_float(xg[r], xbf);
            }
        }
        lds_barrier();
    }

    // ---------------------------------------------------------------- a8: fixed-order sums, store
    if (tid < 4 * kTileRows) {
        // the two lanes that hold row rr in every wave: 4 (rr % 8) + rr / 8 and the same + 32
        const uint32_t l0 = 4 * (rr & 7) + (rr >> 3);
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < W; w += 4) {
            const uint32_t o = lds0 + L::kRed + ((w + rq) * kWave + l0) * 4;
            sum += *(lds_f32_t *)(uintptr_t)o;
            sum += *(lds_f32_t *)(uintptr_t)(o + 32 * 4);
        }
        const int32_t cap = ob + T + kProdMore;                // entries whose products are in LDS
        for (int32_t j = rlo + (int32_t)rq; j < min(rhi, cap); j += 4) {
            const int32_t k = j - ob;
            sum += *(lds_f32_t *)(uintptr_t)(lds0 + (k < T ? L::kProd + k * 4 : (k - T) * 4));
        }
        for (int32_t j = max(rlo, cap) + (int32_t)rq; j < rhi; j += 4)         // beyond even that: never in practice
            sum = fmaf(half_bits_to_float(a.val[j]), x_bits_to_float(x[a.col[j]], xbf), sum);
        sum = dpp_add<0xB1>(sum);                              // the four lanes of a row
        sum = dpp_add<0x4E>(sum);
        const uint32_t n = n0 + rr;
        if (rq == 0 && n < N) store_out(a.y, (int64_t)slot * a.y_stride + n, sum, y_f32 != 0, a.y_bf16 != 0);
    }
}

template <int BITS, int W, bool XBF>
hipError_t launch_tile_x(const DecodeArgs &a, int slots, bool y_f32, hipStream_t s)
{
    constexpr int kLds = TileLds<BITS, W>::kTotal;
    auto kern = decode_tile_kernel<BITS, W, XBF>;
    static std::atomic<int> configured[kMaxDevices];           // per device; idempotent attribute, benign race
    const int dev = current_device();
    if (dev < 0) return hipErrorInvalidDevice;
    if (!configured[dev].load(std::memory_order_relaxed)) {
        // the lookup addresses assume the tables at LDS offset 0: the kernel must have no static LDS
        hipFuncAttributes fa;
        hipError_t err = hipFuncGetAttributes(&fa, reinterpret_cast<const void *>(kern));
        if (err != hipSuccess) return err;
        if (fa.sharedSizeBytes != 0) return hipErrorInvalidValue;
        err = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
        if (err != hipSuccess) return err;
        configured[dev].store(1, std::memory_order_relaxed);
    }
    hipLaunchKernelGGL(kern, dim3((a.N + kTileRows - 1) / kTileRows, slots), dim3(W * kWave), kLds, s, a, (int)y_f32);
    return hipGetLastError();
}

template <int BITS, int W>
hipError_t launch_tile_w(const DecodeArgs &a, int slots, bool y_f32, hipStream_t s)
{
    return a.x_bf16 ? launch_tile_x<BITS, W, true>(a, slots, y_f32, s) : launch_tile_x<BITS, W, false>(a, slots, y_f32, s);
}

}  // namespace

// V2, 4-bit, M = 1 per slot.  Worth it when there are enough tiles to give every compute unit one
// (measured against the streaming kernel; see the dispatch in xfp_api.hip).
bool tile_supports(int bits, int mode, uint32_t N, uint32_t K, int slots)
{
    return mode == 0 && bits == 4 && K >= 2 * kGroup && (uint64_t)(N + kTileRows - 1) / kTileRows * slots <= 0x7fffffffu && slots <= 65535;
}

hipError_t launch_decode_tile(int bits, bool y_f32, const DecodeArgs &a, int slots, hipStream_t s)
{
    if (bits != 4) return hipErrorInvalidValue;
    const uint32_t S = (a.K / kGroup + 1) / 2;
    if (S <= 4) return launch_tile_w<4, 4>(a, slots, y_f32, s);
    if (S <= 8 || (uint64_t)(a.N + kTileRows - 1) / kTileRows * slots > 384) return launch_tile_w<4, 8>(a, slots, y_f32, s);
    return launch_tile_w<4, 16>(a, slots, y_f32, s);
}

}  // namespace xfp
