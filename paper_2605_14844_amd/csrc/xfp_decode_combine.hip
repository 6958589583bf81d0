// Down projection of a routed-expert layer with the router's weighted sum over
// the slots folded in (V2 codebooks, M = 1 per slot):
//     y[n] = sum_t w[t] * ( x_t . W_hat[expert_ids[t]][n][:] ).
// An output row is treated as ONE long row: the concatenation of row n of the
// T active experts, T * K weights, against the concatenation of the T
// activation rows.  That is the streaming kernel's picture again (a wave owns
// output rows, lane l always decodes the same 32-weight units, so its share of
// the activations is loaded once and stays in VGPRs; pair tables in LDS; fp32
// accumulation, DPP reduction, no atomics), with three differences: a lane's
// unit belongs to a slot, so its index pointer, activation pointer and lookup
// table depend on the lane; a row needs T pair tables (one per expert's
// codebook), T <= 8; and each unit's partial sum is scaled by its slot's router
// weight before the lanes are added.  One launch, no per-slot result in memory.
// The paper applies the fused decode to routed experts (sections 1 and 6.1) and
// names launch overhead as what dominates them; it does not describe this
// epilogue, which is this library's addition.
#include "xfp_decode_stream.inc.h"

namespace xfp {
namespace {

constexpr int kMaxSlots = 8;               // pair tables a wave keeps in LDS (plus the all-zero one)

struct CombineArgs {
    const uint32_t *idx;   // [E][N][K*bits/32]
    const uint16_t *cb;    // [E][N][2^b]
    const int32_t *rp;     // [E*N+1]
    const int32_t *col;
    const uint16_t *val;
    const uint16_t *x;     // slot t reads x + t * x_stride
    const int32_t *eids;   // device [T]
    const float *w;        // device [T]
    void *y;               // [N]
    int64_t x_stride;
    uint32_t N, K, T;
    uint32_t rows_per_wave;
    int y_f32, y_bf16;
    int x_bf16;            // x holds bf16 values, converted to fp16 as they are loaded
};

// NCH : 2048-wide chunks of the concatenated row, T * K <= NCH * 2048
// TAIL: T * K is not a multiple of 2048: lanes past the end read a clamped
//       address, zero activations, the all-zero table and weight 0
// U   : output rows a wave decodes at once.  A wave needs the activations of ALL
//       slots (T * K values, 16 KB at C4's shape) however few rows it owns, so
//       with one row per wave the activation traffic through L2 is several times
//       the index stream; U rows share them, and all loads of the U rows are
//       issued before the first is touched.
// Waves per SIMD the registers are budgeted for: every wave should be resident at
// once (one row per wave at the sizes this is for), because each wave pays a chain
// of dependent round trips (expert ids -> row pointers -> col/val -> activations).
constexpr int combine_waves_per_simd(int loads) { return loads <= 2 ? 4 : (loads <= 3 ? 3 : 2); }   // loads: lane-loads of a batch

template <int BITS, int NCH, bool TAIL, int U>
__global__ __launch_bounds__(kWave, combine_waves_per_simd(NCH * U)) void decode_combine_kernel(CombineArgs a)
{
    using Fmt = TableFmt<BITS>;
    constexpr int ENT = Fmt::kEntries, GPL = Fmt::kGroupsPerLaneLoad;
    constexpr int kNumTables = U * kMaxSlots;              // table u * 8 + t: row u of the batch, slot t; then the all-zero one
    constexpr int kTables = (kNumTables + 1) * Fmt::kRowBytes;
    const uint32_t lds_base = static_lds<kTables + kNumTables * Fmt::kRawBytes + 16>();
    const uint32_t raw_base = lds_base + kTables;

    const uint32_t lane = threadIdx.x;
    const uint32_t N = a.N, K = a.K, T = a.T;
    const uint32_t wpr = K / 32 * BITS;                    // dwords of an expert's row
    const uint32_t upr = K / kLaneWeights;                 // 32-weight units of an expert's row
    const uint32_t units = T * upr;
    const uint32_t row_begin = blockIdx.x * a.rows_per_wave;
    const uint32_t row_end = min(N, row_begin + a.rows_per_wave);
    const uint32_t k2 = 2;                                 // SDWA shift amount, kept in a VGPR

    // expert ids and router weights of all slots through the scalar cache (uniform
    // addresses): a vector gather here would put a full memory round trip in front
    // of every other load of the kernel
    typedef __attribute__((address_space(4))) const int32_t const_i32_t;
    typedef __attribute__((address_space(4))) const float const_f32_t;
    const_i32_t *eids_s = (const_i32_t *)(uintptr_t)a.eids;
    const_f32_t *w_s = (const_f32_t *)(uintptr_t)a.w;
    // slot t's values are parked in lane t of one register each; a lane then fetches
    // the values of ITS slot with a lane permute
    uint32_t e_vec = 0u, w_vec = 0u;
    {
        uint32_t ev[kMaxSlots], wv[kMaxSlots];             // all sixteen scalar loads first, one wait
#pragma unroll
        for (int t = 0; t < kMaxSlots; ++t) {
            const uint32_t tc = min((uint32_t)t, T - 1);
            ev[t] = (uint32_t)eids_s[tc];
            wv[t] = __builtin_bit_cast(uint32_t, w_s[tc]);
        }
#pragma unroll
        for (int t = 0; t < kMaxSlots; ++t) {
            asm("v_writelane_b32 %0, %1, %2" : "+v"(e_vec) : "s"(ev[t]), "n"(t));
            asm("v_writelane_b32 %0, %1, %2" : "+v"(w_vec) : "s"(wv[t]), "n"(t));
        }
    }
    auto expert_of = [&](uint32_t t) { return (uint32_t)__builtin_amdgcn_ds_bpermute((int)(t * 4), (int)e_vec); };
    auto weight_of = [&](uint32_t t) {
        return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((int)(t * 4), (int)w_vec));
    };

    // ---- geometry of this lane's units (the same for every row) ----
    bool live[NCH];
    uint32_t slot[NCH];
    const uint32_t *ip[NCH];                               // index words of this lane's unit in row 0 of its expert
    float wt[NCH];
    uint32_t xr[NCH][16];
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const uint32_t unit = c * kWave + lane;
        live[c] = !TAIL || c < NCH - 1 || unit < units;
        const uint32_t ul = live[c] ? unit : 0u;
        slot[c] = ul / upr;
        const uint32_t uo = ul % upr;                      // unit within the expert's row
        const uint32_t e = expert_of(slot[c]);
        ip[c] = a.idx + (size_t)e * N * wpr + (size_t)uo * BITS;
        wt[c] = live[c] ? weight_of(slot[c]) : 0.f;
        const uint4 *xp = reinterpret_cast<const uint4 *>(a.x + (int64_t)slot[c] * a.x_stride + (size_t)uo * kLaneWeights);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint4 v = xp[i];
            xr[c][4 * i] = live[c] ? v.x : 0u; xr[c][4 * i + 1] = live[c] ? v.y : 0u;
            xr[c][4 * i + 2] = live[c] ? v.z : 0u; xr[c][4 * i + 3] = live[c] ? v.w : 0u;
        }
    }
    // codebook dword this lane stages per row: table t = lane / (ENT / 2), dword lane % (ENT / 2)
    static_assert(kMaxSlots * (ENT / 2) <= kWave, "one codebook dword per lane");
    const uint32_t ct = min(lane / (ENT / 2), T - 1);
    const uint32_t *cbp = reinterpret_cast<const uint32_t *>(a.cb) + (size_t)expert_of(ct) * N * (ENT / 2) +
                          lane % (ENT / 2);
    // outliers: the lanes are dealt to the slots, nsub lanes each; a lane walks the CSR
    // entries of its slot's row with stride nsub (a row rarely has more than one or two)
    const uint32_t nsub = kWave / T;
    const uint32_t ot = min(lane / nsub, T - 1), osub = lane % nsub;
    const bool o_on = lane < T * nsub;
    const int32_t *orp = a.rp + (size_t)expert_of(ot) * N;
    const uint16_t *ox = a.x + (int64_t)ot * a.x_stride;
    const float ow = o_on ? weight_of(ot) : 0.f;

    const bool xbf = a.x_bf16 != 0;
    if (xbf) {
#pragma unroll
        for (int c = 0; c < NCH; ++c)
#pragma unroll
            for (int i = 0; i < 16; ++i) xr[c][i] = bf16x2_to_f16x2(xr[c][i]);
    }

    // the all-zero table that dead lanes look up
    if constexpr (TAIL) {
#pragma unroll
        for (int i = lane; i < Fmt::kRowBytes / 4; i += kWave)
            *(lds_u32_w_t *)(uintptr_t)(lds_base + kNumTables * Fmt::kRowBytes + i * 4) = 0u;
    }
    for (uint32_t row0 = row_begin; row0 < row_end; row0 += U) {
        // ---- all loads of the batch up front: codebooks, row pointers, index words ----
        uint32_t cbv[U];
        int32_t r0[U], r1[U];
        LaneWords<BITS> lw[U][NCH];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t row = min(row0 + u, N - 1);         // rows past the end are decoded again and not stored
            cbv[u] = cbp[(size_t)row * (ENT / 2)];
            r0[u] = orp[row];
            r1[u] = orp[row + 1];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t row = min(row0 + u, N - 1);
#pragma unroll
            for (int c = 0; c < NCH; ++c) lw[u][c] = load_lane_words<BITS>(ip[c] + (size_t)row * wpr);
        }
        __builtin_amdgcn_sched_barrier(0);
        // Keep the activations as packed fp16 pairs (the compiler would otherwise hoist
        // their fp32 conversions out of the row loop and double the registers).
#pragma unroll
        for (int c = 0; c < NCH; ++c)
#pragma unroll
            for (int i = 0; i < 16; ++i) asm volatile("" : "+v"(xr[c][i]));

        // ---- a2: eight pair tables per row (slots past T repeat the last one: no branches) ----
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (kMaxSlots * (ENT / 2) == kWave || lane < kMaxSlots * (ENT / 2))
                *(lds_u32_w_t *)(uintptr_t)(raw_base + u * kMaxSlots * Fmt::kRawBytes + lane * 4) = cbv[u];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        constexpr int PE = 1 << (2 * BITS);                    // pair entries per table (16, 64 or 256)
        constexpr int PR = PE >= kWave ? PE / kWave : 1;
        if (PE >= kWave || lane < PE) {
#pragma unroll
            for (int r = 0; r < kNumTables; ++r) {
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

        // ---- a7 (issue): first outlier entry of this lane's slot in every row of the batch ----
        // no branch around the loads: a lane without an entry reads the row-pointer array instead
        int32_t oj[U];
        uint32_t ocol[U], oval[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            oj[u] = r0[u] + (int32_t)osub;
            const bool ohave = o_on && oj[u] < r1[u];
            const int32_t *pc = ohave ? a.col + oj[u] : a.rp;
            const uint16_t *pv = ohave ? a.val + oj[u] : reinterpret_cast<const uint16_t *>(a.rp);
            const uint32_t ocol_raw = (uint32_t)*pc, oval_raw = (uint32_t)*pv;
            ocol[u] = ohave ? ocol_raw : 0u;
            oval[u] = ohave ? oval_raw : 0u;
        }
        __builtin_amdgcn_sched_barrier(0);

        // ---- a4-a6: depack, gather, multiply-accumulate; lookups run one group of eight ahead ----
        float sum[U];
        uint16_t oxv[U];
        {
            constexpr int TPR = NCH * GPL;                     // tasks per row
            constexpr int NT = U * TPR;
            uint32_t val[2][8];
            float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int u = 0; u < U; ++u) sum[u] = 0.f;
            auto issue = [&](int t, uint32_t (&v)[8]) {
                const int u = t / TPR, c = (t % TPR) / GPL, g = t % GPL;
                issue_group<BITS, true, true>(lw[u][c], g, lds_base,
                                              live[c] ? u * kMaxSlots + slot[c] : (uint32_t)kNumTables, v, k2);
            };
            issue(0, val[0]);
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const int u = t / TPR, c = (t % TPR) / GPL, g = t % GPL;
                if (t + 1 < NT) issue(t + 1, val[(t + 1) & 1]);
                if (t == 3 * NT / 4) {                         // x at the outlier columns (see the streaming kernel)
#pragma unroll
                    for (int v = 0; v < U; ++v) oxv[v] = ox[ocol[v]];
                }
                __builtin_amdgcn_sched_barrier(0);
                consume_group<BITS>(g, val[t & 1], xr[c], acc);
                if (g == GPL - 1) {                            // unit finished: scale by its slot's router weight
                    sum[u] = fmaf(wt[c], (acc[0] + acc[1]) + (acc[2] + acc[3]), sum[u]);
                    acc[0] = acc[1] = acc[2] = acc[3] = 0.f;
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // The sums must exist HERE: without this the compiler sinks the whole multiply-accumulate
        // chain below the (rare) loop over further outlier entries, i.e. behind the outlier
        // loads' round trips instead of in front of them.
#pragma unroll
        for (int u = 0; u < U; ++u) asm volatile("" : "+v"(sum[u]));
        // ---- a7 (fold), a8 ----
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float p = half_bits_to_float((uint16_t)oval[u]) * x_bits_to_float(oxv[u], xbf);
            for (int32_t j = oj[u] + (int32_t)nsub; o_on && j < r1[u]; j += (int32_t)nsub)   // more entries than lanes: rare
                p = fmaf(half_bits_to_float(a.val[j]), x_bits_to_float(ox[a.col[j]], xbf), p);
            const float tot = wave_sum(fmaf(ow, p, sum[u]));
            if (lane == 0 && row0 + u < row_end) store_out(a.y, row0 + u, tot, a.y_f32 != 0, a.y_bf16 != 0);
        }
    }
}

template <int BITS, int NCH, bool TAIL, int U>
hipError_t launch_combine_u(CombineArgs a, hipStream_t s)
{
    uint32_t rpw = U;                                      // one batch per wave unless that makes too many waves
    while ((a.N + rpw - 1) / rpw > 8192 && rpw < 64 * U) rpw += U;
    a.rows_per_wave = rpw;
    hipLaunchKernelGGL((decode_combine_kernel<BITS, NCH, TAIL, U>), dim3((a.N + rpw - 1) / rpw), dim3(kWave), 0, s, a);
    return hipGetLastError();
}

// Rows per batch: as many as keep the tables of a wave within 20 KB of LDS (4 for 2 and 3 bits, 2 for
// 4 bits) and the index words of a batch within 64 registers, fewer when the matrix is too small to
// give every CU a few waves that way, or when the concatenated row is long (registers).
template <int BITS, int NCH, bool TAIL>
hipError_t launch_combine_t(const CombineArgs &a, hipStream_t s)
{
    constexpr int kUmax = (BITS == 4 ? 2 : 4);
    constexpr bool f4 = kUmax >= 4 && NCH <= 4, f2 = NCH <= 6;       // beyond that the registers spill
    if constexpr (f4) {
        if (a.N >= 4 * 1024) return launch_combine_u<BITS, NCH, TAIL, 4>(a, s);
    }
    if constexpr (f2) {
        if (a.N >= 2 * 1024) return launch_combine_u<BITS, NCH, TAIL, 2>(a, s);
    }
    return launch_combine_u<BITS, NCH, TAIL, 1>(a, s);
}

template <int BITS, int NCH>
hipError_t launch_combine_n(const CombineArgs &a, hipStream_t s)
{
    if (((uint64_t)a.T * a.K) % 2048 == 0) return launch_combine_t<BITS, NCH, false>(a, s);
    return launch_combine_t<BITS, NCH, true>(a, s);
}

template <int BITS>
hipError_t launch_combine_b(const CombineArgs &a, hipStream_t s)
{
    switch (((uint64_t)a.T * a.K + 2047) / 2048) {
    case 1: return launch_combine_n<BITS, 1>(a, s);
    case 2: return launch_combine_n<BITS, 2>(a, s);
    case 3: return launch_combine_n<BITS, 3>(a, s);
    case 4: return launch_combine_n<BITS, 4>(a, s);
    case 5: return launch_combine_n<BITS, 5>(a, s);
    case 6: return launch_combine_n<BITS, 6>(a, s);
    case 7: return launch_combine_n<BITS, 7>(a, s);
    default: return launch_combine_n<BITS, 8>(a, s);
    }
}

}  // namespace

bool combine_supports(int bits, int mode, uint32_t K, int T)
{
    return mode == 0 && bits >= 2 && bits <= 4 && T >= 1 && T <= kMaxSlots && (uint64_t)T * K <= 8 * 2048;
}

hipError_t launch_decode_combine(int bits, const DecodeArgs &d, int T, const float *w, bool y_f32, bool y_bf16,
                                 hipStream_t s)
{
    CombineArgs a;
    a.idx = d.idx;
    a.cb = d.cb;
    a.rp = d.rp;
    a.col = d.col;
    a.val = d.val;
    a.x = d.x;
    a.eids = d.eids;
    a.w = w;
    a.y = d.y;
    a.x_stride = d.x_stride;
    a.N = d.N;
    a.K = d.K;
    a.T = (uint32_t)T;
    a.rows_per_wave = 1;
    a.y_f32 = (int)y_f32;
    a.y_bf16 = (int)y_bf16;
    a.x_bf16 = (int)d.x_bf16;
    switch (bits) {
    case 2: return launch_combine_b<2>(a, s);
    case 3: return launch_combine_b<3>(a, s);
    default: return launch_combine_b<4>(a, s);
    }
}

}  // namespace xfp
