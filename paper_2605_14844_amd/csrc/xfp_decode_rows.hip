// General fused decode kernel: any K that is a multiple of 128, any N, every bit width of the paper's
// packing table (2 .. 6), and the only kernel for V2a matrices with a scale and a mid-point per group.
//
// One wave owns one output row at a time (no atomics, a fixed summation
// order).  The activation row is staged once per workgroup in LDS (paper
// section 5, activation-row caching), the codebook of the row (V2) or the
// whole library (V2a) sits in LDS next to it, each lane streams 32 indices
// per load, looks its codebook entries up in LDS and accumulates in fp32;
// the row's CSR outliers are folded in before the wave reduction.
#include "xfp_device.h"

namespace xfp {

constexpr int kRowsThreads = 256;
constexpr int kRowsWaves = kRowsThreads / kWave;

template <int BITS, int I>
__device__ __forceinline__ void accumulate_pairs(const LaneWords<BITS> &lw, const _Float16 *tbl,
                                                 const uint32_t *xw, float &acc)
{
    if constexpr (I < 16) {
        half2_t c;
        c.x = tbl[field<BITS, 2 * I>(lw)];
        c.y = tbl[field<BITS, 2 * I + 1>(lw)];
        acc = dot2(c, as_half2(xw[I]), acc);
        accumulate_pairs<BITS, I + 1>(lw, tbl, xw, acc);
    }
}

// AFF (V2a only): every group carries a scale and a mid-point (paper section 3.4; no formula given, reading
// taken: entry * scale + mid).  By linearity a unit of 32 weights inside one group contributes
// scale * sum(x * entry) + mid * sum(x), both sums in fp32, one fused multiply-add on top.
template <int BITS, int MODE, bool YF32, bool AFF>
__global__ __launch_bounds__(kRowsThreads) void decode_rows_kernel(DecodeArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int ENT = 1 << BITS;
    uint32_t *xs = reinterpret_cast<uint32_t *>(smem);                    // K halves
    _Float16 *tables = reinterpret_cast<_Float16 *>(smem + (size_t)a.K * 2);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t slot = blockIdx.y;
    const uint32_t e = a.eids ? (uint32_t)a.eids[slot] : 0u;
    const uint32_t N = a.N, K = a.K;
    const uint32_t wpr = K / 32 * BITS;                                  // words per row
    const uint32_t *idx = a.idx + (size_t)e * N * wpr;
    const int32_t *rp = a.rp + (size_t)e * N;
    const uint16_t *x = a.x + (int64_t)slot * a.x_stride;

    // a1: stage the activation row.
    for (uint32_t i = tid; i < K / 8; i += kRowsThreads) {
        uint4 v = reinterpret_cast<const uint4 *>(x)[i];
        if (a.x_bf16) v = make_uint4(bf16x2_to_f16x2(v.x), bf16x2_to_f16x2(v.y), bf16x2_to_f16x2(v.z), bf16x2_to_f16x2(v.w));
        reinterpret_cast<uint4 *>(xs)[i] = v;
    }
    // a2: V2a library -> LDS once per workgroup.
    if constexpr (MODE == 1) {
        const uint16_t *lib = a.cb + (size_t)e * a.L * ENT;
        for (uint32_t i = tid; i < a.L * ENT; i += kRowsThreads)
            tables[i] = __builtin_bit_cast(_Float16, lib[i]);
    }
    __syncthreads();

    const uint32_t row0 = blockIdx.x * a.rows_per_block;
    const uint32_t row1 = min(N, row0 + a.rows_per_block);
    _Float16 *mytbl = tables + wave * ENT;                                // V2: per-wave table

    for (uint32_t row = row0 + wave; row < row1; row += kRowsWaves) {
        if constexpr (MODE == 0) {
            const uint32_t *cbw = reinterpret_cast<const uint32_t *>(a.cb + ((size_t)e * N + row) * ENT);
            __builtin_amdgcn_wave_barrier();
            if (lane < ENT / 2) reinterpret_cast<uint32_t *>(mytbl)[lane] = cbw[lane];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
        const uint32_t *rw = idx + (size_t)row * wpr;
        float acc = 0.f;
        for (uint32_t u = lane; u < K / kLaneWeights; u += kWave) {
            // a3/a4: stream and depack; a5: gather; a6: multiply-accumulate.
            LaneWords<BITS> lw = load_lane_words<BITS>(rw + (size_t)u * BITS);
            const _Float16 *tbl = mytbl;
            if constexpr (MODE == 1) {
                uint32_t g = a.gid[((size_t)e * N + row) * (K / kGroup) + u / (kGroup / kLaneWeights)];
                tbl = tables + g * ENT;
            }
            uint32_t xw[16];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                uint4 v = reinterpret_cast<const uint4 *>(xs)[u * 4 + i];
                xw[4 * i] = v.x; xw[4 * i + 1] = v.y; xw[4 * i + 2] = v.z; xw[4 * i + 3] = v.w;
            }
            if constexpr (AFF) {
                const size_t g = ((size_t)e * N + row) * (K / kGroup) + u / (kGroup / kLaneWeights);
                const float sc = half_bits_to_float(a.gscale[g]), md = half_bits_to_float(a.gmid[g]);
                float au = 0.f, xs = 0.f;
                accumulate_pairs<BITS, 0>(lw, tbl, xw, au);
                const half2_t ones = {(_Float16)1.0f, (_Float16)1.0f};
#pragma unroll
                for (int i = 0; i < 16; ++i) xs = dot2(ones, as_half2(xw[i]), xs);
                acc += fmaf(sc, au, md * xs);
            } else {
                accumulate_pairs<BITS, 0>(lw, tbl, xw, acc);
            }
        }
        // a7: outlier fold, CSR row owned by this wave.
        const int32_t j1 = rp[row + 1];
        for (int32_t j = rp[row] + lane; j < j1; j += kWave) {
            float v = half_bits_to_float(a.val[j]);
            float xv = (float)reinterpret_cast<const _Float16 *>(xs)[a.col[j]];
            acc = fmaf(v, xv, acc);
        }
        // a8: reduce and store.
        acc = wave_sum(acc);
        if (lane == 0) store_y<YF32>(a.y, (int64_t)slot * a.y_stride + row, acc, a.y_bf16 != 0);
    }
}

template <int BITS, int MODE, bool YF32, bool AFF = false>
static hipError_t launch_rows_t(const DecodeArgs &a, int slots, hipStream_t s)
{
    size_t table_halves = MODE == 1 ? (size_t)a.L << BITS : (size_t)kRowsWaves << BITS;
    size_t smem = (size_t)a.K * 2 + table_halves * 2;
    dim3 grid((a.N + a.rows_per_block - 1) / a.rows_per_block, slots);
    auto kern = decode_rows_kernel<BITS, MODE, YF32, AFF>;
    if (smem > 48 * 1024) {
        hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (err != hipSuccess) return err;
    }
    hipLaunchKernelGGL(kern, grid, dim3(kRowsThreads), smem, s, a);
    return hipGetLastError();
}

template <int BITS>
static hipError_t launch_rows_b(int mode, bool y_f32, const DecodeArgs &a, int slots, hipStream_t s)
{
    if (mode == 0)
        return y_f32 ? launch_rows_t<BITS, 0, true>(a, slots, s) : launch_rows_t<BITS, 0, false>(a, slots, s);
    if (a.gscale)
        return y_f32 ? launch_rows_t<BITS, 1, true, true>(a, slots, s) : launch_rows_t<BITS, 1, false, true>(a, slots, s);
    return y_f32 ? launch_rows_t<BITS, 1, true>(a, slots, s) : launch_rows_t<BITS, 1, false>(a, slots, s);
}

hipError_t launch_decode_rows(int bits, int mode, bool y_f32, const DecodeArgs &a, int slots,
                              hipStream_t s)
{
    switch (bits) {
    case 2: return launch_rows_b<2>(mode, y_f32, a, slots, s);
    case 3: return launch_rows_b<3>(mode, y_f32, a, slots, s);
    case 5: return launch_rows_b<5>(mode, y_f32, a, slots, s);
    case 6: return launch_rows_b<6>(mode, y_f32, a, slots, s);
    default: return launch_rows_b<4>(mode, y_f32, a, slots, s);
    }
}

}  // namespace xfp
