// Small-batch fused decode (2 <= M <= 16 tokens per launch) on the matrix cores,
// V2 codebooks, 4-bit indices, K a multiple of 1024 up to 8192.
//
// The weights are read from HBM once for all tokens.  A workgroup of 8 waves
// owns a tile of 16 output rows at a time; wave w owns the K slice
// [w*K/8, (w+1)*K/8) of every tile, so its share of the 16 activation rows
// stays in VGPRs for the whole kernel as ready-made MFMA B operands.
// v_mfma_f32_16x16x32_f16 contracts 32 k per issue:
//     A (16 rows x 32 k) = dequantised weights, lane (i, q) supplies 8 consecutive
//                          k of row i -- exactly one dword of 4-bit indices;
//     B (32 k x 16 tokens) = activations, lane (m, q) supplies the same 8 k of token m;
//     D (16 x 16 fp32)     = partial y for the wave's K slice.
// Within a lane the k order is free as long as A and B agree, so lane (i, q)
// takes a contiguous run of K/32 weights of row i: 4 lanes cover 4 x 16..128
// contiguous bytes of a row and every index byte is loaded exactly once.
//
// Dequantisation is one LDS lookup per PAIR of weights: a per-row table maps an
// index byte (two 4-bit indices) to two fp16 values, which is already the
// packed form the MFMA operand wants.  The 16 rows of a tile need 16 different
// tables in one wave instruction, so the tables are stored bank-private:
// entry e of row i lives at dword e*32 + bank with bank = i (+16 for odd q), so
// the 32 lanes the LDS serves per clock always hit 32 different banks.  The
// tables of tile t+1 are built (double-buffered) while tile t is decoded.
//
// Per tile, the 8 partial D blocks are summed through LDS in a fixed order
// (deterministic) by 256 threads, which also add the CSR outlier products of
// the tile.  One thread per outlier entry computes its 16 products: col/val
// come through bounds-checked buffer loads one tile ahead, and the 16 tokens'
// activations at that column come as ONE 32-byte read from a k-major
// (transposed) copy of x.  Gathering them from the row-major x instead costs
// 16 cache lines per entry and was measured to triple the kernel time.  The
// transposed copy lives in a small ring of file-scope device buffers and is
// written by a tiny kernel launched in front of the decode kernel on the same
// stream; more than kXtSlots batched calls in flight at once on one GPU would
// reuse a slot that is still being read.
#include "xfp_device.h"

#include <atomic>

namespace xfp {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) const uint32_t lds_cu32_t;
typedef __attribute__((address_space(3))) uint32_t lds_u32_t;
typedef __attribute__((address_space(3))) float lds_f32_t;

constexpr int kMfmaThreads = 512;
constexpr int kMfmaWaves = 8;
constexpr int kTile = 16;                       // rows per tile = tokens per launch
constexpr int kTabBytes = 256 * 32 * 4;         // one pair table set: [256 entries][32 banks] dwords
constexpr int kRedBytes = kMfmaWaves * 256 * 4; // partial D blocks of one tile
constexpr int kProdEntries = 512;               // outlier entries per tile kept in LDS
constexpr int kProdBytes = kProdEntries * 16 * 4;
constexpr int kMfmaLds = 2 * kTabBytes + 2 * kRedBytes + 2 * kProdBytes;

constexpr int kXtSlots = 16;                   // batched calls that may overlap on one GPU
constexpr int kXtMaxK = 8192;
static __device__ __align__(256) uint16_t g_xt[kXtSlots][kXtMaxK * kTile];   // [slot][k][16 tokens]

// x [M][ldx] row-major -> g_xt[slot][k][0..15], tokens >= M zero.
__global__ __launch_bounds__(256) void transpose_x_kernel(const uint16_t *x, int64_t ldx, int M, uint32_t K,
                                                          int slot)
{
    const uint32_t k = blockIdx.x * 256 + threadIdx.x;
    if (k >= K) return;
    uint32_t v[8];
#pragma unroll
    for (int m = 0; m < 16; m += 2) {
        const uint32_t lo = m < M ? x[(size_t)m * ldx + k] : 0u;
        const uint32_t hi = m + 1 < M ? x[(size_t)(m + 1) * ldx + k] : 0u;
        v[m / 2] = lo | (hi << 16);
    }
    uint4 *o = reinterpret_cast<uint4 *>(&g_xt[slot][(size_t)k * kTile]);
    o[0] = make_uint4(v[0], v[1], v[2], v[3]);
    o[1] = make_uint4(v[4], v[5], v[6], v[7]);
}

#define XFP_SDWA_SHL(dst, amount, src, J)                                                         \
    asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_" #J \
        : "=v"(dst) : "v"(amount), "v"(src))

__device__ __forceinline__ uint32_t byte_times_128(uint32_t w, int j, uint32_t seven)
{
    uint32_t r;
    switch (j) {
    case 0: XFP_SDWA_SHL(r, seven, w, 0); break;
    case 1: XFP_SDWA_SHL(r, seven, w, 1); break;
    case 2: XFP_SDWA_SHL(r, seven, w, 2); break;
    default: XFP_SDWA_SHL(r, seven, w, 3); break;
    }
    return r;
}

// KS = K / 1024: each lane owns 32*KS weights of its row per tile (KS dwordx4
// loads), 4*KS MFMA steps, 16*KS VGPRs of activations.
template <int KS>
__global__ __launch_bounds__(kMfmaThreads) void decode_mfma4_kernel(DecodeArgs a, int M, int y_f32, int xt_slot)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    const uint32_t lds_tab = lds0, lds_red = lds0 + 2 * kTabBytes, lds_prod = lds_red + 2 * kRedBytes;

    constexpr int NSTEP = 4 * KS;               // MFMA issues per tile per wave
    constexpr int R = 32 * KS;                  // weights per lane per tile
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t i = lane & 15, q = lane >> 4;
    const uint32_t N = a.N, K = a.K;
    const uint32_t wpr = K / 8;                 // dwords per row (4-bit)
    const uint32_t ntiles = (N + kTile - 1) / kTile;
    const uint32_t k0 = wave * (K / kMfmaWaves) + q * R;        // first k of this lane
    const uint32_t seven = 7;
    const uint32_t bank4 = (((q & 1) << 4) | i) * 4;             // this lane's private bank
    const uint32_t *cbw = reinterpret_cast<const uint32_t *>(a.cb);

    // B operands: this lane's activations, token m = i, k = k0 .. k0 + R.
    uint32_t xr[NSTEP][4];
    {
        const uint32_t m = min(i, (uint32_t)M - 1);
        const uint4 *xp = reinterpret_cast<const uint4 *>(a.x + (size_t)m * a.x_stride + k0);
#pragma unroll
        for (int s = 0; s < NSTEP; ++s) {
            uint4 v = xp[s];
            const bool on = i < (uint32_t)M;
            xr[s][0] = on ? v.x : 0u; xr[s][1] = on ? v.y : 0u;
            xr[s][2] = on ? v.z : 0u; xr[s][3] = on ? v.w : 0u;
        }
    }

    // Table builder role of this thread: bank (-> row) and low-nibble entry are fixed.
    const uint32_t tb_bank = tid & 31, tb_row = tb_bank & 15, tb_lo = tid >> 5;   // tb_lo in [0,16)

    uint32_t t = blockIdx.x;
    if (t >= ntiles) return;

    // ---- prologue: tables, index words and row pointers of the first tile ----
    uint4 iw[KS];
    int32_t rp_lo, rp_hi, rp_base, rp_end;
    auto load_indices = [&](uint32_t tile, int c) {
        const uint32_t row = min(tile * kTile + i, N - 1);
        iw[c] = reinterpret_cast<const uint4 *>(a.idx + (size_t)row * wpr + k0 / 8)[c];
    };
    auto load_rp = [&](uint32_t tile) {
        const uint32_t n0 = tile * kTile, nl = (tid >> 4) & 15;
        rp_lo = a.rp[min(n0 + nl, N)];
        rp_hi = a.rp[min(n0 + nl + 1, N)];
        rp_base = a.rp[min(n0, N)];
        rp_end = a.rp[min(n0 + kTile, N)];
    };
    uint4 cbr[2];
    uint32_t cblo;
    auto load_codebook = [&](uint32_t tile) {
        const uint32_t row = min(tile * kTile + tb_row, N - 1);
        const uint32_t *p = cbw + (size_t)row * 8;
        cbr[0] = reinterpret_cast<const uint4 *>(p)[0];
        cbr[1] = reinterpret_cast<const uint4 *>(p)[1];
        cblo = p[tb_lo >> 1];
    };
    auto build_table = [&](uint32_t buf) {
        const uint32_t lo = (tb_lo & 1) ? (cblo >> 16) : (cblo & 0xFFFFu);
        const uint32_t cw[8] = {cbr[0].x, cbr[0].y, cbr[0].z, cbr[0].w, cbr[1].x, cbr[1].y, cbr[1].z, cbr[1].w};
        const uint32_t base = lds_tab + buf * kTabBytes + tb_lo * 128 + tb_bank * 4;
#pragma unroll
        for (int rep = 0; rep < 16; ++rep) {             // entry = tb_lo + 16*rep: high nibble = rep
            const uint32_t hi = (rep & 1) ? (cw[rep >> 1] & 0xFFFF0000u) : (cw[rep >> 1] << 16);
            *(lds_u32_t *)(uintptr_t)(base + rep * 16 * 128) = lo | hi;
        }
    };
    // Outlier entry `tid` of a tile (the first 512; more are rare and handled by
    // the reducers): col/val are fetched one tile ahead through bounds-checked
    // buffer loads (entries past the end read as zero).
    const uint4 *xt = reinterpret_cast<const uint4 *>(&g_xt[xt_slot][0]);
    uint32_t ocol = 0, oval = 0;
    auto out_issue = [&](int32_t base, int32_t cnt) {
        __amdgpu_buffer_rsrc_t rc = __builtin_amdgcn_make_buffer_rsrc((void *)(a.col + base), 0, cnt * 4, 0x00020000);
        __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc((void *)(a.val + base), 0, cnt * 2, 0x00020000);
        ocol = __builtin_amdgcn_raw_buffer_load_b32(rc, tid * 4, 0, 0);
        oval = __builtin_amdgcn_raw_buffer_load_b16(rv, tid * 2, 0, 0);
    };

    load_rp(t);
    load_codebook(t);
#pragma unroll
    for (int c = 0; c < KS; ++c) load_indices(t, c);
    out_issue(__builtin_amdgcn_readfirstlane(rp_base),
              __builtin_amdgcn_readfirstlane(rp_end) - __builtin_amdgcn_readfirstlane(rp_base));
    build_table(0);
    __syncthreads();

    for (uint32_t it = 0; t < ntiles; t += gridDim.x, ++it) {
        const uint32_t buf = it & 1;
        const uint32_t tn = t + gridDim.x;               // next tile of this workgroup
        const bool has_next = tn < ntiles;
        const uint32_t n0 = t * kTile;
        // metadata of this tile (loaded one iteration ago)
        const int32_t ob0 = __builtin_amdgcn_readfirstlane(rp_base);
        const int32_t ocnt = __builtin_amdgcn_readfirstlane(rp_end) - ob0;
        const int32_t my_lo = rp_lo - ob0, my_hi = rp_hi - ob0;  // reducer's entry range, tile-relative

        // a7: gather x at this tile's outlier columns (col/val were issued one
        // tile ago, so waiting for them waits for nothing newer than this tile's
        // index words); the products go to LDS after a few decode steps, before
        // any load of the next tile is issued.
#ifdef XFP_EXP_MFMA_NO_OUT
        const bool have_out = false;
#else
        const bool have_out = ocnt > 0;
#endif
        uint4 ox0 = make_uint4(0, 0, 0, 0), ox1 = ox0;
        if (have_out) {
            ox0 = xt[(size_t)ocol * 2];
            ox1 = xt[(size_t)ocol * 2 + 1];
        }
        __builtin_amdgcn_sched_barrier(0);
        if (has_next) {
            load_rp(tn);
            load_codebook(tn);
        }
        __builtin_amdgcn_sched_barrier(0);

        // ---- a3-a6: depack, pair lookup, MFMA; lookups run one step ahead ----
        float4_t acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
        const uint32_t tl = lds_tab + buf * kTabBytes + bank4;
        uint32_t av[2][4];
        auto lookup = [&](int s, uint32_t (&v)[4]) {
            const uint4 &q4 = iw[s / 4];
            const uint32_t w = (s & 3) == 0 ? q4.x : ((s & 3) == 1 ? q4.y : ((s & 3) == 2 ? q4.z : q4.w));
#pragma unroll
#ifdef XFP_EXP_MFMA_NO_LOOKUP
            for (int j = 0; j < 4; ++j) v[j] = w + j;
#else
            for (int j = 0; j < 4; ++j) v[j] = *(lds_cu32_t *)(uintptr_t)(tl + byte_times_128(w, j, seven));
#endif
        };
        constexpr int OUT_STEP = 3;                      // step after which the outlier products are stored
        lookup(0, av[0]);
#pragma unroll
        for (int s = 0; s < NSTEP; ++s) {
            if (s + 1 < NSTEP) lookup(s + 1, av[(s + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
            half8_t af = __builtin_bit_cast(half8_t, make_uint4(av[s & 1][0], av[s & 1][1], av[s & 1][2], av[s & 1][3]));
            half8_t bf = __builtin_bit_cast(half8_t, make_uint4(xr[s][0], xr[s][1], xr[s][2], xr[s][3]));
            if (s & 1) acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(af, bf, acc1, 0, 0, 0);
            else acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(af, bf, acc0, 0, 0, 0);
            if (s == OUT_STEP && have_out) {
                const float v = half_bits_to_float((uint16_t)oval);
                const uint32_t xw[8] = {ox0.x, ox0.y, ox0.z, ox0.w, ox1.x, ox1.y, ox1.z, ox1.w};
                float p[16];
#pragma unroll
                for (int m = 0; m < 16; ++m)
                    p[m] = v * half_bits_to_float((uint16_t)(m & 1 ? xw[m / 2] >> 16 : xw[m / 2] & 0xFFFFu));
                typedef __attribute__((address_space(3))) float4_t lds_f4_t;
                lds_f4_t *dst = (lds_f4_t *)(uintptr_t)(lds_prod + buf * kProdBytes + tid * 64);
#pragma unroll
                for (int g = 0; g < 4; ++g) dst[g] = float4_t{p[4 * g], p[4 * g + 1], p[4 * g + 2], p[4 * g + 3]};
            }
            // an index quad is dead after its 4th step: refill it for the next tile
            // (the first refill comes after the outlier products are out of the way)
            if ((s & 3) == 3 && has_next) load_indices(tn, s / 4);
            __builtin_amdgcn_sched_barrier(0);
        }

        // ---- next tile: outlier loads and tables; this tile: partial D ----
        if (has_next) {
#ifndef XFP_EXP_MFMA_NO_OUT
            out_issue(__builtin_amdgcn_readfirstlane(rp_base),
                      __builtin_amdgcn_readfirstlane(rp_end) - __builtin_amdgcn_readfirstlane(rp_base));
#endif
#ifndef XFP_EXP_MFMA_NO_BUILD
            build_table(buf ^ 1);
#endif
        }
        {
            const uint32_t rb = lds_red + buf * kRedBytes + wave * 1024;
#pragma unroll
            for (int r = 0; r < 4; ++r)                   // D[4q + r][i]
                *(lds_f32_t *)(uintptr_t)(rb + ((4 * q + r) * 16 + i) * 4) = acc0[r] + acc1[r];
        }
        __syncthreads();

        // ---- a8: cross-wave reduction, outlier fold, store (256 threads) ----
        if (tid < 256) {
            const uint32_t nl = tid >> 4, m = tid & 15, n = n0 + nl;
            float s = 0.f;
#pragma unroll
            for (int w = 0; w < kMfmaWaves; ++w)
                s += *(lds_f32_t *)(uintptr_t)(lds_red + buf * kRedBytes + w * 1024 + tid * 4);
            const uint16_t *xrow = a.x + (size_t)min(m, (uint32_t)M - 1) * a.x_stride;
#ifndef XFP_EXP_MFMA_NO_OUT
            for (int32_t e = my_lo; e < my_hi; ++e) {
                if (e < kProdEntries)
                    s += *(lds_f32_t *)(uintptr_t)(lds_prod + buf * kProdBytes + (e * 16 + m) * 4);
                else                                       // more than 512 entries in a tile: rare
                    s = fmaf(half_bits_to_float(a.val[ob0 + e]), half_bits_to_float(xrow[a.col[ob0 + e]]), s);
            }
#endif
            if (n < N && m < (uint32_t)M) {
                const int64_t o = (int64_t)m * a.y_stride + n;
                if (y_f32) static_cast<float *>(a.y)[o] = s;
                else static_cast<_Float16 *>(a.y)[o] = (_Float16)s;
            }
        }
    }
}

template <int KS>
static hipError_t launch_mfma_t(const DecodeArgs &a, int M, bool y_f32, hipStream_t s)
{
    static bool configured = false;                      // idempotent attribute, benign race
    auto kern = decode_mfma4_kernel<KS>;
    if (!configured) {
        hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kMfmaLds);
        if (err != hipSuccess) return err;
        configured = true;
    }
    static std::atomic<unsigned> next_slot{0};
    const int slot = (int)(next_slot.fetch_add(1, std::memory_order_relaxed) % kXtSlots);
    hipLaunchKernelGGL(transpose_x_kernel, dim3((a.K + 255) / 256), dim3(256), 0, s, a.x, a.x_stride, M, a.K, slot);
    const uint32_t ntiles = (a.N + kTile - 1) / kTile;
    const uint32_t blocks = ntiles < 256 ? ntiles : 256;
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(kMfmaThreads), kMfmaLds, s, a, M, (int)y_f32, slot);
    return hipGetLastError();
}

bool mfma_supports(int bits, int mode, uint32_t K, int M)
{
    return bits == 4 && mode == 0 && M >= 2 && K % 1024 == 0 && K >= 1024 && K <= 8192;
}

// M <= 16 tokens per launch; the caller loops over chunks of 16.
hipError_t launch_decode_mfma(const DecodeArgs &a, int M, bool y_f32, hipStream_t s)
{
    switch (a.K / 1024) {
    case 1: return launch_mfma_t<1>(a, M, y_f32, s);
    case 2: return launch_mfma_t<2>(a, M, y_f32, s);
    case 3: return launch_mfma_t<3>(a, M, y_f32, s);
    case 4: return launch_mfma_t<4>(a, M, y_f32, s);
    case 5: return launch_mfma_t<5>(a, M, y_f32, s);
    case 6: return launch_mfma_t<6>(a, M, y_f32, s);
    case 7: return launch_mfma_t<7>(a, M, y_f32, s);
    default: return launch_mfma_t<8>(a, M, y_f32, s);
    }
}

}  // namespace xfp
