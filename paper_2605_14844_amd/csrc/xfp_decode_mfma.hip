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

#ifdef XFP_EXP_TIMING
static __device__ unsigned long long g_dbg[8192];
#define XFP_STAMP(phase) do { if (blockIdx.x == 0 && lane == 0 && it < 8) g_dbg[(it * 8 + (phase)) * 8 + wave] = __builtin_amdgcn_s_memrealtime(); } while (0)
extern "C" int xfp_exp_read_debug(void *dst, size_t bytes) { return (int)hipMemcpyFromSymbol(dst, HIP_SYMBOL(g_dbg), bytes); }
#else
#define XFP_STAMP(phase) do { } while (0)
#endif

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits
// for every outstanding global load (vmcnt(0)), which would drain the index
// prefetch of the next tile at every tile boundary.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
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
    const uint32_t tstep = gridDim.x;

    // ---- per-tile loaders ----
    uint4 iw[KS];
    auto load_indices = [&](uint32_t tile, int c) {
        const uint32_t row = min(tile * kTile + i, N - 1);
        iw[c] = reinterpret_cast<const uint4 *>(a.idx + (size_t)row * wpr + k0 / 8)[c];
    };
    // Row pointers a thread needs for a tile: the tile's entry range and the
    // ranges of the two rows it helps reduce (rows `wave` and `wave + 8`).
    struct TileRp { int32_t base, end, lo1, hi1, lo2, hi2; };
    auto load_rp = [&](uint32_t tile) {
        const uint32_t n0 = tile * kTile;
        TileRp r;
        r.base = a.rp[min(n0, N)];
        r.end = a.rp[min(n0 + kTile, N)];
        r.lo1 = a.rp[min(n0 + wave, N)];
        r.hi1 = a.rp[min(n0 + wave + 1, N)];
        r.lo2 = a.rp[min(n0 + wave + 8, N)];
        r.hi2 = a.rp[min(n0 + wave + 9, N)];
        return r;
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
    // Outlier entry `tid` of a tile (the first 512; more are rare and handled in
    // the reduction): col/val through bounds-checked buffer loads (entries past
    // the end read as zero), then the 16 tokens' activations at that column as
    // one 32-byte read of the transposed copy.
    const uint4 *xt = reinterpret_cast<const uint4 *>(&g_xt[xt_slot][0]);
    auto out_issue = [&](const TileRp &r, uint32_t &col, uint32_t &val) {
        const int32_t base = __builtin_amdgcn_readfirstlane(r.base);
        const int32_t cnt = __builtin_amdgcn_readfirstlane(r.end) - base;
        __amdgpu_buffer_rsrc_t rc = __builtin_amdgcn_make_buffer_rsrc((void *)(a.col + base), 0, cnt * 4, 0x00020000);
        __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc((void *)(a.val + base), 0, cnt * 2, 0x00020000);
        col = __builtin_amdgcn_raw_buffer_load_b32(rc, tid * 4, 0, 0);
        val = __builtin_amdgcn_raw_buffer_load_b16(rv, tid * 2, 0, 0);
    };

    // ---- prologue ----
    // Pipeline depths: index words, codebooks/tables and outlier col/val run one
    // tile ahead; row pointers two tiles ahead (they gate the col/val loads).
    const uint32_t t1 = t + tstep < ntiles ? t + tstep : t;
    TileRp rp_cur = load_rp(t);
    TileRp rp_nxt = load_rp(t1);
    load_codebook(t);
#pragma unroll
    for (int c = 0; c < KS; ++c) load_indices(t, c);
    uint32_t ocol_n = 0, oval_n = 0, oval_c = 0;
    uint4 ox0_c, ox1_c;
    out_issue(rp_cur, ocol_n, oval_n);
    build_table(0);
    ox0_c = xt[(size_t)ocol_n * 2];
    ox1_c = xt[(size_t)ocol_n * 2 + 1];
    oval_c = oval_n;
    out_issue(rp_nxt, ocol_n, oval_n);               // the second tile's entries, gathered during pass 0
    __syncthreads();

    for (uint32_t it = 0; t < ntiles; t += tstep, ++it) {
        const uint32_t buf = it & 1;
        // Next tile of this workgroup.  The last pass "prefetches" its own tile
        // again (cache hits, results unused) so that the loop body is one
        // straight line: conditional loads make the compiler wait for every
        // outstanding load (vmcnt(0)) where a partial wait would do.
        const uint32_t tn = t + tstep < ntiles ? t + tstep : t;
        const uint32_t n0 = t * kTile;
        const int32_t ob0 = __builtin_amdgcn_readfirstlane(rp_cur.base);
        const int32_t ocnt = __builtin_amdgcn_readfirstlane(rp_cur.end) - ob0;
#ifdef XFP_EXP_MFMA_NO_OUT
        const bool have_out = false;
#else
        const bool have_out = true;                      // entries past the end read as zero products
#endif
        (void)ocnt;
        XFP_STAMP(0);
        // Loads of this pass, oldest first: the row pointers two tiles ahead and
        // the next tile's codebooks; index refills follow during the decode and
        // the col/val loads of the tile after next close the pass.
        TileRp rp_far = load_rp(tn + tstep < ntiles ? tn + tstep : tn);
        load_codebook(tn);
        __builtin_amdgcn_sched_barrier(0);
        XFP_STAMP(1);

        // ---- a3-a6: depack, pair lookup, MFMA; lookups run two steps ahead ----
        float4_t acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
        const uint32_t tl = lds_tab + buf * kTabBytes + bank4;
        uint32_t av[3][4];
        auto lookup = [&](int s, uint32_t (&v)[4]) {
            const uint4 &q4 = iw[s / 4];
            const uint32_t w = (s & 3) == 0 ? q4.x : ((s & 3) == 1 ? q4.y : ((s & 3) == 2 ? q4.z : q4.w));
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = *(lds_cu32_t *)(uintptr_t)(tl + byte_times_128(w, j, seven));
        };
        constexpr int OUT_STEP = 2;                      // after this step the outlier products are stored
        // From this step on the next tile's loads are issued: first the x gather
        // at its outlier columns (their col loads are the oldest loads of this
        // pass), then the index refills of the quads already consumed.
        constexpr int GATHER_STEP = NSTEP >= 16 ? 11 : NSTEP - 1;
        uint4 ox0_n = ox0_c, ox1_n = ox1_c;
        lookup(0, av[0]);
        if (NSTEP > 1) lookup(1, av[1]);
#pragma unroll
        for (int s = 0; s < NSTEP; ++s) {
            if (s + 2 < NSTEP) lookup(s + 2, av[(s + 2) % 3]);
            __builtin_amdgcn_sched_barrier(0);
            const uint32_t (&cur)[4] = av[s % 3];
            half8_t af = __builtin_bit_cast(half8_t, make_uint4(cur[0], cur[1], cur[2], cur[3]));
            half8_t bf = __builtin_bit_cast(half8_t, make_uint4(xr[s][0], xr[s][1], xr[s][2], xr[s][3]));
            if (s & 1) acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(af, bf, acc1, 0, 0, 0);
            else acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(af, bf, acc0, 0, 0, 0);
            if (s == OUT_STEP && have_out) {
                // a7: this entry's 16 products -> LDS (gathered one tile ago)
                const float v = half_bits_to_float((uint16_t)oval_c);
                const uint32_t xw[8] = {ox0_c.x, ox0_c.y, ox0_c.z, ox0_c.w, ox1_c.x, ox1_c.y, ox1_c.z, ox1_c.w};
                float p[16];
#pragma unroll
                for (int m = 0; m < 16; ++m)
                    p[m] = v * half_bits_to_float((uint16_t)(m & 1 ? xw[m / 2] >> 16 : xw[m / 2] & 0xFFFFu));
                typedef __attribute__((address_space(3))) float4_t lds_f4_t;
                lds_f4_t *dst = (lds_f4_t *)(uintptr_t)(lds_prod + buf * kProdBytes + tid * 64);
#pragma unroll
                for (int g = 0; g < 4; ++g) dst[g] = float4_t{p[4 * g], p[4 * g + 1], p[4 * g + 2], p[4 * g + 3]};
            }
            if (s == GATHER_STEP) {                      // next tile's activations at its outlier columns
                ox0_n = xt[(size_t)ocol_n * 2];
                ox1_n = xt[(size_t)ocol_n * 2 + 1];
            }
            // an index quad is dead after its 4th step: refill it for the next tile
#ifndef XFP_EXP_MFMA_NO_REFILL
            if (s == GATHER_STEP) {
#pragma unroll
                for (int c = 0; c < KS; ++c)
                    if (4 * c + 3 <= GATHER_STEP) load_indices(tn, c);
            } else if (s > GATHER_STEP && (s & 3) == 3) {
                load_indices(tn, s / 4);
            }
#endif
            __builtin_amdgcn_sched_barrier(0);
        }
        XFP_STAMP(2);

        // ---- tables of the next tile, partial D of this one, col/val two tiles ahead ----
        build_table(buf ^ 1);
        oval_c = oval_n;                                 // next tile's values (arrived long ago)
        out_issue(rp_far, ocol_n, oval_n);
        {
            const uint32_t rb = lds_red + buf * kRedBytes + wave * 1024;
#pragma unroll
            for (int r = 0; r < 4; ++r)                   // D[4q + r][i]
                *(lds_f32_t *)(uintptr_t)(rb + ((4 * q + r) * 16 + i) * 4) = acc0[r] + acc1[r];
        }
        XFP_STAMP(3);
        lds_barrier();
        XFP_STAMP(4);

        // ---- a8: cross-wave reduction, outlier fold, store ----
        // Output (row nl, token m) is summed by the 4 lanes of a quad in a fixed
        // pattern (lane j: waves j and j+4, outlier entries lo+j, lo+j+4, ...) and
        // a fixed DPP order, so results are deterministic.  Each thread serves
        // rows `wave` and `wave + 8`.
        {
            const uint32_t sub = tid & 3, m = (tid >> 2) & 15;
            const uint16_t *xrow = a.x + (size_t)min(m, (uint32_t)M - 1) * a.x_stride;
            constexpr int RD = 10;                        // unconditional reads per lane: 4*RD entries per row
            float part[2], pv[2][RD];
            int32_t lo[2], hi[2];
            const uint32_t pbase = lds_prod + buf * kProdBytes + m * 4;
#pragma unroll
            for (int h = 0; h < 2; ++h) {                 // issue every LDS read of both outputs first
                const uint32_t o = (wave + 8 * h) * 16 + m;
                part[h] = *(lds_f32_t *)(uintptr_t)(lds_red + buf * kRedBytes + sub * 1024 + o * 4) +
                          *(lds_f32_t *)(uintptr_t)(lds_red + buf * kRedBytes + (sub + 4) * 1024 + o * 4);
                lo[h] = (h ? rp_cur.lo2 : rp_cur.lo1) - ob0;
                hi[h] = min((h ? rp_cur.hi2 : rp_cur.hi1) - ob0, (int32_t)kProdEntries);
#ifndef XFP_EXP_MFMA_NO_OUT
                // Unclamped: a read past the product buffer lands in LDS that is
                // either allocated or out of range (reads as 0), and is masked below.
                const uint32_t eb = pbase + (uint32_t)(lo[h] + (int32_t)sub) * 64;
#pragma unroll
                for (int j = 0; j < RD; ++j) pv[h][j] = *(lds_f32_t *)(uintptr_t)(eb + j * 256);
#endif
            }
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const uint32_t nl = wave + 8 * h, n = n0 + nl;
                float s = part[h];
#ifndef XFP_EXP_MFMA_NO_OUT
#pragma unroll
                for (int j = 0; j < RD; ++j) s += lo[h] + (int32_t)sub + 4 * j < hi[h] ? pv[h][j] : 0.f;
                for (int32_t e = lo[h] + (int32_t)sub + 4 * RD; e < hi[h]; e += 4)          // long rows: rare
                    s += *(lds_f32_t *)(uintptr_t)(pbase + e * 64);
                const int32_t full_hi = (h ? rp_cur.hi2 : rp_cur.hi1) - ob0;
                for (int32_t e = max(lo[h], (int32_t)kProdEntries) + (int32_t)sub; e < full_hi; e += 4)   // > 512 per tile: rare
                    s = fmaf(half_bits_to_float(a.val[ob0 + e]), half_bits_to_float(xrow[a.col[ob0 + e]]), s);
#endif
                if (h == 0) XFP_STAMP(6); else XFP_STAMP(7);
                s = dpp_add<0xB1>(s);                     // quad_perm [1,0,3,2]
                s = dpp_add<0x4E>(s);                     // quad_perm [2,3,0,1]
                if (sub == 0 && n < N && m < (uint32_t)M) {
                    const int64_t oo = (int64_t)m * a.y_stride + n;
                    if (y_f32) static_cast<float *>(a.y)[oo] = s;
                    else static_cast<_Float16 *>(a.y)[oo] = (_Float16)s;
                }
            }
        }
        XFP_STAMP(5);
        // rotate the pipelines
        rp_cur = rp_nxt;
        rp_nxt = rp_far;
        ox0_c = ox0_n;
        ox1_c = ox1_n;
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
