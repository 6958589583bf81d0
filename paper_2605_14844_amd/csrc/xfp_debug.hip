// Parity hooks (depack and codebook gather on their own) and the streaming
// probes used to calibrate bandwidth figures and profiler byte counters.
#include "xfp_device.h"
#include "../../include/xfp.h"

namespace xfp {

template <int BITS, int F>
__device__ __forceinline__ void emit_fields(const LaneWords<BITS> &lw, uint8_t *q)
{
    if constexpr (F < 32) {
        q[F] = (uint8_t)field<BITS, F>(lw);
        emit_fields<BITS, F + 1>(lw, q);
    }
}

// One thread per 32-weight unit of the flat [rows][K] index stream.
template <int BITS>
__global__ __launch_bounds__(256) void unpack_kernel(const uint32_t *idx, uint64_t units, uint8_t *out)
{
    uint64_t u = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (u >= units) return;
    LaneWords<BITS> lw = load_lane_words<BITS>(idx + u * BITS);
    __align__(16) uint8_t q[32];
    emit_fields<BITS, 0>(lw, q);
    uint4 *o = reinterpret_cast<uint4 *>(out + u * 32);
    o[0] = *reinterpret_cast<uint4 *>(q);
    o[1] = *reinterpret_cast<uint4 *>(q + 16);
}

template <int BITS, int MODE>
__global__ __launch_bounds__(256) void dequant_kernel(DecodeArgs a, uint64_t units, uint16_t *out)
{
    constexpr int ENT = 1 << BITS;
    uint64_t u = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (u >= units) return;
    const uint32_t upr = a.K / kLaneWeights;             // units per row
    uint64_t grow = u / upr;                             // row in the stacked [E*N] space
    uint32_t ur = (uint32_t)(u % upr);
    LaneWords<BITS> lw = load_lane_words<BITS>(a.idx + u * BITS);
    const uint16_t *tbl;
    if constexpr (MODE == 0) {
        tbl = a.cb + grow * ENT;
    } else {
        uint64_t e = grow / a.N;
        uint32_t g = a.gid[grow * (a.K / kGroup) + ur / (kGroup / kLaneWeights)];
        tbl = a.cb + (e * a.L + g) * ENT;
    }
    __align__(16) uint8_t q[32];
    emit_fields<BITS, 0>(lw, q);
    __align__(16) uint16_t w[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) w[i] = tbl[q[i]];
    uint4 *o = reinterpret_cast<uint4 *>(out + u * 32);
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = *reinterpret_cast<uint4 *>(w + 8 * i);
}

hipError_t launch_unpack(int bits, const uint32_t *idx, uint64_t rows, uint32_t K, uint8_t *out,
                         hipStream_t s)
{
    uint64_t units = rows * (K / kLaneWeights);
    if (units == 0) return hipSuccess;
    dim3 grid((unsigned)((units + 255) / 256));
    switch (bits) {
    case 2: hipLaunchKernelGGL(unpack_kernel<2>, grid, dim3(256), 0, s, idx, units, out); break;
    case 3: hipLaunchKernelGGL(unpack_kernel<3>, grid, dim3(256), 0, s, idx, units, out); break;
    case 5: hipLaunchKernelGGL(unpack_kernel<5>, grid, dim3(256), 0, s, idx, units, out); break;
    case 6: hipLaunchKernelGGL(unpack_kernel<6>, grid, dim3(256), 0, s, idx, units, out); break;
    default: hipLaunchKernelGGL(unpack_kernel<4>, grid, dim3(256), 0, s, idx, units, out); break;
    }
    return hipGetLastError();
}

template <int BITS>
static void launch_dequant_b(int mode, const DecodeArgs &a, uint64_t units, uint16_t *out, dim3 grid,
                             hipStream_t s)
{
    if (mode == 0)
        hipLaunchKernelGGL((dequant_kernel<BITS, 0>), grid, dim3(256), 0, s, a, units, out);
    else
        hipLaunchKernelGGL((dequant_kernel<BITS, 1>), grid, dim3(256), 0, s, a, units, out);
}

hipError_t launch_dequant(int bits, int mode, const DecodeArgs &a, uint32_t E, uint16_t *out,
                          hipStream_t s)
{
    uint64_t units = (uint64_t)E * a.N * (a.K / kLaneWeights);
    if (units == 0) return hipSuccess;
    dim3 grid((unsigned)((units + 255) / 256));
    switch (bits) {
    case 2: launch_dequant_b<2>(mode, a, units, out, grid, s); break;
    case 3: launch_dequant_b<3>(mode, a, units, out, grid, s); break;
    case 5: launch_dequant_b<5>(mode, a, units, out, grid, s); break;
    case 6: launch_dequant_b<6>(mode, a, units, out, grid, s); break;
    default: launch_dequant_b<4>(mode, a, units, out, grid, s); break;
    }
    return hipGetLastError();
}

// ---- streaming probes -------------------------------------------------------
constexpr int kProbeBlocks = 4096;

// Plain streaming read: every thread has four independent 16-byte loads in
// flight, a workgroup reads a contiguous 16 KB span per trip.  The XOR of the
// words reaches `sink` only through a branch on its value, so the loads stay
// alive and the kernel has no other work: this is the shape that read fastest
// among those tried (one to eight loads per thread, 64 to 1024 threads,
// persistent loops), and serves as the practical ceiling beside the decode kernels.
constexpr int kProbeLoads = 4;

__global__ __launch_bounds__(256) void probe_read_kernel(const uint4 *src, uint64_t n16, uint32_t *sink)
{
    typedef uint32_t u4 __attribute__((ext_vector_type(4)));
    uint32_t acc = 0;
    const uint64_t span = 256ull * kProbeLoads;
    for (uint64_t b = (uint64_t)blockIdx.x * span; b < n16; b += (uint64_t)gridDim.x * span) {
        u4 v[kProbeLoads];
#pragma unroll
        for (int i = 0; i < kProbeLoads; ++i) {
            uint64_t o = b + threadIdx.x + (uint64_t)i * 256;
            o = o < n16 ? o : n16 - 1;
            v[i] = __builtin_nontemporal_load(reinterpret_cast<const u4 *>(src) + o);
        }
#pragma unroll
        for (int i = 0; i < kProbeLoads; ++i) acc ^= v[i].x ^ v[i].y ^ v[i].z ^ v[i].w;
    }
    if (acc == 0x9e3779b9u) sink[blockIdx.x & (kProbeBlocks - 1)] = acc;
}

__global__ __launch_bounds__(256) void probe_copy_kernel(const uint4 *src, uint4 *dst, uint64_t n16)
{
    for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (uint64_t)gridDim.x * 256)
        dst[i] = src[i];
}

hipError_t launch_probe_read(const void *src, uint64_t bytes, uint32_t *sink, hipStream_t s)
{
    uint64_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    const uint64_t span = 256ull * kProbeLoads, want = (n16 + span - 1) / span;
    unsigned blocks = (unsigned)(want < 4ull * kProbeBlocks ? want : 4ull * kProbeBlocks);
    hipLaunchKernelGGL(probe_read_kernel, dim3(blocks), dim3(256), 0, s,
                       static_cast<const uint4 *>(src), n16, sink);
    return hipGetLastError();
}

hipError_t launch_probe_copy(const void *src, void *dst, uint64_t bytes, hipStream_t s)
{
    uint64_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    unsigned blocks = (unsigned)((n16 + 255) / 256 < kProbeBlocks ? (n16 + 255) / 256 : kProbeBlocks);
    hipLaunchKernelGGL(probe_copy_kernel, dim3(blocks), dim3(256), 0, s,
                       static_cast<const uint4 *>(src), static_cast<uint4 *>(dst), n16);
    return hipGetLastError();
}

// ---------------------------------------------------------------- content check
// What the decode entry points take on trust, checked on the device.
// report[0] violations found; report[1] OR of (1 << kind) over them;
// report[2], report[3] low and high word of the smallest position among them
// (kind 1: group id index; 2: row pointer index; 3, 4: outlier entry index;
// 5: slot).  All three are order-independent, so the report is deterministic.
struct CheckArgs {
    const uint8_t *gid;
    const int32_t *rp, *col, *eids;
    uint64_t n_gid, n_rows, cap;       // group ids, stacked rows, entries allocated in col
    uint32_t K, L, E;
    int T;
    uint32_t *report;
};

__device__ __forceinline__ void check_fail(uint32_t *report, int kind, uint64_t pos)
{
    atomicAdd(&report[0], 1u);
    atomicOr(&report[1], 1u << kind);
    atomicMin(reinterpret_cast<unsigned long long *>(report + 2), (unsigned long long)pos);
}

__global__ void check_init_kernel(uint32_t *report)
{
    report[0] = 0u;
    report[1] = 0u;
    report[2] = 0xFFFFFFFFu;
    report[3] = 0xFFFFFFFFu;
}

__global__ __launch_bounds__(256) void check_contents_kernel(CheckArgs c)
{
    const uint64_t stride = (uint64_t)gridDim.x * 256;
    const uint64_t t0 = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (c.gid)
        for (uint64_t i = t0; i < c.n_gid; i += stride)
            if (c.gid[i] >= c.L) check_fail(c.report, XFP_CHECK_GROUP_ID, i);
    if (t0 == 0 && c.rp[0] != 0) check_fail(c.report, XFP_CHECK_ROW_PTR, 0);
    for (uint64_t r = t0; r < c.n_rows; r += stride) {
        const int64_t a = c.rp[r], b = c.rp[r + 1];
        if (b < a || b < 0 || (uint64_t)b > c.cap) {
            check_fail(c.report, XFP_CHECK_ROW_PTR, r + 1);
            continue;
        }
        if (a < 0) continue;                               // reported at the previous row
        int64_t prev = -1;
        for (int64_t j = a; j < b; ++j) {
            const int64_t k = c.col[j];
            if (k < 0 || k >= (int64_t)c.K) check_fail(c.report, XFP_CHECK_COL_RANGE, (uint64_t)j);
            else if (k <= prev) check_fail(c.report, XFP_CHECK_COL_ORDER, (uint64_t)j);
            prev = k;
        }
    }
    if (c.eids)
        for (uint64_t t = t0; t < (uint64_t)c.T; t += stride)
            if (c.eids[t] < 0 || (uint32_t)c.eids[t] >= c.E) check_fail(c.report, XFP_CHECK_EXPERT_ID, t);
}

hipError_t launch_check_contents(const DecodeArgs &a, uint32_t E, uint64_t nnz_capacity, const int32_t *eids, int T,
                                 uint32_t *report, hipStream_t s)
{
    CheckArgs c;
    c.gid = a.gid;
    c.rp = a.rp;
    c.col = a.col;
    c.eids = eids;
    c.n_rows = (uint64_t)E * a.N;
    c.n_gid = a.gid ? c.n_rows * (a.K / kGroup) : 0;
    c.cap = nnz_capacity;
    c.K = a.K;
    c.L = a.L;
    c.E = E;
    c.T = T;
    c.report = report;
    hipLaunchKernelGGL(check_init_kernel, dim3(1), dim3(1), 0, s, report);
    const uint64_t work = c.n_gid > c.n_rows ? c.n_gid : c.n_rows;
    const unsigned blocks = (unsigned)((work + 255) / 256 < 4096 ? (work + 255) / 256 : 4096);
    hipLaunchKernelGGL(check_contents_kernel, dim3(blocks ? blocks : 1), dim3(256), 0, s, c);
    return hipGetLastError();
}

}  // namespace xfp
