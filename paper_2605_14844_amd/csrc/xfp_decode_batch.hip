// Small-batch fused decode on the matrix cores: the 4-bit instantiation of the
// kernel, the re-laid activation copies it reads, and the host-side dispatch
// over bit widths.
#include "xfp_decode_batch.inc.h"

namespace xfp {

// defined in xfp_decode_batch3.hip, xfp_decode_batch2.hip
hipError_t launch_batch3(const DecodeArgs &a, int M, bool y_f32, float *part, const void *xt, const void *xb,
                         hipStream_t s);
hipError_t launch_batch2(const DecodeArgs &a, int M, bool y_f32, float *part, const void *xt, const void *xb,
                         hipStream_t s);
// defined in xfp_decode_batch_lib3.hip, xfp_decode_batch_lib4.hip
hipError_t launch_batch_lib3(const DecodeArgs &a, int M, bool y_f32, float *part, const void *xt, const void *xb,
                             hipStream_t s);
hipError_t launch_batch_lib4(const DecodeArgs &a, int M, bool y_f32, float *part, const void *xt, const void *xb,
                             hipStream_t s);

namespace {

constexpr int kXtSlots = 16;               // batched calls that may overlap on one GPU
constexpr int kXtMaxK = 32768;
// Two re-laid copies of the 16 x K activations of a call, per ring slot:
//   xt [k][16 tokens]           the outlier products read the 16 tokens of one column as 32 bytes;
//   xb [k / 8][16 tokens][8 k]  the B operand of lane (m, q) for a k block is 16 contiguous bytes and
//                               the 64 lanes of a wave read 1 KB contiguous (from the row-major x the
//                               same load touches 64 different cache lines).
// Tokens >= M are zero in both.  More than kXtSlots batched calls in flight at once on one GPU
// would reuse a slot that is still being read.
struct XCopies {
    uint16_t xt[kXtMaxK * kTile];
    uint16_t xb[kXtMaxK * kTile];
};
__device__ __align__(256) XCopies g_x[kXtSlots];

// blocks [0, K/256): xt, one thread per k;  blocks [K/256, K/256 + K/128): xb, one thread per (k block, token).
__global__ __launch_bounds__(256) void relayout_x_kernel(const uint16_t *x, int64_t ldx, int M, uint32_t K, int slot)
{
    const uint32_t nb_t = (K + 255) / 256;
    if (blockIdx.x < nb_t) {
        const uint32_t k = blockIdx.x * 256 + threadIdx.x;
        if (k >= K) return;
        uint32_t v[8];
#pragma unroll
        for (int m = 0; m < 16; m += 2) {
            const uint32_t lo = m < M ? x[(size_t)m * ldx + k] : 0u;
            const uint32_t hi = m + 1 < M ? x[(size_t)(m + 1) * ldx + k] : 0u;
            v[m / 2] = lo | (hi << 16);
        }
        uint4 *o = reinterpret_cast<uint4 *>(&g_x[slot].xt[(size_t)k * kTile]);
        o[0] = make_uint4(v[0], v[1], v[2], v[3]);
        o[1] = make_uint4(v[4], v[5], v[6], v[7]);
    } else {
        const uint32_t id = (blockIdx.x - nb_t) * 256 + threadIdx.x;      // = k block * 16 + token
        const uint32_t kb = id >> 4, m = id & 15;
        if (kb * 8 >= K) return;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if ((int)m < M) v = *reinterpret_cast<const uint4 *>(x + (size_t)m * ldx + (size_t)kb * 8);
        reinterpret_cast<uint4 *>(g_x[slot].xb)[id] = v;
    }
}

}  // namespace

// V2 at every bit width; V2a at 3 and 4 bits when the library's pair tables fit the 64 KB table region.
bool batch_supports(int bits, int mode, uint32_t L, uint32_t N, uint32_t K, int M)
{
    const bool format = mode == 0 ? bits >= 2 && bits <= 4
                                  : mode == 1 && (bits == 3 || bits == 4) && L >= 1 && ((size_t)L << (2 * bits)) * 4 <= 64 * 1024;
    if (!(format && M >= 2 && K % kGroup == 0 && K >= kGroup && K <= (uint32_t)kXtMaxK))
        return false;
    if (K <= 8192) return true;
    const uint32_t GS = (uint32_t)batch_split_nl(K) * 8;
    const uint32_t S = (K / kGroup + GS - 1) / GS;
    return (uint64_t)S * 16u * N <= scratch_plane_floats();          // the partial planes of 16 tokens fit
}

bool batch_is_split(uint32_t K) { return batch_split_nl(K) != 0; }

// M <= 16 tokens per launch; the caller loops over chunks of 16.  part: an fp32
// scratch plane when batch_is_split(a.K) (calls on one stream may share it).
hipError_t launch_decode_batch(int bits, int mode, const DecodeArgs &a, int M, bool y_f32, float *part, hipStream_t s)
{
    static std::atomic<void *> ring[kMaxDevices];          // device address of g_x, per device (each holds its own copy)
    const int dev = current_device();
    if (dev < 0) return hipErrorInvalidDevice;
    void *p = ring[dev].load(std::memory_order_relaxed);
    if (!p) {
        hipError_t err = hipGetSymbolAddress(&p, HIP_SYMBOL(g_x));
        if (err != hipSuccess) return err;
        ring[dev].store(p, std::memory_order_relaxed);
    }
    static std::atomic<unsigned> next_slot{0};
    const int xs = (int)(next_slot.fetch_add(1, std::memory_order_relaxed) % kXtSlots);
    hipLaunchKernelGGL(relayout_x_kernel, dim3((a.K + 255) / 256 + (a.K * 2 + 255) / 256), dim3(256), 0, s, a.x,
                       a.x_stride, M, a.K, xs);
    const XCopies *xc = static_cast<const XCopies *>(p) + xs;
    if (mode == 1) {
        if (bits == 4) return launch_batch_lib4(a, M, y_f32, part, xc->xt, xc->xb, s);
        return launch_batch_lib3(a, M, y_f32, part, xc->xt, xc->xb, s);
    }
    if (bits == 4) return launch_batch_bits<4>(a, M, y_f32, part, xc->xt, xc->xb, s);
    if (bits == 3) return launch_batch3(a, M, y_f32, part, xc->xt, xc->xb, s);
    return launch_batch2(a, M, y_f32, part, xc->xt, xc->xb, s);
}

}  // namespace xfp
