// Streaming fused decode, plain variant, plus what the variants share on the
// host side: shape support, split-K launch and its sum kernel, the fp32 scratch
// ring, the unfused SiLU(gate) * up kernel.  The kernel itself is in
// xfp_decode_stream.inc.h.
#include "xfp_decode_stream.inc.h"

#include <atomic>

namespace xfp {

// defined in xfp_decode_stream_split.hip / xfp_decode_stream_fused.hip
hipError_t launch_stream_split(int bits, int mode, bool y_f32, const DecodeArgs &a, int slots, hipStream_t s);
hipError_t launch_stream_fused(int bits, int mode, bool y_f32, const DecodeArgs &a, int slots, hipStream_t s);

// V2a needs the library's pair tables in LDS: (L + 1) tables of 64 B / 256 B / 1 KB.
bool stream_supports(int bits, int mode, uint32_t K, uint32_t L)
{
    if (bits < 2 || bits > 4 || K > 8 * 2048) return false;
    if (mode == 0) return true;
    return mode == 1 && (size_t)(L + 1) * (4u << (2 * bits)) <= 64 * 1024;
}

hipError_t launch_decode_stream(int bits, int mode, bool y_f32, const DecodeArgs &a, int slots, hipStream_t s)
{
    if (a.fuse_half) return launch_stream_fused(bits, mode, y_f32, a, slots, s);
    if (a.k_slices) return launch_stream_split(bits, mode, y_f32, a, slots, s);
    return launch_stream_variant<0>(bits, mode, y_f32, a, slots, s);
}

// ---------------------------------------------------------------- split-K
// Rows longer than the streaming kernel holds in registers (K > 16384) are cut
// into S equal slices (S divides K / 128, a slice is at most 8192 columns so
// that four waves fit a SIMD); grid z = slice.  Slice z writes fp32 partial sums
// to its own plane of a file-scope buffer and a second kernel adds the planes in
// slice order: deterministic, no atomics.  A ring of kSplitSlots buffers lets
// that many split-K calls overlap on one GPU before a slot is reused.
constexpr uint32_t kSplitFloats = 1u << 20;            // S * slots * N per call (4 MB per ring slot)
constexpr int kSplitSlots = 4;
__device__ __align__(256) float g_partial[kSplitSlots][kSplitFloats];

__global__ __launch_bounds__(256) void splitk_sum_kernel(const float *part, uint32_t S, uint32_t N, uint32_t slots,
                                                         void *y, int64_t y_stride, int y_f32)
{
    const uint32_t n = blockIdx.x * 256 + threadIdx.x, slot = blockIdx.y;
    if (n >= N) return;
    const size_t plane = (size_t)slots * N;
    float s = part[(size_t)slot * N + n];
    for (uint32_t z = 1; z < S; ++z) s += part[z * plane + (size_t)slot * N + n];
    const int64_t o = (int64_t)slot * y_stride + n;
    if (y_f32) static_cast<float *>(y)[o] = s;
    else static_cast<_Float16 *>(y)[o] = (_Float16)s;
}

int splitk_slices(int bits, int mode, uint32_t N, uint32_t K, uint32_t L, int slots)
{
    const uint32_t G = K / kGroup;
    for (uint32_t S = (K + 8191) / 8192; S <= 16; ++S) {
        if (G % S != 0) continue;
        if (!stream_supports(bits, mode, K / S, L)) return 0;
        if ((uint64_t)S * (uint64_t)slots * N > kSplitFloats) return 0;
        return (int)S;
    }
    return 0;
}

// One slot of the ring of fp32 scratch planes (kSplitFloats floats each), or
// nullptr with *err set.
float *scratch_plane(hipError_t *err)
{
    static std::atomic<void *> ring{nullptr};          // device address of g_partial (one GPU per process)
    void *p = ring.load(std::memory_order_relaxed);
    if (!p) {
        *err = hipGetSymbolAddress(&p, HIP_SYMBOL(g_partial));
        if (*err != hipSuccess) return nullptr;
        ring.store(p, std::memory_order_relaxed);
    }
    static std::atomic<unsigned> next_slot{0};
    return static_cast<float *>(p) + (size_t)(next_slot.fetch_add(1, std::memory_order_relaxed) % kSplitSlots) * kSplitFloats;
}

uint32_t scratch_plane_floats() { return kSplitFloats; }

hipError_t launch_decode_splitk(int bits, int mode, bool y_f32, const DecodeArgs &a, int slots, int slices,
                                hipStream_t s)
{
    hipError_t perr = hipSuccess;
    float *part = scratch_plane(&perr);
    if (!part) return perr;
    DecodeArgs c = a;
    c.k_slices = (uint32_t)slices;
    c.row_words = a.K / 32 * (uint32_t)bits;
    c.gid_row = a.K / kGroup;
    c.K = a.K / (uint32_t)slices;
    c.y = part;
    c.y_stride = a.N;
    c.z_stride = (int64_t)slots * a.N;
    hipError_t err = launch_decode_stream(bits, mode, true, c, slots, s);
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(splitk_sum_kernel, dim3((a.N + 255) / 256, slots), dim3(256), 0, s, part, (uint32_t)slices, a.N,
                       (uint32_t)slots, a.y, a.y_stride, (int)y_f32);
    return hipGetLastError();
}

// h[t][j] = SiLU(y[t][j]) * y[t][half + j] from fp32 sums (the unfused form of
// the streaming kernel's gate/up epilogue, for shapes that kernel does not take).
__global__ __launch_bounds__(256) void silu_mul_kernel(const float *y, uint32_t half, uint32_t slots, void *h,
                                                       int64_t h_stride, int h_f32)
{
    const uint32_t j = blockIdx.x * 256 + threadIdx.x, slot = blockIdx.y;
    if (j >= half) return;
    const float g = y[(size_t)slot * 2 * half + j], up = y[(size_t)slot * 2 * half + half + j];
    const float v = g / (1.0f + __expf(-g)) * up;
    const int64_t o = (int64_t)slot * h_stride + j;
    if (h_f32) static_cast<float *>(h)[o] = v;
    else static_cast<_Float16 *>(h)[o] = (_Float16)v;
}

hipError_t launch_silu_mul(const float *y, uint32_t half, int slots, void *h, int64_t h_stride, bool h_f32,
                           hipStream_t s)
{
    hipLaunchKernelGGL(silu_mul_kernel, dim3((half + 255) / 256, slots), dim3(256), 0, s, y, half, (uint32_t)slots, h,
                       h_stride, (int)h_f32);
    return hipGetLastError();
}

}  // namespace xfp
