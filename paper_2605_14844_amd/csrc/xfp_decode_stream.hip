// Streaming fused decode, plain variant, plus what the variants share on the
// host side: shape support, split-K launch and its sum kernel, the unfused
// SiLU(gate) * up kernel.  The kernel itself is in
// xfp_decode_stream.inc.h.
#include "xfp_decode_stream.inc.h"

namespace xfp {

// defined in xfp_decode_stream_split.hip / xfp_decode_stream_fused.hip / xfp_decode_stream_affine.hip
hipError_t launch_stream_affine(int bits, bool y_f32, const DecodeArgs &a, int slots, hipStream_t s);
hipError_t launch_stream_split(int bits, int mode, bool y_f32, const DecodeArgs &a, int slots, hipStream_t s);
hipError_t launch_stream_fused(int bits, int mode, bool y_f32, const DecodeArgs &a, int slots, hipStream_t s);

// V2a needs the library's pair tables in LDS: (L + 1) tables of 64 B / 256 B / 1 KB.  mode: 0 V2, 1 V2a, 2 V2a with a
// scale and a mid-point per group (plain variant only).
bool stream_supports(int bits, int mode, uint32_t K, uint32_t L)
{
    if (bits < 2 || bits > 4 || K > 8 * 2048) return false;
    if (mode == 0) return true;
    return (mode == 1 || mode == 2) && (size_t)(L + 1) * (4u << (2 * bits)) <= 64 * 1024;
}

hipError_t launch_decode_stream(int bits, int mode, bool y_f32, const DecodeArgs &a, int slots, hipStream_t s)
{
    if (mode == 2) return launch_stream_affine(bits, y_f32, a, slots, s);
    if (a.fuse_half) return launch_stream_fused(bits, mode, y_f32, a, slots, s);
    if (a.k_slices) return launch_stream_split(bits, mode, y_f32, a, slots, s);
    return launch_stream_variant<0>(bits, mode, y_f32, a, slots, s);
}

// ---------------------------------------------------------------- split-K
// Rows longer than the streaming kernel holds in registers (K > 16384) are cut
// into S equal slices (S divides K / 128, a slice is at most 8192 columns so
// that four waves fit a SIMD); grid z = slice.  Slice z writes fp32 partial sums
// to its own part of the call's scratch plane and a second kernel adds the parts
// in slice order: deterministic, no atomics.
__global__ __launch_bounds__(256) void splitk_sum_kernel(const float *part, uint32_t S, uint32_t N, uint32_t slots,
                                                         void *y, int64_t y_stride, int y_f32, int y_bf16)
{
    const uint32_t n = blockIdx.x * 256 + threadIdx.x, slot = blockIdx.y;
    if (n >= N) return;
    const size_t plane = (size_t)slots * N;
    float s = part[(size_t)slot * N + n];
    for (uint32_t z = 1; z < S; ++z) s += part[z * plane + (size_t)slot * N + n];
    const int64_t o = (int64_t)slot * y_stride + n;
    store_out(y, o, s, y_f32 != 0, y_bf16 != 0);
}

int splitk_slices(int bits, int mode, uint32_t N, uint32_t K, uint32_t L, int slots, uint64_t plane_cap)
{
    const uint32_t G = K / kGroup;
    for (uint32_t S = (K + 8191) / 8192; S <= 16; ++S) {
        if (G % S != 0) continue;
        if (!stream_supports(bits, mode, K / S, L)) return 0;
        if ((uint64_t)S * (uint64_t)slots * N > plane_cap) return 0;
        return (int)S;
    }
    return 0;
}

// part: an fp32 scratch plane of kPlaneFloats floats (S * slots * N of them are used)
hipError_t launch_decode_splitk(int bits, int mode, bool y_f32, const DecodeArgs &a, int slots, int slices,
                                float *part, hipStream_t s)
{
    if (!part) return hipErrorInvalidValue;
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
    return launch_splitk_sum(part, (uint32_t)slices, a.N, slots, a.y, a.y_stride, y_f32, a.y_bf16 != 0, s);
}

hipError_t launch_splitk_sum(const float *part, uint32_t slices, uint32_t N, int slots, void *y, int64_t y_stride,
                             bool y_f32, bool y_bf16, hipStream_t s)
{
    hipLaunchKernelGGL(splitk_sum_kernel, dim3((N + 255) / 256, slots), dim3(256), 0, s, part, slices, N,
                       (uint32_t)slots, y, y_stride, (int)y_f32, (int)y_bf16);
    return hipGetLastError();
}

// h[t][j] = SiLU(y[t][j]) * y[t][half + j] from fp32 sums (the unfused form of
// the streaming kernel's gate/up epilogue, for shapes that kernel does not take).
__global__ __launch_bounds__(256) void silu_mul_kernel(const float *y, uint32_t half, uint32_t slots, void *h,
                                                       int64_t h_stride, int h_f32, int h_bf16)
{
    const uint32_t j = blockIdx.x * 256 + threadIdx.x, slot = blockIdx.y;
    if (j >= half) return;
    const float g = y[(size_t)slot * 2 * half + j], up = y[(size_t)slot * 2 * half + half + j];
    const float v = g / (1.0f + __expf(-g)) * up;
    const int64_t o = (int64_t)slot * h_stride + j;
    store_out(h, o, v, h_f32 != 0, h_bf16 != 0);
}

hipError_t launch_silu_mul(const float *y, uint32_t half, int slots, void *h, int64_t h_stride, bool h_f32,
                           bool h_bf16, hipStream_t s)
{
    hipLaunchKernelGGL(silu_mul_kernel, dim3((half + 255) / 256, slots), dim3(256), 0, s, y, half, (uint32_t)slots, h,
                       h_stride, (int)h_f32, (int)h_bf16);
    return hipGetLastError();
}

// bf16 -> fp16, eight values per thread.  A bf16 value is exact in fp32; the
// rounding to fp16 is exact inside fp16's normal range, rounds to a multiple of
// 2^-24 below 2^-14 and saturates at +-65504 (an activation that large would
// otherwise become an infinity and poison every output).
__global__ __launch_bounds__(256) void bf16_to_f16_kernel(const uint16_t *src, int64_t ld, uint16_t *dst, uint32_t rows,
                                                          uint32_t K)
{
    const uint32_t c8 = blockIdx.x * 256 + threadIdx.x, row = blockIdx.y;
    if (c8 * 8 >= K) return;
    const uint4 v = *reinterpret_cast<const uint4 *>(src + (size_t)row * ld + (size_t)c8 * 8);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    uint32_t o[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float lo = __builtin_bit_cast(float, w[i] << 16), hi = __builtin_bit_cast(float, w[i] & 0xFFFF0000u);
        lo = lo != lo ? lo : fminf(fmaxf(lo, -65504.f), 65504.f);      // NaN stays NaN
        hi = hi != hi ? hi : fminf(fmaxf(hi, -65504.f), 65504.f);
        const _Float16 l16 = (_Float16)lo, h16 = (_Float16)hi;
        o[i] = (uint32_t)__builtin_bit_cast(uint16_t, l16) | ((uint32_t)__builtin_bit_cast(uint16_t, h16) << 16);
    }
    *reinterpret_cast<uint4 *>(dst + (size_t)row * K + (size_t)c8 * 8) = make_uint4(o[0], o[1], o[2], o[3]);
}

hipError_t launch_bf16_to_f16(const void *src, int64_t ld, void *dst, uint32_t rows, uint32_t K, hipStream_t s)
{
    hipLaunchKernelGGL(bf16_to_f16_kernel, dim3((K / 8 + 255) / 256, rows), dim3(256), 0, s,
                       static_cast<const uint16_t *>(src), ld, static_cast<uint16_t *>(dst), rows, K);
    return hipGetLastError();
}

// y[n] = sum over slots t, in slot order, of w[t] * part[t][n] (fp32): the combine
// step of a routed-expert layer, for the shapes no fused kernel takes.
__global__ __launch_bounds__(256) void moe_combine_kernel(const float *part, const float *w, uint32_t N, uint32_t slots,
                                                          void *y, int y_f32, int y_bf16)
{
    const uint32_t n = blockIdx.x * 256 + threadIdx.x;
    if (n >= N) return;
    float s = 0.f;
    for (uint32_t t = 0; t < slots; ++t) s = fmaf(w[t], part[(size_t)t * N + n], s);
    store_out(y, n, s, y_f32 != 0, y_bf16 != 0);
}

hipError_t launch_moe_combine(const float *part, const float *w, uint32_t N, int slots, void *y, bool y_f32,
                              bool y_bf16, hipStream_t s)
{
    hipLaunchKernelGGL(moe_combine_kernel, dim3((N + 255) / 256), dim3(256), 0, s, part, w, N, (uint32_t)slots, y,
                       (int)y_f32, (int)y_bf16);
    return hipGetLastError();
}

}  // namespace xfp
