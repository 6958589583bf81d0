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
// defined in xfp_decode_batch_lib2.hip, xfp_decode_batch_lib3.hip, xfp_decode_batch_lib4.hip
hipError_t launch_batch_lib2(const DecodeArgs &a, int M, bool y_f32, float *part, const void *xt, const void *xb,
                             hipStream_t s);
hipError_t launch_batch_lib3(const DecodeArgs &a, int M, bool y_f32, float *part, const void *xt, const void *xb,
                             hipStream_t s);
hipError_t launch_batch_lib4(const DecodeArgs &a, int M, bool y_f32, float *part, const void *xt, const void *xb,
                             hipStream_t s);

namespace {

static_assert(kXtTokens == kTile, "the re-laid copies hold one launch's tokens");

// blocks [0, K/256): xt, one thread per k;  blocks [K/256, K/256 + K/128): xb, one thread per (k block, token).
// bf16 activations are converted to fp16 on the way (bf16: x holds bf16 patterns).
__global__ __launch_bounds__(256) void relayout_x_kernel(const uint16_t *x, int64_t ldx, int M, uint32_t K, int bf16,
                                                         XCopies *xc)
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
            if (bf16) v[m / 2] = bf16x2_to_f16x2(v[m / 2]);
        }
        uint4 *o = reinterpret_cast<uint4 *>(&xc->xt[(size_t)k * kTile]);
        o[0] = make_uint4(v[0], v[1], v[2], v[3]);
        o[1] = make_uint4(v[4], v[5], v[6], v[7]);
    } else {
        const uint32_t id = (blockIdx.x - nb_t) * 256 + threadIdx.x;      // = k block * 16 + token
        const uint32_t kb = id >> 4, m = id & 15;
        if (kb * 8 >= K) return;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if ((int)m < M) v = *reinterpret_cast<const uint4 *>(x + (size_t)m * ldx + (size_t)kb * 8);
        if (bf16) v = make_uint4(bf16x2_to_f16x2(v.x), bf16x2_to_f16x2(v.y), bf16x2_to_f16x2(v.z), bf16x2_to_f16x2(v.w));
        reinterpret_cast<uint4 *>(xc->xb)[id] = v;
    }
}

}  // namespace

// V2 and V2a at 2, 3 and 4 bits; V2a when the library's pair tables fit the 64 KB table region.
// k_cap, plane_cap: what the workspace holds (columns of the re-laid copies, floats of a partial-sum plane).
bool batch_supports(int bits, int mode, uint32_t L, uint32_t N, uint32_t K, int M, uint64_t k_cap, uint64_t plane_cap)
{
    const bool format = mode == 0 ? bits >= 2 && bits <= 4
                                  : mode == 1 && bits >= 2 && bits <= 4 && L >= 1 && ((size_t)L << (2 * bits)) * 4 <= 64 * 1024;
    if (!(format && M >= 2 && K % kGroup == 0 && K >= kGroup && K <= k_cap))
        return false;
    if (K <= 8192) return true;
    const uint32_t GS = (uint32_t)batch_split_nl(K) * 8;
    const uint32_t S = (K / kGroup + GS - 1) / GS;
    return (uint64_t)S * 16u * N <= plane_cap;                       // the partial planes of 16 tokens fit
}

bool batch_is_split(uint32_t K) { return batch_split_nl(K) != 0; }

// M <= 16 tokens per launch; the caller loops over chunks of 16.  xc: the workspace's
// re-laid activation copies, written by a small kernel in front of the decode kernel
// (launches on one stream may share them).  part: an fp32 scratch plane when
// batch_is_split(a.K).
hipError_t launch_decode_batch(int bits, int mode, const DecodeArgs &a, int M, bool y_f32, float *part, XCopies *xc,
                               hipStream_t s)
{
    if (!xc) return hipErrorInvalidValue;
    hipLaunchKernelGGL(relayout_x_kernel, dim3((a.K + 255) / 256 + (a.K * 2 + 255) / 256), dim3(256), 0, s, a.x,
                       a.x_stride, M, a.K, (int)a.x_bf16, xc);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    if (mode == 1) {
        if (bits == 4) return launch_batch_lib4(a, M, y_f32, part, xc->xt, xc->xb, s);
        if (bits == 2) return launch_batch_lib2(a, M, y_f32, part, xc->xt, xc->xb, s);
        return launch_batch_lib3(a, M, y_f32, part, xc->xt, xc->xb, s);
    }
    if (bits == 4) return launch_batch_bits<4>(a, M, y_f32, part, xc->xt, xc->xb, s);
    if (bits == 3) return launch_batch3(a, M, y_f32, part, xc->xt, xc->xb, s);
    return launch_batch2(a, M, y_f32, part, xc->xt, xc->xb, s);
}

}  // namespace xfp
