// One-time format conversion at load: indices in the word forms of the paper's
// packing table (section 3.3, table 2: 16 / 10 / 8 / 5 values per uint32 at 2 / 3 /
// 4 / 6 bits, 3 per uint16 at 5 bits; reserve bits on top of a word) -> the dense
// stream the decode kernels read (6.25 % fewer bytes per decode call at 3, 5 and
// 6 bits; a plain copy at 2 and 4, which have no reserve bits).
#include "xfp_internal.h"

namespace xfp {
namespace {

// One thread per destination dword d of a row: bits [32 d, 32 d + 32) of the
// dense stream hold (parts of) values floor(32 d / b) .. floor((32 d + 31) / b).
// Value v comes from source word v / PER, bits [b (v % PER), + b).
template <int BITS, int PER, typename WORD>
__global__ __launch_bounds__(256) void repack_words_kernel(const WORD *src, uint64_t rows, uint32_t K, uint32_t *dst)
{
    const uint32_t dw = K / 32 * BITS, sw = (K + PER - 1) / PER;
    const uint64_t id = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= rows * dw) return;
    const uint64_t r = id / dw;
    const uint32_t d = (uint32_t)(id - r * dw);
    const WORD *s = src + r * sw;
    const int32_t bit0 = 32 * (int32_t)d;
    uint32_t out = 0;
    for (int32_t v = bit0 / BITS; BITS * v < bit0 + 32; ++v) {   // v < K: the last dword ends with value K - 1
        const uint32_t q = ((uint32_t)s[v / PER] >> (BITS * (v % PER))) & ((1u << BITS) - 1u);
        const int32_t sh = BITS * v - bit0;
        out |= sh >= 0 ? q << sh : q >> -sh;
    }
    dst[id] = out;
}

template <int BITS, int PER, typename WORD>
hipError_t launch_t(const void *src, uint64_t rows, uint32_t K, uint32_t *dst, hipStream_t s)
{
    const uint64_t total = rows * (K / 32 * BITS);
    hipLaunchKernelGGL((repack_words_kernel<BITS, PER, WORD>), dim3((uint32_t)((total + 255) / 256)), dim3(256), 0, s,
                       static_cast<const WORD *>(src), rows, K, dst);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_repack_words(const void *src, uint64_t rows, uint32_t K, int bits, uint32_t *dst, hipStream_t s)
{
    switch (bits) {
    case 2: return launch_t<2, 16, uint32_t>(src, rows, K, dst, s);
    case 3: return launch_t<3, 10, uint32_t>(src, rows, K, dst, s);
    case 4: return launch_t<4, 8, uint32_t>(src, rows, K, dst, s);
    case 5: return launch_t<5, 3, uint16_t>(src, rows, K, dst, s);
    case 6: return launch_t<6, 5, uint32_t>(src, rows, K, dst, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace xfp
