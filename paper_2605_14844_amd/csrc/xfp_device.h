// Device-side building blocks for the gfx950 decode kernels: index-stream
// loads, b-bit field extraction, fp16 pair math and wave64 reductions.
#pragma once
#include "xfp_internal.h"

namespace xfp {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

// One lane's share of the index stream: 32 consecutive b-bit fields = BITS dwords.
template <int BITS>
struct LaneWords {
    uint32_t w[BITS];
};

// The index stream is read exactly once: the loads carry the non-temporal hint
// so that the stream does not displace the activations and codebooks in L2.
template <int BITS>
__device__ __forceinline__ LaneWords<BITS> load_lane_words(const uint32_t *p)
{
    LaneWords<BITS> r;
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    if constexpr (BITS == 4) {
        u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
        r.w[0] = v.x; r.w[1] = v.y; r.w[2] = v.z; r.w[3] = v.w;
    } else if constexpr (BITS == 2) {
        u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(p));
        r.w[0] = v.x; r.w[1] = v.y;
    } else {
#pragma unroll
        for (int i = 0; i < BITS; ++i) r.w[i] = __builtin_nontemporal_load(p + i);
    }
    return r;
}

// Field F (0..31) of a lane's words: bits [F*BITS, F*BITS + BITS) of the
// little-endian stream.  Fields that cross a dword boundary (3-bit only) are
// taken from the 64-bit window with a funnel shift.
template <int BITS, int F>
__device__ __forceinline__ uint32_t field(const LaneWords<BITS> &lw)
{
    constexpr int bit = F * BITS;
    constexpr int word = bit / 32;
    constexpr int sh = bit % 32;
    constexpr uint32_t mask = (1u << BITS) - 1u;
    if constexpr (sh + BITS <= 32) {
        return (lw.w[word] >> sh) & mask;
    } else {
        return __builtin_amdgcn_alignbit(lw.w[word + 1], lw.w[word], sh) & mask;
    }
}

__device__ __forceinline__ float dot2(half2_t a, half2_t b, float acc)
{
    return __builtin_amdgcn_fdot2(a, b, acc, false);   // v_dot2_f32_f16: fp32 accumulate
}

__device__ __forceinline__ half2_t as_half2(uint32_t u) { return __builtin_bit_cast(half2_t, u); }
__device__ __forceinline__ float half_bits_to_float(uint16_t h)
{
    return (float)__builtin_bit_cast(_Float16, h);
}

// bf16 activations (paper section 5: the kernel takes bf16).  A bf16 value is exact
// in fp32; the rounding to fp16 (nearest even) is exact inside fp16's normal
// range, rounds to a multiple of 2^-24 below 2^-14 and saturates at +-65504 (an
// activation that large would otherwise become an infinity and poison every
// output); NaN stays NaN.  Every kernel converts with these two functions, so a
// call with bf16 x gives bit for bit what the same call gives on the converted x.
__device__ __forceinline__ _Float16 bf16_bits_to_half(uint32_t b)      // b: bf16 pattern in the low 16 bits
{
    float f = __builtin_bit_cast(float, b << 16);
    f = f != f ? f : fminf(fmaxf(f, -65504.f), 65504.f);
    return (_Float16)f;
}
__device__ __forceinline__ uint32_t bf16x2_to_f16x2(uint32_t w)
{
    float lo = __builtin_bit_cast(float, w << 16), hi = __builtin_bit_cast(float, w & 0xFFFF0000u);
    lo = lo != lo ? lo : fminf(fmaxf(lo, -65504.f), 65504.f);
    hi = hi != hi ? hi : fminf(fmaxf(hi, -65504.f), 65504.f);
    const _Float16 l16 = (_Float16)lo, h16 = (_Float16)hi;
    return (uint32_t)__builtin_bit_cast(uint16_t, l16) | ((uint32_t)__builtin_bit_cast(uint16_t, h16) << 16);
}
// one activation as fp32, from its fp16 or bf16 pattern.  Both readings are
// computed and one is picked bit-wise: as a branch, this handful of instructions
// cost the streaming kernel 35 registers (and with them a wave per SIMD).
__device__ __forceinline__ float x_bits_to_float(uint16_t h, bool bf16)
{
    const uint32_t a = __builtin_bit_cast(uint32_t, (float)__builtin_bit_cast(_Float16, h));
    const uint32_t b = __builtin_bit_cast(uint32_t, (float)bf16_bits_to_half(h));
    const uint32_t m = bf16 ? 0xFFFFFFFFu : 0u;
    return __builtin_bit_cast(float, (b & m) | (a & ~m));
}

template <int CTRL>
__device__ __forceinline__ float dpp_add(float v)
{
    int t = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true);
    return v + __builtin_bit_cast(float, t);
}

// Sum over the 64 lanes in a fixed order (deterministic); every lane gets it.
__device__ __forceinline__ float wave_sum(float v)
{
    v = dpp_add<0xB1>(v);    // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);    // quad_perm [2,3,0,1]
    v = dpp_add<0x141>(v);   // row_half_mirror: other quad of the 8
    v = dpp_add<0x140>(v);   // row_mirror: other half of the 16
    int b = __builtin_bit_cast(int, v);
    float s0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0));
    float s1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16));
    float s2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32));
    float s3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48));
    return (s0 + s1) + (s2 + s3);
}

// Sum over aligned segments of SEG lanes (SEG = 4, 8, 16, 32, 64); every lane
// of a segment gets its segment's sum.
template <int SEG>
__device__ __forceinline__ float segment_sum(float v)
{
    if constexpr (SEG == 64) return wave_sum(v);
    v = dpp_add<0xB1>(v);
    v = dpp_add<0x4E>(v);
    if constexpr (SEG >= 8) v = dpp_add<0x141>(v);
    if constexpr (SEG >= 16) v = dpp_add<0x140>(v);
    if constexpr (SEG == 32) {
        int b = __builtin_bit_cast(int, v);
        float s0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0));
        float s1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16));
        float s2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32));
        float s3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48));
        v = (threadIdx.x & 32) ? (s2 + s3) : (s0 + s1);
    }
    return v;
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits
// for every outstanding global load, which would drain the index prefetch.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Exchange a register-index bit with lane-index bit 0 (HIGH = 0, quad_perm
// [1,0,3,2]) or bit 1 (HIGH = 1, quad_perm [2,3,0,1]) for two register pairs
// (x0, y0) and (x1, y1): afterwards x holds, in the lanes whose bit is set, what
// y held in the partner lane, and y holds, in the lanes whose bit is clear, what
// x held in the partner lane.  One v_cndmask_b32 with a DPP source per output;
// the two scalar moves in front also cover the wait states a DPP read needs
// after a vector write.
#define XFP_EXCHANGE_ASM(QP, MASK)                                                                   \
    asm volatile("s_nop 1\n\t"                                                                       \
                 "s_mov_b32 vcc_lo, " MASK "\n\ts_mov_b32 vcc_hi, " MASK "\n\t"                        \
                 "v_cndmask_b32_dpp %0, %5, %4, vcc quad_perm:" QP " row_mask:0xf bank_mask:0xf\n\t" \
                 "v_cndmask_b32_dpp %2, %7, %6, vcc quad_perm:" QP " row_mask:0xf bank_mask:0xf\n\t" \
                 "s_not_b64 vcc, vcc\n\t"                                                            \
                 "v_cndmask_b32_dpp %1, %4, %5, vcc quad_perm:" QP " row_mask:0xf bank_mask:0xf\n\t" \
                 "v_cndmask_b32_dpp %3, %6, %7, vcc quad_perm:" QP " row_mask:0xf bank_mask:0xf"      \
                 : "=&v"(o0), "=&v"(o1), "=&v"(o2), "=&v"(o3)                                        \
                 : "v"(x0), "v"(y0), "v"(x1), "v"(y1)                                                \
                 : "vcc", "scc")
template <int HIGH>
__device__ __forceinline__ void lane_reg_exchange(uint32_t &x0, uint32_t &y0, uint32_t &x1, uint32_t &y1)
{
    uint32_t o0, o1, o2, o3;
    if constexpr (HIGH) XFP_EXCHANGE_ASM("[2,3,0,1]", "0x33333333");    // vcc: lanes whose bit 1 is clear
    else XFP_EXCHANGE_ASM("[1,0,3,2]", "0x55555555");                   // vcc: lanes whose bit 0 is clear
    x0 = o0; y0 = o1; x1 = o2; y1 = o3;
}

// Index words from the coalesced load layout to the MFMA A-operand layout (matrix-core kernels).
// Before: lane l = 4a + b holds pieces d = 0..3 (v[d], 8 weights each) of chunk b of tile row a (a tile
// is 16 rows, a chunk 32 weights).  Afterwards lane (i, q) = i + 16 q holds, in v[b], piece q of chunk b
// of tile row 4 (i % 4) + i / 4.
__device__ __forceinline__ void to_operand_layout(uint32_t (&v)[4])
{
    // lane bit 5 <-> register bit 1, lane bit 4 <-> register bit 0
    auto s02 = __builtin_amdgcn_permlane32_swap(v[0], v[2], false, false);
    auto s13 = __builtin_amdgcn_permlane32_swap(v[1], v[3], false, false);
    auto s01 = __builtin_amdgcn_permlane16_swap(s02[0], s13[0], false, false);
    auto s23 = __builtin_amdgcn_permlane16_swap(s02[1], s13[1], false, false);
    v[0] = s01[0]; v[1] = s01[1]; v[2] = s23[0]; v[3] = s23[1];
    // lane bit 1 <-> register bit 1, lane bit 0 <-> register bit 0
    lane_reg_exchange<1>(v[0], v[2], v[1], v[3]);
    lane_reg_exchange<0>(v[0], v[1], v[2], v[3]);
}

// fp32 -> bf16 bit pattern, round to nearest even, NaN stays NaN
__device__ __forceinline__ uint16_t float_to_bf16_bits(float v)
{
    uint32_t u = __builtin_bit_cast(uint32_t, v);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// One output element: fp32 as it is, else one rounding (to nearest even) to fp16 or bf16.
__device__ __forceinline__ void store_out(void *y, int64_t i, float v, bool f32, bool bf16)
{
    if (f32) static_cast<float *>(y)[i] = v;
    else if (bf16) static_cast<uint16_t *>(y)[i] = float_to_bf16_bits(v);
    else static_cast<_Float16 *>(y)[i] = (_Float16)v;
}

template <bool YF32>
__device__ __forceinline__ void store_y(void *y, int64_t i, float v, bool bf16)
{
    store_out(y, i, v, YF32, bf16);
}

}  // namespace xfp
