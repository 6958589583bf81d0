// Internal declarations shared by the host dispatcher and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace xfp {

constexpr int kGroup = 128;
constexpr int kWave = 64;
constexpr int kMaxDevices = 64;   // GPUs of one process whose static scratch addresses are remembered
constexpr int kLaneWeights = 32;   // weights one lane decodes per index load (all bit widths)

// Everything a decode kernel needs, passed by value.  gridDim.y enumerates
// "slots": tokens of a batched call (eids == nullptr) or MoE slots.
struct DecodeArgs {
    const uint32_t *idx;   // [E][N][K*bits/32]
    const uint16_t *cb;    // V2 [E][N][2^b]   V2a [E][L][2^b]
    const uint8_t *gid;    // V2a [E][N][K/128]
    const int32_t *rp;     // [E*N+1]
    const int32_t *col;
    const uint16_t *val;
    const uint16_t *x;     // slot s reads x + s * x_stride
    void *y;               // slot s writes y + s * y_stride (elements of the y dtype)
    const int32_t *eids;   // device [slots] or nullptr (matrix 0 for every slot)
    int64_t x_stride;
    int64_t y_stride;
    uint32_t N, K, L;
    uint32_t rows_per_block;
    // Split-K launches of the streaming kernel (zero otherwise): K above is then the
    // length of one slice, workgroup z decodes columns [z K, (z + 1) K) of every row.
    uint32_t k_slices;     // slices (grid z)
    uint32_t row_words;    // dwords of a full index row
    uint32_t gid_row;      // library ids of a full row
    int64_t z_stride;      // slice z writes y + z * z_stride (fp32 partial sums)
    // Fused SiLU(gate) * up (zero otherwise): rows [0, fuse_half) are gate rows, rows
    // [fuse_half, 2 fuse_half) up rows; y gets fuse_half values per slot.
    uint32_t fuse_half;
    uint32_t y_bf16;       // the 16-bit output type is bf16 instead of fp16
    uint32_t x_bf16;       // x holds bf16 values; every kernel converts them to fp16 as it loads them
    const uint16_t *gscale;   // V2a with a scale and a mid-point per group (general kernel only): fp16 [E][N][K/128]
    const uint16_t *gmid;
};

// Device memory a call may need beyond its inputs and outputs.  One call gets ONE
// workspace and carves every plane it needs out of it, so a call never holds
// more than one unit of whatever the workspaces come from (a ring slot, or the
// static array of the entry point that allocates nothing).
constexpr uint32_t kPlaneFloats = 1u << 20;        // floats of an fp32 scratch plane (4 MB)
constexpr int kXtMaxK = 32768;                     // longest row the batched kernel takes
constexpr int kXtTokens = 16;                      // tokens per launch of the batched kernel
// Two re-laid copies of the activations of a batched launch (16 tokens x K <= 32768, or up to 64 tokens with
// 16 ceil(M / 16) K <= 16 * 32768 for the wide kernel, whose copies are [k][16 T tokens] and [T][k / 8][16][8]):
//   xt [k][16 tokens]           the outlier products read the 16 tokens of one column as 32 bytes;
//   xb [k / 8][16 tokens][8 k]  the B operand of lane (m, q) for a k block is 16 contiguous bytes and
//                               the 64 lanes of a wave read 1 KB contiguous (from the row-major x the
//                               same load touches 64 different cache lines).
// Tokens >= M are zero in both.
struct XCopies {
    uint16_t xt[kXtMaxK * kXtTokens];
    uint16_t xb[kXtMaxK * kXtTokens];
};
struct WorkspaceLayout {
    XCopies xc;                  // batched kernel: re-laid activations (2 MB)
    float epi[kPlaneFloats];     // unfused epilogues: per-slot fp32 results
    float part[kPlaneFloats];    // split-K: per-slice fp32 partial sums
};
struct Workspace {
    XCopies *xc;
    float *epi;
    float *part;
};
inline Workspace workspace_at(void *base)
{
    WorkspaceLayout *l = static_cast<WorkspaceLayout *>(base);
    return Workspace{&l->xc, l->epi, l->part};
}
// One slot of the static ring of workspaces on the current device.  Calls on a
// stream that is being captured into a graph cycle through slots of their own,
// which eager calls never take.
hipError_t ring_workspace(hipStream_t s, Workspace *out);
// Resolves the ring's address on the current device (no-op once done).
hipError_t ring_resolve();
// Pure slot arithmetic of the ring (exposed for a host-only test): ticket-th call
// of its kind -> slot index.
int ring_slot_index(unsigned ticket, bool capturing);
int ring_slots(bool capturing);

// Index of the current device for per-device host-side state, or -1.
inline int current_device()
{
    int d = 0;
    return hipGetDevice(&d) == hipSuccess && d >= 0 && d < kMaxDevices ? d : -1;
}

// Launchers, one per kernel family (defined in the .hip files).
hipError_t launch_decode_rows(int bits, int mode, bool y_f32, const DecodeArgs &a, int slots,
                              hipStream_t s);
// Streaming kernel (K <= 16384; V2, or V2a whose library tables fit in LDS): x in
// registers, pair tables in LDS.
bool stream_supports(int bits, int mode, uint32_t K, uint32_t L);
hipError_t launch_decode_stream(int bits, int mode, bool y_f32, const DecodeArgs &a, int slots, hipStream_t s);
// Tile kernel (V2, 4-bit, M = 1 per slot): rows across lanes, one pair table per lane, conflict-free lookups.
bool tile_supports(int bits, int mode, uint32_t N, uint32_t K, int slots);
hipError_t launch_decode_tile(int bits, bool y_f32, const DecodeArgs &a, int slots, hipStream_t s);
// Split-K form of the streaming kernel for rows longer than it holds in registers:
// S equal slices of K, fp32 partial sums in a file-scope device buffer, summed in
// slice order by a second kernel.  splitk_slices returns S, or 0 if the shape does
// not fit (then the general kernel runs).
// plane_cap: floats of the scratch plane that takes the partial sums (S * slots * N of them).
int splitk_slices(int bits, int mode, uint32_t N, uint32_t K, uint32_t L, int slots, uint64_t plane_cap = kPlaneFloats);
hipError_t launch_decode_splitk(int bits, int mode, bool y_f32, const DecodeArgs &a, int slots, int slices,
                                float *part, hipStream_t s);
// y[slot][n] = sum over slices z, in order, of part[z][slot][n]
hipError_t launch_splitk_sum(const float *part, uint32_t slices, uint32_t N, int slots, void *y, int64_t y_stride,
                             bool y_f32, bool y_bf16, hipStream_t s);
// Matrix-core kernel for 2..16 tokens per launch (V2 and V2a at 2..4 bits
// with a library whose pair tables fit 64 KB of LDS; K <= 32768; rows
// above 8192 columns in slices whose partial sums go through a scratch plane).
bool batch_supports(int bits, int mode, uint32_t L, uint32_t N, uint32_t K, int M, uint64_t k_cap = kXtMaxK,
                    uint64_t plane_cap = kPlaneFloats);
bool batch_is_split(uint32_t K);
hipError_t launch_decode_batch(int bits, int mode, const DecodeArgs &a, int M, bool y_f32, float *part, XCopies *xc,
                               hipStream_t s);
// Wide matrix-core kernel: up to 64 tokens in ONE pass over the weights (V2 and V2a at 2..4 bits, a V2a library's
// pair tables within 64 KB; mode 2 = V2a with a scale and a mid-point per group, 16 tokens per launch, sx = 16 K / 128
// floats of scratch; the re-laid copies of 16 ceil(M / 16) x K activations must fit copy_cap halves each).
bool wide_supports(int bits, int mode, uint32_t L, uint32_t N, uint32_t K, int M,
                   uint64_t copy_cap = (uint64_t)kXtMaxK * kXtTokens);
hipError_t launch_decode_wide(int bits, int mode, const DecodeArgs &a, int M, bool y_f32, XCopies *xc, float *sx,
                              hipStream_t s);
hipError_t launch_silu_mul(const float *y, uint32_t half, int slots, void *h, int64_t h_stride, bool h_f32,
                           bool h_bf16, hipStream_t s);
// Down projection with the router's weighted sum over the slots in one launch (V2, T <= 8, T * K <= 16384)
bool combine_supports(int bits, int mode, uint32_t K, int T);
hipError_t launch_decode_combine(int bits, const DecodeArgs &d, int T, const float *w, bool y_f32, bool y_bf16,
                                 hipStream_t s);
hipError_t launch_moe_combine(const float *part, const float *w, uint32_t N, int slots, void *y, bool y_f32,
                              bool y_bf16, hipStream_t s);
// bf16 [rows][ld] -> fp16 [rows][K] (exact inside fp16's normal range, saturating beyond it);
// the stand-alone form of the conversion every decode kernel applies when x_bf16 is set
hipError_t launch_bf16_to_f16(const void *src, int64_t ld, void *dst, uint32_t rows, uint32_t K, hipStream_t s);
// indices in a word form of the packing table [rows][ceil(K/per)] -> dense stream [rows][K*bits/32]
hipError_t launch_repack_words(const void *src, uint64_t rows, uint32_t K, int bits, uint32_t *dst, hipStream_t s);
hipError_t launch_unpack(int bits, const uint32_t *idx, uint64_t rows, uint32_t K, uint8_t *out,
                         hipStream_t s);
hipError_t launch_dequant(int bits, int mode, const DecodeArgs &a, uint32_t E, uint16_t *out,
                          hipStream_t s);
hipError_t launch_check_contents(const DecodeArgs &a, uint32_t E, uint64_t nnz_capacity, const int32_t *eids, int T,
                                 uint32_t *report, hipStream_t s);
hipError_t launch_probe_read(const void *src, uint64_t bytes, uint32_t *sink, hipStream_t s);
hipError_t launch_probe_copy(const void *src, void *dst, uint64_t bytes, hipStream_t s);

}  // namespace xfp
