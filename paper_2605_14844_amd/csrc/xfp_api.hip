// Host side of the C ABI: argument validation, kernel selection, launch.
// Nothing here allocates, copies or synchronises.
#include "../../include/xfp.h"
#include "xfp_internal.h"

#include <atomic>
#include <cstdio>
#include <cstring>

// The one workspace of xfp_gemv_noalloc: a file-scope device array (each GPU of the
// process holds its own copy at its own address).  Host code never passes the
// array's name to a kernel or a runtime call: it resolves the address once per
// device, with that device current, and uses the resolved pointer.
static __device__ __align__(256) unsigned char scratch[sizeof(xfp::WorkspaceLayout)];
static std::atomic<void *> g_scratch_ptr[xfp::kMaxDevices];

static hipError_t scratch_resolve(void **out)
{
    const int dev = xfp::current_device();
    if (dev < 0) return hipErrorInvalidDevice;
    void *ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        hipError_t err = hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch));
        if (err != hipSuccess) return err;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);
    }
    if (out) *out = ptr;
    return hipSuccess;
}

namespace {

thread_local hipError_t g_last_hip = hipSuccess;
thread_local char g_msg[256];

inline bool misaligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

int check_weights(const xfp_weights *W)
{
    if (!W) return XFP_ERR_NULL;
    if (W->struct_size != sizeof(xfp_weights)) return XFP_ERR_UNSUPPORTED;
    if (W->mode != XFP_MODE_V2 && W->mode != XFP_MODE_V2A) return XFP_ERR_UNSUPPORTED;
    if (W->bits < 2 || W->bits > 6) return XFP_ERR_UNSUPPORTED;
    if (W->group != XFP_GROUP || (W->flags & ~XFP_FLAG_GROUP_AFFINE) != 0 || W->reserved != 0) return XFP_ERR_UNSUPPORTED;
    if ((W->flags & XFP_FLAG_GROUP_AFFINE) && W->mode != XFP_MODE_V2A) return XFP_ERR_UNSUPPORTED;
    if (W->N == 0 || W->K == 0 || W->E == 0) return XFP_ERR_SHAPE;
    if (W->K % XFP_GROUP != 0) return XFP_ERR_SHAPE;
    if ((uint64_t)W->E * W->N > 0x7fffffffull) return XFP_ERR_SHAPE;
    if (W->mode == XFP_MODE_V2A) {
        if (W->L == 0 || W->L > XFP_MAX_LIBRARY) return XFP_ERR_UNSUPPORTED;
        if (!W->group_ids) return XFP_ERR_NULL;
    } else if (W->L != 0) {
        return XFP_ERR_UNSUPPORTED;
    }
    if (W->flags & XFP_FLAG_GROUP_AFFINE) {
        if (!W->group_scale || !W->group_mid) return XFP_ERR_NULL;
        if (misaligned(W->group_scale, 2) || misaligned(W->group_mid, 2)) return XFP_ERR_ALIGN;
    } else if (W->group_scale || W->group_mid) {
        return XFP_ERR_UNSUPPORTED;                            // arrays given but not announced in flags
    }
    if (!W->indices || !W->codebooks || !W->out_row_ptr) return XFP_ERR_NULL;
    if (misaligned(W->indices, 16) || misaligned(W->codebooks, 16) || misaligned(W->out_row_ptr, 4) ||
        misaligned(W->out_col, 4) || misaligned(W->out_val, 2))
        return XFP_ERR_ALIGN;
    return XFP_OK;
}

xfp::DecodeArgs base_args(const xfp_weights *W)
{
    xfp::DecodeArgs a;
    std::memset(&a, 0, sizeof(a));
    a.idx = W->indices;
    a.cb = W->codebooks;
    a.gid = W->group_ids;
    a.rp = W->out_row_ptr;
    a.col = W->out_col;
    a.val = W->out_val;
    a.N = W->N;
    a.K = W->K;
    a.L = W->L;
    a.gscale = W->group_scale;
    a.gmid = W->group_mid;
    return a;
}

int finish(hipError_t err)
{
    if (err == hipSuccess) return XFP_OK;
    g_last_hip = err;
    return XFP_ERR_HIP;
}

// y_dtype argument: an xfp_dtype, optionally OR-ed with XFP_X_BF16
bool dtype_ok(int y_dtype)
{
    return (y_dtype & ~(0xFF | XFP_X_BF16)) == 0 && (y_dtype & 0xFF) <= XFP_BF16;
}

// Where a call's scratch memory comes from: one slot of the static ring, taken
// the first time some path asks for it (most calls never do), or a workspace
// the entry point fixed beforehand.
struct Scratch {
    hipStream_t stream;
    bool have = false;
    xfp::Workspace ws{};
    explicit Scratch(hipStream_t s) : stream(s) {}
    Scratch(hipStream_t s, const xfp::Workspace &fixed) : stream(s), have(true), ws(fixed) {}
    hipError_t get(const xfp::Workspace **out)
    {
        if (!have) {
            hipError_t err = xfp::ring_workspace(stream, &ws);
            if (err != hipSuccess) return err;
            have = true;
        }
        *out = &ws;
        return hipSuccess;
    }
};

// Formats outside the batched, split and fused kernels: 5- and 6-bit indices, a scale and a mid-point per group.
// (The latter has ONE tuned kernel, the plain streaming one: stream_affine below.)
bool general_only(const xfp_weights *W) { return W->bits > 4 || (W->flags & XFP_FLAG_GROUP_AFFINE) != 0; }

// V2a with a scale and a mid-point per group, 2..4 bits, rows the streaming kernel holds: its MODE 2
bool stream_affine(const xfp_weights *W)
{
    return (W->flags & XFP_FLAG_GROUP_AFFINE) != 0 && W->mode == XFP_MODE_V2A && W->bits <= 4 &&
           xfp::stream_supports((int)W->bits, 2, W->K, W->L);
}

// Longest row the general kernel can stage: x (2 K bytes) and its tables share the
// 160 KB of LDS of a compute unit.
bool rows_fits(const xfp_weights *W)
{
    const size_t tables = (W->mode == XFP_MODE_V2A ? (size_t)W->L : 4u) * (2u << W->bits);
    return (size_t)W->K * 2 + tables <= 160 * 1024;
}

// Shapes no kernel takes (checked before anything is launched): rows beyond the
// streaming and split-K kernels that the general kernel cannot stage either.
bool prefer_tile(const xfp_weights *W, int slots);

bool decodable(const xfp_weights *W, int slots)
{
    const int bits = (int)W->bits, mode = (int)W->mode;
    if (general_only(W)) return stream_affine(W) || rows_fits(W);
    return prefer_tile(W, slots) || xfp::stream_supports(bits, mode, W->K, W->L) ||
           xfp::splitk_slices(bits, mode, W->N, W->K, W->L, slots) || rows_fits(W);
}

int check_io(const xfp_weights *W, const void *x, const void *y, int y_dtype, int64_t ldy)
{
    if (!x || !y) return XFP_ERR_NULL;
    if (!dtype_ok(y_dtype)) return XFP_ERR_UNSUPPORTED;
    if (ldy < (int64_t)W->N) return XFP_ERR_SHAPE;
    if (misaligned(x, 16) || misaligned(y, 16)) return XFP_ERR_ALIGN;
    return XFP_OK;
}

// Rows one workgroup of the general kernel walks: enough workgroups to cover
// the chip several times over, few enough that staging x is amortised.
uint32_t rows_per_block(uint32_t N, int slots)
{
    uint64_t total = (uint64_t)N * slots;
    uint32_t r = 4;
    while (r < 64 && total / r > 4096) r *= 2;
    return r;
}

// M = 1 per slot: the tile kernel or the streaming kernel?  Measured on MI355X (4-bit V2, one call per
// matrix, graph replay over a ring of copies, us streaming / tile): 8192 x 4096 6.2 / 6.7; 16384 x 4096
// 10.0 / 9.2; 8192 x 8192 10.9 / 10.7; 4096 x 16384 14.8 / 14.5; 28672 x 4096 17.4 / 15.7; 32768 x 4096
// 19.5 / 16.7; 16384 x 8192 20.0 / 17.7; 8192 x 16384 22.2 / 18.2; 28672 x 8192 31.0 / 30.2.  The streaming
// kernel wins while a call is a few waves per SIMD (nothing to build per tile, no barrier); from 2^26
// weights per call on the tile kernel's conflict-free lookups win or tie everywhere.  Rows beyond what
// the streaming kernel holds in registers, which it can only take as split-K slices plus a second launch,
// are the tile kernel's at any size (8192 x 28672: 32.9 / 25.2 us).
constexpr uint64_t kTileFromWeights = 1ull << 26;
std::atomic<int> g_kernel_choice{XFP_KERNEL_AUTO};

bool prefer_tile(const xfp_weights *W, int slots)
{
    if (general_only(W) || !xfp::tile_supports((int)W->bits, (int)W->mode, W->N, W->K, slots)) return false;
    const int choice = g_kernel_choice.load(std::memory_order_relaxed);
    if (choice == XFP_KERNEL_TILE) return true;
    if (choice == XFP_KERNEL_STREAM) return false;
    return W->K > 16384 || (uint64_t)W->N * W->K * (uint64_t)slots >= kTileFromWeights;
}

// What the next launch of a plain decode call is: the kernel family and how many of the remaining slots it
// takes.  The one place the dispatch rule lives: decode() executes it, xfp_route() reports it.
struct Plan {
    int route;      // an xfp_route_id, or a negative status
    int take;       // slots (tokens) the launch covers
    int slices;     // split-K: slices of K
};

// 2 .. 16 tokens on rows above 8192 columns, in a matrix of 256 tiles of 32 rows or more: the wide kernel
bool long_rows_go_wide(const xfp_weights *W, int tokens)
{
    return tokens >= 2 && tokens <= 16 && xfp::batch_is_split(W->K) && (W->N + 31) / 32 >= 256 &&
           xfp::wide_supports((int)W->bits, (int)W->mode, W->L, W->N, W->K, tokens);
}

// V2a with a scale and a mid-point per group, 2 .. 16 tokens of one matrix: the wide kernel's MODE 2, from 2^27
// weights x tokens on (measured against the streaming kernel's mode run once per token, us for 2 / 4 / 8 / 16
// tokens: 28672 x 8192 at 3 bits 59 / 59 / 60 / 60 against 71 / 134 / 242 / 413; 4096 x 4096 14 / 14 / 14 / 15
// against 8 / 11 / 22 / 39; 1024 x 4096 at 4 bits 14 .. 15 against 5 / 6 / 8 / 12)
bool wide_affine(const xfp_weights *W, bool expert_indexed, int tokens)
{
    return !expert_indexed && tokens >= 2 && tokens <= 16 && (W->flags & XFP_FLAG_GROUP_AFFINE) != 0 &&
           W->mode == XFP_MODE_V2A && W->bits <= 4 && (uint64_t)W->N * W->K * (uint64_t)tokens >= (1ull << 27) &&
           xfp::wide_supports((int)W->bits, 2, W->L, W->N, W->K, tokens);
}

Plan plan(const xfp_weights *W, bool expert_indexed, int slots)
{
    const int bits = (int)W->bits, mode = (int)W->mode;
    const bool gen = general_only(W);
    if (!gen && !expert_indexed && slots >= 2) {
        // batched tokens: the weights are read once per 16 tokens, once per up to 64 where the wide kernel takes
        // the format and its re-laid copies fit the workspace
        int wide = slots < 64 ? slots : 64;
        while (wide > 16 && !xfp::wide_supports(bits, mode, W->L, W->N, W->K, wide)) wide -= 16;
        if (wide > 16) return Plan{XFP_ROUTE_WIDE, wide, 0};
        // rows the 16-token kernel would cut into slices of K (three launches, partial planes): the wide kernel
        // takes any row length in one launch and is faster once its 32-row tiles fill the chip (measured, 16 tokens:
        // 8192 x 28672 at 4 bits 52 against 54 us, at 3 bits 48 against 55, 16384 x 12288 40 against 44, but
        // 4096 x 16384 with its 128 tiles 31 against 24)
        if (long_rows_go_wide(W, slots < 16 ? slots : 16)) return Plan{XFP_ROUTE_WIDE, slots < 16 ? slots : 16, 0};
        if (xfp::batch_supports(bits, mode, W->L, W->N, W->K, slots)) return Plan{XFP_ROUTE_BATCH, slots < 16 ? slots : 16, 0};
    }
    // a scale and a mid-point per group with several tokens: the wide kernel's mode for it, 16 tokens per launch
    if (wide_affine(W, expert_indexed, slots < 16 ? slots : 16)) return Plan{XFP_ROUTE_WIDE, slots < 16 ? slots : 16, 0};
    // M = 1 per slot: every remaining slot in one launch (also the odd token left over after chunks of 16)
    const int take = slots;
    if (prefer_tile(W, take)) return Plan{XFP_ROUTE_TILE, take, 0};
    if (stream_affine(W)) return Plan{XFP_ROUTE_STREAM, take, 0};
    if (!gen && xfp::stream_supports(bits, mode, W->K, W->L)) return Plan{XFP_ROUTE_STREAM, take, 0};
    if (const int S = gen ? 0 : xfp::splitk_slices(bits, mode, W->N, W->K, W->L, take)) return Plan{XFP_ROUTE_SPLIT_K, take, S};
    if (!rows_fits(W)) return Plan{XFP_ERR_UNSUPPORTED, 0, 0};
    return Plan{XFP_ROUTE_GENERAL, take, 0};
}

// y_dtype: an xfp_dtype, optionally OR-ed with XFP_X_BF16
int decode(const xfp_weights *W, const int32_t *eids, int slots, const void *x, int64_t x_stride,
           void *y, int y_dtype, int64_t ldy, Scratch &sc, hipStream_t s)
{
    const bool x_bf16 = (y_dtype & XFP_X_BF16) != 0;
    y_dtype &= 0xFF;
    const int bits = (int)W->bits, mode = (int)W->mode;
    const bool y_f32 = y_dtype == XFP_F32;
    xfp::DecodeArgs a = base_args(W);
    a.x = static_cast<const uint16_t *>(x);
    a.y = y;
    a.eids = eids;
    a.x_stride = x_stride;
    a.y_stride = ldy;
    a.y_bf16 = y_dtype == XFP_BF16;
    a.x_bf16 = x_bf16;
    const size_t ysz = y_f32 ? 4 : 2;
    // the launches of a call run in stream order, so they share the call's workspace
    for (int m0 = 0; m0 < slots;) {
        const Plan p = plan(W, eids != nullptr, slots - m0);
        if (p.route < 0) return p.route;
        xfp::DecodeArgs c = a;
        c.x = a.x + (int64_t)m0 * x_stride;
        c.y = static_cast<char *>(y) + (size_t)m0 * (size_t)ldy * ysz;
        if (eids) c.eids = eids + m0;
        const xfp::Workspace *ws = nullptr;
        if (p.route == XFP_ROUTE_WIDE || p.route == XFP_ROUTE_BATCH || p.route == XFP_ROUTE_SPLIT_K) {
            hipError_t werr = sc.get(&ws);
            if (werr != hipSuccess) return finish(werr);
        }
        hipError_t err = hipSuccess;
        switch (p.route) {
        case XFP_ROUTE_WIDE:
            err = xfp::launch_decode_wide(bits, (W->flags & XFP_FLAG_GROUP_AFFINE) ? 2 : mode, c, p.take, y_f32, ws->xc, ws->part, s);
            break;
        case XFP_ROUTE_BATCH: err = xfp::launch_decode_batch(bits, mode, c, p.take, y_f32, ws->part, ws->xc, s); break;
        case XFP_ROUTE_TILE: err = xfp::launch_decode_tile(bits, y_f32, c, p.take, s); break;
        case XFP_ROUTE_STREAM: err = xfp::launch_decode_stream(bits, stream_affine(W) ? 2 : mode, y_f32, c, p.take, s); break;
        case XFP_ROUTE_SPLIT_K: err = xfp::launch_decode_splitk(bits, mode, y_f32, c, p.take, p.slices, ws->part, s); break;
        default:
            c.rows_per_block = rows_per_block(W->N, p.take);
            err = xfp::launch_decode_rows(bits, mode, y_f32, c, p.take, s);
            break;
        }
        if (err != hipSuccess) return finish(err);
        m0 += p.take;
    }
    return XFP_OK;
}

// h[t][j] = SiLU(y[t][j]) * y[t][N/2 + j]: in the streaming kernel's store when it
// takes the shape, else the plain decode into a scratch plane plus a small kernel.
int decode_silu_mul(const xfp_weights *W, const int32_t *eids, int slots, const void *x, int64_t x_stride,
                    void *h, int h_dtype, int64_t ldh, Scratch &sc, hipStream_t s)
{
    const int x_flag = h_dtype & XFP_X_BF16;
    h_dtype &= 0xFF;
    if (!general_only(W) && xfp::stream_supports((int)W->bits, (int)W->mode, W->K, W->L)) {
        xfp::DecodeArgs a = base_args(W);
        a.y_bf16 = h_dtype == XFP_BF16;
        a.x_bf16 = x_flag != 0;
        a.x = static_cast<const uint16_t *>(x);
        a.y = h;
        a.eids = eids;
        a.x_stride = x_stride;
        a.y_stride = ldh;
        a.fuse_half = W->N / 2;
        hipError_t err = xfp::launch_decode_stream((int)W->bits, (int)W->mode, h_dtype == XFP_F32, a, slots, s);
        if (err != hipErrorInvalidValue) return finish(err);     // InvalidValue: no even batch fits, nothing launched
    }
    if ((uint64_t)slots * W->N > xfp::kPlaneFloats || !decodable(W, slots)) return XFP_ERR_UNSUPPORTED;
    const xfp::Workspace *ws = nullptr;
    hipError_t werr = sc.get(&ws);
    if (werr != hipSuccess) return finish(werr);
    int rc = decode(W, eids, slots, x, x_stride, ws->epi, XFP_F32 | x_flag, (int64_t)W->N, sc, s);
    if (rc) return rc;
    return finish(xfp::launch_silu_mul(ws->epi, W->N / 2, slots, h, ldh, h_dtype == XFP_F32, h_dtype == XFP_BF16, s));
}

}  // namespace

extern "C" {

int xfp_gemv(const xfp_weights *W, const void *x, int M, int64_t ldx, void *y, int y_dtype,
             int64_t ldy, void *hip_stream)
{
    int rc = check_weights(W);
    if (rc) return rc;
    if (W->E != 1) return XFP_ERR_SHAPE;
    if (M <= 0 || M > 65535) return XFP_ERR_SHAPE;
    rc = check_io(W, x, y, y_dtype, ldy);
    if (rc) return rc;
    if (ldx < (int64_t)W->K) return XFP_ERR_SHAPE;
    if (ldx % 8 != 0) return XFP_ERR_ALIGN;
    if (!decodable(W, M)) return XFP_ERR_UNSUPPORTED;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    Scratch sc(s);
    return decode(W, nullptr, M, x, ldx, y, y_dtype, ldy, sc, s);
}

int xfp_gemv_noalloc(const xfp_weights *W, const void *x, int M, int64_t ldx, void *y, int y_dtype,
                     int64_t ldy, void *hip_stream)
{
    int rc = check_weights(W);
    if (rc) return rc;
    if (W->E != 1) return XFP_ERR_SHAPE;
    if (M <= 0 || M > 65535) return XFP_ERR_SHAPE;
    rc = check_io(W, x, y, y_dtype, ldy);
    if (rc) return rc;
    if (ldx < (int64_t)W->K) return XFP_ERR_SHAPE;
    if (ldx % 8 != 0) return XFP_ERR_ALIGN;
    // a route that only the size of the scratch planes closes is refused, not replaced
    const int bits = (int)W->bits, mode = (int)W->mode;
    constexpr uint64_t kNoCap = ~0ull;
    if (!general_only(W) && !long_rows_go_wide(W, M < 16 ? M : 16) &&
        xfp::batch_supports(bits, mode, W->L, W->N, W->K, M, kNoCap, kNoCap) != xfp::batch_supports(bits, mode, W->L, W->N, W->K, M))
        return XFP_ERR_SCRATCH;
    if (!general_only(W) && !prefer_tile(W, M) &&
        !xfp::batch_supports(bits, mode, W->L, W->N, W->K, M) && !xfp::stream_supports(bits, mode, W->K, W->L) &&
        xfp::splitk_slices(bits, mode, W->N, W->K, W->L, M, kNoCap) != xfp::splitk_slices(bits, mode, W->N, W->K, W->L, M))
        return XFP_ERR_SCRATCH;
    if (!decodable(W, M)) return XFP_ERR_UNSUPPORTED;
    void *ptr = nullptr;
    hipError_t err = scratch_resolve(&ptr);
    if (err != hipSuccess) return finish(err);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    Scratch sc(s, xfp::workspace_at(ptr));
    return decode(W, nullptr, M, x, ldx, y, y_dtype, ldy, sc, s);
}

int xfp_gemv_moe(const xfp_weights *bank, const int32_t *expert_ids, int T, const void *x,
                 int64_t x_slot_stride, void *y, int y_dtype, int64_t ldy, void *hip_stream)
{
    int rc = check_weights(bank);
    if (rc) return rc;
    if (T < 0 || T > 65535) return XFP_ERR_SHAPE;
    if (T == 0) return XFP_OK;
    if (!expert_ids) return XFP_ERR_NULL;
    rc = check_io(bank, x, y, y_dtype, ldy);
    if (rc) return rc;
    if (x_slot_stride != 0 && x_slot_stride < (int64_t)bank->K) return XFP_ERR_SHAPE;
    if (x_slot_stride % 8 != 0 || misaligned(expert_ids, 4)) return XFP_ERR_ALIGN;
    if (!decodable(bank, T)) return XFP_ERR_UNSUPPORTED;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    Scratch sc(s);
    return decode(bank, expert_ids, T, x, x_slot_stride, y, y_dtype, ldy, sc, s);
}

int xfp_gemv_moe_silu_mul(const xfp_weights *bank, const int32_t *expert_ids, int T, const void *x,
                          int64_t x_slot_stride, void *h, int h_dtype, int64_t ldh, void *hip_stream)
{
    int rc = check_weights(bank);
    if (rc) return rc;
    if (bank->N % 2 != 0) return XFP_ERR_SHAPE;
    if (T < 0 || T > 65535) return XFP_ERR_SHAPE;
    if (T == 0) return XFP_OK;
    if (!expert_ids && bank->E != 1) return XFP_ERR_NULL;
    if (!x || !h) return XFP_ERR_NULL;
    if (!dtype_ok(h_dtype)) return XFP_ERR_UNSUPPORTED;
    if (ldh < (int64_t)(bank->N / 2)) return XFP_ERR_SHAPE;
    if (x_slot_stride != 0 && x_slot_stride < (int64_t)bank->K) return XFP_ERR_SHAPE;
    if (misaligned(x, 16) || misaligned(h, 16) || x_slot_stride % 8 != 0 || misaligned(expert_ids, 4))
        return XFP_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    Scratch sc(s);
    return decode_silu_mul(bank, expert_ids, T, x, x_slot_stride, h, h_dtype, ldh, sc, s);
}

int xfp_gemv_moe_combine(const xfp_weights *bank, const int32_t *expert_ids, int T, const void *x,
                         int64_t x_slot_stride, const float *slot_weights, void *y, int y_dtype, void *hip_stream)
{
    int rc = check_weights(bank);
    if (rc) return rc;
    if (T <= 0 || T > 65535) return XFP_ERR_SHAPE;
    if (!expert_ids || !slot_weights) return XFP_ERR_NULL;
    rc = check_io(bank, x, y, y_dtype, (int64_t)bank->N);
    if (rc) return rc;
    if (x_slot_stride != 0 && x_slot_stride < (int64_t)bank->K) return XFP_ERR_SHAPE;
    if (x_slot_stride % 8 != 0 || misaligned(expert_ids, 4) || misaligned(slot_weights, 4)) return XFP_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int yd = y_dtype & 0xFF;
    if (!general_only(bank) && xfp::combine_supports((int)bank->bits, (int)bank->mode, bank->K, T)) {
        xfp::DecodeArgs a = base_args(bank);
        a.x = static_cast<const uint16_t *>(x);
        a.y = y;
        a.eids = expert_ids;
        a.x_stride = x_slot_stride;
        a.x_bf16 = (y_dtype & XFP_X_BF16) != 0;
        return finish(xfp::launch_decode_combine((int)bank->bits, a, T, slot_weights, yd == XFP_F32, yd == XFP_BF16, s));
    }
    // other shapes: per-slot fp32 results in a scratch plane, added by a second kernel
    if ((uint64_t)T * bank->N > xfp::kPlaneFloats || !decodable(bank, T)) return XFP_ERR_UNSUPPORTED;
    Scratch sc(s);
    const xfp::Workspace *ws = nullptr;
    hipError_t werr = sc.get(&ws);
    if (werr != hipSuccess) return finish(werr);
    rc = decode(bank, expert_ids, T, x, x_slot_stride, ws->epi, XFP_F32 | (y_dtype & XFP_X_BF16), (int64_t)bank->N, sc, s);
    if (rc) return rc;
    return finish(xfp::launch_moe_combine(ws->epi, slot_weights, bank->N, T, y, yd == XFP_F32, yd == XFP_BF16, s));
}

int xfp_repack_words(const void *src, int64_t rows, int K, int bits, uint32_t *dst, void *hip_stream)
{
    if (!src || !dst) return XFP_ERR_NULL;
    if (bits < 2 || bits > 6) return XFP_ERR_UNSUPPORTED;
    if (rows < 0 || K <= 0 || K % xfp::kGroup != 0) return XFP_ERR_SHAPE;
    if ((uint64_t)rows * (uint64_t)(K / 32 * bits) >= (1ull << 40)) return XFP_ERR_SHAPE;
    if (misaligned(src, bits == 5 ? 2 : 4) || misaligned(dst, 4)) return XFP_ERR_ALIGN;
    if (rows == 0) return XFP_OK;
    return finish(xfp::launch_repack_words(src, (uint64_t)rows, (uint32_t)K, bits, dst, static_cast<hipStream_t>(hip_stream)));
}

int xfp_repack_word10(const uint32_t *src, int64_t rows, int K, uint32_t *dst, void *hip_stream)
{
    return xfp_repack_words(src, rows, K, 3, dst, hip_stream);
}

int xfp_convert_bf16_to_f16(const void *src, int64_t ld_src, void *dst, int rows, int cols, void *hip_stream)
{
    if (!src || !dst) return XFP_ERR_NULL;
    if (rows < 0 || cols < 0 || cols % 8 != 0 || rows > 65535 || ld_src < cols) return XFP_ERR_SHAPE;
    if (misaligned(src, 16) || misaligned(dst, 16) || ld_src % 8 != 0) return XFP_ERR_ALIGN;
    if (rows == 0 || cols == 0) return XFP_OK;
    return finish(xfp::launch_bf16_to_f16(src, ld_src, dst, (uint32_t)rows, (uint32_t)cols,
                                          static_cast<hipStream_t>(hip_stream)));
}

int xfp_unpack_indices(const xfp_weights *W, uint8_t *idx_out, void *hip_stream)
{
    int rc = check_weights(W);
    if (rc) return rc;
    if (!idx_out) return XFP_ERR_NULL;
    if (misaligned(idx_out, 16)) return XFP_ERR_ALIGN;
    return finish(xfp::launch_unpack((int)W->bits, W->indices, (uint64_t)W->E * W->N, W->K, idx_out,
                                     static_cast<hipStream_t>(hip_stream)));
}

int xfp_dequant_bulk(const xfp_weights *W, uint16_t *w_out, void *hip_stream)
{
    int rc = check_weights(W);
    if (rc) return rc;
    if (!w_out) return XFP_ERR_NULL;
    if (misaligned(w_out, 16)) return XFP_ERR_ALIGN;
    xfp::DecodeArgs a = base_args(W);
    return finish(xfp::launch_dequant((int)W->bits, (int)W->mode, a, W->E, w_out,
                                      static_cast<hipStream_t>(hip_stream)));
}

int xfp_check_contents(const xfp_weights *W, int64_t nnz_capacity, const int32_t *expert_ids, int T,
                       uint32_t *report, void *hip_stream)
{
    int rc = check_weights(W);
    if (rc) return rc;
    if (!report) return XFP_ERR_NULL;
    if (nnz_capacity < 0 || T < 0) return XFP_ERR_SHAPE;
    if (nnz_capacity > 0 && !W->out_col) return XFP_ERR_NULL;
    if (misaligned(report, 8) || misaligned(expert_ids, 4)) return XFP_ERR_ALIGN;
    xfp::DecodeArgs a = base_args(W);
    return finish(xfp::launch_check_contents(a, W->E, (uint64_t)nnz_capacity, expert_ids, expert_ids ? T : 0, report,
                                             static_cast<hipStream_t>(hip_stream)));
}

int xfp_probe_read(const void *src, uint64_t bytes, uint32_t *sink, void *hip_stream)
{
    if (!src || !sink) return XFP_ERR_NULL;
    if (bytes % 16 != 0) return XFP_ERR_SHAPE;
    if (misaligned(src, 16) || misaligned(sink, 4)) return XFP_ERR_ALIGN;
    return finish(xfp::launch_probe_read(src, bytes, sink, static_cast<hipStream_t>(hip_stream)));
}

int xfp_probe_copy(const void *src, void *dst, uint64_t bytes, void *hip_stream)
{
    if (!src || !dst) return XFP_ERR_NULL;
    if (bytes % 16 != 0) return XFP_ERR_SHAPE;
    if (misaligned(src, 16) || misaligned(dst, 16)) return XFP_ERR_ALIGN;
    return finish(xfp::launch_probe_copy(src, dst, bytes, static_cast<hipStream_t>(hip_stream)));
}

const char *xfp_strerror(int status)
{
    switch (status) {
    case XFP_OK: return "ok";
    case XFP_ERR_NULL: return "a required pointer is NULL";
    case XFP_ERR_SHAPE: return "bad shape (sizes must be positive, K a multiple of 128, leading dimensions large enough)";
    case XFP_ERR_UNSUPPORTED: return "unsupported format or shape (bits 2..6, mode V2/V2a, group 128, flags 0 or 1 (V2a only), output fp16/bf16/fp32; a row too long for every kernel; a result too large for the scratch plane)";
    case XFP_ERR_ALIGN: return "a pointer or leading dimension is misaligned";
    case XFP_ERR_SCRATCH: return "the call needs more scratch memory than xfp_gemv_noalloc's static array holds (M >= 2: K <= 32768; sliced rows of M = 1 calls: S * M * N <= 2^20)";
    case XFP_ERR_HIP:
        std::snprintf(g_msg, sizeof(g_msg), "HIP launch failed: %s", hipGetErrorString(g_last_hip));
        return g_msg;
    default: return "unknown status";
    }
}

int xfp_init(void)
{
    hipError_t err = xfp::ring_resolve();
    if (err == hipSuccess) err = scratch_resolve(nullptr);
    return finish(err);
}

int xfp_select_kernel(int which)
{
    if (which != XFP_KERNEL_AUTO && which != XFP_KERNEL_STREAM && which != XFP_KERNEL_TILE) return XFP_ERR_UNSUPPORTED;
    g_kernel_choice.store(which, std::memory_order_relaxed);
    return XFP_OK;
}

int xfp_route(const xfp_weights *W, int M, int expert_indexed, int *tokens)
{
    int rc = check_weights(W);
    if (rc) return rc;
    if (M < 1 || M > 65535) return XFP_ERR_SHAPE;
    if (!expert_indexed && W->E != 1) return XFP_ERR_SHAPE;
    const Plan p = plan(W, expert_indexed != 0, M);
    if (tokens) *tokens = p.take;
    return p.route;
}

int xfp_ring_slot(unsigned ticket, int capturing) { return xfp::ring_slot_index(ticket, capturing != 0); }

int xfp_version(void) { return (0 << 16) | (2 << 8) | 0; }

}  // extern "C"
