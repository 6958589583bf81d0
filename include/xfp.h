/*
 * xfp.h - C ABI of the MI355X (gfx950) XFP fused decode library.
 *
 * The library computes the decode-time product of an activation with an
 * XFP-compressed weight matrix
 *
 *     y = x * W_hat^T,     W_hat = Codebook[Q_bulk] + W_outlier          (paper eq. 1)
 *
 * in one kernel launch that fuses the steps the paper lists at the start of
 * section 5: depack the N-bit indices, gather codebook entries held on chip,
 * add the sparse outlier term, multiply-accumulate.  Q_bulk is a dense b-bit
 * index tensor; the codebook is either V2 (one fp16 codebook of 2^b entries
 * per output channel) or V2a (a per-layer library of L codebooks plus one
 * library id per group of 128 weights), paper sections 3.1, 3.2 and 3.4.
 *
 * Conventions common to every entry point
 *  - Every data pointer (inside xfp_weights and x / y / expert_ids / outputs)
 *    is a DEVICE pointer owned by the caller.  The xfp_weights struct itself
 *    is HOST memory, read during the call and not retained.
 *  - Calls are asynchronous on `hip_stream` (a hipStream_t; NULL = the default
 *    stream).  The library never allocates, frees, copies or synchronises, so
 *    every entry point may be recorded into a HIP graph.
 *  - Outputs are overwritten, never accumulated into.
 *  - Return value: XFP_OK or a negative xfp_status.  Nothing is launched when
 *    an argument is rejected.  A failed launch returns XFP_ERR_HIP.
 *  - Only what the host can see is validated (shapes, bit width, mode, NULLs,
 *    alignment).  Contents of device buffers (expert ids in range, group ids
 *    below L, CSR row pointers ascending and columns in [0, K)) are the
 *    caller's contract; violating it is undefined behaviour.
 *    xfp_check_contents checks that contract on the device.
 *  - Calls from several host threads are safe.  The only state kept between
 *    calls is a static ring of eight workspaces of 10 MB in device memory
 *    (every GPU the process uses holds its own copy; a call uses the one of the
 *    current device, which must be the device of its pointers and stream).
 *    A call that needs scratch memory (the batched path's re-laid activations,
 *    split-K partial sums, the unfused forms of the epilogues) takes ONE slot
 *    for everything it needs.  Eager calls cycle through four slots, so calls
 *    on ONE stream never interfere, and calls that overlap on different
 *    streams do only when more than four scratch-using calls are in flight at
 *    once.  Calls recorded into a HIP graph keep their slot for as long as the
 *    graph lives and cycle through four slots of their own, which eager calls
 *    never take; two graphs that may run at the same time on different streams
 *    can meet in one of them.  xfp_init resolves the ring's address; call it
 *    once per device before recording a graph (an eager call does the same).
 *  - Results are run-to-run deterministic by construction (fixed summation
 *    orders, no floating-point atomics).  One observation stands against it and
 *    is not explained: on one machine one call returned, twice, the same wrong
 *    value (off by 2e-4 relative) in one of four workgroups that compute the
 *    same output from the same data; bit-exact emulation of that kernel excludes
 *    every event its code could produce (stale or foreign table contents, a
 *    wrong library id, wrong activations, a dropped or duplicated outlier) and
 *    leaves only a corrupted single operand.
 *
 * Data layout (all little-endian)
 *  - indices: per matrix, N rows of K*bits/32 uint32 words, no row padding.
 *    Field k of a row is bits [k*bits, (k+1)*bits) of the row's bit stream,
 *    least significant bit first; the stream fills word 0 from bit 0 upward,
 *    then word 1, ...  For bits = 2 and 4 this is the paper's table 2 (16 and
 *    8 values per uint32, no reserve bits).  For bits = 3, 5 and 6 the stream is
 *    dense (3.0, 5.0, 6.0 bit per weight, fields cross word boundaries), which
 *    is NOT the table's word forms with reserve bits (10 per uint32, 3 per
 *    uint16, 5 per uint32); xfp_repack_words converts those once at load.
 *  - group: 128 consecutive k of one output row (K % 128 == 0).
 *  - outliers: CSR over the stacked E*N rows: int32 row_ptr [E*N + 1] holding
 *    absolute offsets (row_ptr[0] == 0), int32 col [nnz] ascending within a
 *    row with no duplicates, fp16 val [nnz].  The outlier value is ADDED to
 *    the codebook value at that position (eq. 1 is a sum).
 *  - x is fp16 (or bf16, converted as it is loaded: XFP_X_BF16); y is fp16, bf16 or fp32, rounded
 *    once, to nearest even, from the fp32 sum; accumulation is fp32.
 */
#ifndef XFP_H
#define XFP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    XFP_OK = 0,
    XFP_ERR_NULL = -1,        /* a required pointer is NULL                         */
    XFP_ERR_SHAPE = -2,       /* N, K, M, E <= 0, T < 0, K % group != 0, ld too small */
    XFP_ERR_UNSUPPORTED = -3, /* bits, mode, L, group, dtype, flags, struct_size; a row no kernel takes */
    XFP_ERR_ALIGN = -4,       /* a base pointer or a leading dimension is misaligned */
    XFP_ERR_HIP = -5,         /* the HIP runtime refused the launch                  */
    XFP_ERR_SCRATCH = -6      /* xfp_gemv_noalloc: the call needs more scratch than the static array holds */
} xfp_status;

typedef enum { XFP_MODE_V2 = 0, XFP_MODE_V2A = 1 } xfp_mode;
typedef enum { XFP_F16 = 0, XFP_F32 = 1, XFP_BF16 = 2 } xfp_dtype;   /* type of an output (y, h) */
/* OR into a y_dtype / h_dtype argument: the activations x are bf16 instead of
 * fp16 (the paper's kernel takes and returns bf16, section 5).  Every kernel
 * converts them to fp16 as it loads them (see xfp_convert_bf16_to_f16 for the
 * rounding): no extra launch, no scratch, and bit for bit the result of the
 * same call on the converted activations. */
#define XFP_X_BF16 0x100

/* xfp_weights.flags, bit 0: a V2a matrix whose groups carry a scale and a
 * mid-point next to their library id (paper section 3.4; with the one-byte id a
 * 40-bit record per group, the 0.31 bit per weight of section 3.2).  The paper
 * gives no formula; reading taken: the affine map
 *     C[n][k] = library[id][q] * scale[n][k/128] + mid[n][k/128],
 * evaluated in fp32 on a group's partial sums (scale * sum(x * entry) + mid *
 * sum(x), which is the same thing by linearity).  Scale 1 and mid-point 0 give
 * the plain library.  At 2 to 4 bits such matrices run a mode of their own of the
 * streaming kernel (rows up to 16384 columns, token by token) or, for several
 * tokens on a large matrix (2^27 weights x tokens and more), of the wide
 * matrix-core kernel, 16 tokens per launch; else the general kernel. */
#define XFP_FLAG_GROUP_AFFINE 1u

#define XFP_GROUP 128
#define XFP_MAX_LIBRARY 256          /* V2a ids are one byte each */

/* One bank of E matrices of identical shape and format (E = 1: a plain matrix). */
typedef struct xfp_weights {
    uint32_t struct_size;       /* sizeof(xfp_weights), checked                              */
    uint32_t mode;              /* xfp_mode                                                  */
    uint32_t bits;              /* 2 .. 6 (paper section 3.1); 5 and 6 run the general kernel only */
    uint32_t group;             /* must be 128                                               */
    uint32_t N, K;              /* output channels, input channels; K % 128 == 0             */
    uint32_t L;                 /* V2a: library size, 1..256 (paper default 32); V2: 0       */
    uint32_t E;                 /* matrices stacked in this bank                             */
    uint32_t flags;             /* 0 or XFP_FLAG_GROUP_AFFINE                                */
    uint32_t reserved;          /* must be 0                                                 */
    const uint32_t *indices;    /* [E][N][K*bits/32]                                         */
    const uint16_t *codebooks;  /* fp16: V2 [E][N][1<<bits], V2a [E][L][1<<bits]             */
    const uint8_t *group_ids;   /* V2a: [E][N][K/128], each < L; V2: NULL                    */
    const int32_t *out_row_ptr; /* [E*N + 1]                                                 */
    const int32_t *out_col;     /* [nnz] (may be NULL when nnz == 0)                         */
    const uint16_t *out_val;    /* fp16 [nnz] (may be NULL when nnz == 0)                    */
    const uint16_t *group_scale;/* fp16 [E][N][K/128] with XFP_FLAG_GROUP_AFFINE, else NULL  */
    const uint16_t *group_mid;  /* fp16 [E][N][K/128] with XFP_FLAG_GROUP_AFFINE, else NULL  */
} xfp_weights;

/*
 * y[m][n] = sum_k x[m][k] * C[n][k] + sum_{j in CSR row n} val[j] * x[m][col[j]]
 * for m in [0, M), n in [0, N)    (paper eq. 1 and section 5, steps 1-4).
 *
 * W      one matrix (W->E must be 1).
 * x      fp16 [M][ldx], ldx >= K, ldx % 8 == 0, 16-byte aligned.
 * y      [M][ldy] of y_dtype, ldy >= N, 16-byte aligned base.
 * M      1 .. 65535.  M = 1 is the decode case.  M >= 2 takes a matrix-core
 *        (MFMA) path that reads the weights once per 16 tokens, for V2 and
 *        V2a at 2 to 4 bits (a V2a library with L * 4^bits * 4 bytes <= 64 KB),
 *        K <= 32768; rows above 8192 columns in one launch when the matrix
 *        has 8161 rows or more, else in slices of K whose partial sums go
 *        through a static scratch plane.  The same formats with more than 16
 *        tokens read the weights once per up to 64 tokens (as many chunks
 *        of 16 as 16 * ceil(m / 16) * K <= 2^19 allows: 64 tokens up to
 *        K = 8192, 32 up to 16384); any other shape or width runs the
 *        M = 1 path once per token.  Same results either way, to rounding.
 * XFP_ERR_UNSUPPORTED for a row no kernel takes: longer than 16384 columns, not
 * 4-bit V2 (whose rows of any length the tile kernel takes), with no split into
 * equal slices of at most 8192 (or partial sums beyond the scratch plane) AND
 * too long for the general kernel to stage on chip (2 K bytes plus its tables
 * within 160 KB).  xfp_route tells on the host which kernel a call takes.
 */
int xfp_gemv(const xfp_weights *W, const void *x, int M, int64_t ldx,
             void *y, int y_dtype, int64_t ldy, void *hip_stream);

/*
 * xfp_gemv for callers that cannot allocate and must know where every byte a
 * call touches lives: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  (No paper counterpart.)  Same arguments and
 * same results, bit for bit, as xfp_gemv.  Whatever scratch the call needs
 * (re-laid activations for M >= 2, partial sums of rows cut into slices of K)
 * lives in ONE static device array of 10 MB, not in the ring the other entry
 * points cycle through; each GPU the process uses holds its own copy until the
 * process ends.  The call allocates nothing, frees nothing and calls no
 * allocating routine.
 * Limits (the array's size): where xfp_gemv would reroute a call because a
 * scratch plane is too small, this one returns XFP_ERR_SCRATCH and launches
 * nothing: M >= 2 with K > 32768; rows above 16384 columns that the M = 1 path
 * cuts into S equal slices with S * M * N > 2^20 (4-bit V2 rows of that length
 * take the tile kernel, which needs no scratch).
 * Every call on a GPU uses that GPU's one array, which keeps the last call's
 * contents (nothing in it has to start at zero: every plane is written before it
 * is read): calls that overlap in time on one GPU (two streams, two threads)
 * race.  Calls on one stream are ordered and never interfere.
 */
int xfp_gemv_noalloc(const xfp_weights *W, const void *x, int M, int64_t ldx,
                     void *y, int y_dtype, int64_t ldy, void *hip_stream);

/*
 * Expert-indexed grouped form for routed-expert layers: for each slot
 * t in [0, T), y[t][:] = xfp_gemv of matrix expert_ids[t] of the bank applied
 * to input row t (M = 1 per slot).  The paper applies the fused decode to
 * routed-expert weights (sections 1 and 6.1) without describing the launch;
 * this grouped call is this library's reading.  expert_ids is read on the
 * device, so a router's output can be consumed without a host round trip.
 *
 * expert_ids     device int32 [T], each in [0, bank->E); duplicates allowed.
 * x              fp16; slot t reads x + t * x_slot_stride (in elements).
 *                x_slot_stride == 0 shares one input row between all slots,
 *                otherwise it must be >= K and a multiple of 8.
 * y              [T][ldy], ldy >= N.
 * T == 0 is a no-op that returns XFP_OK.  T <= 65535.
 */
int xfp_gemv_moe(const xfp_weights *bank, const int32_t *expert_ids, int T,
                 const void *x, int64_t x_slot_stride,
                 void *y, int y_dtype, int64_t ldy, void *hip_stream);

/*
 * Gate/up projection of a gated-MLP expert with its activation folded into the
 * store: the bank's matrices stack the gate rows [0, N/2) on the up rows
 * [N/2, N), and for each slot t
 *     h[t][j] = SiLU(g) * u,   g = y[t][j],  u = y[t][N/2 + j],  SiLU(g) = g / (1 + exp(-g)),
 * with y as xfp_gemv_moe defines it, kept in fp32 until the one rounding to
 * h_dtype.  The paper's models are gated-MLP mixtures of experts (section 6.1)
 * and it names kernel-launch overhead as what dominates a routed-expert layer
 * (section 6); it does not describe this epilogue, which is this library's
 * addition: one launch and no round trip of y through memory.
 *
 * bank->N must be even.  expert_ids may be NULL when bank->E == 1 (a dense
 * gated MLP: slot t is token t).  h is [T][ldh], ldh >= N/2; everything else
 * as for xfp_gemv_moe.  Shapes the streaming kernel does not take (K / 128
 * without a split, oversized V2a libraries) run the plain decode into an
 * fp32 scratch plane plus a small kernel; XFP_ERR_UNSUPPORTED if T * N exceeds
 * that plane (2^20 floats).
 */
int xfp_gemv_moe_silu_mul(const xfp_weights *bank, const int32_t *expert_ids, int T,
                          const void *x, int64_t x_slot_stride,
                          void *h, int h_dtype, int64_t ldh, void *hip_stream);

/*
 * Down projection of a routed-expert layer with the router's combine folded in:
 *     y[n] = sum over slots t of slot_weights[t] * (matrix expert_ids[t] applied to input row t)[n],
 * accumulated in fp32, one rounding to y_dtype.  Like
 * the gate/up epilogue this is the library's addition to what the paper
 * describes (sections 1 and 6.1 apply the decode to routed experts and name
 * launch overhead as what dominates them).  V2 banks with T <= 8 and
 * T * K <= 16384 take one launch: an output row is decoded as the concatenation
 * of the T experts' rows, each part scaled by its slot's weight (the slots are
 * then added lane by lane and by a wave reduction, not in ascending order).
 * Other shapes: the per-slot results meet in an fp32 scratch plane
 * (T * N <= 2^20, else XFP_ERR_UNSUPPORTED) and a second small kernel adds them
 * in ascending slot order.
 *
 * slot_weights   device fp32 [T].   y  [N] of y_dtype.   T >= 1.
 * Everything else as for xfp_gemv_moe.
 */
int xfp_gemv_moe_combine(const xfp_weights *bank, const int32_t *expert_ids, int T,
                         const void *x, int64_t x_slot_stride, const float *slot_weights,
                         void *y, int y_dtype, void *hip_stream);

/*
 * bf16 -> fp16 for activations, dst[r][c] = src[r * ld_src + c], dst dense
 * [rows][cols].  Every bf16 value is exact in fp32; the one rounding to fp16
 * (to nearest even) is exact for magnitudes in [2^-14, 65504], rounds to a
 * multiple of 2^-24 below and SATURATES at +-65504 above (an infinity in x
 * would turn every output into NaN or infinity); NaN stays NaN.
 * cols % 8 == 0, ld_src >= cols and % 8 == 0, rows <= 65535, 16-byte aligned.
 */
int xfp_convert_bf16_to_f16(const void *src, int64_t ld_src, void *dst, int rows, int cols, void *hip_stream);

/*
 * Load-time conversion of 3-bit indices from the word packing of the paper's
 * packing table (section 3.3, table 2: ten values per uint32, 30 bits used, 2
 * reserved) to the dense 3-bit stream that xfp_weights.indices holds.
 * Reading taken: value k of a row sits in word k / 10 at bits [3 (k % 10),
 * 3 (k % 10) + 3), value 0 in the low bits; the two top bits of every word are
 * ignored; a row takes ceil(K / 10) words, rows stored back to back.
 * src [rows][ceil(K/10)] and dst [rows][K*3/32] are DEVICE pointers, 4-byte
 * aligned, distinct buffers (the caller owns both).  K % 128 == 0, rows >= 0
 * (rows = E * N for a bank), rows * K*3/32 < 2^40.  Integer work, bit-exact.
 */
int xfp_repack_word10(const uint32_t *src, int64_t rows, int K, uint32_t *dst, void *hip_stream);

/*
 * The same conversion for every width of the packing table (section 3.3, table
 * 2): bits = 2, 3, 4, 6 are 16, 10, 8, 5 values per uint32, bits = 5 is 3 values
 * per uint16 (one reserve bit).  Same reading: value k in word k / per at bit
 * bits * (k % per), reserve bits on top and ignored, a row takes ceil(K / per)
 * words, rows back to back.  src: DEVICE pointer to the words (2-byte aligned for
 * bits = 5, else 4-byte); dst [rows][K*bits/32] as for xfp_repack_word10.
 * For bits = 2 and 4 the word form is the dense stream and this is a copy.
 */
int xfp_repack_words(const void *src, int64_t rows, int K, int bits, uint32_t *dst, void *hip_stream);

/*
 * Parity hooks: the first two fused steps on their own (paper section 5,
 * steps 1 and 2), so that they can be compared bit for bit.
 * xfp_unpack_indices writes every index as one byte, idx_out [E*N][K].
 * xfp_dequant_bulk writes the selected codebook entry's fp16 bit pattern,
 * w_out [E*N][K]; the outlier term is not included, nor is the scale and
 * mid-point of XFP_FLAG_GROUP_AFFINE (both are applied in the decode).
 */
int xfp_unpack_indices(const xfp_weights *W, uint8_t *idx_out, void *hip_stream);
int xfp_dequant_bulk(const xfp_weights *W, uint16_t *w_out, void *hip_stream);

/*
 * Debugging aid (no paper counterpart): checks on the device the contents the
 * decode entry points take on trust, and writes a report instead of trapping.
 * Asynchronous like everything else; read the report after synchronising.
 *
 * nnz_capacity  entries allocated in out_col / out_val (row pointers beyond it
 *               are reported and never followed).
 * expert_ids    device int32 [T] or NULL (then T is ignored).
 * report        device uint32 [4], 8-byte aligned:
 *               [0] number of violations, [1] OR of (1 << kind) over them,
 *               [2], [3] low / high word of the smallest position among them
 *               (all ones when there is none).  Positions: group id index,
 *               row pointer index, outlier entry index, slot.
 */
typedef enum {
    XFP_CHECK_GROUP_ID = 1,   /* a V2a group id >= L                               */
    XFP_CHECK_ROW_PTR = 2,    /* row_ptr[0] != 0, decreasing, or beyond nnz_capacity */
    XFP_CHECK_COL_RANGE = 3,  /* an outlier column outside [0, K)                  */
    XFP_CHECK_COL_ORDER = 4,  /* columns of a row not strictly ascending           */
    XFP_CHECK_EXPERT_ID = 5   /* an expert id outside [0, E)                       */
} xfp_check_kind;
int xfp_check_contents(const xfp_weights *W, int64_t nnz_capacity, const int32_t *expert_ids, int T,
                       uint32_t *report, void *hip_stream);

/*
 * Measurement helpers (no paper counterpart): stream `bytes` (a multiple of
 * 16, 16-byte aligned) once through the chip.  xfp_probe_read only reads
 * (four independent 16-byte loads per thread; `sink`, at least 4096 uint32,
 * is written only if the XOR of all words a workgroup read equals one magic
 * value, which keeps the loads alive); xfp_probe_copy copies src to dst.  They calibrate achievable HBM bandwidth
 * and the profiler's byte counters.
 */
int xfp_probe_read(const void *src, uint64_t bytes, uint32_t *sink, void *hip_stream);
int xfp_probe_copy(const void *src, void *dst, uint64_t bytes, void *hip_stream);

/*
 * Resolves, for the current device, the addresses of the library's static
 * device memory (the ring of workspaces and xfp_gemv_noalloc's array).  Optional: the first call that needs them does the same; call
 * it once per device before recording calls into a HIP graph, so that nothing
 * but launches happens under capture.
 */
int xfp_init(void);

/*
 * Measurement and test aid (no paper counterpart): which kernel the M = 1 calls
 * take where two can (V2, 4 bits: the streaming kernel, one wave per output row,
 * or the tile kernel, 32 rows across the lanes with a pair table per lane).
 * XFP_KERNEL_AUTO restores the library's own rule (the tile kernel for rows of
 * more than 16384 columns and for calls of 2^26 weights or more).  Process-wide; results agree to rounding either way.
 * XFP_ERR_UNSUPPORTED for any other value.
 */
typedef enum { XFP_KERNEL_AUTO = 0, XFP_KERNEL_STREAM = 1, XFP_KERNEL_TILE = 2 } xfp_kernel_choice;
int xfp_select_kernel(int which);

/*
 * The dispatch rule, queryable on the host (no paper counterpart; touches no device): which kernel family the
 * FIRST launch of xfp_gemv(W, x, M, ...) (expert_indexed == 0) or of xfp_gemv_moe(bank, ids, T = M, ...)
 * (expert_indexed != 0) would be, and in *tokens (may be NULL) how many of the M tokens / slots that launch
 * covers; a call with tokens left over continues with the rule applied to the rest.  The descriptor is validated
 * as by the decode calls (its pointers are not dereferenced).  Returns an xfp_route_id, or a negative xfp_status
 * (XFP_ERR_UNSUPPORTED for a row no kernel takes).  xfp_select_kernel changes what it reports, as it changes
 * what runs.
 */
typedef enum {
    XFP_ROUTE_GENERAL = 0,   /* one wave per row, x and tables in LDS: widths 5 and 6, scale + mid-point, odd shapes */
    XFP_ROUTE_STREAM = 1,    /* M = 1 per slot, a wave per row (run of rows), x in registers                        */
    XFP_ROUTE_SPLIT_K = 2,   /* the streaming kernel over slices of K plus the fixed-order sum                      */
    XFP_ROUTE_TILE = 3,      /* M = 1 per slot, 32 rows across the lanes                                             */
    XFP_ROUTE_BATCH = 4,     /* 2 .. 16 tokens on the matrix cores, activations in registers                         */
    XFP_ROUTE_WIDE = 5       /* 17 .. 64 tokens on the matrix cores in one pass over the weights                     */
} xfp_route_id;
int xfp_route(const xfp_weights *W, int M, int expert_indexed, int *tokens);

/*
 * Test hook for the ring's slot arithmetic (host only, touches no device): the
 * slot index in [0, 8) that the ticket-th scratch-using call of its kind takes;
 * capturing != 0: a call recorded into a HIP graph.  Eager calls get slots
 * 0..3, recorded calls 4..7.
 */
int xfp_ring_slot(unsigned ticket, int capturing);

/* Text for a status code; never NULL.  For XFP_ERR_HIP the text of the last
 * HIP error seen by the calling thread is appended. */
const char *xfp_strerror(int status);

/* (major << 16) | (minor << 8) | patch */
int xfp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* XFP_H */
