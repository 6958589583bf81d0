/*
 * CPU oracle for the XFP fused decode path.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the checker, not the product: only the tests, the smoke
 * check and the benchmark's cpu_baseline leg may build or call it.  It
 * shares no code, header, table or helper with the HIP library.
 *
 * The decode path has a plain definition (paper section 3.1, eq. 1, and the
 * four fused steps listed at the start of section 5), so the oracle is that
 * definition written out in fp64, one element at a time:
 *
 *     q[n,k]  = the b-bit field k of row n of the packed index tensor
 *     C[n,k]  = V2 : codebook of output channel n, entry q[n,k]
 *               V2a: library codebook id[n, k/128], entry q[n,k];
 *                    with the scale and mid-point that section 3.4 gives every
 *                    group: that entry * scale[n, k/128] + mid[n, k/128]
 *     y[m,n]  = sum_k x[m,k] * C[n,k]  +  sum_{j in CSR row n} val[j] * x[m,col[j]]
 *
 * with every fp16 input widened exactly to double and both sums taken in
 * ascending order.  No blocking, no fusion, no reordering.  Threads (OpenMP)
 * split the output rows only; each row is computed start to finish by one
 * thread in the order above.
 *
 * Pins (tests/test_oracle_pins.py): hand-written packed words including a
 * field that straddles two words, pack/unpack round trips, the per-word
 * counts of the paper's packing table (also for its word forms with reserve
 * bits, ten 3-bit values per uint32, three 5-bit per uint16, five 6-bit per uint32:
 * hand-written words, reserved bits ignored, an independent packer), the affine
 * group map against a dense numpy build and exact rational arithmetic (scale 1,
 * mid 0 is the plain library), all 65536 fp16 patterns against an
 * independent converter, all-ones codebooks (row sums of x), zero codebooks
 * (outlier term alone against a dense scatter), a uniform-grid codebook
 * against textbook symmetric int4 dequantisation, V2a with one id against V2,
 * entry-permutation invariance, linearity, and brute-force dense matmul.
 * The paper prints no numeric input/output example of the kernel, so y is
 * pinned by definition, invariants and brute force only.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define XFP_ORACLE_GROUP 128

/* fp16 bit pattern -> double, exact (IEEE binary16 is a subset of binary64). */
static double half_bits_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int mant = h & 0x3ff;
    double v;
    if (expo == 0) {
        v = ldexp((double)mant, -24);              /* zero and subnormals */
    } else if (expo == 31) {
        v = mant ? NAN : INFINITY;
    } else {
        v = ldexp(1.0 + (double)mant / 1024.0, expo - 15);
    }
    return sign ? -v : v;
}

void xfp_oracle_half_to_double(const uint16_t *h, int64_t n, double *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = half_bits_to_double(h[i]);
}

/* Bit p of a row's little-endian bitstream stored as uint32 words. */
static unsigned stream_bit(const uint32_t *row_words, int64_t p)
{
    return (row_words[p / 32] >> (p % 32)) & 1u;
}

/* Field k = bits [k*b, k*b + b) of the row stream, least significant first
 * (for b = 2 and 4 this is the paper's 16 / 8 values per uint32 with value 0
 * in the low bits; for b = 3 the stream is dense, so fields cross words). */
static unsigned stream_field(const uint32_t *row_words, int64_t k, int bits)
{
    unsigned q = 0;
    for (int j = 0; j < bits; ++j) q |= stream_bit(row_words, k * bits + j) << j;
    return q;
}

void xfp_oracle_unpack(const uint32_t *words, int64_t rows, int64_t K, int bits, uint8_t *q)
{
    int64_t wpr = K * bits / 32;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t k = 0; k < K; ++k)
            q[r * K + k] = (uint8_t)stream_field(words + r * wpr, k, bits);
}

/* The word packing of 3-bit indices in the paper's packing table (section 3.3,
 * table 2): ten values per uint32, 30 bits used, 2 reserved.  Reading taken:
 * value k of a row sits in word k / 10 at bits [3 (k % 10), 3 (k % 10) + 3),
 * value 0 in the low bits as for the other widths, the reserved bits on top and
 * ignored; a row of K values takes ceil(K / 10) words, the last one part-filled. */
void xfp_oracle_unpack_word10(const uint32_t *words, int64_t rows, int64_t K, uint8_t *q)
{
    int64_t wpr = (K + 9) / 10;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t k = 0; k < K; ++k)
            q[r * K + k] = (uint8_t)((words[r * wpr + k / 10] >> (3 * (k % 10))) & 7u);
}

/* The other word forms of the same table: bits = 5, three values per uint16 (15
 * bits used, 1 reserved); bits = 6, five per uint32 (30 used, 2 reserved); bits =
 * 3 as above; bits = 2 and 4 fill their uint32 (16 and 8 values, no reserve bits).
 * Same reading: value k in word k / per at bit bits * (k % per), reserve bits on
 * top and ignored, a row takes ceil(K / per) words.  `words` is the raw byte
 * image (little-endian words).  Returns the values per word, 0 for other widths. */
int xfp_oracle_unpack_wordform(const uint8_t *words, int64_t rows, int64_t K, int bits, uint8_t *q)
{
    int per, wbytes;
    switch (bits) {
    case 2: per = 16; wbytes = 4; break;
    case 3: per = 10; wbytes = 4; break;
    case 4: per = 8; wbytes = 4; break;
    case 5: per = 3; wbytes = 2; break;
    case 6: per = 5; wbytes = 4; break;
    default: return 0;
    }
    int64_t wpr = (K + per - 1) / per;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t k = 0; k < K; ++k) {
            const uint8_t *wp = words + (r * wpr + k / per) * wbytes;
            uint32_t w = 0;
            for (int b = 0; b < wbytes; ++b) w |= (uint32_t)wp[b] << (8 * b);
            q[r * K + k] = (uint8_t)((w >> (bits * (k % per))) & ((1u << bits) - 1u));
        }
    return per;
}

void xfp_oracle_pack(const uint8_t *q, int64_t rows, int64_t K, int bits, uint32_t *words)
{
    int64_t wpr = K * bits / 32;
    memset(words, 0, (size_t)(rows * wpr) * sizeof(uint32_t));
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t k = 0; k < K; ++k)
            for (int j = 0; j < bits; ++j) {
                int64_t p = k * bits + j;
                uint32_t bit = (q[r * K + k] >> j) & 1u;
                words[r * wpr + p / 32] |= bit << (p % 32);
            }
}

/* Codebook that row n, position k selects (pointer to its 2^b fp16 entries). */
static const uint16_t *codebook_of(int mode, int bits, int64_t K, const uint16_t *codebooks,
                                   const uint8_t *group_ids, int64_t n, int64_t k)
{
    int64_t entries = (int64_t)1 << bits;
    if (mode == 0) return codebooks + n * entries;                 /* V2: per output channel */
    int64_t gpr = K / XFP_ORACLE_GROUP;                            /* V2a: library[id of the group] */
    return codebooks + (int64_t)group_ids[n * gpr + k / XFP_ORACLE_GROUP] * entries;
}

/* Bulk value at (n, k): the selected entry, mapped by the group's scale and
 * mid-point when the matrix carries them (section 3.4 names a scale and a
 * mid-point per group without a formula; reading taken: the affine map
 * entry * scale + mid, the only map two such numbers define; scale 1 and mid 0
 * give the plain library value). */
static double bulk_value(uint16_t c, int64_t K, const uint16_t *gscale, const uint16_t *gmid, int64_t n, int64_t k)
{
    double v = half_bits_to_double(c);
    if (gscale && gmid) {
        int64_t g = n * (K / XFP_ORACLE_GROUP) + k / XFP_ORACLE_GROUP;
        v = v * half_bits_to_double(gscale[g]) + half_bits_to_double(gmid[g]);
    }
    return v;
}

/* Bulk term only: selected fp16 bit patterns (the codebook entries themselves)
 * and/or the bulk values as doubles (with the group map applied, if any). */
int xfp_oracle_dequant_bulk(int mode, int bits, int64_t N, int64_t K,
                            const uint32_t *words, const uint16_t *codebooks,
                            const uint8_t *group_ids, const uint16_t *gscale, const uint16_t *gmid,
                            uint16_t *w_bits, double *w)
{
    if ((mode != 0 && mode != 1) || bits < 1 || bits > 8 || K % XFP_ORACLE_GROUP) return -1;
    int64_t wpr = K * bits / 32;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            unsigned q = stream_field(words + n * wpr, k, bits);
            uint16_t c = codebook_of(mode, bits, K, codebooks, group_ids, n, k)[q];
            if (w_bits) w_bits[n * K + k] = c;
            if (w) w[n * K + k] = bulk_value(c, K, gscale, gmid, n, k);
        }
    return 0;
}

/* y[m][n] for one matrix whose CSR rows start at row_ptr[0] (absolute offsets
 * into col/val).  x is fp16 bits [M][ldx]; y is double [M][ldy]. */
static void gemv_one_matrix(int mode, int bits, int64_t N, int64_t K,
                            const uint32_t *words, const uint16_t *codebooks,
                            const uint8_t *group_ids, const uint16_t *gscale, const uint16_t *gmid,
                            const int32_t *row_ptr,
                            const int32_t *col, const uint16_t *val,
                            const uint16_t *x, int64_t M, int64_t ldx,
                            double *y, int64_t ldy, int nthreads)
{
    int64_t wpr = K * bits / 32;
    double *xd = (double *)malloc((size_t)(M * K) * sizeof(double));
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k) xd[m * K + k] = half_bits_to_double(x[m * ldx + k]);

#ifdef _OPENMP
#pragma omp parallel num_threads(nthreads > 0 ? nthreads : 1)
#endif
    {
        double *C = (double *)malloc((size_t)K * sizeof(double));
#ifdef _OPENMP
#pragma omp for schedule(static)
#endif
        for (int64_t n = 0; n < N; ++n) {
            for (int64_t k = 0; k < K; ++k) {
                unsigned q = stream_field(words + n * wpr, k, bits);
                C[k] = bulk_value(codebook_of(mode, bits, K, codebooks, group_ids, n, k)[q], K, gscale, gmid, n, k);
            }
            for (int64_t m = 0; m < M; ++m) {
                double bulk = 0.0;
                for (int64_t k = 0; k < K; ++k) bulk += xd[m * K + k] * C[k];
                double outl = 0.0;
                for (int32_t j = row_ptr[n]; j < row_ptr[n + 1]; ++j)
                    outl += half_bits_to_double(val[j]) * xd[m * K + col[j]];
                y[m * ldy + n] = bulk + outl;
            }
        }
        free(C);
    }
    free(xd);
}

int xfp_oracle_gemv(int mode, int bits, int64_t N, int64_t K,
                    const uint32_t *words, const uint16_t *codebooks, const uint8_t *group_ids,
                    const uint16_t *gscale, const uint16_t *gmid,
                    const int32_t *row_ptr, const int32_t *col, const uint16_t *val,
                    const uint16_t *x, int64_t M, int64_t ldx, double *y, int64_t ldy,
                    int nthreads)
{
    if ((mode != 0 && mode != 1) || bits < 1 || bits > 8 || K % XFP_ORACLE_GROUP) return -1;
    if ((gscale != NULL) != (gmid != NULL) || (gscale && mode != 1)) return -1;
    gemv_one_matrix(mode, bits, N, K, words, codebooks, group_ids, gscale, gmid, row_ptr, col, val,
                    x, M, ldx, y, ldy, nthreads);
    return 0;
}

/* Expert-indexed form: slot t uses matrix expert_ids[t] of the bank and input
 * row t (or the one shared row when x_slot_stride == 0); M = 1 per slot.
 * The paper applies the same decode to routed-expert weights (section 1) and
 * gives no further launch detail; this is the grouped reading. */
int xfp_oracle_gemv_moe(int mode, int bits, int64_t N, int64_t K, int64_t L, int64_t E,
                        const uint32_t *words, const uint16_t *codebooks,
                        const uint8_t *group_ids, const uint16_t *gscale, const uint16_t *gmid,
                        const int32_t *row_ptr, const int32_t *col,
                        const uint16_t *val, const int32_t *expert_ids, int64_t T,
                        const uint16_t *x, int64_t x_slot_stride, double *y, int64_t ldy,
                        int nthreads)
{
    if ((mode != 0 && mode != 1) || bits < 1 || bits > 8 || K % XFP_ORACLE_GROUP) return -1;
    int64_t wpr = K * bits / 32, entries = (int64_t)1 << bits;
    for (int64_t t = 0; t < T; ++t) {
        int64_t e = expert_ids[t];
        if (e < 0 || e >= E) return -2;
        const uint16_t *cb = mode == 0 ? codebooks + e * N * entries : codebooks + e * L * entries;
        const uint8_t *ids = mode == 0 ? NULL : group_ids + e * N * (K / XFP_ORACLE_GROUP);
        const uint16_t *gs = gscale ? gscale + e * N * (K / XFP_ORACLE_GROUP) : NULL;
        const uint16_t *gm = gmid ? gmid + e * N * (K / XFP_ORACLE_GROUP) : NULL;
        gemv_one_matrix(mode, bits, N, K, words + e * N * wpr, cb, ids, gs, gm, row_ptr + e * N, col, val,
                        x + t * x_slot_stride, 1, K, y + t * ldy, ldy, nthreads);
    }
    return 0;
}

int xfp_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
