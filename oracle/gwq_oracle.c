/*
 * CPU oracle for the GWQ linear-layer hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain statement of what the GPU library must compute.  It is
 * used by the tests, by the smoke check and by the benchmark's CPU-baseline leg; the
 * product path never calls it and shares no code with it.
 *
 * Source: "Gradient-Aware Weight Quantization for Large Language Models" (GWQ),
 * Sec. 3.2 "Gradient Aware Quantization":
 *   Eq. 6  scale       s = (max W - min W) / (number of steps)
 *   Eq. 7  zero point  z = -min W / s
 *   Eq. 8  outliers    O = 1(|W_grad| >= quantile): the largest 1 % of |gradient| stay FP16
 *   Eq. 9  quantise    q = round(W / s) + z        (non-outliers only)
 *   Eq. 10 dequantise  Q(W) = s * (q - z)
 * and the layer it serves, y = x * (Q(W) + outliers)^T, with no bias (Sec. 3.1 disables it);
 * and Sec. 3.1 for the two figures of merit of a packed layer:
 *   Eq. 4  squared error           || W - W_Q ||^2
 *   Eq. 3, 5  first-order change   g^T (W - W_Q) of the loss (its Taylor expansion around W)
 * and for the score itself, Eq. 2: g = grad_W L.  For one linear layer Y = X W^T the chain rule
 * gives g[n][k] = sum_m (dL/dY)[m][n] * X[m][k]; the mean over calibration samples (Sec. 4.3, ablation on the number of calibration samples)
 * is a scaled accumulation of that.
 *
 * Readings taken where the text is silent or garbled (each is also listed in the design
 * notes of the repository):
 *   - Eq. 6 prints 2^(b-1) in the denominator; the quantiser is called round-to-nearest
 *     min-max (caption of the first table), so the number of steps is maxq = 2^b - 1.
 *   - z is rounded to an integer, z and q are clamped to [0, maxq].
 *   - round() is round-half-to-even.
 *   - the scale is stored as FP16, the smallest FP16 value s with s*maxq >= range, so that
 *     the top code never clips.
 *   - min/max run over the non-outlier members of a group and are widened to contain 0.
 *   - exactly ceil(ppm * N * K / 1e6) outliers per matrix; ties on |score| go to the lowest
 *     flat index n*K + k.
 *   - the code stored under an outlier is z (it decodes to 0), so "add" and "replace" agree.
 *
 * Parity pins (tests marked "not gpu"): selection against a full lexicographic sort in numpy,
 * scale against an exhaustive search over every FP16 value with exact rationals, zero point
 * and codes against exact-rational rounding, the |w - Q(w)| <= s/2 bound, the special cases
 * ppm = 0 (plain group-wise RTN) and ppm = 1e6 (y = x W^T by numpy's fp64 matmul), word
 * layouts against hand-assembled words, the linear map against numpy on decoded weights, and
 * the figures of merit against exact rationals on the hand-worked groups.
 * Parity with the paper's model-level results (perplexity, accuracy, the 1.2x speedup) is
 * parity unpinned: it needs the models and datasets, which are not available.
 *
 * Build:  gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC gwq_oracle.c -o libgwq_oracle.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define GWQ_ORACLE_OK 0
#define GWQ_ORACLE_BAD_ARG (-1)
#define GWQ_ORACLE_NO_MEM (-2)

/* ---------------------------------------------------------------- FP16 <-> FP64 ---- */

/* Exact value of an IEEE binary16 bit pattern. */
double gwq_oracle_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1F;
    int f = h & 0x3FF;
    double v;
    if (e == 0)
        v = ldexp((double)f, -24);               /* zero and subnormals            */
    else if (e == 31)
        v = f ? NAN : INFINITY;
    else
        v = ldexp((double)(f | 0x400), e - 25);  /* 1.f * 2^(e-15)                 */
    return sign ? -v : v;
}

/* Nearest binary16 (ties to even) of a finite non-negative double; overflow gives +inf. */
static uint16_t double_to_half_nonneg(double x)
{
    if (!(x > 0.0)) return 0;
    if (x >= 65520.0) return 0x7C00;             /* halfway between 65504 and 2^16 */
    int e;
    (void)frexp(x, &e);                          /* x = m * 2^e, m in [0.5, 1)     */
    int q = e - 11;                              /* ulp exponent for a normal      */
    if (q < -24) q = -24;                        /* subnormal grid                 */
    double scaled = ldexp(x, -q);                /* exact: power-of-two scaling    */
    double r = rint(scaled);                     /* ties to even                   */
    /* r is an integer in [0, 2048]; value = r * 2^q.  Re-encode through the exact decoder. */
    uint16_t lo = 0, hi = 0x7C00;
    while (lo < hi) {                            /* smallest pattern with value >= r*2^q */
        uint16_t mid = (uint16_t)((lo + hi) / 2);
        if (gwq_oracle_half_to_double(mid) < ldexp(r, q)) lo = (uint16_t)(mid + 1); else hi = mid;
    }
    return lo;
}

/* ---------------------------------------------------------------- outlier count ---- */

/* ceil(ppm * N * K / 1e6): "the largest 1 %" (Eq. 8) as an exact count, ppm = 10000. */
int64_t gwq_oracle_outlier_count(int64_t N, int64_t K, uint32_t ppm)
{
    return ((int64_t)ppm * N * K + 999999) / 1000000;
}

/* ---------------------------------------------------------------- selection -------- */

/* Ranking key of a score: the bit pattern of |score| as binary32.  It orders all
 * non-NaN magnitudes like the reals, treats -0 as +0 and puts NaN above +inf. */
static uint32_t key_of_f32(uint32_t bits) { return bits & 0x7FFFFFFFu; }

static uint32_t half_bits_to_float_bits(uint16_t h)
{
    float f = (float)gwq_oracle_half_to_double(h);   /* exact: every binary16 is a binary32 */
    uint32_t b;
    if (((h >> 10) & 0x1F) == 31 && (h & 0x3FF)) {   /* NaN: keep it a NaN with its payload */
        b = 0x7F800000u | ((uint32_t)(h & 0x3FF) << 13) | ((uint32_t)(h >> 15) << 31);
        return b;
    }
    memcpy(&b, &f, 4);
    return b;
}

static int cmp_u64_desc(const void *a, const void *b)
{
    uint64_t x = *(const uint64_t *)a, y = *(const uint64_t *)b;
    return (x < y) - (x > y);
}

/* Eq. 8 with an exact count: order all entries by (|score| descending, flat index
 * ascending) and mark the first k_out.  mask[n*K+k] = 1 for an outlier, else 0.
 * score_is_f16: 0 = binary32 scores, 1 = binary16 scores. */
int gwq_oracle_select(const void *score, int score_is_f16, int64_t N, int64_t K,
                      uint32_t ppm, uint8_t *mask)
{
    if (!score || !mask || N <= 0 || K <= 0 || ppm > 1000000u) return GWQ_ORACLE_BAD_ARG;
    int64_t total = N * K;
    if (total > (int64_t)0xFFFFFFFF) return GWQ_ORACLE_BAD_ARG;
    int64_t k_out = gwq_oracle_outlier_count(N, K, ppm);
    uint64_t *order = (uint64_t *)malloc((size_t)total * sizeof(uint64_t));
    if (!order) return GWQ_ORACLE_NO_MEM;
    for (int64_t i = 0; i < total; ++i) {
        uint32_t bits = score_is_f16 ? half_bits_to_float_bits(((const uint16_t *)score)[i])
                                     : ((const uint32_t *)score)[i];
        /* Descending sort of this composite = key descending, then flat index ascending. */
        order[i] = ((uint64_t)key_of_f32(bits) << 32) | (uint64_t)(0xFFFFFFFFu - (uint32_t)i);
    }
    qsort(order, (size_t)total, sizeof(uint64_t), cmp_u64_desc);
    memset(mask, 0, (size_t)total);
    for (int64_t r = 0; r < k_out; ++r) {
        uint32_t idx = 0xFFFFFFFFu - (uint32_t)(order[r] & 0xFFFFFFFFu);
        mask[idx] = 1;
    }
    free(order);
    return GWQ_ORACLE_OK;
}

/* ---------------------------------------------------------------- CSR of outliers -- */

/* Outliers keep their FP16 bit pattern (abstract and Sec. 1: outliers stay at FP16).
 * Rows in order, columns ascending within a row. */
int gwq_oracle_csr(const uint16_t *W, const uint8_t *mask, int64_t N, int64_t K,
                   int32_t *row_ptr, uint16_t *col_idx, uint16_t *out_val)
{
    if (!W || !mask || !row_ptr || N <= 0 || K <= 0 || K > 65536) return GWQ_ORACLE_BAD_ARG;
    int64_t pos = 0;
    for (int64_t n = 0; n < N; ++n) {
        row_ptr[n] = (int32_t)pos;
        for (int64_t k = 0; k < K; ++k)
            if (mask[n * K + k]) {
                col_idx[pos] = (uint16_t)k;
                out_val[pos] = W[n * K + k];
                ++pos;
            }
    }
    row_ptr[N] = (int32_t)pos;
    return GWQ_ORACLE_OK;
}

/* ---------------------------------------------------------------- one group -------- */

/* Quantise one group of `len` consecutive weights of one output channel (Eq. 6, 7, 9).
 * w: FP16 bit patterns; mask: 1 = outlier (excluded from min/max, gets code z).
 * Outputs: scale as FP16 bits, zero point, one code per member. */
int gwq_oracle_quant_group(const uint16_t *w, const uint8_t *mask, int len, int bits,
                           uint16_t *scale_out, uint8_t *zero_out, uint8_t *codes)
{
    if (!w || !mask || !scale_out || !zero_out || !codes || len <= 0 || (bits != 3 && bits != 4))
        return GWQ_ORACLE_BAD_ARG;
    const int maxq = (1 << bits) - 1;
    double mn = 0.0, mx = 0.0;                    /* range always contains 0        */
    for (int i = 0; i < len; ++i) {
        if (mask[i]) continue;
        double v = gwq_oracle_half_to_double(w[i]);
        if (v < mn) mn = v;
        if (v > mx) mx = v;
    }
    double R = mx - mn;                           /* exact: both are multiples of 2^-24 below 2^17 */
    uint16_t s_bits;
    int z;
    if (R == 0.0) {
        s_bits = 0x3C00;                          /* 1.0 */
        z = 0;
    } else {
        /* Eq. 6 with maxq steps, stored as the smallest FP16 s such that s*maxq >= R. */
        s_bits = double_to_half_nonneg(R / maxq);
        if (s_bits == 0) s_bits = 1;
        while (s_bits < 0x7BFF && gwq_oracle_half_to_double(s_bits) * maxq < R) ++s_bits;
        while (s_bits > 1 && gwq_oracle_half_to_double((uint16_t)(s_bits - 1)) * maxq >= R) --s_bits;
        double s = gwq_oracle_half_to_double(s_bits);
        /* Eq. 7, rounded half-to-even and clamped. */
        double zr = rint(-mn / s);
        z = !(zr > 0.0) ? 0 : (zr > maxq ? maxq : (int)zr);   /* NaN (non-finite weights) -> 0 */
    }
    double s = gwq_oracle_half_to_double(s_bits);
    for (int i = 0; i < len; ++i) {
        if (mask[i]) { codes[i] = (uint8_t)z; continue; }
        /* Eq. 9, clamped to the code range. */
        double qr = rint(gwq_oracle_half_to_double(w[i]) / s) + z;
        int q = !(qr > 0.0) ? 0 : (qr > maxq ? maxq : (int)qr);
        codes[i] = (uint8_t)q;
    }
    *scale_out = s_bits;
    *zero_out = (uint8_t)z;
    return GWQ_ORACLE_OK;
}

/* ---------------------------------------------------------------- word layout ------ */

/* Packed layout of one group of 128 codes (k_local = 0..127), as 32-bit words.
 *
 * The group is cut into four slots of 32 consecutive codes, slot b = k_local / 32.
 * Inside a word, codes with an even position sit in the low 16 bits and codes with an odd
 * position in the high 16 bits, `bits` bits apiece, ascending.
 *
 * 4-bit: 16 words; word 4b+j (j = 0..3) holds codes 32b+8j+t, t = 0..7:
 *        t even -> bit 4*(t/2), t odd -> bit 16 + 4*(t/2).
 * 3-bit: 13 words; word 3b+i (i = 0..2) holds codes 32b+10i+t, t = 0..9:
 *        t even -> bit 3*(t/2), t odd -> bit 16 + 3*(t/2); bits 15 and 31 are zero.
 *        Word 12 (the tail) holds the last two codes of every slot:
 *        code 32b+30 -> bit 3b, code 32b+31 -> bit 16 + 3b; all other bits are zero.
 */
#define GWQ_GROUP 128   /* codes per block of the word layout */

/* The quantisation group (Sec. 3.2, first paragraph: scale and zero point are per group of beta weights of an
 * output channel along the input dimension; the paper sets beta = 16) is 16, 32, 64 or 128: a whole number of
 * groups per 128-code block of the word layout, which does not depend on it. */
static int group_ok(int group) { return group == 16 || group == 32 || group == 64 || group == 128; }

static int words_per_group(int bits) { return bits == 4 ? 16 : 13; }

static void pack_group(const uint8_t *c, int bits, uint32_t *out)
{
    int nw = words_per_group(bits);
    for (int j = 0; j < nw; ++j) out[j] = 0;
    for (int kl = 0; kl < GWQ_GROUP; ++kl) {
        int b = kl / 32, r = kl % 32;
        int word, t, shift;
        if (bits == 4) {
            word = 4 * b + r / 8;
            t = r % 8;
            shift = (t % 2 ? 16 : 0) + 4 * (t / 2);
        } else if (r < 30) {
            word = 3 * b + r / 10;
            t = r % 10;
            shift = (t % 2 ? 16 : 0) + 3 * (t / 2);
        } else {
            word = 12;
            shift = (r == 31 ? 16 : 0) + 3 * b;
        }
        out[word] |= (uint32_t)c[kl] << shift;
    }
}

static void unpack_group(const uint32_t *in, int bits, uint8_t *c)
{
    uint32_t m = (1u << bits) - 1u;
    for (int kl = 0; kl < GWQ_GROUP; ++kl) {
        int b = kl / 32, r = kl % 32;
        int word, t, shift;
        if (bits == 4) {
            word = 4 * b + r / 8;
            t = r % 8;
            shift = (t % 2 ? 16 : 0) + 4 * (t / 2);
        } else if (r < 30) {
            word = 3 * b + r / 10;
            t = r % 10;
            shift = (t % 2 ? 16 : 0) + 3 * (t / 2);
        } else {
            word = 12;
            shift = (r == 31 ? 16 : 0) + 3 * b;
        }
        c[kl] = (uint8_t)((in[word] >> shift) & m);
    }
}

int gwq_oracle_pack_codes(const uint8_t *codes, int64_t N, int64_t K, int bits, uint32_t *qweight)
{
    if (!codes || !qweight || N <= 0 || K <= 0 || K % GWQ_GROUP || (bits != 3 && bits != 4))
        return GWQ_ORACLE_BAD_ARG;
    int nw = words_per_group(bits);
    int64_t groups = N * (K / GWQ_GROUP);
    for (int64_t g = 0; g < groups; ++g) pack_group(codes + g * GWQ_GROUP, bits, qweight + g * nw);
    return GWQ_ORACLE_OK;
}

int gwq_oracle_unpack_codes(const uint32_t *qweight, int64_t N, int64_t K, int bits, uint8_t *codes)
{
    if (!codes || !qweight || N <= 0 || K <= 0 || K % GWQ_GROUP || (bits != 3 && bits != 4))
        return GWQ_ORACLE_BAD_ARG;
    int nw = words_per_group(bits);
    int64_t groups = N * (K / GWQ_GROUP);
    for (int64_t g = 0; g < groups; ++g) unpack_group(qweight + g * nw, bits, codes + g * GWQ_GROUP);
    return GWQ_ORACLE_OK;
}

/* ---------------------------------------------------------------- gwq_pack twin ---- */

/* Everything after the selection: CSR of the marked entries, then per (row, group of `group`
 * consecutive weights along K) scale, zero, codes (Eq. 6, 7, 9), and the word layout above per
 * block of 128 codes.  `mask` is the outlier indicator [N*K]; col_idx/out_val must hold as many
 * entries as the mask marks; scales/zeros are [N][K/group]. */
int gwq_oracle_encode(const uint16_t *W, const uint8_t *mask, int64_t N, int64_t K, int bits, int group,
                      uint32_t *qweight, uint16_t *scales, uint8_t *zeros,
                      int32_t *row_ptr, uint16_t *col_idx, uint16_t *out_val)
{
    if (!W || !mask || !qweight || !scales || !zeros || !row_ptr) return GWQ_ORACLE_BAD_ARG;
    if (N <= 0 || K <= 0 || K % GWQ_GROUP || K > 65536 || (bits != 3 && bits != 4) || !group_ok(group))
        return GWQ_ORACLE_BAD_ARG;
    int rc = gwq_oracle_csr(W, mask, N, K, row_ptr, col_idx, out_val);
    int nw = words_per_group(bits);
    int64_t bpr = K / GWQ_GROUP, gpr = K / group;       /* blocks and groups per row */
    uint8_t codes[GWQ_GROUP];
    for (int64_t n = 0; n < N && rc == GWQ_ORACLE_OK; ++n)
        for (int64_t blk = 0; blk < bpr && rc == GWQ_ORACLE_OK; ++blk) {
            for (int64_t k = blk * GWQ_GROUP; k < (blk + 1) * GWQ_GROUP && rc == GWQ_ORACLE_OK; k += group)
                rc = gwq_oracle_quant_group(W + n * K + k, mask + n * K + k, group, bits,
                                            &scales[n * gpr + k / group], &zeros[n * gpr + k / group],
                                            codes + (k - blk * GWQ_GROUP));
            pack_group(codes, bits, qweight + (n * bpr + blk) * nw);
        }
    return rc;
}

/* Whole encoding: selection (Eq. 8) followed by gwq_oracle_encode.
 * Output sizes: qweight N*(K/128)*wpg words, scales/zeros N*(K/group), row_ptr N+1,
 * col_idx/out_val k_out = gwq_oracle_outlier_count(N, K, ppm).
 * mask_out (optional, N*K bytes) receives the outlier indicator. */
int gwq_oracle_pack(const uint16_t *W, const void *score, int score_is_f16,
                    int64_t N, int64_t K, int bits, int group, uint32_t ppm,
                    uint32_t *qweight, uint16_t *scales, uint8_t *zeros,
                    int32_t *row_ptr, uint16_t *col_idx, uint16_t *out_val, uint8_t *mask_out)
{
    if (!W || !score || N <= 0 || K <= 0) return GWQ_ORACLE_BAD_ARG;
    uint8_t *mask = mask_out ? mask_out : (uint8_t *)malloc((size_t)(N * K));
    if (!mask) return GWQ_ORACLE_NO_MEM;
    int rc = gwq_oracle_select(score, score_is_f16, N, K, ppm, mask);
    if (rc == GWQ_ORACLE_OK)
        rc = gwq_oracle_encode(W, mask, N, K, bits, group, qweight, scales, zeros, row_ptr, col_idx, out_val);
    if (!mask_out) free(mask);
    return rc;
}

/* ---------------------------------------------------------------- decode + linear -- */

/* Decoded row n of the layer's weight in fp64: Eq. 10 for the codes, plus the FP16
 * outliers of that row (the code under an outlier decodes to 0). */
static void decode_row(int64_t n, int64_t K, int bits, int group, const uint32_t *qweight,
                       const uint16_t *scales, const uint8_t *zeros, const int32_t *row_ptr,
                       const uint16_t *col_idx, const uint16_t *out_val, double *w_hat)
{
    int nw = words_per_group(bits);
    int64_t bpr = K / GWQ_GROUP, gpr = K / group;
    uint8_t codes[GWQ_GROUP];
    for (int64_t blk = 0; blk < bpr; ++blk) {
        unpack_group(qweight + (n * bpr + blk) * nw, bits, codes);
        for (int i = 0; i < GWQ_GROUP; ++i) {
            int64_t k = blk * GWQ_GROUP + i;
            double s = gwq_oracle_half_to_double(scales[n * gpr + k / group]);
            int z = zeros[n * gpr + k / group];
            w_hat[k] = s * (double)(codes[i] - z);
        }
    }
    for (int32_t j = row_ptr[n]; j < row_ptr[n + 1]; ++j)
        w_hat[col_idx[j]] += gwq_oracle_half_to_double(out_val[j]);
}

int gwq_oracle_decode(int64_t N, int64_t K, int bits, int group, const uint32_t *qweight,
                      const uint16_t *scales, const uint8_t *zeros, const int32_t *row_ptr,
                      const uint16_t *col_idx, const uint16_t *out_val, double *W_hat)
{
    if (!qweight || !scales || !zeros || !row_ptr || !W_hat) return GWQ_ORACLE_BAD_ARG;
    if (N <= 0 || K <= 0 || K % GWQ_GROUP || (bits != 3 && bits != 4) || !group_ok(group)) return GWQ_ORACLE_BAD_ARG;
    for (int64_t n = 0; n < N; ++n)
        decode_row(n, K, bits, group, qweight, scales, zeros, row_ptr, col_idx, out_val, W_hat + n * K);
    return GWQ_ORACLE_OK;
}

/* Y[m, j] = sum_k X[m, k] * W_hat[rows[j], k] in fp64, k ascending; Y is [M][n_rows].
 * rows == NULL means rows 0..n_rows-1 (n_rows = N gives the full product Y[M][N]). */
static int linear_checked(int64_t N, int64_t K, int bits, int group, const uint32_t *qweight,
                          const uint16_t *scales, const uint8_t *zeros, const int32_t *row_ptr,
                          const uint16_t *col_idx, const uint16_t *out_val,
                          const double *Xd, int64_t M, const int32_t *rows, int64_t n_rows,
                          double *Y);

int gwq_oracle_linear_f64(int64_t N, int64_t K, int bits, int group, const uint32_t *qweight,
                          const uint16_t *scales, const uint8_t *zeros, const int32_t *row_ptr,
                          const uint16_t *col_idx, const uint16_t *out_val,
                          const uint16_t *X, int64_t M, const int32_t *rows, int64_t n_rows,
                          double *Y)
{
    if (!X || M <= 0 || K <= 0) return GWQ_ORACLE_BAD_ARG;
    double *Xd = (double *)malloc((size_t)(M * K) * sizeof(double));
    if (!Xd) return GWQ_ORACLE_NO_MEM;
    for (int64_t i = 0; i < M * K; ++i) Xd[i] = gwq_oracle_half_to_double(X[i]);
    int rc = linear_checked(N, K, bits, group, qweight, scales, zeros, row_ptr, col_idx, out_val, Xd, M, rows, n_rows, Y);
    free(Xd);
    return rc;
}

/* The same product for activations given as fp64 values (any 16-bit type widens to fp64 exactly; the caller
 * widens): the method fixes the weights' format, not the activations' (Sec. 3.2 quantises W only). */
int gwq_oracle_linear_f64_x(int64_t N, int64_t K, int bits, int group, const uint32_t *qweight,
                            const uint16_t *scales, const uint8_t *zeros, const int32_t *row_ptr,
                            const uint16_t *col_idx, const uint16_t *out_val,
                            const double *Xd, int64_t M, const int32_t *rows, int64_t n_rows,
                            double *Y)
{
    if (!Xd) return GWQ_ORACLE_BAD_ARG;
    return linear_checked(N, K, bits, group, qweight, scales, zeros, row_ptr, col_idx, out_val, Xd, M, rows, n_rows, Y);
}

static int linear_checked(int64_t N, int64_t K, int bits, int group, const uint32_t *qweight,
                          const uint16_t *scales, const uint8_t *zeros, const int32_t *row_ptr,
                          const uint16_t *col_idx, const uint16_t *out_val,
                          const double *Xd, int64_t M, const int32_t *rows, int64_t n_rows,
                          double *Y)
{
    if (!qweight || !scales || !zeros || !row_ptr || !Xd || !Y) return GWQ_ORACLE_BAD_ARG;
    if (N <= 0 || K <= 0 || K % GWQ_GROUP || M <= 0 || n_rows < 0 || (bits != 3 && bits != 4) || !group_ok(group))
        return GWQ_ORACLE_BAD_ARG;
    if (rows)
        for (int64_t j = 0; j < n_rows; ++j)
            if (rows[j] < 0 || rows[j] >= N) return GWQ_ORACLE_BAD_ARG;
    if (!rows && n_rows > N) return GWQ_ORACLE_BAD_ARG;
    int failed = 0;
#pragma omp parallel
    {
        double *w_hat = (double *)malloc((size_t)K * sizeof(double));
        if (!w_hat) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for schedule(static)
            for (int64_t j = 0; j < n_rows; ++j) {
                int64_t n = rows ? rows[j] : j;
                decode_row(n, K, bits, group, qweight, scales, zeros, row_ptr, col_idx, out_val, w_hat);
                for (int64_t m = 0; m < M; ++m) {
                    double acc = 0.0;
                    for (int64_t k = 0; k < K; ++k) acc += Xd[m * K + k] * w_hat[k];
                    Y[m * n_rows + j] = acc;
                }
            }
        }
        free(w_hat);
    }
    return failed ? GWQ_ORACLE_NO_MEM : GWQ_ORACLE_OK;
}

/* ---------------------------------------------------------------- figures of merit -- */

/* Sec. 3.1: with W_Q the decoded layer (Eq. 10 plus the FP16 outliers) and D = W - W_Q,
 *   out[0] = sum D^2          (Eq. 4: what the quantiser minimises)
 *   out[1] = sum score * D    (Eq. 3 and 5: g^T (W - W_Q), the first-order change of the loss
 *                              when `score` is the gradient g)
 *   out[2] = max |D|
 * Every D is computed in fp64 from exact operands; the sums run in fp64 over n, then k, ascending. */
int gwq_oracle_quality(int64_t N, int64_t K, int bits, int group, const uint32_t *qweight,
                       const uint16_t *scales, const uint8_t *zeros, const int32_t *row_ptr,
                       const uint16_t *col_idx, const uint16_t *out_val,
                       const uint16_t *W, const void *score, int score_is_f16, double *out)
{
    if (!qweight || !scales || !zeros || !row_ptr || !W || !score || !out) return GWQ_ORACLE_BAD_ARG;
    if (N <= 0 || K <= 0 || K % GWQ_GROUP || (bits != 3 && bits != 4) || !group_ok(group)) return GWQ_ORACLE_BAD_ARG;
    double *w_hat = (double *)malloc((size_t)K * sizeof(double));
    if (!w_hat) return GWQ_ORACLE_NO_MEM;
    double sq = 0.0, first = 0.0, mx = 0.0;
    for (int64_t n = 0; n < N; ++n) {
        decode_row(n, K, bits, group, qweight, scales, zeros, row_ptr, col_idx, out_val, w_hat);
        for (int64_t k = 0; k < K; ++k) {
            double d = gwq_oracle_half_to_double(W[n * K + k]) - w_hat[k];
            double g = score_is_f16 ? gwq_oracle_half_to_double(((const uint16_t *)score)[n * K + k])
                                    : (double)((const float *)score)[n * K + k];
            sq += d * d;
            first += g * d;
            if (fabs(d) > mx) mx = fabs(d);
        }
    }
    free(w_hat);
    out[0] = sq; out[1] = first; out[2] = mx;
    return GWQ_ORACLE_OK;
}

/* ---------------------------------------------------------------- gated pair of the MLP -- */

/* The layers the paper quantises sit in decoder blocks whose MLP is down(silu(gate(x)) * up(x)); its
 * efficiency table (Sec. 4.2) times generation through all of them.  Given the two products G = X Wg^T and
 * U = X Wu^T (as gwq_oracle_linear_f64 returns them), H[i] = silu(G[i]) * U[i] with
 * silu(x) = x / (1 + exp(-x)), in fp64, element by element. */
int gwq_oracle_gate_up(const double *G, const double *U, int64_t count, double *H)
{
    if (!G || !U || !H || count < 0) return GWQ_ORACLE_BAD_ARG;
    for (int64_t i = 0; i < count; ++i) H[i] = G[i] / (1.0 + exp(-G[i])) * U[i];
    return GWQ_ORACLE_OK;
}

/* ---------------------------------------------------------------- score production -- */

/* Eq. 2 for one linear layer Y = X W^T (no bias, Sec. 3.1): the gradient of the loss with respect to
 * W, given the gradient dY[M][N] of the loss with respect to Y and the layer's input X[M][K], is
 *   g[n][k] = sum_m dY[m][n] * X[m][k]          (chain rule; m ascending, fp64, products exact)
 * and out[n][k] = beta * prev[n][k] + alpha * g[n][k]: with alpha = 1 / samples, beta = 0 for the
 * first sample and 1 afterwards this is the mean gradient over calibration samples (Sec. 4.3, ablation on the number of calibration samples).
 * prev may be NULL when beta == 0. */
int gwq_oracle_score(const uint16_t *dY, const uint16_t *X, int64_t M, int64_t N, int64_t K,
                     double alpha, double beta, const float *prev, double *out)
{
    if (!dY || !X || !out || (beta != 0.0 && !prev)) return GWQ_ORACLE_BAD_ARG;
    if (M <= 0 || N <= 0 || K <= 0) return GWQ_ORACLE_BAD_ARG;
#pragma omp parallel for schedule(static)           /* rows are independent; each sum keeps its order */
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            double g = 0.0;
            for (int64_t m = 0; m < M; ++m)
                g += gwq_oracle_half_to_double(dY[m * N + n]) * gwq_oracle_half_to_double(X[m * K + k]);
            out[n * K + k] = (beta != 0.0 ? beta * (double)prev[n * K + k] : 0.0) + alpha * g;
        }
    return GWQ_ORACLE_OK;
}
