/*
 * bdr_ref.c -- CPU oracle for the BDR / shared-microexponent quantizer.
 *
 * TEST INFRASTRUCTURE ONLY (see bdr_ref.h).  Plain C99, one element at a time,
 * integer arithmetic on FP32 bit patterns for everything that decides a code,
 * fp64 for the QSNR sums and the GEMM.  No blocking, no fusion, no threads.
 *
 * The method is a deterministic encoding, so this file takes the steps in the
 * order the paper gives them (Sec. IX, proof of Theorem 1):
 *
 *   step 1  private exponent of every element            (Eq. "max_exp")
 *   step 2  shared exponent E = exponent of the block max (text after "max_exp")
 *   step 3  sub-block shift tau                           (Eq. "q_error_max-1" and
 *                                                          the paragraph after "q_error_all")
 *   step 4  magnitude rounded to m bits at weight 2^(E-tau) (Eq. "max_exp_round")
 *   step 5  packing into (m+1) + d1/k1 + d2/k2 bits/element (Sec. III)
 *   step 6  descaling                                     (Sec. II, "descaling step")
 *   step 7  QSNR                                          (Sec. IV-A, Eq. 3)
 *
 * Readings taken where the paper is silent (each is a choice, not a quotation):
 *
 *   R1  m counts the stored magnitude bits; the top one has weight 2^(E-tau).
 *       There is no implicit leading one.  (Eq. "max_exp_round" sums j=0..m-1;
 *       the footnote in Sec. III says the implicit bit belongs to scalar FP.)
 *   R2  "nearest" is nearest, ties to even magnitude, unless the format asks
 *       for ties-away (RNA) or truncation (RTZ).
 *   R3  A magnitude that rounds up to 2^m is held at 2^m - 1; E is not bumped,
 *       so E stays the exponent of the block maximum and Q(Q(x)) = Q(x).
 *   R4  tau is subtracted from E; a sub-block more than beta binades below the
 *       block maximum gets tau = beta.
 *   R5  An FP32 exponent field of 0 (zero or subnormal) counts as 1, which is
 *       the true exponent -126 of subnormals; the significand then has no
 *       implicit one.  An all-zero block gets the exponent code 1.
 *   R6  Exponent field 255 (Inf/NaN) counts as 254 and the magnitude saturates
 *       at 2^m - 1 with the sign kept.  Outside the supported domain.
 *   R7  The sign bit is copied from the input even when the magnitude is 0.
 *   R8  A row whose length is not a multiple of k1 is padded with +0 to the
 *       next multiple; pads are stored (as code 0).  (End of Sec. IX: a vector
 *       shorter than k1 behaves as a smaller block.)
 *   R9  Only d1 = 8 is implemented (Theorem 1 fixes d1 = 8): the shared
 *       exponent code is the biased FP32 exponent itself.
 *   R10 log in Eq. 3 is log10 (the proof turns 10 m log 4 into 6.02 m), and the
 *       expectation is taken as the ratio of the two sums over the whole tensor.
 *   R11 Packed image, three planes, each a little-endian bit stream (bit b of
 *       the stream is bit b%8 of byte b/8):
 *         codes: element t = r * Cp + c holds bits [t(m+1), (t+1)(m+1)), the
 *                magnitude in the low m bits and the sign above it;
 *         sexp : one byte per block, block index r * (Cp/k1) + c / k1;
 *         mexp : sub-block u = r * (Cp/k2) + c / k2 holds bits [u d2, (u+1) d2);
 *       Cp is the row length rounded up to a multiple of k1.
 *   R12 Quantizing along columns is quantizing the transposed tensor along its
 *       rows, plane indices included (Sec. V: transpose first, then quantize).
 */
#include "bdr_ref.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

#define BDR_REF_MAX_K1 4096

/* ------------------------------------------------------------------ helpers */

static int is_pow2(int32_t v) { return v > 0 && (v & (v - 1)) == 0; }

static uint32_t bits_of_float(float v)
{
    uint32_t b;
    memcpy(&b, &v, sizeof b);
    return b;
}

static float float_of_bits(uint32_t b)
{
    float v;
    memcpy(&v, &b, sizeof v);
    return v;
}

/* FP32 bit pattern of element idx of a buffer of the given dtype.  BF16 is the
 * upper half of an FP32, so widening is exact. */
static uint32_t load_bits(const void *x, int dtype, int64_t idx)
{
    if (dtype == BDR_REF_BF16)
        return (uint32_t)((const uint16_t *)x)[idx] << 16;
    return ((const uint32_t *)x)[idx];
}

static void store_value(void *y, int dtype, int64_t idx, double v)
{
    uint32_t b = bits_of_float((float)v); /* exact, see bdr_ref_decode */
    if (dtype == BDR_REF_BF16)
        ((uint16_t *)y)[idx] = (uint16_t)(b >> 16);
    else
        ((uint32_t *)y)[idx] = b;
}

/* step 1: private exponent, as the biased FP32 field, with R5 and R6. */
static int private_exponent(uint32_t bits)
{
    int e = (int)((bits >> 23) & 0xFFu);
    if (e < 1) e = 1;
    if (e > 254) e = 254;
    return e;
}

static void put_bits(uint8_t *buf, uint64_t bitpos, int nbits, uint32_t value)
{
    for (int i = 0; i < nbits; ++i) {
        uint64_t p = bitpos + (uint64_t)i;
        uint8_t mask = (uint8_t)(1u << (p & 7u));
        if ((value >> i) & 1u)
            buf[p >> 3] |= mask;
        else
            buf[p >> 3] &= (uint8_t)~mask;
    }
}

static uint32_t get_bits(const uint8_t *buf, uint64_t bitpos, int nbits)
{
    uint32_t v = 0;
    for (int i = 0; i < nbits; ++i) {
        uint64_t p = bitpos + (uint64_t)i;
        v |= (uint32_t)((buf[p >> 3] >> (p & 7u)) & 1u) << i;
    }
    return v;
}

/* ------------------------------------------------------------------- format */

int bdr_ref_format_validate(const bdr_ref_format *f)
{
    if (!f) return BDR_REF_ERR_NULL;
    if (!is_pow2(f->k1) || f->k1 > BDR_REF_MAX_K1) return BDR_REF_ERR_FORMAT;
    if (!is_pow2(f->k2) || f->k2 > f->k1) return BDR_REF_ERR_FORMAT;
    if (f->d1 != 8) return BDR_REF_ERR_FORMAT; /* R9 */
    if (f->d2 < 0 || f->d2 > 3) return BDR_REF_ERR_FORMAT;
    if (f->m < 1 || f->m > 8) return BDR_REF_ERR_FORMAT;
    if (f->rounding != BDR_REF_RNE && f->rounding != BDR_REF_RNA && f->rounding != BDR_REF_RTZ)
        return BDR_REF_ERR_FORMAT;
    return BDR_REF_OK;
}

double bdr_ref_bits_per_element(const bdr_ref_format *f)
{
    return (double)(f->m + 1) + (double)f->d1 / (double)f->k1 + (double)f->d2 / (double)f->k2;
}

/* Logical view used by everything below: the tensor as [R x C] with blocks
 * along C.  For AXIS_ROW that is the tensor itself, for AXIS_COL its
 * transpose (R12).  Element (r, c) of the view sits at r*sr + c*sc. */
typedef struct {
    int64_t R, C, Cp, sr, sc;
} view_t;

static view_t make_view(const bdr_ref_format *f, int64_t rows, int64_t cols, int64_t ld, int axis)
{
    view_t v;
    if (axis == BDR_REF_AXIS_COL) {
        v.R = cols; v.C = rows; v.sr = 1; v.sc = ld;
    } else {
        v.R = rows; v.C = cols; v.sr = ld; v.sc = 1;
    }
    v.Cp = (v.C + f->k1 - 1) / f->k1 * f->k1; /* R8 */
    return v;
}

int bdr_ref_packed_sizes(const bdr_ref_format *f, int64_t rows, int64_t cols, int axis,
                         size_t *codes_bytes, size_t *sexp_bytes, size_t *mexp_bytes)
{
    int st = bdr_ref_format_validate(f);
    if (st) return st;
    if (rows < 0 || cols < 0) return BDR_REF_ERR_SHAPE;
    if (axis != BDR_REF_AXIS_ROW && axis != BDR_REF_AXIS_COL) return BDR_REF_ERR_SHAPE;
    view_t v = make_view(f, rows, cols, cols, axis);
    uint64_t n = (uint64_t)v.R * (uint64_t)v.Cp;
    if (codes_bytes) *codes_bytes = (size_t)((n * (uint64_t)(f->m + 1) + 7u) / 8u);
    if (sexp_bytes) *sexp_bytes = (size_t)(n / (uint64_t)f->k1);
    if (mexp_bytes) *mexp_bytes = (size_t)((n / (uint64_t)f->k2 * (uint64_t)f->d2 + 7u) / 8u);
    return BDR_REF_OK;
}

/* -------------------------------------------------------------- one block */

/* step 4: |x| / 2^q rounded to an integer, from the 24-bit significand.
 * |x| = sig * 2^(e-150) with e the private exponent, so the quotient is
 * sig * 2^(e-150-q) = sig >> s with s = q + 150 - e.  s >= 16 always, because
 * q >= e - 127 - (m-1) (tau never exceeds E minus the sub-block maximum). */
static uint32_t round_magnitude(uint32_t bits, int q, int m, int rounding)
{
    uint32_t raw = (bits >> 23) & 0xFFu;
    uint32_t top = (1u << m) - 1u;
    if (raw == 255u) return top; /* R6 */
    uint32_t sig = bits & 0x7FFFFFu;
    if (raw != 0u) sig |= 0x800000u; /* R5: no implicit one for subnormals */
    int e = private_exponent(bits);
    int s = q + 150 - e;
    uint32_t M;
    if (s >= 32) {
        /* everything is below half a step, except that RNA/RNE still see it
         * as "less than half" because sig < 2^24 <= 2^(s-1) */
        M = 0;
    } else {
        uint32_t floor_part = sig >> s;
        uint32_t rem = sig & ((1u << s) - 1u);
        uint32_t half = 1u << (s - 1);
        M = floor_part;
        if (rounding == BDR_REF_RNE) {
            if (rem > half || (rem == half && (floor_part & 1u))) M += 1u; /* R2 */
        } else if (rounding == BDR_REF_RNA) {
            if (rem >= half) M += 1u;
        }
    }
    if (M > top) M = top; /* R3 */
    return M;
}

void bdr_ref_quantize_block(const bdr_ref_format *f, const uint32_t *xbits, int n, uint8_t *sexp,
                            uint8_t *tau, uint16_t *code)
{
    const int k1 = f->k1, k2 = f->k2, m = f->m;
    const int beta = (1 << f->d2) - 1;
    uint32_t xb[BDR_REF_MAX_K1];
    for (int i = 0; i < k1; ++i) xb[i] = i < n ? xbits[i] : 0u; /* R8 */

    /* step 2: E is the private exponent of the element of largest magnitude,
     * which is the largest private exponent in the block. */
    int SE = 1;
    for (int i = 0; i < k1; ++i) {
        int e = private_exponent(xb[i]);
        if (e > SE) SE = e;
    }
    *sexp = (uint8_t)SE;

    for (int j = 0; j < k1 / k2; ++j) {
        /* step 3: a sub-block whose largest exponent is E - t gets tau = t,
         * unless t exceeds beta, then tau = beta (R4). */
        int esub = 1;
        for (int i = 0; i < k2; ++i) {
            int e = private_exponent(xb[j * k2 + i]);
            if (e > esub) esub = e;
        }
        int t = SE - esub;
        if (t > beta) t = beta;
        tau[j] = (uint8_t)t;

        /* step 4: the m magnitude bits have weights 2^(E-tau) ... 2^(E-tau-(m-1)),
         * so the magnitude is an integer count of steps of 2^q. */
        int q = (SE - 127) - t - (m - 1);
        for (int i = 0; i < k2; ++i) {
            uint32_t b = xb[j * k2 + i];
            uint32_t M = round_magnitude(b, q, m, f->rounding);
            uint32_t sign = b >> 31; /* R7 */
            code[j * k2 + i] = (uint16_t)((sign << m) | M);
        }
    }
}

double bdr_ref_decode(const bdr_ref_format *f, uint8_t sexp, uint8_t tau, uint16_t code)
{
    /* step 6: descale.  M < 2^8 and q >= 1 - 127 - 7 - 7 = -140, so M * 2^q is
     * a multiple of 2^-149 below 2^128: exact in fp32, and in bf16 whenever
     * m + beta <= 8. */
    const int m = f->m;
    uint32_t M = code & ((1u << m) - 1u);
    int sign = (code >> m) & 1;
    int q = ((int)sexp - 127) - (int)tau - (m - 1);
    double mag = ldexp((double)M, q);
    return sign ? -mag : mag;
}

/* ------------------------------------------------------------ whole tensor */

static int check_tensor_args(const bdr_ref_format *f, int dtype, int64_t rows, int64_t cols,
                             int64_t ld, int axis)
{
    int st = bdr_ref_format_validate(f);
    if (st) return st;
    if (dtype != BDR_REF_F32 && dtype != BDR_REF_BF16) return BDR_REF_ERR_DTYPE;
    if (axis != BDR_REF_AXIS_ROW && axis != BDR_REF_AXIS_COL) return BDR_REF_ERR_SHAPE;
    if (rows < 0 || cols < 0 || ld < cols) return BDR_REF_ERR_SHAPE;
    return BDR_REF_OK;
}

int bdr_ref_quantize(const bdr_ref_format *f, const void *x, int dtype, int64_t rows,
                     int64_t cols, int64_t ld, int axis, uint8_t *codes, uint8_t *sexp,
                     uint8_t *mexp)
{
    int st = check_tensor_args(f, dtype, rows, cols, ld, axis);
    if (st) return st;
    if (rows == 0 || cols == 0) return BDR_REF_OK;
    if (!x || !codes || !sexp || (f->d2 > 0 && !mexp)) return BDR_REF_ERR_NULL;

    const int k1 = f->k1, k2 = f->k2, m = f->m, d2 = f->d2;
    view_t v = make_view(f, rows, cols, ld, axis);
    uint32_t xb[BDR_REF_MAX_K1];
    uint8_t tau[BDR_REF_MAX_K1];
    uint16_t code[BDR_REF_MAX_K1];

    for (int64_t r = 0; r < v.R; ++r) {
        for (int64_t c0 = 0; c0 < v.Cp; c0 += k1) {
            int n = (int)(v.C - c0 < k1 ? v.C - c0 : k1);
            for (int i = 0; i < n; ++i)
                xb[i] = load_bits(x, dtype, r * v.sr + (c0 + i) * v.sc);
            uint8_t se;
            bdr_ref_quantize_block(f, xb, n, &se, tau, code);

            /* step 5: R11 */
            sexp[r * (v.Cp / k1) + c0 / k1] = se;
            for (int i = 0; i < k1; ++i) {
                uint64_t t = (uint64_t)r * (uint64_t)v.Cp + (uint64_t)(c0 + i);
                put_bits(codes, t * (uint64_t)(m + 1), m + 1, code[i]);
            }
            if (d2 > 0) {
                for (int j = 0; j < k1 / k2; ++j) {
                    uint64_t u = (uint64_t)r * (uint64_t)(v.Cp / k2) + (uint64_t)(c0 / k2 + j);
                    put_bits(mexp, u * (uint64_t)d2, d2, tau[j]);
                }
            }
        }
    }
    return BDR_REF_OK;
}

int bdr_ref_dequantize(const bdr_ref_format *f, const uint8_t *codes, const uint8_t *sexp,
                       const uint8_t *mexp, int64_t rows, int64_t cols, int axis, void *y,
                       int dtype, int64_t ld)
{
    int st = check_tensor_args(f, dtype, rows, cols, ld, axis);
    if (st) return st;
    if (dtype == BDR_REF_BF16 && f->m + ((1 << f->d2) - 1) > 8) return BDR_REF_ERR_DTYPE;
    if (rows == 0 || cols == 0) return BDR_REF_OK;
    if (!y || !codes || !sexp || (f->d2 > 0 && !mexp)) return BDR_REF_ERR_NULL;

    const int k1 = f->k1, k2 = f->k2, m = f->m, d2 = f->d2;
    view_t v = make_view(f, rows, cols, ld, axis);
    for (int64_t r = 0; r < v.R; ++r) {
        for (int64_t c = 0; c < v.C; ++c) {
            uint64_t t = (uint64_t)r * (uint64_t)v.Cp + (uint64_t)c;
            uint16_t code = (uint16_t)get_bits(codes, t * (uint64_t)(m + 1), m + 1);
            uint8_t se = sexp[r * (v.Cp / k1) + c / k1];
            uint8_t tau = 0;
            if (d2 > 0) {
                uint64_t u = (uint64_t)r * (uint64_t)(v.Cp / k2) + (uint64_t)(c / k2);
                tau = (uint8_t)get_bits(mexp, u * (uint64_t)d2, d2);
            }
            store_value(y, dtype, r * v.sr + c * v.sc, bdr_ref_decode(f, se, tau, code));
        }
    }
    return BDR_REF_OK;
}

int bdr_ref_quantize_dequantize(const bdr_ref_format *f, const void *x, void *y, int dtype,
                                int64_t rows, int64_t cols, int64_t ld, int axis)
{
    int st = check_tensor_args(f, dtype, rows, cols, ld, axis);
    if (st) return st;
    if (dtype == BDR_REF_BF16 && f->m + ((1 << f->d2) - 1) > 8) return BDR_REF_ERR_DTYPE;
    if (rows == 0 || cols == 0) return BDR_REF_OK;
    if (!x || !y) return BDR_REF_ERR_NULL;

    size_t nc, ns, nm;
    bdr_ref_packed_sizes(f, rows, cols, axis, &nc, &ns, &nm);
    uint8_t *codes = (uint8_t *)calloc(nc ? nc : 1, 1);
    uint8_t *sexp = (uint8_t *)calloc(ns ? ns : 1, 1);
    uint8_t *mexp = (uint8_t *)calloc(nm ? nm : 1, 1);
    st = BDR_REF_ERR_NULL;
    if (codes && sexp && mexp) {
        st = bdr_ref_quantize(f, x, dtype, rows, cols, ld, axis, codes, sexp, mexp);
        if (!st) st = bdr_ref_dequantize(f, codes, sexp, mexp, rows, cols, axis, y, dtype, ld);
    }
    free(codes);
    free(sexp);
    free(mexp);
    return st;
}

/* --------------------------------------------------------------------- QSNR */

int bdr_ref_qsnr_sweep(const bdr_ref_format *fmts, int32_t n_fmts, const void *x, int dtype,
                       int64_t rows, int64_t cols, int64_t ld, double *qsnr_db, double *sums)
{
    if (n_fmts < 0) return BDR_REF_ERR_SHAPE;
    if (!fmts || !x || !qsnr_db || !sums) return BDR_REF_ERR_NULL;
    for (int32_t k = 0; k < n_fmts; ++k) {
        int st = check_tensor_args(&fmts[k], dtype, rows, cols, ld, BDR_REF_AXIS_ROW);
        if (st) return st;
    }
    if (dtype != BDR_REF_F32 && dtype != BDR_REF_BF16) return BDR_REF_ERR_DTYPE;

    /* step 7, signal power: sum of squares of the FP32 values, in index order */
    double s_sig = 0.0;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            double xv = (double)float_of_bits(load_bits(x, dtype, r * ld + c));
            s_sig += xv * xv;
        }
    sums[n_fmts] = s_sig;

    /* Q(x) is held in FP32 whatever the input type: BF16 widens exactly and
     * every BDR value is exact in FP32. */
    size_t n = (size_t)rows * (size_t)cols;
    float *xf = (float *)malloc((n ? n : 1) * sizeof(float));
    float *yf = (float *)malloc((n ? n : 1) * sizeof(float));
    if (!xf || !yf) {
        free(xf);
        free(yf);
        return BDR_REF_ERR_NULL;
    }
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c)
            xf[r * cols + c] = float_of_bits(load_bits(x, dtype, r * ld + c));

    int st = BDR_REF_OK;
    for (int32_t k = 0; k < n_fmts && !st; ++k) {
        st = bdr_ref_quantize_dequantize(&fmts[k], xf, yf, BDR_REF_F32, rows, cols, cols,
                                         BDR_REF_AXIS_ROW);
        if (st) break;
        /* step 7, noise power */
        double s_err = 0.0;
        for (size_t i = 0; i < n; ++i) {
            double d = (double)yf[i] - (double)xf[i];
            s_err += d * d;
        }
        sums[k] = s_err;
        qsnr_db[k] = s_err > 0.0 ? 10.0 * log10(s_sig / s_err) : INFINITY; /* R10 */
    }
    free(xf);
    free(yf);
    return st;
}

/* ------------------------------------------------------------------ mx_gemm */

/* One row of a row-wise packed [R x K] operand, dequantized into out[K]. */
static void dequant_row(const bdr_ref_format *f, const uint8_t *codes, const uint8_t *sexp,
                        const uint8_t *mexp, int64_t K, int64_t r, double *out)
{
    const int k1 = f->k1, k2 = f->k2, m = f->m, d2 = f->d2;
    int64_t Kp = (K + k1 - 1) / k1 * k1;
    for (int64_t c = 0; c < K; ++c) {
        uint64_t t = (uint64_t)r * (uint64_t)Kp + (uint64_t)c;
        uint16_t code = (uint16_t)get_bits(codes, t * (uint64_t)(m + 1), m + 1);
        uint8_t se = sexp[r * (Kp / k1) + c / k1];
        uint8_t tau = 0;
        if (d2 > 0)
            tau = (uint8_t)get_bits(
                mexp, ((uint64_t)r * (uint64_t)(Kp / k2) + (uint64_t)(c / k2)) * (uint64_t)d2, d2);
        out[c] = bdr_ref_decode(f, se, tau, code);
    }
}

int bdr_ref_mx_gemm_sampled(const bdr_ref_format *fa, const bdr_ref_format *fb,
                            const uint8_t *a_codes, const uint8_t *a_sexp, const uint8_t *a_mexp,
                            const uint8_t *b_codes, const uint8_t *b_sexp, const uint8_t *b_mexp,
                            int64_t M, int64_t N, int64_t K, int64_t n_samples,
                            const int64_t *idx_i, const int64_t *idx_j, float *out,
                            double *absdot)
{
    int st = bdr_ref_format_validate(fa);
    if (st) return st;
    st = bdr_ref_format_validate(fb);
    if (st) return st;
    if (M < 0 || N < 0 || K < 0 || n_samples < 0) return BDR_REF_ERR_SHAPE;
    if (n_samples == 0) return BDR_REF_OK;
    if (!a_codes || !a_sexp || !b_codes || !b_sexp || !idx_i || !idx_j || !out)
        return BDR_REF_ERR_NULL;
    if ((fa->d2 > 0 && !a_mexp) || (fb->d2 > 0 && !b_mexp)) return BDR_REF_ERR_NULL;

    double *ar = (double *)malloc((size_t)(K ? K : 1) * sizeof(double));
    double *br = (double *)malloc((size_t)(K ? K : 1) * sizeof(double));
    if (!ar || !br) {
        free(ar);
        free(br);
        return BDR_REF_ERR_NULL;
    }
    for (int64_t s = 0; s < n_samples; ++s) {
        int64_t i = idx_i[s], j = idx_j[s];
        if (i < 0 || i >= M || j < 0 || j >= N) {
            free(ar);
            free(br);
            return BDR_REF_ERR_SHAPE;
        }
        dequant_row(fa, a_codes, a_sexp, a_mexp, K, i, ar);
        dequant_row(fb, b_codes, b_sexp, b_mexp, K, j, br);
        double acc = 0.0, aabs = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double p = ar[k] * br[k]; /* exact: two 8-bit significands */
            acc += p;
            aabs += fabs(p);
        }
        out[s] = (float)acc;
        if (absdot) absdot[s] = aabs;
    }
    free(ar);
    free(br);
    return BDR_REF_OK;
}

int bdr_ref_mx_gemm(const bdr_ref_format *fa, const bdr_ref_format *fb, const uint8_t *a_codes,
                    const uint8_t *a_sexp, const uint8_t *a_mexp, const uint8_t *b_codes,
                    const uint8_t *b_sexp, const uint8_t *b_mexp, int64_t M, int64_t N, int64_t K,
                    float *C, int64_t ldc)
{
    int st = bdr_ref_format_validate(fa);
    if (st) return st;
    st = bdr_ref_format_validate(fb);
    if (st) return st;
    if (M < 0 || N < 0 || K < 0 || ldc < N) return BDR_REF_ERR_SHAPE;
    if (M == 0 || N == 0) return BDR_REF_OK;
    if (!a_codes || !a_sexp || !b_codes || !b_sexp || !C) return BDR_REF_ERR_NULL;
    if ((fa->d2 > 0 && !a_mexp) || (fb->d2 > 0 && !b_mexp)) return BDR_REF_ERR_NULL;

    size_t kk = (size_t)(K ? K : 1);
    double *ah = (double *)malloc((size_t)M * kk * sizeof(double));
    double *bh = (double *)malloc((size_t)N * kk * sizeof(double));
    if (!ah || !bh) {
        free(ah);
        free(bh);
        return BDR_REF_ERR_NULL;
    }
    for (int64_t i = 0; i < M; ++i) dequant_row(fa, a_codes, a_sexp, a_mexp, K, i, ah + i * kk);
    for (int64_t j = 0; j < N; ++j) dequant_row(fb, b_codes, b_sexp, b_mexp, K, j, bh + j * kk);
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k) acc += ah[i * kk + k] * bh[j * kk + k];
            C[i * ldc + j] = (float)acc;
        }
    free(ah);
    free(bh);
    return BDR_REF_OK;
}

/* --------------------------------------------------- dot-product pipeline */

/*
 * Sec. IV-B, "Dot Product Architecture" (and the caption of the pipeline figure): for k1 > 1
 * the first part of the pipeline reduces the Hadamard product of the k1 elements of a block to
 * a single element, with a conditional right shift of up to 2^d2 - 1 bits at depth log2(k2)
 * when there are sub-blocks; there are r / k1 such reductions, whose results are normalized to
 * the largest element and reduced in fixed point with f bits.  The text stops there (the figure
 * is not part of it), so what follows is a reading, step by step:
 *
 *   D1  Element products are exact integers: P_i = (+-Ma_i)(+-Mb_i), the sign-magnitude
 *       mantissas of the two codes.
 *   D2  The k2 products of a sub-block share their shifts and are added exactly:
 *       S_j = sum of P_i over sub-block j (adder tree of depth log2 k2).
 *   D3  At that depth sub-block j is shifted right by tau_a[j] + tau_b[j] bits (each operand
 *       contributes up to its own 2^d2 - 1) and the k1 / k2 results are added.  The datapath
 *       keeps the bits that are shifted out (it is beta_a + beta_b bits wider below the binary
 *       point), so the block result is the exact integer
 *       T = sum_j S_j 2^(beta_a + beta_b - tau_a[j] - tau_b[j])
 *       in units of 2^(Ea + Eb - (ma - 1) - (mb - 1) - beta_a - beta_b), Ea, Eb the shared
 *       exponents of the two blocks.  |T| < 2^W, W = ma + mb + log2(k1) + beta_a + beta_b.
 *   D4  "Normalized to the largest element": the r / k1 block results of a pass are aligned to
 *       the largest exponent sum e_max = max_b (SEa_b + SEb_b) (exponents are compared, as in a
 *       floating-point adder; the values are not inspected); block b is shifted right by
 *       s_b = e_max - (SEa_b + SEb_b).
 *   D5  The f-bit fixed-point word is a two's complement number with f - 1 magnitude bits whose
 *       top magnitude bit is aligned with bit W - 1 of a block result that has the largest
 *       exponent sum: g = f - 1 - W guard bits lie below the integer T (g may be negative).
 *       U_b = floor(T_b 2^(g - s_b)): bits that fall below the word are dropped (arithmetic
 *       shift of a two's complement number: towards minus infinity).
 *   D6  V = sum_b U_b exactly (the adder tree grows by log2(r / k1) carry bits; nothing
 *       saturates).
 *   D7  The result of the pass is V 2^(e_max - 254 - (ma-1) - (mb-1) - beta_a - beta_b - g),
 *       rounded once to FP32, nearest even.
 *   D8  The K / r passes of a longer dot product are added in FP32, in order of increasing k
 *       (the text's remark on scalar formats, "serially accumulating in a floating-point type"
 *       with f - 2 mantissa bits: FP32 for f = 25).
 */

/* floor(t * 2^sh) for |t| < 2^63 and any sh; sh > 0 only where the result fits. */
static __int128 shift_floor(__int128 t, int sh)
{
    if (sh >= 0) return t * ((__int128)1 << sh);
    int n = -sh;
    if (n >= 100) return t < 0 ? -1 : 0;
    __int128 d = (__int128)1 << n;
    __int128 q = t / d; /* truncates towards zero */
    if (t < 0 && q * d != t) q -= 1;
    return q;
}

/* v * 2^x rounded once to FP32, nearest even, subnormals and overflow included. */
static float round_scaled_to_float(__int128 v, int x)
{
    if (v == 0) return 0.0f;
    int neg = v < 0;
    unsigned __int128 mag = neg ? (unsigned __int128)(-v) : (unsigned __int128)v;
    int nb = 0;
    for (unsigned __int128 t = mag; t; t >>= 1) ++nb;
    int e = nb - 1 + x;                            /* exponent of the leading bit */
    int keep = e >= -126 ? 24 : 24 - (-126 - e);   /* significant bits FP32 holds there */
    float out;
    if (keep <= 0) {
        /* below half of the smallest subnormal, or exactly at it: ties go to even (zero) */
        out = (keep == 0 && mag > ((unsigned __int128)1 << (nb - 1))) ? ldexpf(1.0f, -149) : 0.0f;
    } else if (nb <= keep) {
        out = ldexpf((float)(uint64_t)mag, x); /* nb <= 24: exact */
    } else {
        int drop = nb - keep;
        unsigned __int128 q = mag >> drop, rem = mag - (q << drop);
        unsigned __int128 half = (unsigned __int128)1 << (drop - 1);
        if (rem > half || (rem == half && (q & 1))) q += 1;
        out = ldexpf((float)(uint64_t)q, x + drop); /* q <= 2^24: exact; overflow gives inf */
    }
    return neg ? -out : out;
}

static int ilog2_i32(int32_t v)
{
    int l = 0;
    while ((1 << l) < v) ++l;
    return l;
}

int bdr_ref_dot_pipeline_sampled(const bdr_ref_format *fa, const bdr_ref_format *fb,
                                 const uint8_t *a_codes, const uint8_t *a_sexp,
                                 const uint8_t *a_mexp, const uint8_t *b_codes,
                                 const uint8_t *b_sexp, const uint8_t *b_mexp, int64_t M,
                                 int64_t N, int64_t K, int64_t r, int32_t f_bits,
                                 int64_t n_samples, const int64_t *idx_i, const int64_t *idx_j,
                                 float *out)
{
    int st = bdr_ref_format_validate(fa);
    if (st) return st;
    st = bdr_ref_format_validate(fb);
    if (st) return st;
    if (fa->k1 != fb->k1 || fa->k2 != fb->k2) return BDR_REF_ERR_FORMAT;
    if (M < 0 || N < 0 || K < 0 || n_samples < 0) return BDR_REF_ERR_SHAPE;
    if (r < 1 || r % fa->k1 != 0 || K % r != 0) return BDR_REF_ERR_SHAPE;
    if (f_bits < 2 || f_bits > 64) return BDR_REF_ERR_SHAPE;
    if (n_samples == 0) return BDR_REF_OK;
    if (!idx_i || !idx_j || !out) return BDR_REF_ERR_NULL;
    if (K > 0 && (!a_codes || !a_sexp || !b_codes || !b_sexp)) return BDR_REF_ERR_NULL;
    if (K > 0 && ((fa->d2 > 0 && !a_mexp) || (fb->d2 > 0 && !b_mexp))) return BDR_REF_ERR_NULL;

    const int k1 = fa->k1, k2 = fa->k2, ma = fa->m, mb = fb->m;
    const int beta_a = (1 << fa->d2) - 1, beta_b = (1 << fb->d2) - 1;
    const int W = ma + mb + ilog2_i32(k1) + beta_a + beta_b;
    const int g = f_bits - 1 - W;
    const int64_t blocks_per_row = K / k1, subs_per_row = K / k2;

    for (int64_t s = 0; s < n_samples; ++s) {
        const int64_t i = idx_i[s], j = idx_j[s];
        if (i < 0 || i >= M || j < 0 || j >= N) return BDR_REF_ERR_SHAPE;
        float acc = 0.0f;
        for (int64_t k0 = 0; k0 < K; k0 += r) {
            /* D4: the largest exponent sum among the blocks of this pass */
            int e_max = 0;
            for (int64_t b = k0 / k1; b < (k0 + r) / k1; ++b) {
                int e = (int)a_sexp[i * blocks_per_row + b] + (int)b_sexp[j * blocks_per_row + b];
                if (e > e_max) e_max = e;
            }
            __int128 V = 0;
            for (int64_t b = k0 / k1; b < (k0 + r) / k1; ++b) {
                /* D1-D3: the block's integer result */
                int64_t T = 0;
                for (int u = 0; u < k1 / k2; ++u) {
                    const int64_t su = b * (k1 / k2) + u; /* sub-block index within the row */
                    int64_t S = 0;
                    for (int t = 0; t < k2; ++t) {
                        const uint64_t ea = (uint64_t)i * (uint64_t)K + (uint64_t)(su * k2 + t);
                        const uint64_t eb = (uint64_t)j * (uint64_t)K + (uint64_t)(su * k2 + t);
                        const uint32_t ca = get_bits(a_codes, ea * (uint64_t)(ma + 1), ma + 1);
                        const uint32_t cb = get_bits(b_codes, eb * (uint64_t)(mb + 1), mb + 1);
                        int64_t pa = (int64_t)(ca & ((1u << ma) - 1u)), pb = (int64_t)(cb & ((1u << mb) - 1u));
                        if ((ca >> ma) & 1u) pa = -pa;
                        if ((cb >> mb) & 1u) pb = -pb;
                        S += pa * pb;
                    }
                    int ta = 0, tb = 0;
                    if (fa->d2 > 0)
                        ta = (int)get_bits(a_mexp, ((uint64_t)i * (uint64_t)subs_per_row + (uint64_t)su) * (uint64_t)fa->d2, fa->d2);
                    if (fb->d2 > 0)
                        tb = (int)get_bits(b_mexp, ((uint64_t)j * (uint64_t)subs_per_row + (uint64_t)su) * (uint64_t)fb->d2, fb->d2);
                    T += S * ((int64_t)1 << (beta_a + beta_b - ta - tb));
                }
                /* D4-D6: align to e_max inside the f-bit word, drop what falls below it, add */
                const int e = (int)a_sexp[i * blocks_per_row + b] + (int)b_sexp[j * blocks_per_row + b];
                V += shift_floor((__int128)T, g - (e_max - e));
            }
            /* D7, D8 */
            const float pass = round_scaled_to_float(
                V, e_max - 254 - (ma - 1) - (mb - 1) - beta_a - beta_b - g);
            acc = k0 == 0 ? pass : acc + pass;
        }
        out[s] = acc;
    }
    return BDR_REF_OK;
}
