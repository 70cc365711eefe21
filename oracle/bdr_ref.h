/*
 * bdr_ref.h -- CPU oracle for the Block Data Representation (BDR) quantizer.
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, slow, scalar implementation of
 * what the two-level shared-microexponent quantizer computes, written from the
 * paper's definitions (arXiv 2302.08007).  It exists so that the GPU library
 * can be checked against something that can be verified by eye.  It shares no
 * code with the GPU library and must never be called from the product path.
 *
 * Every pointer here is a HOST pointer.  Nothing is allocated on behalf of the
 * caller except short-lived scratch that is freed before return.
 *
 * Passages followed (all from the paper):
 *   - format tuple (k1, k2, d1, d2, m) and bits/element:
 *       Sec. III, "Block Data Representations"
 *   - MX9 / MX6 / MX4 instances: Table II
 *   - shared exponent E, m-bit rounded magnitude, per-element error bound,
 *     sub-block shift tau <= beta = 2^d2 - 1:
 *       Sec. IX (proof of Theorem 1), Eq. "max_exp", "max_exp_round",
 *       "q_error_max", "q_error_max-1" and the paragraph after "q_error_all"
 *   - QSNR: Sec. IV-A, Eq. 3
 *   - quantize along the reduction axis; transpose before quantizing:
 *       Sec. V, "Training"
 *
 * Readings taken where the paper is silent are stated beside the code that
 * implements them in bdr_ref.c.
 *
 * What pins it (tests/test_oracle_pins.py, tests/test_oracle_properties.py; none of
 * them calls the function under test to make its expected value): figures the
 * paper prints for its design-space workload (Sec. IV-C: MX9 about 3.6 dB above
 * MSFP16; a second microexponent bit 0.5 dB, k2 8 -> 2 about 2 dB, k2 2 -> 1
 * 0.7 dB; MX9 about 16 dB above scalar FP8 E4M3), Table II's bits per element,
 * hand-worked blocks, brute force over every representable value, the shift rule
 * and the error bound of Sec. IX, Theorem 1, the symmetries of the definition,
 * textbook block floating point for d2 = 0, and numpy for the product.  Every
 * function has such a pin; absolute QSNR values other than the printed
 * differences are not printed anywhere in the paper.
 *
 * bdr_ref_dot_pipeline_sampled (the dot-product pipeline of Sec. IV-B) is PARITY UNPINNED in
 * the part only a reading decides: the paper gives the pipeline in one paragraph and a figure
 * that is not in the text, and prints no worked value.  What the arithmetic fixes is pinned
 * (tests/test_oracle_dot_pipeline.py): the exact integer block product for d2 = 0, the shift
 * tau_a + tau_b per sub-block pair, equality with the exactly rounded dot product of the
 * dequantized operands once f is large enough, the error bound of one unit per block, and
 * power-of-two scale equivariance.  Where the dropped bits go (floor), what the partial
 * results are aligned to (the largest exponent sum) and where the f-bit word sits are
 * readings, checked only against hand-worked examples derived from those same readings.
 */
#ifndef BDR_REF_H
#define BDR_REF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* A BDR format, Sec. III: block size k1, sub-block size k2, d1 bits of shared
 * exponent per block, d2 bits of microexponent per sub-block, m magnitude bits
 * (plus one sign bit) per element, and the rounding rule for the magnitude. */
typedef struct {
    int32_t k1, d1, k2, d2, m, rounding;
} bdr_ref_format;

enum { BDR_REF_RNE = 0, BDR_REF_RNA = 1, BDR_REF_RTZ = 2 };
enum { BDR_REF_F32 = 0, BDR_REF_BF16 = 1 };
enum { BDR_REF_AXIS_ROW = 0, BDR_REF_AXIS_COL = 1 };
enum {
    BDR_REF_OK = 0,
    BDR_REF_ERR_NULL = 1,
    BDR_REF_ERR_FORMAT = 2,
    BDR_REF_ERR_SHAPE = 3,
    BDR_REF_ERR_DTYPE = 5
};

/* 0 when the tuple is a format this oracle implements:
 * k1, k2 powers of two, k2 divides k1, 1 <= k1 <= 4096, d1 == 8,
 * 0 <= d2 <= 3, 1 <= m <= 8, rounding in {RNE, RNA, RTZ}. */
int bdr_ref_format_validate(const bdr_ref_format *f);

/* Bits per element of the format, Sec. III: (m+1) + d1/k1 + d2/k2. */
double bdr_ref_bits_per_element(const bdr_ref_format *f);

/* Byte sizes of the three packed planes for a [rows x cols] tensor quantized
 * along `axis`.  A row (of the transposed tensor when axis is COL) whose
 * length is not a multiple of k1 is padded with zeros to the next multiple. */
int bdr_ref_packed_sizes(const bdr_ref_format *f, int64_t rows, int64_t cols, int axis,
                         size_t *codes_bytes, size_t *sexp_bytes, size_t *mexp_bytes);

/* Quantize one block of n <= k1 elements given as FP32 bit patterns.
 * Outputs are unpacked: the shared exponent code (biased, 8 bit), one shift
 * tau per sub-block (k1/k2 of them) and one (m+1)-bit sign|magnitude code per
 * element (k1 of them; positions >= n are the codes of +0). */
void bdr_ref_quantize_block(const bdr_ref_format *f, const uint32_t *xbits, int n,
                            uint8_t *sexp, uint8_t *tau, uint16_t *code);

/* Value of one code: (-1)^s * M * 2^(sexp - 127 - tau - (m-1)), as a double
 * (exact).  The caller narrows it. */
double bdr_ref_decode(const bdr_ref_format *f, uint8_t sexp, uint8_t tau, uint16_t code);

/* Quantize x ([rows x cols], leading dimension ld elements, dtype F32 or BF16)
 * into the three planes (sizes from bdr_ref_packed_sizes; mexp may be NULL when
 * d2 == 0).  AXIS_COL gives exactly what AXIS_ROW gives on the transpose. */
int bdr_ref_quantize(const bdr_ref_format *f, const void *x, int dtype, int64_t rows,
                     int64_t cols, int64_t ld, int axis, uint8_t *codes, uint8_t *sexp,
                     uint8_t *mexp);

/* Inverse of the packing: rebuild y ([rows x cols], leading dimension ld) from
 * the planes.  BF16 output requires m + (2^d2 - 1) <= 8, for which it is exact. */
int bdr_ref_dequantize(const bdr_ref_format *f, const uint8_t *codes, const uint8_t *sexp,
                       const uint8_t *mexp, int64_t rows, int64_t cols, int axis, void *y,
                       int dtype, int64_t ld);

/* y = dequantize(quantize(x)); same dtype and leading dimension on both sides. */
int bdr_ref_quantize_dequantize(const bdr_ref_format *f, const void *x, void *y, int dtype,
                                int64_t rows, int64_t cols, int64_t ld, int axis);

/* Eq. 3 over the whole tensor, one value per format, quantizing along rows.
 * sums (n_fmts + 1 doubles) receives S_err[f] = sum (Q(x)-x)^2 per format and
 * then S_sig = sum x^2; qsnr_db[f] = 10 log10(S_sig / S_err[f]) (+inf when
 * S_err is 0). */
int bdr_ref_qsnr_sweep(const bdr_ref_format *fmts, int32_t n_fmts, const void *x, int dtype,
                       int64_t rows, int64_t cols, int64_t ld, double *qsnr_db, double *sums);

/* C[i,j] = sum_k Ahat[i,k] * Bhat[j,k] in fp64, rounded once to fp32, where
 * Ahat ([M x K]) and Bhat ([N x K]) are the dequantized operands, both packed
 * row-wise (blocks along K).  Evaluates only the n_samples entries
 * (idx_i[s], idx_j[s]); out[s] gets the value and, when absdot is not NULL,
 * absdot[s] = sum_k |Ahat[i,k] * Bhat[j,k]|. */
int bdr_ref_mx_gemm_sampled(const bdr_ref_format *fa, const bdr_ref_format *fb,
                            const uint8_t *a_codes, const uint8_t *a_sexp, const uint8_t *a_mexp,
                            const uint8_t *b_codes, const uint8_t *b_sexp, const uint8_t *b_mexp,
                            int64_t M, int64_t N, int64_t K, int64_t n_samples,
                            const int64_t *idx_i, const int64_t *idx_j, float *out,
                            double *absdot);

/* The full [M x N] product of the same definition (row-major, ldc elements). */
int bdr_ref_mx_gemm(const bdr_ref_format *fa, const bdr_ref_format *fb, const uint8_t *a_codes,
                    const uint8_t *a_sexp, const uint8_t *a_mexp, const uint8_t *b_codes,
                    const uint8_t *b_sexp, const uint8_t *b_mexp, int64_t M, int64_t N, int64_t K,
                    float *C, int64_t ldc);

/* The dot-product pipeline the paper outlines for BDR formats (Sec. IV-B, "Dot Product
 * Architecture", and the caption of the pipeline figure there), modelled bit for bit under the
 * readings D1-D8 stated in bdr_ref.c.  A and B are packed row-wise ([M x K] and [N x K], blocks
 * along K) in formats with the same k1 and k2 (a symmetric unit).  A dot product of length K is
 * taken in K / r passes of the pipeline, r the "dot product length" of the unit (a multiple of
 * k1 that divides K); f_bits is its "fixed-point reduction accumulation precision" (2 .. 64;
 * the paper uses min(25, dynamic range), i.e. 25 for every d1 = 8 format).  Evaluates the
 * n_samples entries (idx_i[s], idx_j[s]) of C = A B^T into out[s]. */
int bdr_ref_dot_pipeline_sampled(const bdr_ref_format *fa, const bdr_ref_format *fb,
                                 const uint8_t *a_codes, const uint8_t *a_sexp,
                                 const uint8_t *a_mexp, const uint8_t *b_codes,
                                 const uint8_t *b_sexp, const uint8_t *b_mexp, int64_t M,
                                 int64_t N, int64_t K, int64_t r, int32_t f_bits,
                                 int64_t n_samples, const int64_t *idx_i, const int64_t *idx_j,
                                 float *out);

#ifdef __cplusplus
}
#endif
#endif /* BDR_REF_H */
