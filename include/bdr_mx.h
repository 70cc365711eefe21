/*
 * bdr_mx.h -- C ABI of the MI355X (gfx950) library for Block Data Representations
 * and shared microexponents (arXiv 2302.08007).
 *
 * The library holds the data-parallel hot path of the two-level quantizer: shared
 * exponent per k1-block, microexponent per k2-sub-block, m-bit sign-magnitude
 * elements; bit-packing; dequantization; the QSNR reduction over a sweep of
 * formats; and a GEMM on MX-quantized operands.
 *
 * Conventions that hold for every entry point unless it says otherwise:
 *   - `const bdr_format *` arguments point to HOST memory and are read before the
 *     call returns.  Every other pointer is a DEVICE pointer owned by the caller.
 *   - The library allocates nothing, frees nothing and never synchronizes: work is
 *     enqueued on `hip_stream` (a hipStream_t passed as void*, NULL = the null
 *     stream) and the call returns at once.
 *   - Every function returns a bdr_status; nothing throws or aborts.  All argument
 *     checks, and every request for a resource a kernel needs (more than 64 KiB of
 *     LDS per workgroup), are made before the first launch of a call: on any status
 *     other than BDR_OK and BDR_ERR_LAUNCH nothing was launched and no output was
 *     touched, and the same holds for a BDR_ERR_LAUNCH that comes from such a
 *     request.  BDR_ERR_LAUNCH can also mean that the HIP runtime refused a launch
 *     itself; in a call that enqueues several kernels (bdr_qsnr_sweep, mx_gemm with a
 *     workspace) the earlier ones may then already be enqueued, and workspace and
 *     outputs hold unspecified data.  A HIP error that was already pending when the
 *     call was made is reported, and consumed, as this call's BDR_ERR_LAUNCH.
 *   - A tensor is [rows x cols], row-major, with `ld` elements between the starts
 *     of consecutive rows (ld >= cols).
 *
 * Packed image (three planes, each a little-endian bit stream: bit b of a stream
 * is bit b % 8 of byte b / 8).  For blocks along the rows of an [R x C] tensor:
 *   codes : element t = r * C + c holds bits [t (m+1), (t+1)(m+1)): the magnitude
 *           M in the low m bits, the sign above it;
 *   sexp  : one byte per k1-block, block index r * (C / k1) + c / k1: the biased
 *           FP32 exponent of the block maximum (d1 = 8);
 *   mexp  : sub-block u = r * (C / k2) + c / k2 holds bits [u d2, (u+1) d2): the
 *           shift tau of that sub-block.  Absent (may be NULL) when d2 = 0.
 * The value of an element is (-1)^sign * M * 2^(sexp - 127 - tau - (m - 1)).
 * When the row length is not a multiple of k1, C above is the row length rounded up
 * to the next multiple of k1: the last block of a row is stored whole, the elements
 * it lacks as code 0 (see bdr_packed_sizes).
 * BDR_AXIS_COL means: exactly what BDR_AXIS_ROW gives on the transposed tensor
 * ([cols x rows]), plane indices included.
 */
#ifndef BDR_MX_H
#define BDR_MX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* A BDR format (Sec. III, "Block Data Representations"): k1 elements share one
 * d1-bit exponent, every k2 of them share one d2-bit microexponent, each element
 * has m magnitude bits and a sign; bits/element = (m+1) + d1/k1 + d2/k2.
 * `rounding` says how the magnitude is rounded (Sec. IX says "nearest"). */
typedef struct {
    int32_t k1, d1, k2, d2, m, rounding;
} bdr_format;

enum bdr_rounding { BDR_RNE = 0 /* nearest, ties to even */, BDR_RNA = 1 /* ties away */, BDR_RTZ = 2 /* truncate */ };
enum bdr_dtype { BDR_F32 = 0, BDR_BF16 = 1 };
enum bdr_axis { BDR_AXIS_ROW = 0 /* blocks along the contiguous axis */, BDR_AXIS_COL = 1 /* blocks down the columns */ };
enum bdr_status {
    BDR_OK = 0,
    BDR_ERR_NULL = 1,   /* a required pointer is NULL */
    BDR_ERR_FORMAT = 2, /* the format tuple is not one this library implements */
    BDR_ERR_SHAPE = 3,  /* negative size, ld < cols, or a size the call does not take */
    BDR_ERR_ALIGN = 4,  /* a pointer or row pitch is not aligned as the call asks */
    BDR_ERR_DTYPE = 5,  /* unknown dtype, or BF16 output asked for a format it cannot hold exactly */
    BDR_ERR_LAUNCH = 6, /* the HIP runtime refused a launch (hipGetLastError was consumed) */
    BDR_ERR_WORKSPACE = 7 /* workspace missing or too small */
};

/* Table II: MX9, MX6 and MX4 are (k1 16, d1 8, k2 2, d2 1, m 7 / 4 / 2). */
#define BDR_FORMAT_MX9 { 16, 8, 2, 1, 7, BDR_RNE }
#define BDR_FORMAT_MX6 { 16, 8, 2, 1, 4, BDR_RNE }
#define BDR_FORMAT_MX4 { 16, 8, 2, 1, 2, BDR_RNE }

/* Human-readable name of a status.  Never NULL; static storage. */
const char *bdr_status_string(int status);

/* Host only.  BDR_OK when the tuple is implemented: k1 and k2 powers of two,
 * k2 divides k1, 1 <= k1 <= 256, d1 = 8 (Theorem 1 fixes d1 = 8), 0 <= d2 <= 3,
 * 1 <= m <= 8, rounding one of bdr_rounding.  (Sec. III.) */
int bdr_format_validate(const bdr_format *fmt);

/* Host only.  Byte sizes of the three planes of a [rows x cols] tensor blocked
 * along `axis`; the three together hold (m+1) + d1/k1 + d2/k2 bits per element
 * (Sec. III).  A blocked axis that is not a whole number of blocks is stored
 * padded with +0 to the next multiple of k1, the pads as code 0 (Sec. IX, the
 * remark after Theorem 1: fewer than k1 elements form a block of their own
 * length, and zeros change neither its maximum nor its error); the sizes are those
 * of the padded tensor.  The padded length must be a multiple of 8, which only
 * k1 < 8 can miss (BDR_ERR_SHAPE).  Any of the three outputs may be NULL. */
int bdr_packed_sizes(const bdr_format *fmt, int64_t rows, int64_t cols, int axis,
                     size_t *codes_bytes, size_t *sexp_bytes, size_t *mexp_bytes);

/* Quantize x into the packed image (Sec. IX: shared exponent from the block
 * maximum, Eq. "max_exp"; sub-block shift tau <= 2^d2 - 1, Eq. "q_error_max-1";
 * magnitude rounded to m bits, Eq. "max_exp_round"; Sec. V for the axis).
 *   x      device, [rows x cols] of `dtype`, pitch ld elements, 16-byte aligned,
 *          ld * sizeof(element) a multiple of 16
 *   codes, sexp, mexp   device, sizes from bdr_packed_sizes, 16-byte aligned,
 *          fully overwritten; mexp may be NULL when d2 = 0
 * Whole shapes - the blocked axis a multiple of max(k1, 8) and, for BDR_AXIS_COL,
 * cols a multiple of 8 - run on the fast kernels.  Any other shape whose padded
 * blocked axis (see bdr_packed_sizes) is a multiple of 8 is taken too, element by
 * element: correct, several times slower, and x then needs only the alignment of
 * one element and any ld >= cols.  rows = 0 or cols = 0 is BDR_OK and launches
 * nothing. */
int bdr_quantize(const bdr_format *fmt, const void *x, int dtype, int64_t rows, int64_t cols,
                 int64_t ld, int axis, void *codes, void *sexp, void *mexp, void *hip_stream);

/* Rebuild y from the packed image: y = (-1)^sign * M * 2^(sexp-127-tau-(m-1))
 * (the descaling step of Sec. II / Fig. 4).  Exact in FP32 for every format; BF16
 * output needs m + 2^d2 - 1 <= 8 (then it is exact too), else BDR_ERR_DTYPE.
 * Same shape and alignment rules as bdr_quantize; the [rows x cols] elements of y
 * are all written and nothing else is (the pads of a short last block are not
 * part of y). */
int bdr_dequantize(const bdr_format *fmt, const void *codes, const void *sexp, const void *mexp,
                   int64_t rows, int64_t cols, int axis, void *y, int dtype, int64_t ld,
                   void *hip_stream);

/* Gather + dequantize: y[j, :] = dequantized row indices[j] of a packed table
 * (MX as a storage format for embedding tables, Sec. V "Inferencing": "quantizing both
 * storage and compute" for recommendation models).  The table is the row-wise packed
 * image of a [table_rows x cols] tensor in one of Table II's formats (else
 * BDR_ERR_FORMAT); cols must be a multiple of 32.
 *   indices : device, n_indices int64 values, 8-byte aligned; an index outside
 *             [0, table_rows) yields a row of +0 (it is never dereferenced)
 *   y       : device, [n_indices x cols] of `dtype`, contiguous, 16-byte aligned,
 *             fully overwritten; values are exact in FP32 and in BF16 */
int bdr_gather_dequantize(const bdr_format *fmt, const void *codes, const void *sexp,
                          const void *mexp, int64_t table_rows, int64_t cols, const int64_t *indices,
                          int64_t n_indices, void *y, int dtype, void *hip_stream);

/* The same lookup on a table that keeps each row's bytes together.  A lookup in the
 * three-plane image reads three separate runs per row (codes, exponent bytes,
 * microexponent bytes), each at least one memory line; for embedding rows of a few
 * hundred elements that is several times the bytes a row holds.  In the table image a
 * row is bdr_table_row_bytes(fmt, cols) consecutive bytes: the row's run of the codes
 * plane, then its run of the exponent plane, then its run of the microexponent plane,
 * unchanged; rows follow each other without gaps.  (Storage of embedding tables,
 * Sec. V "Inferencing"; the bytes are those of Sec. III's format, (m+1) + d1/k1 + d2/k2
 * bits per element.)  Table II's formats only (else BDR_ERR_FORMAT); cols a multiple
 * of 64 (else BDR_ERR_SHAPE).
 *
 * bdr_table_row_bytes: host only; 0 for a format or cols the table image does not take.
 * bdr_table_pack: planes (device, as bdr_quantize wrote them for [table_rows x cols],
 *   row blocks) -> table (device, table_rows * row bytes, 16-byte aligned, fully
 *   overwritten).
 * bdr_table_gather_dequantize: as bdr_gather_dequantize, reading the table image. */
size_t bdr_table_row_bytes(const bdr_format *fmt, int64_t cols);
int bdr_table_pack(const bdr_format *fmt, const void *codes, const void *sexp, const void *mexp,
                   int64_t table_rows, int64_t cols, void *table, void *hip_stream);
int bdr_table_gather_dequantize(const bdr_format *fmt, const void *table, int64_t table_rows,
                                int64_t cols, const int64_t *indices, int64_t n_indices, void *y,
                                int dtype, void *hip_stream);

/* Host only.  Memory-interface packing of one tile (Sec. IV-B, "Memory Footprint": a
 * tile of 256 elements into a 64-byte interface): bytes the tile's packed image takes,
 * interface transfers needed, and efficiency = bytes / (transfers * interface_bytes).
 * Any of the three outputs may be NULL. */
int bdr_tile_packing(const bdr_format *fmt, int64_t tile_elements, int64_t interface_bytes,
                     int64_t *packed_bytes, int64_t *transfers, double *efficiency);

/* y = dequantize(quantize(x)) in one pass, without the packed image -- what an
 * emulation library does around every tensor operation (Sec. VI, "Experimental
 * Setup").  x and y have the same dtype, shape and pitch; y may alias x. */
int bdr_quantize_dequantize(const bdr_format *fmt, const void *x, void *y, int dtype,
                            int64_t rows, int64_t cols, int64_t ld, int axis, void *hip_stream);

/* Bytes of device workspace bdr_qsnr_sweep needs for n_fmts formats. */
size_t bdr_qsnr_sweep_workspace_bytes(int32_t n_fmts);

/* QSNR (Sec. IV-A, Eq. 3) of every format in fmts[0..n_fmts) on one tensor, blocks
 * along rows, reading x once:
 *   sums[f]      = sum over the tensor of (Q_f(x) - x)^2      (f < n_fmts)
 *   sums[n_fmts] = sum over the tensor of x^2
 *   qsnr_db[f]   = 10 log10(sums[n_fmts] / sums[f]), +inf when sums[f] = 0
 * fmts is a host array; qsnr_db (n_fmts doubles), sums (n_fmts + 1 doubles) and
 * workspace are device memory; workspace need not be cleared by the caller.
 * cols must be a multiple of max(8, every k1).  1 <= n_fmts <= 1024. */
int bdr_qsnr_sweep(const bdr_format *fmts, int32_t n_fmts, const void *x, int dtype, int64_t rows,
                   int64_t cols, int64_t ld, double *qsnr_db, double *sums, void *workspace,
                   size_t workspace_bytes, void *hip_stream);

/* bdr_qsnr_sweep for callers that cannot allocate device memory and have no workspace
 * to bring: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments without the workspace, same kernels, same results bit for
 * bit; the scratch is a fixed array of bdr_qsnr_sweep_static_scratch_bytes() bytes
 * (under 1 MiB) that is part of the library's device image: every GPU the library runs
 * on holds one until the process ends.  Nothing is allocated or freed, by this call
 * or by anything it calls, and the scratch needs no clearing between calls.  The
 * limit is the one of bdr_qsnr_sweep: 1 <= n_fmts <= 1024, else BDR_ERR_SHAPE
 * (longer lists reuse the array chunk by chunk, so the tensor and the list may have
 * any size the other entry point takes).  All calls on one GPU share that GPU's
 * array: calls that overlap in time on one GPU (two streams, two host threads) race
 * on it and give undefined sums; order them on one stream.  BDR_ERR_LAUNCH when the
 * array's address cannot be resolved on the current device. */
int bdr_qsnr_sweep_static(const bdr_format *fmts, int32_t n_fmts, const void *x, int dtype,
                          int64_t rows, int64_t cols, int64_t ld, double *qsnr_db, double *sums,
                          void *hip_stream);

/* Host only.  Size of the fixed scratch array bdr_qsnr_sweep_static works in. */
size_t bdr_qsnr_sweep_static_scratch_bytes(void);

/* Host only.  Bytes of device workspace with which mx_gemm runs in its two-pass
 * form: (M + N) * K BF16 values, each operand rounded up to 256 bytes (the FP6 and FP4
 * block images need less).  0 when a size is negative or above 2^20. */
size_t mx_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K);

/* C = Ahat * Bhat^T in FP32, where Ahat [M x K] and Bhat [N x K] are the values of
 * two packed images blocked along K (Sec. V: both inputs of a tensor operation are
 * MX-quantized, along the reduction dimension).  Operands are brought, exactly, to a
 * form the matrix cores take and the products are accumulated in FP32: BF16 (8
 * significant bits hold any MX element), or, in the two-pass form when both formats
 * have m <= 4, FP6 elements under one power-of-two scale
 * per block of 16 (M 2^-tau has at most 4 significant bits over 5 binades, which
 * sign + 2 exponent + 3 fraction bits hold), at twice the BF16 rate; when both have
 * m = 2 and M, N, K are at least 128, FP4 elements (M 2^-tau is one of 0, 0.5, 1, 1.5, 2, 3,
 * which sign + 2 exponent + 1 fraction bit hold) at the same rate and half the bytes.
 *   fa, fb : formats of A and B; the two may differ.  Table II's family (k1 16, d1 8,
 *            k2 2, d2 1, m 7, 4 or 2) has kernels of its own in every form.  Any other
 *            format whose elements BF16 holds exactly (m + 2^d2 - 1 <= 8: e.g. block
 *            floating point, d2 = 0, which Sec. IV compares against) is taken in the
 *            two-pass BF16 form, so it needs the workspace (BDR_ERR_WORKSPACE without)
 *            and K a multiple of its k1; anything else is BDR_ERR_FORMAT.  The rounding
 *            rule plays no part here
 *   a_*, b_* : device, the three planes of each image as bdr_quantize wrote them
 *            (B is what BDR_AXIS_COL gives on a [K x N] tensor), 16-byte aligned
 *   C      : device, [M x N] floats, pitch ldc >= N elements, fully overwritten
 *   workspace : device, 16-byte aligned, or NULL.  With at least
 *            mx_gemm_workspace_bytes(M, N, K) bytes (less is BDR_ERR_WORKSPACE) each
 *            operand is rewritten once into it (as BF16, FP6 blocks or FP4 blocks) and
 *            a plain GEMM kernel does the products (the faster form: 2.9x at 8192^3 for
 *            MX6); it is scratch, overwritten, and calls that share it must be
 *            ordered on one stream.  With NULL the expansion to BF16 happens inside
 *            the GEMM kernel, once per tile of C, and no memory beyond the arguments
 *            is touched.  Every product is exact in all forms; the forms differ only
 *            in where the FP32 sum over K is rounded (for M > 64 the BF16 forms give
 *            the same bits as each other).  With M <= 64 the two-pass form does not
 *            tile: it streams once over B's rewritten image (over B's planes
 *            themselves, expanded in registers, when the product is the BF16 one), so
 *            such a call (a decoding step) costs about the time those bytes take; the
 *            sum over K is then added in another, equally fixed, order.
 * K must be a multiple of 64 and M, N, K at most 2^20 each, else BDR_ERR_SHAPE; M and N
 * are free (tiles that hang over the edge of C cost as much as full ones: multiples of 256,
 * else of 128, waste nothing).  M = 0 or N = 0 launches nothing; K = 0 writes zeros.  Block
 * exponent codes from 1 up are exact in every form: the matrix cores take BF16 subnormals
 * (elements of blocks with the lowest codes) as they are.  Inf/NaN codes and sums that are
 * FP32 subnormals are outside the supported domain. */
int mx_gemm(const bdr_format *fa, const bdr_format *fb, const void *a_codes, const void *a_sexp,
            const void *a_mexp, const void *b_codes, const void *b_sexp, const void *b_mexp,
            int64_t M, int64_t N, int64_t K, float *C, int64_t ldc, void *workspace,
            size_t workspace_bytes, void *hip_stream);

/* mx_gemm with the type of C chosen by the caller: c_dtype BDR_F32 is mx_gemm itself;
 * with BDR_BF16 each FP32 sum is rounded once more, to nearest even, as it is stored
 * (the tensors between tensor operations are BF16 in the paper's compute flow, Sec. V
 * "Training": this is the cast the consumer of the product would otherwise make in a pass
 * of its own).  C then needs the alignment of one element; everything else as for
 * mx_gemm.  Any other c_dtype is BDR_ERR_DTYPE. */
int mx_gemm_to(const bdr_format *fa, const bdr_format *fb, const void *a_codes, const void *a_sexp,
               const void *a_mexp, const void *b_codes, const void *b_sexp, const void *b_mexp,
               int64_t M, int64_t N, int64_t K, void *C, int c_dtype, int64_t ldc, void *workspace,
               size_t workspace_bytes, void *hip_stream);

/* Operands made by the quantizer itself.  A tensor that is quantized only to be multiplied
 * (Sec. V: both inputs of each of the three tensor operations of a training iteration,
 * quantized along that operation's reduction axis) need not pass through the three planes:
 * bdr_quantize_operand quantizes x (Sec. IX, as bdr_quantize does, nearest even) straight
 * into an image the product kernel reads - what mx_gemm's two-pass form would make of the
 * planes in its workspace, byte for byte - and mx_gemm_operands multiplies two such images.
 * Table II's formats with nearest-even rounding only (BDR_ERR_FORMAT otherwise); three kinds
 * of image, and both operands of a product must be of the same kind:
 *   BDR_OPERAND_FP6  : MX6 and MX4 (m <= 4): 16 E2M3 codes and a scale byte per block, for
 *                      the block-scaled FP6 product (one byte per element)
 *   BDR_OPERAND_BF16 : MX9, MX6, MX4: the dequantized values in BF16 (exact), for the BF16
 *                      product (two bytes per element)
 *   BDR_OPERAND_FP4  : MX4 only: 16 E2M1 codes per block (half a byte per element), followed
 *                      by an image of one scale byte per block whose rows are padded to a
 *                      multiple of 128, for the block-scaled FP4 product
 *   mx_operand_bytes : host only; bytes of the image of an operand of `rows` rows and
 *            reduction length K (a multiple of 64; of 128 for FP4); 0 for what is not taken
 *   bdr_quantize_operand : x device, [rows x cols] of dtype, pitch ld, aligned as for
 *            bdr_quantize.  BDR_AXIS_ROW: the operand is x, its K is cols (a multiple of
 *            64; of 128 for FP4).  BDR_AXIS_COL: the operand is the transpose of x, [cols x
 *            rows], its K is rows (a multiple of 128; cols a multiple of 64 for FP32, of
 *            128 for BF16 and for FP4 images).
 *            b_operand: 0 for the image of A, 1 for the image of B (FP6 images differ in
 *            where the block's scale byte sits; the others do not).  out: device, 16-byte
 *            aligned, mx_operand_bytes(fmt, operand rows, K, image) bytes, fully overwritten
 *   mx_gemm_operands : C [M x N] = A B^T from the image of A [M x K] and the image of B
 *            [N x K]; C, c_dtype, ldc as for mx_gemm_to.  No workspace is needed.
 * Other shapes, or an unknown image kind, are BDR_ERR_SHAPE. */
enum bdr_operand_image { BDR_OPERAND_FP6 = 0, BDR_OPERAND_BF16 = 1, BDR_OPERAND_FP4 = 2 };
size_t mx_operand_bytes(const bdr_format *fmt, int64_t rows, int64_t K, int image);
int bdr_quantize_operand(const bdr_format *fmt, const void *x, int dtype, int64_t rows, int64_t cols,
                         int64_t ld, int axis, int image, int b_operand, void *out, void *hip_stream);
int mx_gemm_operands(const bdr_format *fa, const bdr_format *fb, const void *image_a, const void *image_b,
                     int image, int64_t M, int64_t N, int64_t K, void *C, int c_dtype, int64_t ldc,
                     void *hip_stream);

/* Host only.  Bytes of device workspace mx_dot_pipeline needs: (M + N) * K BF16 values, each
 * operand rounded up to 256 bytes.  0 when a size is negative or above 2^20. */
size_t mx_dot_pipeline_workspace_bytes(int64_t M, int64_t N, int64_t K);

/* C = Ahat * Bhat^T through a bit-true model of the dot-product pipeline the paper outlines
 * for BDR formats (Sec. IV-B, "Dot Product Architecture" and the caption of the pipeline
 * figure): the Hadamard product of every block of k1 elements is reduced to one integer, each
 * sub-block shifted right by its two microexponents on the way; the r / k1 block results of a
 * pass are aligned to the largest exponent among them and added in a fixed-point word of
 * f_bits bits; a dot product longer than r takes K / r passes, added in FP32.  Where the text
 * leaves the arithmetic open the model takes these readings: nothing is lost inside a block
 * (the datapath is two bits wider below the binary point); blocks are aligned to the largest
 * SEa + SEb of the pass; the word has f_bits - 1 magnitude bits, the top one level with the
 * top bit a block result can have (ma + mb + 6 bits), and what falls below the word is dropped
 * towards minus infinity; a pass is rounded once to FP32, nearest even.  With f_bits = 25 (the
 * paper's choice for every d1 = 8 format) and r = 64 this is what the paper's evaluation
 * assumes a native unit does; mx_gemm adds the same exact products in FP32 instead.
 *   fa, fb, planes, M, N, C, ldc : as for mx_gemm (Table II formats, images blocked along K)
 *   K      : a multiple of 64, at least 64
 *   r      : the unit's dot-product length: a multiple of 64 that divides K (r = K: one pass)
 *   f_bits : 2 .. 26
 *   workspace : device, 16-byte aligned, mx_dot_pipeline_workspace_bytes(M, N, K) bytes; scratch
 * Results that are FP32 subnormals and Inf/NaN codes are outside the supported domain. */
int mx_dot_pipeline(const bdr_format *fa, const bdr_format *fb, const void *a_codes,
                    const void *a_sexp, const void *a_mexp, const void *b_codes, const void *b_sexp,
                    const void *b_mexp, int64_t M, int64_t N, int64_t K, int64_t r, int32_t f_bits,
                    float *C, int64_t ldc, void *workspace, size_t workspace_bytes,
                    void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* BDR_MX_H */
