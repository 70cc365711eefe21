// Host-side declarations shared by the translation units of libbdr_mx.so.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bdr_mx.h"

namespace bdr {

// Table II family by layout alone: k1 16, k2 2, d1 8, d2 1; m 7, 4 or 2.  This is all
// that reading a packed image depends on (decoding never looks at the rounding rule).
inline bool is_mx_layout(const bdr_format &f)
{
    return f.k1 == 16 && f.k2 == 2 && f.d1 == 8 && f.d2 == 1 && (f.m == 7 || f.m == 4 || f.m == 2);
}

// ... and rounded to nearest even: what the specialised quantizers implement.
inline bool is_mx(const bdr_format &f) { return is_mx_layout(f) && f.rounding == BDR_RNE; }

inline int launch_status()
{
    return hipGetLastError() == hipSuccess ? BDR_OK : BDR_ERR_LAUNCH;
}

// A workgroup may use more than 64 KiB of dynamic LDS only after the kernel has been
// given that limit on the device it is launched on.  `state` (one per kernel, zero
// initialised) remembers the answer per device: 0 not asked, 1 granted, -1 refused.
// Two host threads that race on the first call both ask and get the same answer.
constexpr int kMaxDevices = 64;
inline bool grant_dynamic_lds(const void *kernel, size_t bytes, signed char (&state)[kMaxDevices])
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0) return false;
    signed char local = 0;
    signed char &st = dev < kMaxDevices ? state[dev] : local;
    if (st == 0) {
        int lds = 0;
        const bool ok =
            hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) == hipSuccess &&
            (size_t)lds >= bytes &&
            hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) == hipSuccess;
        (void)hipGetLastError();
        st = ok ? 1 : -1;
    }
    return st > 0;
}

// Blocks along the contiguous axis.  All arguments were validated by the caller.
int quantize_row(const bdr_format &f, const void *x, int dtype, int64_t rows, int64_t cols,
                 int64_t ld, void *codes, void *sexp, void *mexp, hipStream_t s);
int dequantize_row(const bdr_format &f, const void *codes, const void *sexp, const void *mexp,
                   int64_t rows, int64_t cols, void *y, int dtype, int64_t ld, hipStream_t s);
// Table II operand -> BF16, every block taking the exponent code se_code instead of its own
// (rows * cols a multiple of 32; the exponent plane is not read).
int dequantize_row_fixed_exponent(const bdr_format &f, const void *codes, const void *mexp, int64_t rows,
                                  int64_t cols, void *y, int se_code, hipStream_t s);
int gather_dequantize_row(const bdr_format &f, const void *codes, const void *sexp, const void *mexp,
                          int64_t table_rows, int64_t cols, const int64_t *idx, int64_t n_idx, void *y,
                          int dtype, hipStream_t s);
// tables whose rows keep their three runs together (cols a multiple of 64)
int table_pack(const bdr_format &f, const void *codes, const void *sexp, const void *mexp, int64_t rows,
               int64_t cols, void *table, hipStream_t s);
int table_gather_dequantize(const bdr_format &f, const void *table, int64_t table_rows, int64_t cols,
                            const int64_t *idx, int64_t n_idx, void *y, int dtype, hipStream_t s);
int qdq_row(const bdr_format &f, const void *x, void *y, int dtype, int64_t rows, int64_t cols,
            int64_t ld, hipStream_t s);

// Blocks down the columns (planes indexed as for the transposed tensor).
int quantize_col(const bdr_format &f, const void *x, int dtype, int64_t rows, int64_t cols,
                 int64_t ld, void *codes, void *sexp, void *mexp, hipStream_t s);
int dequantize_col(const bdr_format &f, const void *codes, const void *sexp, const void *mexp,
                   int64_t rows, int64_t cols, void *y, int dtype, int64_t ld, hipStream_t s);
int qdq_col(const bdr_format &f, const void *x, void *y, int dtype, int64_t rows, int64_t cols,
            int64_t ld, hipStream_t s);

// Column blocks through the general (one element at a time) kernels.
// what: 0 quantize (x -> planes), 1 dequantize (planes -> y), 2 fused (x -> y).
int generic_col(int what, const bdr_format &f, const void *x, void *y, int dtype, int64_t rows,
                int64_t cols, int64_t ld, void *codes, void *sexp, void *mexp, hipStream_t s);

size_t sweep_workspace_bytes(int32_t n_fmts);
int qsnr_sweep(const bdr_format *fmts, int32_t n_fmts, const void *x, int dtype, int64_t rows,
               int64_t cols, int64_t ld, double *qsnr_db, double *sums, void *workspace,
               hipStream_t s);

// The same with the library's own fixed scratch array (no workspace argument, nothing allocated).
size_t sweep_static_scratch_bytes();
int qsnr_sweep_static(const bdr_format *fmts, int32_t n_fmts, const void *x, int dtype, int64_t rows,
                      int64_t cols, int64_t ld, double *qsnr_db, double *sums, hipStream_t s);

int gemm(const bdr_format &fa, const bdr_format &fb, const void *a_codes, const void *a_sexp,
         const void *a_mexp, const void *b_codes, const void *b_sexp, const void *b_mexp,
         int64_t M, int64_t N, int64_t K, void *C, int64_t ldc, int c_bf16, hipStream_t s);
// (`dry`: only request what the kernel needs, launch nothing; the same for the products below)
int gemm_bf16(const void *A, const void *B, int64_t M, int64_t N, int64_t K, void *C, int64_t ldc, int c_bf16,
              bool dry, hipStream_t s);
// Table II planes of a [rows x K] operand -> BF16 tiled along K ([K / 32][rows][32 elements]),
// and the GEMM on two such images.
int to_bf16_tiled(const bdr_format &f, const void *codes, const void *sexp, const void *mexp, int64_t rows,
                  int64_t K, void *out, hipStream_t s);
int gemm_bf16_tiled(const void *A, const void *B, int64_t M, int64_t N, int64_t K, void *C, int64_t ldc, int c_bf16,
                    bool dry, hipStream_t s);
// MX6 / MX4 planes of a [rows x K] operand (K % 64 == 0) -> one 16-byte FP6 chunk per block,
// tiled along K ([K / 64][rows][4 chunks]), and the GEMM on two such images.
int to_fp6(const bdr_format &f, const void *codes, const void *sexp, const void *mexp,
           int64_t rows, int64_t K, void *out, bool b_operand, hipStream_t s);
int gemm_fp6(const void *A, const void *B, int64_t M, int64_t N, int64_t K, void *C, int64_t ldc, int c_bf16,
             bool dry, hipStream_t s);
// Quantize (Table II, nearest even) straight into an operand image: kind 0 / 1 the FP6 image of an
// A / B operand (MX6, MX4), kind 2 the BF16 image (to_bf16_tiled's).  Blocks along the rows of x
// [rows x cols] (the operand is x, K = cols), or down its columns (the operand is the transpose,
// K = rows; whole tiles only: quantize_operand_col_ok).
int quantize_operand_row(const bdr_format &f, const void *x, int dtype, int64_t rows, int64_t cols, int64_t ld,
                         void *out, int kind, hipStream_t s);
bool quantize_operand_col_ok(int dtype, int64_t rows, int64_t cols);
int quantize_operand_col(const bdr_format &f, const void *x, int dtype, int64_t rows, int64_t cols, int64_t ld,
                         void *out, int kind, hipStream_t s);
// The FP4 form of the two-pass product (MX4 x MX4): image writer, size of its scale image,
// and the product on two such images (K_out % 128 == 0).
bool gemm_bf16_planes_ok(int64_t M, int64_t K);
int gemm_bf16_planes(const void *A, const bdr_format &fb, const void *b_codes, const void *b_sexp,
                     const void *b_mexp, int64_t M, int64_t N, int64_t K, void *C, int64_t ldc, int c_bf16,
                     hipStream_t s);
int to_fp4(const void *codes, const void *sexp, const void *mexp, int64_t rows, int64_t K, int64_t K_out,
           void *out, void *scales, hipStream_t s);
size_t fp4_scale_bytes(int64_t rows, int64_t K_out);
int gemm_fp4(const void *A, const void *SA, const void *B, const void *SB, int64_t M, int64_t N, int64_t K,
             void *C, int64_t ldc, int c_bf16, bool dry, hipStream_t s);

// The dot-product pipeline model (mx_dot_pipeline.hip); arguments validated by the caller.
int dot_pipeline(const bdr_format &fa, const bdr_format &fb, const void *a_codes, const void *a_sexp,
                 const void *a_mexp, const void *b_codes, const void *b_sexp, const void *b_mexp,
                 int64_t M, int64_t N, int64_t K, int64_t r, int f_bits, float *C, int64_t ldc,
                 void *workspace, hipStream_t s);

}  // namespace bdr
