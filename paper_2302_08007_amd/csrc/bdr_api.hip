// C ABI of libbdr_mx.so: argument checking and dispatch.  No kernel lives here.
//
// Every entry point validates on the host first and returns a status; nothing is
// launched unless every check passed, because a kernel that is handed a shape it
// does not expect can fault the GPU.
#include "bdr_internal.hpp"

namespace {

inline bool is_pow2(int32_t v) { return v > 0 && (v & (v - 1)) == 0; }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t elem_size(int dtype) { return dtype == BDR_F32 ? 4 : 2; }

int check_format(const bdr_format *f)
{
    if (!f) return BDR_ERR_NULL;
    if (!is_pow2(f->k1) || f->k1 > 256) return BDR_ERR_FORMAT;
    if (!is_pow2(f->k2) || f->k2 > f->k1) return BDR_ERR_FORMAT;
    if (f->d1 != 8) return BDR_ERR_FORMAT;
    if (f->d2 < 0 || f->d2 > 3) return BDR_ERR_FORMAT;
    if (f->m < 1 || f->m > 8) return BDR_ERR_FORMAT;
    if (f->rounding != BDR_RNE && f->rounding != BDR_RNA && f->rounding != BDR_RTZ)
        return BDR_ERR_FORMAT;
    return BDR_OK;
}

// Length of the blocked axis as the planes store it: a short last block is stored whole, its
// pads as code 0 (Sec. IX, the remark after Theorem 1: a vector shorter than k1 is a block of
// its own length).
inline int64_t padded_len(const bdr_format *f, int64_t n) { return (n + f->k1 - 1) / f->k1 * f->k1; }

// Shape rules common to quantize / dequantize / fused.  Whole shapes: the blocked axis is a
// multiple of max(k1, 8) (a lane owns 8 consecutive elements of a block row), and for column
// blocks the contiguous axis is a multiple of 8 as well.  Other shapes are taken when `loose`
// is given (it is set for them): they run element by element, so all they need is a padded
// length that is a multiple of 8, which only k1 < 8 can miss.
int check_shape(const bdr_format *f, int dtype, int64_t rows, int64_t cols, int64_t ld, int axis,
                bool *loose = nullptr)
{
    if (loose) *loose = false;
    if (dtype != BDR_F32 && dtype != BDR_BF16) return BDR_ERR_DTYPE;
    if (axis != BDR_AXIS_ROW && axis != BDR_AXIS_COL) return BDR_ERR_SHAPE;
    if (rows < 0 || cols < 0 || ld < cols) return BDR_ERR_SHAPE;
    if (rows > 0 && cols > 0 && rows > ((int64_t)1 << 40) / cols) return BDR_ERR_SHAPE;
    const int64_t unit = f->k1 > 8 ? f->k1 : 8;
    const int64_t blocked = axis == BDR_AXIS_ROW ? cols : rows;
    if (blocked % unit != 0 || (axis == BDR_AXIS_COL && cols % 8 != 0)) {
        if (!loose || padded_len(f, blocked) % 8 != 0) return BDR_ERR_SHAPE;
        *loose = true;
    }
    return BDR_OK;
}

// Whole shapes move in 16-byte pieces; loose ones element by element.
int check_tensor_ptr(const void *p, int dtype, int64_t ld, bool loose = false)
{
    if (!p) return BDR_ERR_NULL;
    if (loose) return reinterpret_cast<uintptr_t>(p) % elem_size(dtype) ? BDR_ERR_ALIGN : BDR_OK;
    if (!aligned16(p) || (ld * (int64_t)elem_size(dtype)) % 16 != 0) return BDR_ERR_ALIGN;
    return BDR_OK;
}

int check_planes(const bdr_format *f, const void *codes, const void *sexp, const void *mexp)
{
    if (!codes || !sexp || (f->d2 > 0 && !mexp)) return BDR_ERR_NULL;
    if (!aligned16(codes) || !aligned16(sexp) || (f->d2 > 0 && !aligned16(mexp)))
        return BDR_ERR_ALIGN;
    return BDR_OK;
}

inline bool bf16_exact(const bdr_format *f) { return f->m + ((1 << f->d2) - 1) <= 8; }

}  // namespace

extern "C" {

const char *bdr_status_string(int status)
{
    switch (status) {
    case BDR_OK: return "ok";
    case BDR_ERR_NULL: return "a required pointer is NULL";
    case BDR_ERR_FORMAT: return "BDR format not implemented";
    case BDR_ERR_SHAPE: return "bad shape for this format";
    case BDR_ERR_ALIGN: return "pointer or pitch not 16-byte aligned";
    case BDR_ERR_DTYPE: return "bad dtype for this call";
    case BDR_ERR_LAUNCH: return "HIP launch failed";
    case BDR_ERR_WORKSPACE: return "workspace missing or too small";
    default: return "unknown status";
    }
}

int bdr_format_validate(const bdr_format *fmt) { return check_format(fmt); }

int bdr_packed_sizes(const bdr_format *fmt, int64_t rows, int64_t cols, int axis,
                     size_t *codes_bytes, size_t *sexp_bytes, size_t *mexp_bytes)
{
    int st = check_format(fmt);
    if (st) return st;
    bool loose;
    st = check_shape(fmt, BDR_F32, rows, cols, cols, axis, &loose);
    if (st) return st;
    const uint64_t n = axis == BDR_AXIS_ROW ? (uint64_t)rows * (uint64_t)padded_len(fmt, cols)
                                            : (uint64_t)cols * (uint64_t)padded_len(fmt, rows);
    if (codes_bytes) *codes_bytes = (size_t)(n * (uint64_t)(fmt->m + 1) / 8u);  // n % 8 == 0
    if (sexp_bytes) *sexp_bytes = (size_t)(n / (uint64_t)fmt->k1);
    if (mexp_bytes) *mexp_bytes = (size_t)((n / (uint64_t)fmt->k2 * (uint64_t)fmt->d2 + 7u) / 8u);
    return BDR_OK;
}

int bdr_quantize(const bdr_format *fmt, const void *x, int dtype, int64_t rows, int64_t cols,
                 int64_t ld, int axis, void *codes, void *sexp, void *mexp, void *hip_stream)
{
    int st = check_format(fmt);
    if (st) return st;
    bool loose;
    st = check_shape(fmt, dtype, rows, cols, ld, axis, &loose);
    if (st) return st;
    if (rows == 0 || cols == 0) return BDR_OK;
    st = check_tensor_ptr(x, dtype, ld, loose);
    if (st) return st;
    st = check_planes(fmt, codes, sexp, mexp);
    if (st) return st;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (axis == BDR_AXIS_ROW)
        return bdr::quantize_row(*fmt, x, dtype, rows, cols, ld, codes, sexp, mexp, s);
    return bdr::quantize_col(*fmt, x, dtype, rows, cols, ld, codes, sexp, mexp, s);
}

int bdr_dequantize(const bdr_format *fmt, const void *codes, const void *sexp, const void *mexp,
                   int64_t rows, int64_t cols, int axis, void *y, int dtype, int64_t ld,
                   void *hip_stream)
{
    int st = check_format(fmt);
    if (st) return st;
    bool loose;
    st = check_shape(fmt, dtype, rows, cols, ld, axis, &loose);
    if (st) return st;
    if (dtype == BDR_BF16 && !bf16_exact(fmt)) return BDR_ERR_DTYPE;
    if (rows == 0 || cols == 0) return BDR_OK;
    st = check_tensor_ptr(y, dtype, ld, loose);
    if (st) return st;
    st = check_planes(fmt, codes, sexp, mexp);
    if (st) return st;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (axis == BDR_AXIS_ROW)
        return bdr::dequantize_row(*fmt, codes, sexp, mexp, rows, cols, y, dtype, ld, s);
    return bdr::dequantize_col(*fmt, codes, sexp, mexp, rows, cols, y, dtype, ld, s);
}

int bdr_gather_dequantize(const bdr_format *fmt, const void *codes, const void *sexp,
                          const void *mexp, int64_t table_rows, int64_t cols, const int64_t *indices,
                          int64_t n_indices, void *y, int dtype, void *hip_stream)
{
    int st = check_format(fmt);
    if (st) return st;
    if (!bdr::is_mx_layout(*fmt)) return BDR_ERR_FORMAT;
    if (dtype != BDR_F32 && dtype != BDR_BF16) return BDR_ERR_DTYPE;
    if (table_rows < 0 || cols < 0 || n_indices < 0 || cols % 32 != 0) return BDR_ERR_SHAPE;
    if (cols > ((int64_t)1 << 24) || table_rows > ((int64_t)1 << 40) / (cols > 0 ? cols : 1) ||
        n_indices > ((int64_t)1 << 40) / (cols > 0 ? cols : 1))
        return BDR_ERR_SHAPE;
    if (n_indices == 0 || cols == 0) return BDR_OK;
    if (!indices) return BDR_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(indices) & 7u) != 0) return BDR_ERR_ALIGN;
    st = check_tensor_ptr(y, dtype, cols);
    if (st) return st;
    if (table_rows > 0) {
        st = check_planes(fmt, codes, sexp, mexp);
        if (st) return st;
    }
    return bdr::gather_dequantize_row(*fmt, codes, sexp, mexp, table_rows, cols, indices, n_indices, y,
                                      dtype, static_cast<hipStream_t>(hip_stream));
}

// Checks shared by the two calls on tables that keep a row's runs together.
static int check_table(const bdr_format *fmt, int64_t table_rows, int64_t cols)
{
    int st = check_format(fmt);
    if (st) return st;
    if (!bdr::is_mx_layout(*fmt)) return BDR_ERR_FORMAT;
    if (table_rows < 0 || cols < 0 || cols % 64 != 0) return BDR_ERR_SHAPE;
    if (cols > ((int64_t)1 << 24) || table_rows > ((int64_t)1 << 40) / (cols > 0 ? cols : 1)) return BDR_ERR_SHAPE;
    return BDR_OK;
}

size_t bdr_table_row_bytes(const bdr_format *fmt, int64_t cols)
{
    if (check_table(fmt, 0, cols) != BDR_OK) return 0;
    return (size_t)(cols / 8 * (fmt->m + 1) + 2 * (cols / 16));
}

int bdr_table_pack(const bdr_format *fmt, const void *codes, const void *sexp, const void *mexp,
                   int64_t table_rows, int64_t cols, void *table, void *hip_stream)
{
    int st = check_table(fmt, table_rows, cols);
    if (st) return st;
    if (table_rows == 0 || cols == 0) return BDR_OK;
    st = check_planes(fmt, codes, sexp, mexp);
    if (st) return st;
    if (!table) return BDR_ERR_NULL;
    if (!aligned16(table)) return BDR_ERR_ALIGN;
    return bdr::table_pack(*fmt, codes, sexp, mexp, table_rows, cols, table, static_cast<hipStream_t>(hip_stream));
}

int bdr_table_gather_dequantize(const bdr_format *fmt, const void *table, int64_t table_rows, int64_t cols,
                                const int64_t *indices, int64_t n_indices, void *y, int dtype,
                                void *hip_stream)
{
    int st = check_table(fmt, table_rows, cols);
    if (st) return st;
    if (dtype != BDR_F32 && dtype != BDR_BF16) return BDR_ERR_DTYPE;
    if (n_indices < 0 || n_indices > ((int64_t)1 << 40) / (cols > 0 ? cols : 1)) return BDR_ERR_SHAPE;
    if (n_indices == 0 || cols == 0) return BDR_OK;
    if (!indices) return BDR_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(indices) & 7u) != 0) return BDR_ERR_ALIGN;
    st = check_tensor_ptr(y, dtype, cols);
    if (st) return st;
    if (table_rows > 0) {
        if (!table) return BDR_ERR_NULL;
        if (!aligned16(table)) return BDR_ERR_ALIGN;
    }
    return bdr::table_gather_dequantize(*fmt, table, table_rows, cols, indices, n_indices, y, dtype,
                                        static_cast<hipStream_t>(hip_stream));
}

int bdr_tile_packing(const bdr_format *fmt, int64_t tile_elements, int64_t interface_bytes,
                     int64_t *packed_bytes, int64_t *transfers, double *efficiency)
{
    int st = check_format(fmt);
    if (st) return st;
    if (tile_elements < 1 || interface_bytes < 1 || tile_elements > ((int64_t)1 << 40) ||
        interface_bytes > ((int64_t)1 << 20))
        return BDR_ERR_SHAPE;
    // bits = tile * ((m+1) + d1/k1 + d2/k2), taken over whole blocks and sub-blocks
    const int64_t nb = (tile_elements + fmt->k1 - 1) / fmt->k1, ns = (tile_elements + fmt->k2 - 1) / fmt->k2;
    const int64_t bits = tile_elements * (fmt->m + 1) + nb * fmt->d1 + ns * fmt->d2;
    const int64_t bytes = (bits + 7) / 8;
    const int64_t lines = (bytes + interface_bytes - 1) / interface_bytes;
    if (packed_bytes) *packed_bytes = bytes;
    if (transfers) *transfers = lines;
    if (efficiency) *efficiency = (double)bytes / (double)(lines * interface_bytes);
    return BDR_OK;
}

int bdr_quantize_dequantize(const bdr_format *fmt, const void *x, void *y, int dtype,
                            int64_t rows, int64_t cols, int64_t ld, int axis, void *hip_stream)
{
    int st = check_format(fmt);
    if (st) return st;
    bool loose;
    st = check_shape(fmt, dtype, rows, cols, ld, axis, &loose);
    if (st) return st;
    if (dtype == BDR_BF16 && !bf16_exact(fmt)) return BDR_ERR_DTYPE;
    if (rows == 0 || cols == 0) return BDR_OK;
    st = check_tensor_ptr(x, dtype, ld, loose);
    if (st) return st;
    st = check_tensor_ptr(y, dtype, ld, loose);
    if (st) return st;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (axis == BDR_AXIS_ROW) return bdr::qdq_row(*fmt, x, y, dtype, rows, cols, ld, s);
    return bdr::qdq_col(*fmt, x, y, dtype, rows, cols, ld, s);
}

size_t bdr_qsnr_sweep_workspace_bytes(int32_t n_fmts)
{
    if (n_fmts < 1 || n_fmts > 1024) return 0;
    return bdr::sweep_workspace_bytes(n_fmts);
}

// Argument checks shared by the two sweep entry points: formats and outputs ...
static int check_sweep_head(const bdr_format *fmts, int32_t n_fmts, int dtype, int64_t rows,
                            int64_t cols, int64_t ld, const double *qsnr_db, const double *sums)
{
    if (!fmts) return BDR_ERR_NULL;
    if (n_fmts < 1 || n_fmts > 1024) return BDR_ERR_SHAPE;
    for (int32_t k = 0; k < n_fmts; ++k) {
        int st = check_format(&fmts[k]);
        if (st) return st;
        st = check_shape(&fmts[k], dtype, rows, cols, ld, BDR_AXIS_ROW);
        if (st) return st;
    }
    if (!qsnr_db || !sums) return BDR_ERR_NULL;
    return BDR_OK;
}

// ... then alignment and the tensor.
static int check_sweep_tail(const void *x, int dtype, int64_t rows, int64_t cols, int64_t ld,
                            const double *qsnr_db, const double *sums)
{
    if ((reinterpret_cast<uintptr_t>(qsnr_db) & 7u) || (reinterpret_cast<uintptr_t>(sums) & 7u))
        return BDR_ERR_ALIGN;
    if (rows > 0 && cols > 0) return check_tensor_ptr(x, dtype, ld);
    return BDR_OK;
}

int bdr_qsnr_sweep(const bdr_format *fmts, int32_t n_fmts, const void *x, int dtype, int64_t rows,
                   int64_t cols, int64_t ld, double *qsnr_db, double *sums, void *workspace,
                   size_t workspace_bytes, void *hip_stream)
{
    int st = check_sweep_head(fmts, n_fmts, dtype, rows, cols, ld, qsnr_db, sums);
    if (st) return st;
    if (!workspace || workspace_bytes < bdr::sweep_workspace_bytes(n_fmts)) return BDR_ERR_WORKSPACE;
    if (!aligned16(workspace)) return BDR_ERR_ALIGN;
    st = check_sweep_tail(x, dtype, rows, cols, ld, qsnr_db, sums);
    if (st) return st;
    return bdr::qsnr_sweep(fmts, n_fmts, x, dtype, rows, cols, ld, qsnr_db, sums, workspace,
                           static_cast<hipStream_t>(hip_stream));
}

size_t bdr_qsnr_sweep_static_scratch_bytes(void) { return bdr::sweep_static_scratch_bytes(); }

int bdr_qsnr_sweep_static(const bdr_format *fmts, int32_t n_fmts, const void *x, int dtype,
                          int64_t rows, int64_t cols, int64_t ld, double *qsnr_db, double *sums,
                          void *hip_stream)
{
    int st = check_sweep_head(fmts, n_fmts, dtype, rows, cols, ld, qsnr_db, sums);
    if (st) return st;
    st = check_sweep_tail(x, dtype, rows, cols, ld, qsnr_db, sums);
    if (st) return st;
    return bdr::qsnr_sweep_static(fmts, n_fmts, x, dtype, rows, cols, ld, qsnr_db, sums,
                                  static_cast<hipStream_t>(hip_stream));
}

static size_t gemm_ws_half(int64_t rows, int64_t K)
{
    return ((size_t)rows * (size_t)K * 2 + 255) & ~(size_t)255;
}

size_t mx_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    if (M < 0 || N < 0 || K < 0 || M > (1 << 20) || N > (1 << 20) || K > (1 << 20)) return 0;
    return gemm_ws_half(M, K) + gemm_ws_half(N, K);
}

int mx_gemm_to(const bdr_format *fa, const bdr_format *fb, const void *a_codes, const void *a_sexp,
               const void *a_mexp, const void *b_codes, const void *b_sexp, const void *b_mexp,
               int64_t M, int64_t N, int64_t K, void *C, int c_dtype, int64_t ldc, void *workspace,
               size_t workspace_bytes, void *hip_stream)
{
    if (c_dtype != BDR_F32 && c_dtype != BDR_BF16) return BDR_ERR_DTYPE;
    const int c_bf16 = c_dtype == BDR_BF16;
    int st = check_format(fa);
    if (st) return st;
    st = check_format(fb);
    if (st) return st;
    // Table II's formats have kernels of their own.  Any other pair of formats whose elements
    // BF16 holds exactly goes through the two-pass BF16 form (general dequantize to BF16,
    // then the BF16 product kernel) and therefore needs the workspace.
    const bool both_mx = bdr::is_mx_layout(*fa) && bdr::is_mx_layout(*fb);
    if (!both_mx && (!bf16_exact(fa) || !bf16_exact(fb))) return BDR_ERR_FORMAT;
    if (M < 0 || N < 0 || K < 0 || ldc < N) return BDR_ERR_SHAPE;
    if (K % 64 != 0) return BDR_ERR_SHAPE;
    if (!both_mx && (K % fa->k1 != 0 || K % fb->k1 != 0)) return BDR_ERR_SHAPE;
    if (M > (1 << 20) || N > (1 << 20) || K > (1 << 20)) return BDR_ERR_SHAPE;
    if (M == 0 || N == 0) return BDR_OK;
    if (!C) return BDR_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(C) % elem_size(c_dtype) != 0) return BDR_ERR_ALIGN;
    if (K > 0) {
        st = check_planes(fa, a_codes, a_sexp, a_mexp);
        if (st) return st;
        st = check_planes(fb, b_codes, b_sexp, b_mexp);
        if (st) return st;
    }
    if (!both_mx && K > 0 && !workspace) return BDR_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (workspace && K > 0) {
        // two passes: each operand is rewritten once in the form the matrix cores take, then
        // a plain GEMM kernel runs on the two images
        if (workspace_bytes < mx_gemm_workspace_bytes(M, N, K)) return BDR_ERR_WORKSPACE;
        if (!aligned16(workspace)) return BDR_ERR_ALIGN;
        char *wa = static_cast<char *>(workspace), *wb = wa + gemm_ws_half(M, K);
        // In each form the product kernel's resources are asked for first (a dry call), so that a
        // refusal comes back before anything is enqueued.
        if (both_mx && fa->m == 2 && fb->m == 2 && M >= 128 && N >= 128 && K >= 128) {
            // MX4 x MX4: both operands as 4-bit E2M1 images, half a byte per element plus one
            // scale byte per block in an image of its own (rows padded to 128, K to 128).  The
            // size conditions keep both inside the operand's half of the workspace.
            const int64_t Kp = (K + 127) / 128 * 128;
            char *sa = wa + (size_t)M * (size_t)(Kp / 2), *sb = wb + (size_t)N * (size_t)(Kp / 2);
            st = bdr::gemm_fp4(wa, sa, wb, sb, M, N, Kp, C, ldc, c_bf16, true, s);
            if (st) return st;
            st = bdr::to_fp4(a_codes, a_sexp, a_mexp, M, K, Kp, wa, sa, s);
            if (st) return st;
            st = bdr::to_fp4(b_codes, b_sexp, b_mexp, N, K, Kp, wb, sb, s);
            if (st) return st;
            return bdr::gemm_fp4(wa, sa, wb, sb, M, N, Kp, C, ldc, c_bf16, false, s);
        }
        if (both_mx && fa->m <= 4 && fb->m <= 4) {
            // MX6 and MX4 elements are exact FP6 values under a per-block power of two:
            // block-scaled FP6 MFMAs, twice the rate of BF16.  One byte per element of workspace.
            st = bdr::gemm_fp6(wa, wb, M, N, K, C, ldc, c_bf16, true, s);
            if (st) return st;
            st = bdr::to_fp6(*fa, a_codes, a_sexp, a_mexp, M, K, wa, false, s);
            if (st) return st;
            st = bdr::to_fp6(*fb, b_codes, b_sexp, b_mexp, N, K, wb, true, s);
            if (st) return st;
            return bdr::gemm_fp6(wa, wb, M, N, K, C, ldc, c_bf16, false, s);
        }
        if (both_mx && bdr::gemm_bf16_planes_ok(M, K)) {
            // few rows of A (a decoding step): only A is expanded; B is streamed once as it is
            // stored and expanded in registers
            st = bdr::to_bf16_tiled(*fa, a_codes, a_sexp, a_mexp, M, K, wa, s);
            if (st) return st;
            return bdr::gemm_bf16_planes(wa, *fb, b_codes, b_sexp, b_mexp, M, N, K, C, ldc, c_bf16, s);
        }
        if (both_mx) {
            // MX9 has 8 significant bits with the sign: each operand is expanded to BF16 (exact),
            // in the K-tiled layout of the ring kernel
            st = bdr::gemm_bf16_tiled(wa, wb, M, N, K, C, ldc, c_bf16, true, s);
            if (st) return st;
            st = bdr::to_bf16_tiled(*fa, a_codes, a_sexp, a_mexp, M, K, wa, s);
            if (st) return st;
            st = bdr::to_bf16_tiled(*fb, b_codes, b_sexp, b_mexp, N, K, wb, s);
            if (st) return st;
            return bdr::gemm_bf16_tiled(wa, wb, M, N, K, C, ldc, c_bf16, false, s);
        }
        // any other format that passed the check above: general dequantize to row-major BF16
        st = bdr::gemm_bf16(wa, wb, M, N, K, C, ldc, c_bf16, true, s);
        if (st) return st;
        st = bdr::dequantize_row(*fa, a_codes, a_sexp, a_mexp, M, K, wa, BDR_BF16, K, s);
        if (st) return st;
        st = bdr::dequantize_row(*fb, b_codes, b_sexp, b_mexp, N, K, wb, BDR_BF16, K, s);
        if (st) return st;
        return bdr::gemm_bf16(wa, wb, M, N, K, C, ldc, c_bf16, false, s);
    }
    return bdr::gemm(*fa, *fb, a_codes, a_sexp, a_mexp, b_codes, b_sexp, b_mexp, M, N, K, C, ldc, c_bf16, s);
}

int mx_gemm(const bdr_format *fa, const bdr_format *fb, const void *a_codes, const void *a_sexp,
            const void *a_mexp, const void *b_codes, const void *b_sexp, const void *b_mexp,
            int64_t M, int64_t N, int64_t K, float *C, int64_t ldc, void *workspace,
            size_t workspace_bytes, void *hip_stream)
{
    return mx_gemm_to(fa, fb, a_codes, a_sexp, a_mexp, b_codes, b_sexp, b_mexp, M, N, K, C, BDR_F32, ldc,
                      workspace, workspace_bytes, hip_stream);
}

// ---- operands made by the quantizer itself

// FP6 images hold MX6 and MX4; BF16 images any of Table II's formats.  Nearest even only: that is
// what the specialised quantizers implement.
static bool operand_format(const bdr_format *f, int image)
{
    if (!bdr::is_mx(*f)) return false;
    return image == BDR_OPERAND_BF16 || (image == BDR_OPERAND_FP6 && f->m <= 4) || (image == BDR_OPERAND_FP4 && f->m == 2);
}
static bool operand_image(int image)
{
    return image == BDR_OPERAND_FP6 || image == BDR_OPERAND_BF16 || image == BDR_OPERAND_FP4;
}
// K of an operand image: whole K steps of the product kernel that takes it
static int64_t operand_k_multiple(int image) { return image == BDR_OPERAND_FP4 ? 128 : 64; }

size_t mx_operand_bytes(const bdr_format *fmt, int64_t rows, int64_t K, int image)
{
    if (check_format(fmt) != BDR_OK || !operand_image(image) || !operand_format(fmt, image)) return 0;
    if (rows < 0 || K < 0 || K % operand_k_multiple(image) != 0 || rows > (1 << 20) || K > (1 << 20)) return 0;
    // FP6: a 16-byte chunk per block of 16; BF16: two bytes per element; FP4: half a byte per
    // element, then one scale byte per block with the rows padded to a multiple of 128
    if (image == BDR_OPERAND_FP4) return (size_t)rows * (size_t)(K / 2) + bdr::fp4_scale_bytes(rows, K);
    return (size_t)rows * (size_t)K * (image == BDR_OPERAND_BF16 ? 2u : 1u);
}

int bdr_quantize_operand(const bdr_format *fmt, const void *x, int dtype, int64_t rows, int64_t cols,
                         int64_t ld, int axis, int image, int b_operand, void *out, void *hip_stream)
{
    int st = check_format(fmt);
    if (st) return st;
    if (!operand_image(image)) return BDR_ERR_SHAPE;
    if (!operand_format(fmt, image)) return BDR_ERR_FORMAT;
    if (dtype != BDR_F32 && dtype != BDR_BF16) return BDR_ERR_DTYPE;
    if (axis != BDR_AXIS_ROW && axis != BDR_AXIS_COL) return BDR_ERR_SHAPE;
    if (rows < 0 || cols < 0 || ld < cols || rows > (1 << 20) || cols > (1 << 20)) return BDR_ERR_SHAPE;
    if (axis == BDR_AXIS_ROW ? cols % operand_k_multiple(image) != 0 : !bdr::quantize_operand_col_ok(dtype, rows, cols))
        return BDR_ERR_SHAPE;
    // (column blocks: the operand's rows are the tensor's columns; the FP4 scale image wants whole groups of 128)
    if (image == BDR_OPERAND_FP4 && axis == BDR_AXIS_COL && cols % 128 != 0) return BDR_ERR_SHAPE;
    if (rows == 0 || cols == 0) return BDR_OK;
    st = check_tensor_ptr(x, dtype, ld);
    if (st) return st;
    if (!out) return BDR_ERR_NULL;
    if (!aligned16(out)) return BDR_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int kind = image == BDR_OPERAND_BF16 ? 2 : image == BDR_OPERAND_FP4 ? 3 : (b_operand ? 1 : 0);
    if (axis == BDR_AXIS_ROW) return bdr::quantize_operand_row(*fmt, x, dtype, rows, cols, ld, out, kind, s);
    return bdr::quantize_operand_col(*fmt, x, dtype, rows, cols, ld, out, kind, s);
}

int mx_gemm_operands(const bdr_format *fa, const bdr_format *fb, const void *image_a, const void *image_b,
                     int image, int64_t M, int64_t N, int64_t K, void *C, int c_dtype, int64_t ldc,
                     void *hip_stream)
{
    if (c_dtype != BDR_F32 && c_dtype != BDR_BF16) return BDR_ERR_DTYPE;
    int st = check_format(fa);
    if (st) return st;
    st = check_format(fb);
    if (st) return st;
    if (!operand_image(image)) return BDR_ERR_SHAPE;
    if (!operand_format(fa, image) || !operand_format(fb, image)) return BDR_ERR_FORMAT;
    if (M < 0 || N < 0 || K < 0 || ldc < N || K % operand_k_multiple(image) != 0) return BDR_ERR_SHAPE;
    if (M > (1 << 20) || N > (1 << 20) || K > (1 << 20)) return BDR_ERR_SHAPE;
    if (M == 0 || N == 0) return BDR_OK;
    if (!C) return BDR_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(C) % elem_size(c_dtype) != 0) return BDR_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int c_bf16 = c_dtype == BDR_BF16;
    if (K == 0)  // the empty sum: mx_gemm's own path for it (no operand is read)
        return bdr::gemm(*fa, *fb, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, M, N, 0, C, ldc, c_bf16, s);
    if (!image_a || !image_b) return BDR_ERR_NULL;
    if (!aligned16(image_a) || !aligned16(image_b)) return BDR_ERR_ALIGN;
    if (image == BDR_OPERAND_FP4) {  // chunks, then the scale image
        const char *sa = static_cast<const char *>(image_a) + (size_t)M * (size_t)(K / 2);
        const char *sb = static_cast<const char *>(image_b) + (size_t)N * (size_t)(K / 2);
        st = bdr::gemm_fp4(image_a, sa, image_b, sb, M, N, K, C, ldc, c_bf16, true, s);
        if (st) return st;
        return bdr::gemm_fp4(image_a, sa, image_b, sb, M, N, K, C, ldc, c_bf16, false, s);
    }
    if (image == BDR_OPERAND_BF16) {
        st = bdr::gemm_bf16_tiled(image_a, image_b, M, N, K, C, ldc, c_bf16, true, s);
        if (st) return st;
        return bdr::gemm_bf16_tiled(image_a, image_b, M, N, K, C, ldc, c_bf16, false, s);
    }
    st = bdr::gemm_fp6(image_a, image_b, M, N, K, C, ldc, c_bf16, true, s);
    if (st) return st;
    return bdr::gemm_fp6(image_a, image_b, M, N, K, C, ldc, c_bf16, false, s);
}

size_t mx_dot_pipeline_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    return mx_gemm_workspace_bytes(M, N, K);
}

int mx_dot_pipeline(const bdr_format *fa, const bdr_format *fb, const void *a_codes,
                    const void *a_sexp, const void *a_mexp, const void *b_codes, const void *b_sexp,
                    const void *b_mexp, int64_t M, int64_t N, int64_t K, int64_t r, int32_t f_bits,
                    float *C, int64_t ldc, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    int st = check_format(fa);
    if (st) return st;
    st = check_format(fb);
    if (st) return st;
    if (!bdr::is_mx_layout(*fa) || !bdr::is_mx_layout(*fb)) return BDR_ERR_FORMAT;
    if (M < 0 || N < 0 || K < 64 || ldc < N) return BDR_ERR_SHAPE;
    if (M > (1 << 20) || N > (1 << 20) || K > (1 << 20)) return BDR_ERR_SHAPE;
    if (K % 64 != 0 || r < 64 || r % 64 != 0 || K % r != 0) return BDR_ERR_SHAPE;
    if (f_bits < 2 || f_bits > 26) return BDR_ERR_SHAPE;
    if (M == 0 || N == 0) return BDR_OK;
    if (!C) return BDR_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(C) % 4 != 0) return BDR_ERR_ALIGN;
    st = check_planes(fa, a_codes, a_sexp, a_mexp);
    if (st) return st;
    st = check_planes(fb, b_codes, b_sexp, b_mexp);
    if (st) return st;
    if (!workspace || workspace_bytes < mx_gemm_workspace_bytes(M, N, K)) return BDR_ERR_WORKSPACE;
    if (!aligned16(workspace)) return BDR_ERR_ALIGN;
    return bdr::dot_pipeline(*fa, *fb, a_codes, a_sexp, a_mexp, b_codes, b_sexp, b_mexp, M, N, K, r,
                             f_bits, C, ldc, workspace, static_cast<hipStream_t>(hip_stream));
}

}  // extern "C"
