"""MI355X (gfx950) library for Block Data Representations / shared microexponents (MX).

This package is a thin ctypes binding over ``libbdr_mx.so`` (C ABI in ``include/bdr_mx.h``).
It only marshals arguments: tensors must already live on the GPU, every step of the path runs
in the library's HIP kernels, and work is enqueued on torch's current stream.  There is no CPU
fallback -- if the library has not been built, importing fails.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbdr_mx.so")

RNE, RNA, RTZ = 0, 1, 2
F32, BF16 = 0, 1
AXIS_ROW, AXIS_COL = 0, 1
OPERAND_FP6, OPERAND_BF16, OPERAND_FP4 = 0, 1, 2
OK = 0

EXPORTS = (
    "bdr_status_string", "bdr_format_validate", "bdr_packed_sizes", "bdr_quantize",
    "bdr_dequantize", "bdr_gather_dequantize", "bdr_table_row_bytes", "bdr_table_pack",
    "bdr_table_gather_dequantize", "bdr_tile_packing", "bdr_quantize_dequantize",
    "bdr_qsnr_sweep_workspace_bytes",
    "bdr_qsnr_sweep", "bdr_qsnr_sweep_static", "bdr_qsnr_sweep_static_scratch_bytes",
    "mx_gemm_workspace_bytes", "mx_gemm", "mx_gemm_to", "mx_operand_bytes", "bdr_quantize_operand", "mx_gemm_operands", "mx_dot_pipeline_workspace_bytes", "mx_dot_pipeline",
)


class Format(ctypes.Structure):
    """BDR format tuple (Sec. III of the paper): k1, d1, k2, d2, m and the rounding rule."""

    _fields_ = [(n, ctypes.c_int32) for n in ("k1", "d1", "k2", "d2", "m", "rounding")]

    def __repr__(self):
        return "Format(k1=%d,d1=%d,k2=%d,d2=%d,m=%d,rnd=%d)" % (
            self.k1, self.d1, self.k2, self.d2, self.m, self.rounding)


def fmt(k1, k2, d2, m, d1=8, rounding=RNE):
    return Format(k1, d1, k2, d2, m, rounding)


# Table II
MX9 = fmt(16, 2, 1, 7)
MX6 = fmt(16, 2, 1, 4)
MX4 = fmt(16, 2, 1, 2)


class BdrError(RuntimeError):
    def __init__(self, status):
        super().__init__("libbdr_mx: %s (status %d)" % (status_string(status), status))
        self.status = status


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            "%s is missing: build it with `python paper_2302_08007_amd/build.py` "
            "(there is no fallback path)" % LIB_PATH)
    L = ctypes.CDLL(LIB_PATH)
    P, I32, I64, SZ = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    FP = ctypes.POINTER(Format)
    L.bdr_status_string.argtypes = [ctypes.c_int]
    L.bdr_status_string.restype = ctypes.c_char_p
    L.bdr_format_validate.argtypes = [FP]
    L.bdr_packed_sizes.argtypes = [FP, I64, I64, I32, P, P, P]
    L.bdr_quantize.argtypes = [FP, P, I32, I64, I64, I64, I32, P, P, P, P]
    L.bdr_dequantize.argtypes = [FP, P, P, P, I64, I64, I32, P, I32, I64, P]
    L.bdr_quantize_dequantize.argtypes = [FP, P, P, I32, I64, I64, I64, I32, P]
    L.bdr_gather_dequantize.argtypes = [FP, P, P, P, I64, I64, P, I64, P, I32, P]
    L.bdr_table_row_bytes.argtypes = [FP, I64]
    L.bdr_table_row_bytes.restype = SZ
    L.bdr_table_pack.argtypes = [FP, P, P, P, I64, I64, P, P]
    L.bdr_table_gather_dequantize.argtypes = [FP, P, I64, I64, P, I64, P, I32, P]
    L.bdr_tile_packing.argtypes = [FP, I64, I64, P, P, P]
    L.bdr_qsnr_sweep_workspace_bytes.argtypes = [I32]
    L.bdr_qsnr_sweep_workspace_bytes.restype = SZ
    L.bdr_qsnr_sweep.argtypes = [FP, I32, P, I32, I64, I64, I64, P, P, P, SZ, P]
    L.bdr_qsnr_sweep_static.argtypes = [FP, I32, P, I32, I64, I64, I64, P, P, P]
    L.bdr_qsnr_sweep_static_scratch_bytes.argtypes = []
    L.bdr_qsnr_sweep_static_scratch_bytes.restype = SZ
    L.mx_gemm_workspace_bytes.argtypes = [I64, I64, I64]
    L.mx_gemm_workspace_bytes.restype = SZ
    L.mx_gemm.argtypes = [FP, FP, P, P, P, P, P, P, I64, I64, I64, P, I64, P, SZ, P]
    L.mx_gemm_to.argtypes = [FP, FP, P, P, P, P, P, P, I64, I64, I64, P, I32, I64, P, SZ, P]
    L.mx_operand_bytes.argtypes = [FP, I64, I64, I32]
    L.mx_operand_bytes.restype = SZ
    L.bdr_quantize_operand.argtypes = [FP, P, I32, I64, I64, I64, I32, I32, I32, P, P]
    L.mx_gemm_operands.argtypes = [FP, FP, P, P, I32, I64, I64, I64, P, I32, I64, P]
    L.mx_dot_pipeline_workspace_bytes.argtypes = [I64, I64, I64]
    L.mx_dot_pipeline_workspace_bytes.restype = SZ
    L.mx_dot_pipeline.argtypes = [FP, FP, P, P, P, P, P, P, I64, I64, I64, I64, I32, P, I64, P, SZ, P]
    return L


lib = _load()


def status_string(status):
    return lib.bdr_status_string(int(status)).decode()


def _check(status):
    if status != OK:
        raise BdrError(status)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype_code(t):
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError("expected a float32 or bfloat16 tensor, got %s" % t.dtype)


def _dev2d(t):
    if not (t.is_cuda and t.dim() == 2 and t.stride(1) == 1):
        raise ValueError("expected a 2-D GPU tensor with unit column stride")
    return t.shape[0], t.shape[1], t.stride(0)


def _p(t):
    return ctypes.c_void_p(0 if t is None or t.numel() == 0 else t.data_ptr())


def _check_planes(f, planes, rows, cols, axis=AXIS_ROW):
    """The C ABI takes bare pointers, so buffer sizes are verified here: a plane shorter than
    bdr_packed_sizes says would be written (or read) past its end."""
    need = bdr_packed_sizes(f, rows, cols, axis)
    if len(planes) != 3:
        raise ValueError("expected (codes, sexp, mexp)")
    for name, t, n in zip(("codes", "sexp", "mexp"), planes, need):
        if n == 0:
            continue
        if t is None or not (t.is_cuda and t.dtype == torch.uint8 and t.is_contiguous()):
            raise ValueError("%s plane must be a contiguous uint8 GPU tensor" % name)
        if t.numel() < n:
            raise ValueError("%s plane holds %d bytes, %d needed" % (name, t.numel(), n))


def _check_buffer(name, t, dtype, numel):
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous() and t.numel() >= numel):
        raise ValueError("%s must be a contiguous %s GPU tensor of at least %d elements"
                         % (name, dtype, numel))


def bdr_format_validate(f):
    return lib.bdr_format_validate(ctypes.byref(f))


def bdr_packed_sizes(f, rows, cols, axis=AXIS_ROW):
    c, s, m = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib.bdr_packed_sizes(ctypes.byref(f), rows, cols, axis, ctypes.byref(c),
                                ctypes.byref(s), ctypes.byref(m)))
    return c.value, s.value, m.value


def alloc_planes(f, rows, cols, axis=AXIS_ROW, device="cuda"):
    """Uninitialised uint8 tensors for the codes, shared-exponent and microexponent planes."""
    nc, ns, nm = bdr_packed_sizes(f, rows, cols, axis)
    return tuple(torch.empty(n, dtype=torch.uint8, device=device) for n in (nc, ns, nm))


def bdr_quantize(f, x, axis=AXIS_ROW, out=None):
    """Quantize a 2-D GPU tensor into (codes, sexp, mexp) uint8 planes."""
    rows, cols, ld = _dev2d(x)
    planes = out if out is not None else alloc_planes(f, rows, cols, axis, x.device)
    if out is not None:
        _check_planes(f, planes, rows, cols, axis)
    _check(lib.bdr_quantize(ctypes.byref(f), _p(x), _dtype_code(x), rows, cols, ld, axis,
                            _p(planes[0]), _p(planes[1]), _p(planes[2]), _stream()))
    return planes


def bdr_dequantize(f, planes, rows, cols, axis=AXIS_ROW, dtype=torch.float32, out=None):
    y = out if out is not None else torch.empty((rows, cols), dtype=dtype, device=planes[0].device)
    r, c, ld = _dev2d(y)
    if (r, c) != (rows, cols):
        raise ValueError("output must be [rows x cols]")
    _check_planes(f, planes, rows, cols, axis)
    _check(lib.bdr_dequantize(ctypes.byref(f), _p(planes[0]), _p(planes[1]), _p(planes[2]), rows,
                              cols, axis, _p(y), _dtype_code(y), ld, _stream()))
    return y


def bdr_quantize_dequantize(f, x, axis=AXIS_ROW, out=None):
    rows, cols, ld = _dev2d(x)
    y = out if out is not None else torch.empty_like(x)
    if _dev2d(y) != (rows, cols, ld) or y.dtype != x.dtype:
        raise ValueError("output must match the input's shape, pitch and dtype")
    _check(lib.bdr_quantize_dequantize(ctypes.byref(f), _p(x), _p(y), _dtype_code(x), rows, cols,
                                       ld, axis, _stream()))
    return y


def bdr_qsnr_sweep(fmts, x, workspace=None, out=None):
    """QSNR (dB) of every format on a 2-D GPU tensor.  Returns (qsnr_db[n], sums[n+1]) float64."""
    rows, cols, ld = _dev2d(x)
    n = len(fmts)
    arr = (Format * max(n, 1))(*fmts)
    need = lib.bdr_qsnr_sweep_workspace_bytes(n)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=x.device)
    if out is None:
        out = (torch.empty(n, dtype=torch.float64, device=x.device),
               torch.empty(n + 1, dtype=torch.float64, device=x.device))
    _check_buffer("qsnr_db", out[0], torch.float64, n)
    _check_buffer("sums", out[1], torch.float64, n + 1)
    _check_buffer("workspace", workspace, torch.uint8, 0)
    _check(lib.bdr_qsnr_sweep(arr, n, _p(x), _dtype_code(x), rows, cols, ld, _p(out[0]),
                              _p(out[1]), _p(workspace), workspace.numel(), _stream()))
    return out


def bdr_qsnr_sweep_static(fmts, x, out):
    """bdr_qsnr_sweep without a workspace: the library's own fixed scratch array is used and
    nothing is allocated, so `out` = (qsnr_db[n], sums[n+1]) float64 tensors must be given.
    Calls that overlap in time on one GPU race on that array."""
    rows, cols, ld = _dev2d(x)
    n = len(fmts)
    arr = (Format * max(n, 1))(*fmts)
    _check_buffer("qsnr_db", out[0], torch.float64, n)
    _check_buffer("sums", out[1], torch.float64, n + 1)
    _check(lib.bdr_qsnr_sweep_static(arr, n, _p(x), _dtype_code(x), rows, cols, ld, _p(out[0]),
                                     _p(out[1]), _stream()))
    return out


def bdr_gather_dequantize(fmt, planes, table_rows, cols, indices, dtype=None, out=None):
    """out[j, :] = dequantized row indices[j] of the packed table (indices: int64 tensor)."""
    dtype = dtype or torch.float32
    n = indices.numel()
    y = out if out is not None else torch.empty((n, cols), dtype=dtype, device=indices.device)
    _check_buffer("indices", indices, torch.int64, n)
    if not (y.is_cuda and y.is_contiguous() and tuple(y.shape) == (n, cols)):
        raise ValueError("output must be a contiguous [n_indices x cols] GPU tensor")
    _check_planes(fmt, planes, table_rows, cols)
    _check(lib.bdr_gather_dequantize(ctypes.byref(fmt), _p(planes[0]), _p(planes[1]), _p(planes[2]),
                                     table_rows, cols, _p(indices), n, _p(y), _dtype_code(y),
                                     _stream()))
    return y


def bdr_table_row_bytes(fmt, cols):
    """Bytes of one row of the table image that keeps a row's runs together (0: not taken)."""
    return int(lib.bdr_table_row_bytes(ctypes.byref(fmt), cols))


def bdr_table_pack(fmt, planes, table_rows, cols, out=None):
    """Three-plane image of a [table_rows x cols] table -> the image whose rows are
    [codes | exponent bytes | microexponent bytes] (uint8 tensor of table_rows * row bytes)."""
    rb = bdr_table_row_bytes(fmt, cols)
    if rb == 0 and cols != 0:
        raise ValueError("the table image takes Table II's formats with cols a multiple of 64")
    _check_planes(fmt, planes, table_rows, cols)
    t = out if out is not None else torch.empty(table_rows * rb, dtype=torch.uint8, device=planes[0].device)
    _check_buffer("table", t, torch.uint8, table_rows * rb)
    _check(lib.bdr_table_pack(ctypes.byref(fmt), _p(planes[0]), _p(planes[1]), _p(planes[2]), table_rows,
                              cols, _p(t), _stream()))
    return t


def bdr_table_gather_dequantize(fmt, table, table_rows, cols, indices, dtype=None, out=None):
    """bdr_gather_dequantize on the image bdr_table_pack made."""
    dtype = dtype or torch.float32
    n = indices.numel()
    y = out if out is not None else torch.empty((n, cols), dtype=dtype, device=indices.device)
    _check_buffer("indices", indices, torch.int64, n)
    if not (y.is_cuda and y.is_contiguous() and tuple(y.shape) == (n, cols)):
        raise ValueError("output must be a contiguous [n_indices x cols] GPU tensor")
    rb = bdr_table_row_bytes(fmt, cols)
    if rb == 0 and cols != 0:
        raise ValueError("the table image takes Table II's formats with cols a multiple of 64")
    _check_buffer("table", table, torch.uint8, table_rows * rb)
    _check(lib.bdr_table_gather_dequantize(ctypes.byref(fmt), _p(table), table_rows, cols, _p(indices), n,
                                           _p(y), _dtype_code(y), _stream()))
    return y


def bdr_tile_packing(fmt, tile_elements=256, interface_bytes=64):
    """(packed bytes, interface transfers, efficiency) of one tile (Sec. IV-B, Memory Footprint)."""
    b, t, e = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_double()
    _check(lib.bdr_tile_packing(ctypes.byref(fmt), tile_elements, interface_bytes, ctypes.byref(b),
                                ctypes.byref(t), ctypes.byref(e)))
    return b.value, t.value, e.value


def mx_gemm_workspace_bytes(M, N, K):
    return lib.mx_gemm_workspace_bytes(M, N, K)


def mx_gemm(fa, fb, a_planes, b_planes, M, N, K, out=None, workspace=None, dtype=None):
    """C[M, N] = Ahat @ Bhat^T for two packed operands blocked along K.  `workspace`: a
    uint8 tensor of at least mx_gemm_workspace_bytes(M, N, K) bytes selects the two-pass
    form, None the single-kernel form (Table II formats only; other BF16-exact formats need
    the workspace).  C is float32, or bfloat16 (the sums rounded once more as they are stored)
    when `out` or `dtype` says so."""
    dtype = out.dtype if out is not None else (dtype or torch.float32)
    C = out if out is not None else torch.empty((M, N), dtype=dtype, device=a_planes[0].device)
    if not (C.is_cuda and C.dtype in (torch.float32, torch.bfloat16) and C.dim() == 2
            and tuple(C.shape) == (M, N) and C.stride(1) == 1):
        raise ValueError("output must be an [M x N] float32 or bfloat16 GPU tensor with unit column stride")
    if K > 0:
        _check_planes(fa, a_planes, M, K)
        _check_planes(fb, b_planes, N, K)
    if workspace is not None:
        _check_buffer("workspace", workspace, torch.uint8, 0)
    ws, wsb = (_p(workspace), workspace.numel()) if workspace is not None else (None, 0)
    args = (ctypes.byref(fa), ctypes.byref(fb), _p(a_planes[0]), _p(a_planes[1]), _p(a_planes[2]),
            _p(b_planes[0]), _p(b_planes[1]), _p(b_planes[2]), M, N, K, _p(C))
    if C.dtype == torch.float32:
        _check(lib.mx_gemm(*args, C.stride(0), ws, wsb, _stream()))
    else:
        _check(lib.mx_gemm_to(*args, _dtype_code(C), C.stride(0), ws, wsb, _stream()))
    return C


def mx_operand_bytes(fmt, rows, K, image=OPERAND_FP6):
    return int(lib.mx_operand_bytes(ctypes.byref(fmt), rows, K, image))


def bdr_quantize_operand(fmt, x, axis=AXIS_ROW, image=OPERAND_FP6, b_operand=False, out=None):
    """Quantize x straight into an image the product kernel reads (OPERAND_FP6: MX6 / MX4 for the
    block-scaled FP6 product; OPERAND_BF16: any Table II format for the BF16 product; OPERAND_FP4:
    MX4 for the block-scaled FP4 product, K a multiple of 128): the image
    of x itself (axis ROW, K = columns) or of its transpose (axis COL, K = rows).  Returns a
    uint8 tensor."""
    rows, cols, ld = _dev2d(x)
    op_rows, K = (rows, cols) if axis == AXIS_ROW else (cols, rows)
    need = mx_operand_bytes(fmt, op_rows, K, image)
    img = out if out is not None else torch.empty(max(need, 16), dtype=torch.uint8, device=x.device)
    _check_buffer("image", img, torch.uint8, need)
    _check(lib.bdr_quantize_operand(ctypes.byref(fmt), _p(x), _dtype_code(x), rows, cols, ld, axis, image,
                                    int(b_operand), _p(img), _stream()))
    return img


def mx_gemm_operands(fa, fb, image_a, image_b, M, N, K, image=OPERAND_FP6, out=None, dtype=None):
    """C[M, N] = A B^T from two operand images of the same kind made by bdr_quantize_operand."""
    dtype = out.dtype if out is not None else (dtype or torch.float32)
    C = out if out is not None else torch.empty((M, N), dtype=dtype, device=image_a.device)
    if not (C.is_cuda and C.dtype in (torch.float32, torch.bfloat16) and C.dim() == 2
            and tuple(C.shape) == (M, N) and C.stride(1) == 1):
        raise ValueError("output must be an [M x N] float32 or bfloat16 GPU tensor with unit column stride")
    _check_buffer("image_a", image_a, torch.uint8, mx_operand_bytes(fa, M, K, image))
    _check_buffer("image_b", image_b, torch.uint8, mx_operand_bytes(fb, N, K, image))
    _check(lib.mx_gemm_operands(ctypes.byref(fa), ctypes.byref(fb), _p(image_a), _p(image_b), image, M, N, K,
                                _p(C), _dtype_code(C), C.stride(0), _stream()))
    return C


def mx_dot_pipeline(fa, fb, a_planes, b_planes, M, N, K, r=None, f_bits=25, out=None, workspace=None):
    """C[M, N] = Ahat @ Bhat^T through the bit-true model of the paper's dot-product pipeline
    (Sec. IV-B): r = dot-product length of the unit (default K: one pass), f_bits = width of its
    fixed-point accumulation word."""
    C = out if out is not None else torch.empty((M, N), dtype=torch.float32,
                                                device=a_planes[0].device)
    if not (C.is_cuda and C.dtype == torch.float32 and C.dim() == 2 and tuple(C.shape) == (M, N)
            and C.stride(1) == 1):
        raise ValueError("output must be an [M x N] float32 GPU tensor with unit column stride")
    _check_planes(fa, a_planes, M, K)
    _check_planes(fb, b_planes, N, K)
    need = lib.mx_dot_pipeline_workspace_bytes(M, N, K)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=C.device)
    _check_buffer("workspace", workspace, torch.uint8, need)
    _check(lib.mx_dot_pipeline(ctypes.byref(fa), ctypes.byref(fb), _p(a_planes[0]), _p(a_planes[1]),
                               _p(a_planes[2]), _p(b_planes[0]), _p(b_planes[1]), _p(b_planes[2]),
                               M, N, K, K if r is None else r, f_bits, _p(C), C.stride(0),
                               _p(workspace), workspace.numel(), _stream()))
    return C
