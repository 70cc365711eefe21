"""CPU oracle for the BDR / shared-microexponent quantizer -- TEST INFRASTRUCTURE ONLY.

Thin ctypes access to ``libbdr_ref.so`` (built from ``bdr_ref.c`` by ``oracle/build.py``).
All arrays are numpy host arrays.  Nothing in the product package may import this module;
only the tests, the smoke check and the bench's CPU-baseline leg do.
"""
import ctypes
import os

import numpy as np

from . import build as _build

RNE, RNA, RTZ = 0, 1, 2
F32, BF16 = 0, 1
AXIS_ROW, AXIS_COL = 0, 1
OK, ERR_NULL, ERR_FORMAT, ERR_SHAPE, ERR_DTYPE = 0, 1, 2, 3, 5


class Format(ctypes.Structure):
    """BDR format tuple (Sec. III): k1, d1, k2, d2, m and the rounding rule."""

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

_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_build.LIB):
            _build.build()
        L = ctypes.CDLL(_build.LIB)
        P, I32, I64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        FP = ctypes.POINTER(Format)
        L.bdr_ref_format_validate.argtypes = [FP]
        L.bdr_ref_bits_per_element.argtypes = [FP]
        L.bdr_ref_bits_per_element.restype = ctypes.c_double
        L.bdr_ref_packed_sizes.argtypes = [FP, I64, I64, I32, P, P, P]
        L.bdr_ref_quantize_block.argtypes = [FP, P, I32, P, P, P]
        L.bdr_ref_quantize_block.restype = None
        L.bdr_ref_decode.argtypes = [FP, ctypes.c_uint8, ctypes.c_uint8, ctypes.c_uint16]
        L.bdr_ref_decode.restype = ctypes.c_double
        L.bdr_ref_quantize.argtypes = [FP, P, I32, I64, I64, I64, I32, P, P, P]
        L.bdr_ref_dequantize.argtypes = [FP, P, P, P, I64, I64, I32, P, I32, I64]
        L.bdr_ref_quantize_dequantize.argtypes = [FP, P, P, I32, I64, I64, I64, I32]
        L.bdr_ref_qsnr_sweep.argtypes = [FP, I32, P, I32, I64, I64, I64, P, P]
        L.bdr_ref_mx_gemm_sampled.argtypes = [FP, FP, P, P, P, P, P, P, I64, I64, I64, I64,
                                              P, P, P, P]
        L.bdr_ref_mx_gemm.argtypes = [FP, FP, P, P, P, P, P, P, I64, I64, I64, P, I64]
        L.bdr_ref_dot_pipeline_sampled.argtypes = [FP, FP, P, P, P, P, P, P, I64, I64, I64, I64,
                                                   I32, I64, P, P, P]
        _lib = L
    return _lib


class OracleError(RuntimeError):
    def __init__(self, status):
        super().__init__("oracle status %d" % status)
        self.status = status


def _check(st):
    if st != OK:
        raise OracleError(st)


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _dtype_of(a):
    """numpy float32 -> F32; numpy uint16 holding bf16 bit patterns -> BF16."""
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError("expected float32 or uint16 (bf16 bits), got %s" % a.dtype)


def validate(f):
    return lib().bdr_ref_format_validate(ctypes.byref(f))


def bits_per_element(f):
    return lib().bdr_ref_bits_per_element(ctypes.byref(f))


def packed_sizes(f, rows, cols, axis=AXIS_ROW):
    c, s, m = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib().bdr_ref_packed_sizes(ctypes.byref(f), rows, cols, axis, ctypes.byref(c),
                                      ctypes.byref(s), ctypes.byref(m)))
    return c.value, s.value, m.value


def quantize_block(f, x):
    """x: 1-D float32 of length <= k1.  Returns (sexp, tau[k1/k2], code[k1])."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    assert x.ndim == 1 and x.size <= f.k1
    se = np.zeros(1, np.uint8)
    tau = np.zeros(f.k1 // f.k2, np.uint8)
    code = np.zeros(f.k1, np.uint16)
    lib().bdr_ref_quantize_block(ctypes.byref(f), _ptr(x.view(np.uint32)), x.size, _ptr(se),
                                 _ptr(tau), _ptr(code))
    return int(se[0]), tau, code


def decode(f, sexp, tau, code):
    return lib().bdr_ref_decode(ctypes.byref(f), int(sexp), int(tau), int(code))


def quantize(f, x, axis=AXIS_ROW):
    """x: 2-D C-contiguous float32 or uint16(bf16 bits).  Returns (codes, sexp, mexp) uint8."""
    assert x.ndim == 2 and x.flags.c_contiguous
    rows, cols = x.shape
    nc, ns, nm = packed_sizes(f, rows, cols, axis)
    codes, sexp, mexp = np.zeros(nc, np.uint8), np.zeros(ns, np.uint8), np.zeros(nm, np.uint8)
    _check(lib().bdr_ref_quantize(ctypes.byref(f), _ptr(x), _dtype_of(x), rows, cols, cols, axis,
                                  _ptr(codes), _ptr(sexp), _ptr(mexp)))
    return codes, sexp, mexp


def dequantize(f, codes, sexp, mexp, rows, cols, axis=AXIS_ROW, out_dtype=np.float32):
    y = np.zeros((rows, cols), out_dtype)
    _check(lib().bdr_ref_dequantize(ctypes.byref(f), _ptr(codes), _ptr(sexp), _ptr(mexp), rows,
                                    cols, axis, _ptr(y), _dtype_of(y), cols))
    return y


def quantize_dequantize(f, x, axis=AXIS_ROW):
    assert x.ndim == 2 and x.flags.c_contiguous
    y = np.zeros_like(x)
    _check(lib().bdr_ref_quantize_dequantize(ctypes.byref(f), _ptr(x), _ptr(y), _dtype_of(x),
                                             x.shape[0], x.shape[1], x.shape[1], axis))
    return y


def qsnr_sweep(fmts, x):
    """Returns (qsnr_db[n], sums[n+1]) for a 2-D tensor, blocks along rows."""
    assert x.ndim == 2 and x.flags.c_contiguous
    n = len(fmts)
    arr = (Format * max(n, 1))(*fmts)
    q, s = np.zeros(n, np.float64), np.zeros(n + 1, np.float64)
    _check(lib().bdr_ref_qsnr_sweep(arr, n, _ptr(x), _dtype_of(x), x.shape[0], x.shape[1],
                                    x.shape[1], _ptr(q), _ptr(s)))
    return q, s


def mx_gemm_sampled(fa, fb, a_planes, b_planes, M, N, K, idx_i, idx_j):
    idx_i = np.ascontiguousarray(idx_i, np.int64)
    idx_j = np.ascontiguousarray(idx_j, np.int64)
    out = np.zeros(idx_i.size, np.float32)
    absdot = np.zeros(idx_i.size, np.float64)
    _check(lib().bdr_ref_mx_gemm_sampled(
        ctypes.byref(fa), ctypes.byref(fb), _ptr(a_planes[0]), _ptr(a_planes[1]),
        _ptr(a_planes[2]), _ptr(b_planes[0]), _ptr(b_planes[1]), _ptr(b_planes[2]), M, N, K,
        idx_i.size, _ptr(idx_i), _ptr(idx_j), _ptr(out), _ptr(absdot)))
    return out, absdot


def mx_gemm(fa, fb, a_planes, b_planes, M, N, K):
    C = np.zeros((M, N), np.float32)
    _check(lib().bdr_ref_mx_gemm(
        ctypes.byref(fa), ctypes.byref(fb), _ptr(a_planes[0]), _ptr(a_planes[1]),
        _ptr(a_planes[2]), _ptr(b_planes[0]), _ptr(b_planes[1]), _ptr(b_planes[2]), M, N, K,
        _ptr(C), N))
    return C


def dot_pipeline_sampled(fa, fb, a_planes, b_planes, M, N, K, idx_i, idx_j, r=None, f_bits=25):
    """Entries (idx_i[s], idx_j[s]) of C = A B^T through the dot-product pipeline model."""
    idx_i = np.ascontiguousarray(idx_i, np.int64)
    idx_j = np.ascontiguousarray(idx_j, np.int64)
    out = np.zeros(idx_i.size, np.float32)
    _check(lib().bdr_ref_dot_pipeline_sampled(
        ctypes.byref(fa), ctypes.byref(fb), _ptr(a_planes[0]), _ptr(a_planes[1]),
        _ptr(a_planes[2]), _ptr(b_planes[0]), _ptr(b_planes[1]), _ptr(b_planes[2]), M, N, K,
        K if r is None else r, f_bits, idx_i.size, _ptr(idx_i), _ptr(idx_j), _ptr(out)))
    return out


def dot_pipeline(fa, fb, a_planes, b_planes, M, N, K, r=None, f_bits=25):
    """The full [M x N] matrix of the same."""
    ii, jj = [a.reshape(-1) for a in np.meshgrid(np.arange(M), np.arange(N), indexing="ij")]
    return dot_pipeline_sampled(fa, fb, a_planes, b_planes, M, N, K, ii, jj, r, f_bits).reshape(M, N)
