"""Host-side tests of the C ABI: the library loads, exports what include/bdr_mx.h declares, and
every argument check answers with the right status before anything is launched (no GPU needed:
none of these calls reaches a kernel)."""
import ctypes
import os
import re

import pytest

import oracle as O
import paper_2302_08007_amd as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = ctypes.c_void_p(0x10000)       # 16-byte aligned, never dereferenced on the host
FAKE_ODD = ctypes.c_void_p(0x10004)
NULL = ctypes.c_void_p(0)
OK, ERR_NULL, ERR_FORMAT, ERR_SHAPE, ERR_ALIGN, ERR_DTYPE, ERR_LAUNCH, ERR_WS = range(8)


def test_exports_match_header():
    text = open(os.path.join(ROOT, "include", "bdr_mx.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(bdr_\w+|mx_\w+)\s*\(", text))
    names -= {"bdr_format"}
    assert names == set(B.EXPORTS)
    for n in names:
        assert getattr(B.lib, n) is not None


def test_status_strings():
    seen = {B.status_string(s) for s in range(8)}
    assert len(seen) == 8 and B.status_string(99) == "unknown status"


def test_format_validate():
    assert B.bdr_format_validate(B.MX9) == OK
    assert B.lib.bdr_format_validate(None) == ERR_NULL
    for bad in (B.fmt(12, 2, 1, 4), B.fmt(16, 3, 1, 4), B.fmt(16, 32, 1, 4), B.fmt(16, 2, 4, 4),
                B.fmt(16, 2, -1, 4), B.fmt(16, 2, 1, 0), B.fmt(16, 2, 1, 9), B.fmt(512, 2, 1, 4),
                B.fmt(16, 2, 1, 4, d1=7), B.fmt(16, 2, 1, 4, rounding=3)):
        assert B.bdr_format_validate(bad) == ERR_FORMAT, bad
    for good in (B.fmt(1, 1, 0, 1), B.fmt(256, 256, 3, 8, rounding=B.RTZ), B.fmt(64, 1, 2, 5)):
        assert B.bdr_format_validate(good) == OK, good


@pytest.mark.parametrize("f", [B.MX9, B.MX6, B.MX4, B.fmt(64, 4, 1, 4), B.fmt(8, 1, 3, 2),
                               B.fmt(256, 128, 1, 8), B.fmt(2, 1, 1, 3)], ids=repr)
def test_packed_sizes_formula_and_oracle(f):
    rows, cols = 256, 1024
    nc, ns, nm = B.bdr_packed_sizes(f, rows, cols)
    n = rows * cols
    # Sec. III: (m + 1) + d1 / k1 + d2 / k2 bits per element
    assert 8 * nc == n * (f.m + 1) and 8 * ns == n * 8 // f.k1 and 8 * nm == n * f.d2 // f.k2
    assert (nc, ns, nm) == O.packed_sizes(O.Format(f.k1, f.d1, f.k2, f.d2, f.m, f.rounding), rows, cols)
    assert B.bdr_packed_sizes(f, rows, cols, B.AXIS_COL) == B.bdr_packed_sizes(f, cols, rows)
    # Table II: 9, 6 and 4 bits per element
    if f.k1 == 16 and f.k2 == 2 and f.d2 == 1:
        assert 8 * (nc + ns + nm) == n * (f.m + 2)


def test_packed_sizes_of_ragged_shapes():
    """A row whose length is not a whole number of blocks is stored padded to the next multiple
    of k1 (Sec. IX, the remark after Theorem 1); the sizes agree with the oracle's."""
    for f, rows, cols in ((B.MX6, 4, 24), (B.MX9, 7, 1000), (B.fmt(64, 4, 1, 4), 3, 65),
                          (B.fmt(4, 2, 1, 3), 5, 14), (B.fmt(128, 128, 0, 7), 9, 1)):
        of = O.Format(f.k1, f.d1, f.k2, f.d2, f.m, f.rounding)
        pc = -(-cols // f.k1) * f.k1
        assert B.bdr_packed_sizes(f, rows, cols) == O.packed_sizes(of, rows, cols) == \
            B.bdr_packed_sizes(f, rows, pc)
        assert B.bdr_packed_sizes(f, cols, rows, B.AXIS_COL) == O.packed_sizes(of, cols, rows, O.AXIS_COL)
    # column blocks with a ragged contiguous axis: every column is a padded row of the transpose
    assert B.bdr_packed_sizes(B.MX6, 50, 7, B.AXIS_COL) == B.bdr_packed_sizes(B.MX6, 7, 64)


def test_packed_sizes_errors():
    with pytest.raises(B.BdrError) as e:
        B.bdr_packed_sizes(B.fmt(4, 2, 1, 3), 4, 12)   # 12 is whole blocks of 4, but not a multiple of 8
    assert e.value.status == ERR_SHAPE
    with pytest.raises(B.BdrError):
        B.bdr_packed_sizes(B.fmt(4, 2, 1, 3), 4, 9)    # padded to 12: still not a multiple of 8
    with pytest.raises(B.BdrError):
        B.bdr_packed_sizes(B.MX6, -1, 16)
    with pytest.raises(B.BdrError):
        B.bdr_packed_sizes(B.MX6, 16, 16, 2)
    assert B.bdr_packed_sizes(B.MX6, 0, 16) == (0, 0, 0)


def _q(f, x=FAKE, dtype=0, rows=4, cols=64, ld=64, axis=0, codes=FAKE, sexp=FAKE, mexp=FAKE):
    return B.lib.bdr_quantize(ctypes.byref(f), x, dtype, rows, cols, ld, axis, codes, sexp, mexp, NULL)


def test_quantize_argument_checks():
    f = B.MX6
    assert B.lib.bdr_quantize(None, FAKE, 0, 4, 64, 64, 0, FAKE, FAKE, FAKE, NULL) == ERR_NULL
    assert _q(B.fmt(16, 2, 1, 12)) == ERR_FORMAT
    assert _q(f, dtype=2) == ERR_DTYPE
    assert _q(f, axis=5) == ERR_SHAPE
    assert _q(B.fmt(4, 2, 1, 3), cols=12, ld=12) == ERR_SHAPE   # k1 < 8: padded length not a multiple of 8
    assert _q(f, cols=40, ld=40, x=ctypes.c_void_p(0x10002)) == ERR_ALIGN   # a short last block: the alignment of an element
    assert _q(f, cols=40, ld=40, codes=FAKE_ODD) == ERR_ALIGN
    assert _q(f, ld=32) == ERR_SHAPE                     # ld < cols
    assert _q(f, rows=-1) == ERR_SHAPE
    assert _q(B.fmt(2, 1, 1, 3), rows=6, axis=1) == ERR_SHAPE   # blocked axis = rows
    assert _q(f, rows=1 << 30, cols=1 << 20, ld=1 << 20) == ERR_SHAPE   # too large
    assert _q(f, x=NULL) == ERR_NULL
    assert _q(f, codes=NULL) == ERR_NULL
    assert _q(f, mexp=NULL) == ERR_NULL
    assert _q(B.fmt(16, 16, 0, 4), mexp=NULL, x=FAKE_ODD) == ERR_ALIGN    # mexp may be NULL for d2 = 0
    assert _q(f, x=FAKE_ODD) == ERR_ALIGN
    assert _q(f, ld=66) == ERR_ALIGN                     # pitch not a multiple of 16 bytes
    assert _q(f, sexp=FAKE_ODD) == ERR_ALIGN
    assert _q(f, rows=0) == OK                           # empty: nothing to launch
    assert _q(f, rows=0, x=NULL, codes=NULL, sexp=NULL, mexp=NULL) == OK


def test_dequantize_and_fused_argument_checks():
    L, f = B.lib, B.MX6
    deq = lambda f, y=FAKE, dtype=0, rows=4, cols=64, ld=64: L.bdr_dequantize(
        ctypes.byref(f), FAKE, FAKE, FAKE, rows, cols, 0, y, dtype, ld, NULL)
    assert deq(f, y=NULL) == ERR_NULL
    assert deq(f, y=FAKE_ODD) == ERR_ALIGN
    assert deq(B.fmt(2, 2, 0, 3), cols=6, ld=8) == ERR_SHAPE
    assert deq(f, cols=8, ld=8, y=ctypes.c_void_p(0x10002)) == ERR_ALIGN   # half a block is taken (stored as a whole one)
    assert deq(B.fmt(16, 2, 2, 7), dtype=1) == ERR_DTYPE         # m + beta = 10 > 8: not exact in bf16
    assert deq(B.fmt(16, 2, 3, 2), dtype=1) == ERR_DTYPE
    assert deq(f, rows=0) == OK
    qdq = lambda f, x=FAKE, y=FAKE, dtype=0: L.bdr_quantize_dequantize(
        ctypes.byref(f), x, y, dtype, 4, 64, 64, 0, NULL)
    assert qdq(f, x=NULL) == ERR_NULL and qdq(f, y=NULL) == ERR_NULL
    assert qdq(B.fmt(8, 2, 3, 8), dtype=1) == ERR_DTYPE
    assert qdq(f, dtype=7) == ERR_DTYPE


def test_sweep_and_gemm_argument_checks():
    L = B.lib
    arr = (B.Format * 2)(B.MX6, B.fmt(64, 4, 1, 4))
    need = L.bdr_qsnr_sweep_workspace_bytes(2)
    assert need > 0 and L.bdr_qsnr_sweep_workspace_bytes(0) == 0
    assert L.bdr_qsnr_sweep_workspace_bytes(2000) == 0
    sw = lambda n=2, x=FAKE, cols=64, q=FAKE, s=FAKE, ws=FAKE, wsb=need: L.bdr_qsnr_sweep(
        arr, n, x, 0, 4, cols, cols, q, s, ws, wsb, NULL)
    assert L.bdr_qsnr_sweep(None, 2, FAKE, 0, 4, 64, 64, FAKE, FAKE, FAKE, need, NULL) == ERR_NULL
    assert sw(n=0) == ERR_SHAPE
    assert sw(cols=32) == ERR_SHAPE                      # 32 % 64 != 0 for the second format
    assert sw(q=NULL) == ERR_NULL
    assert sw(ws=NULL) == ERR_WS and sw(wsb=need - 1) == ERR_WS
    assert sw(x=NULL) == ERR_NULL
    assert sw(s=FAKE_ODD) == ERR_ALIGN
    # the entry point without a workspace checks the same things (its limit on n_fmts included)
    st = lambda n=2, x=FAKE, cols=64, q=FAKE, s=FAKE: L.bdr_qsnr_sweep_static(
        arr, n, x, 0, 4, cols, cols, q, s, NULL)
    assert st(n=0) == ERR_SHAPE and st(n=1025) == ERR_SHAPE and st(cols=32) == ERR_SHAPE
    assert st(q=NULL) == ERR_NULL and st(x=NULL) == ERR_NULL and st(s=FAKE_ODD) == ERR_ALIGN
    assert L.bdr_qsnr_sweep_static(None, 2, FAKE, 0, 4, 64, 64, FAKE, FAKE, NULL) == ERR_NULL
    assert 0 < L.bdr_qsnr_sweep_static_scratch_bytes() <= 1 << 20
    f = B.MX6
    gm = lambda fa=f, fb=f, M=128, N=128, K=64, C=FAKE, ldc=128, a=FAKE, ws=NULL, wsb=0: L.mx_gemm(
        ctypes.byref(fa), ctypes.byref(fb), a, FAKE, FAKE, FAKE, FAKE, FAKE, M, N, K, C, ldc, ws,
        wsb, NULL)
    assert gm(fa=B.fmt(32, 2, 3, 4)) == ERR_FORMAT       # m + beta = 11: BF16 cannot hold it
    assert gm(fa=B.fmt(32, 2, 1, 4)) == ERR_WS           # other BF16-exact formats need the workspace
    assert gm(fa=B.fmt(128, 2, 1, 4), ws=FAKE, wsb=1 << 20) == ERR_SHAPE    # K = 64 is not a multiple of k1
    assert gm(M=-1) == ERR_SHAPE and gm(K=48) == ERR_SHAPE and gm(ldc=64) == ERR_SHAPE
    assert gm(N=(1 << 20) + 1, ldc=(1 << 20) + 1) == ERR_SHAPE
    assert gm(C=NULL) == ERR_NULL and gm(a=NULL) == ERR_NULL
    assert gm(C=ctypes.c_void_p(0x10002)) == ERR_ALIGN   # C needs only the alignment of a float
    assert gm(M=0) == OK
    gt = lambda C=FAKE, cd=1, ldc=128, M=128: L.mx_gemm_to(
        ctypes.byref(f), ctypes.byref(f), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, M, 128, 64, C, cd, ldc, NULL, 0, NULL)
    assert gt(cd=2) == ERR_DTYPE and gt(cd=-1) == ERR_DTYPE
    assert gt(C=ctypes.c_void_p(0x10001)) == ERR_ALIGN      # a BF16 C needs the alignment of two bytes
    assert gt(C=ctypes.c_void_p(0x10002), cd=0) == ERR_ALIGN and gt(C=NULL) == ERR_NULL
    assert gt(ldc=64) == ERR_SHAPE and gt(M=0) == OK
    need = L.mx_gemm_workspace_bytes(128, 128, 64)
    assert need == 2 * 128 * 64 * 2 and L.mx_gemm_workspace_bytes(-1, 128, 64) == 0
    assert L.mx_gemm_workspace_bytes(128, 384, 64) == (128 + 384) * 64 * 2
    assert gm(ws=FAKE, wsb=need - 1) == ERR_WS
    assert gm(ws=FAKE_ODD, wsb=need) == ERR_ALIGN


def test_dot_pipeline_argument_checks():
    L, f = B.lib, B.MX6
    need = L.mx_dot_pipeline_workspace_bytes(128, 128, 128)
    assert need == 2 * 128 * 128 * 2 == L.mx_gemm_workspace_bytes(128, 128, 128)
    dp = lambda fa=f, fb=f, M=128, N=128, K=128, r=64, fbits=25, C=FAKE, ldc=128, a=FAKE, ws=FAKE, wsb=need: \
        L.mx_dot_pipeline(ctypes.byref(fa), ctypes.byref(fb), a, FAKE, FAKE, FAKE, FAKE, FAKE, M, N, K, r,
                          fbits, C, ldc, ws, wsb, NULL)
    assert dp(fa=B.fmt(32, 2, 1, 4)) == ERR_FORMAT and dp(fb=B.fmt(16, 2, 2, 4)) == ERR_FORMAT
    assert dp(K=0) == ERR_SHAPE and dp(K=96) == ERR_SHAPE and dp(M=-1) == ERR_SHAPE and dp(ldc=64) == ERR_SHAPE
    assert dp(r=32) == ERR_SHAPE and dp(r=96) == ERR_SHAPE and dp(r=0) == ERR_SHAPE and dp(r=256) == ERR_SHAPE
    assert dp(fbits=1) == ERR_SHAPE and dp(fbits=27) == ERR_SHAPE
    assert dp(C=NULL) == ERR_NULL and dp(a=NULL) == ERR_NULL
    assert dp(ws=NULL) == ERR_WS and dp(wsb=need - 1) == ERR_WS and dp(ws=FAKE_ODD) == ERR_ALIGN
    assert dp(M=0) == OK


def test_resources_are_asked_for_before_the_first_launch():
    # A sweep of more than 63 distinct quantizers needs more than 64 KiB of LDS per workgroup,
    # which a kernel has to be granted once per device.  That request is made for every chunk of
    # the format list before the first kernel of the call is enqueued; without a device it is
    # refused, and the call must come back with BDR_ERR_LAUNCH from that request.
    import torch
    if torch.cuda.device_count() > 0:
        pytest.skip("needs a machine without a GPU: with one, the placeholder pointers would be used")
    fmts = [B.fmt(k1, k2, 1, m) for k1 in (16, 32, 64) for k2 in (1, 2, 4) for m in range(1, 9)]
    assert len(fmts) == 72
    arr = (B.Format * len(fmts))(*fmts)
    need = B.lib.bdr_qsnr_sweep_workspace_bytes(len(fmts))
    assert B.lib.bdr_qsnr_sweep(arr, len(fmts), FAKE, 0, 4, 64, 64, FAKE, FAKE, FAKE, need, NULL) == ERR_LAUNCH
    # ... also when only the last chunk of a long list needs it
    small = [B.MX6] * 128 + fmts
    arr = (B.Format * len(small))(*small)
    need = B.lib.bdr_qsnr_sweep_workspace_bytes(len(small))
    assert B.lib.bdr_qsnr_sweep(arr, len(small), FAKE, 0, 4, 64, 64, FAKE, FAKE, FAKE, need, NULL) == ERR_LAUNCH
    # the two-pass mx_gemm asks for its product kernel's LDS before it enqueues the image writers
    # (MX4 x MX4 on FP4 images: 72 KiB even with the small tile)
    f = B.MX4
    need = B.lib.mx_gemm_workspace_bytes(128, 128, 128)
    assert B.lib.mx_gemm(ctypes.byref(f), ctypes.byref(f), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 128, 128, 128,
                         FAKE, 128, FAKE, need, NULL) == ERR_LAUNCH


def test_tile_packing_of_the_paper_formats():
    # Sec. IV-B "Memory Footprint": a 256-element tile into a 64-byte interface.  Table II gives
    # 9 / 6 / 4 bits per element, so the tile is 288 / 192 / 128 bytes: 5 / 3 / 2 transfers,
    # i.e. MX9 fills 4.5 of 5 (90 %), MX6 and MX4 fill theirs completely.
    assert B.bdr_tile_packing(B.MX9) == (288, 5, 0.9)
    assert B.bdr_tile_packing(B.MX6) == (192, 3, 1.0)
    assert B.bdr_tile_packing(B.MX4) == (128, 2, 1.0)
    # block floating point with 8-bit mantissas and sign over 16 elements: 9.5 bits per element
    assert B.bdr_tile_packing(B.fmt(16, 16, 0, 8))[0] == 304
    # a tile that is not a whole number of blocks still pays for the last block's exponent
    assert B.bdr_tile_packing(B.MX9, tile_elements=8)[0] == (8 * 8 + 8 + 4 + 7) // 8
    L = B.lib
    assert L.bdr_tile_packing(ctypes.byref(B.MX9), 0, 64, NULL, NULL, NULL) == ERR_SHAPE
    assert L.bdr_tile_packing(ctypes.byref(B.fmt(16, 3, 1, 7)), 256, 64, NULL, NULL, NULL) == ERR_FORMAT
    assert L.bdr_tile_packing(ctypes.byref(B.MX9), 256, 64, NULL, NULL, NULL) == OK


def test_table_image_argument_checks():
    L, f = B.lib, B.MX6
    assert B.bdr_table_row_bytes(B.MX9, 128) == 144 and B.bdr_table_row_bytes(B.MX6, 128) == 96
    assert B.bdr_table_row_bytes(B.MX4, 64) == 32
    for f2, cols in ((B.MX6, 128), (B.MX9, 64), (B.MX4, 1024)):
        assert 1000 * B.bdr_table_row_bytes(f2, cols) == sum(B.bdr_packed_sizes(f2, 1000, cols))
    assert B.bdr_table_row_bytes(B.MX6, 96) == 0 and B.bdr_table_row_bytes(B.fmt(32, 2, 1, 4), 128) == 0
    assert B.bdr_table_row_bytes(B.MX6, 0) == 0 and B.bdr_table_row_bytes(B.MX6, -64) == 0
    pk = lambda fm=f, rows=10, cols=128, codes=FAKE, sexp=FAKE, mexp=FAKE, t=FAKE: L.bdr_table_pack(
        ctypes.byref(fm), codes, sexp, mexp, rows, cols, t, NULL)
    assert pk(fm=B.fmt(16, 16, 0, 4)) == ERR_FORMAT and pk(cols=96) == ERR_SHAPE and pk(rows=-1) == ERR_SHAPE
    assert pk(codes=NULL) == ERR_NULL and pk(t=NULL) == ERR_NULL and pk(mexp=NULL) == ERR_NULL
    assert pk(t=FAKE_ODD) == ERR_ALIGN and pk(sexp=FAKE_ODD) == ERR_ALIGN
    assert pk(rows=0) == OK and pk(rows=0, codes=NULL, t=NULL) == OK
    tg = lambda fm=f, t=FAKE, rows=100, cols=128, idx=FAKE, n=10, y=FAKE, dtype=0: L.bdr_table_gather_dequantize(
        ctypes.byref(fm), t, rows, cols, idx, n, y, dtype, NULL)
    assert tg(fm=B.fmt(32, 2, 1, 4)) == ERR_FORMAT and tg(dtype=3) == ERR_DTYPE
    assert tg(cols=32) == ERR_SHAPE and tg(n=-1) == ERR_SHAPE and tg(rows=-1) == ERR_SHAPE
    assert tg(idx=NULL) == ERR_NULL and tg(y=NULL) == ERR_NULL and tg(t=NULL) == ERR_NULL
    assert tg(idx=FAKE_ODD) == ERR_ALIGN and tg(y=FAKE_ODD) == ERR_ALIGN and tg(t=FAKE_ODD) == ERR_ALIGN
    assert tg(n=0) == OK and tg(n=0, idx=NULL, y=NULL, t=NULL) == OK


def test_operand_image_argument_checks():
    L, f = B.lib, B.MX6
    FP6, BF = B.OPERAND_FP6, B.OPERAND_BF16
    assert B.mx_operand_bytes(B.MX6, 128, 256) == 128 * 256 == B.mx_operand_bytes(B.MX4, 128, 256, FP6)
    assert B.mx_operand_bytes(B.MX9, 128, 256, FP6) == 0               # MX9 does not fit E2M3
    assert B.mx_operand_bytes(B.MX9, 128, 256, BF) == 2 * 128 * 256 == B.mx_operand_bytes(B.MX4, 128, 256, BF)
    assert B.mx_operand_bytes(B.fmt(16, 2, 1, 4, rounding=B.RTZ), 128, 256) == 0
    assert B.mx_operand_bytes(B.MX6, 128, 100) == 0 and B.mx_operand_bytes(B.MX6, -1, 64) == 0
    F4 = B.OPERAND_FP4
    assert B.mx_operand_bytes(B.MX6, 128, 256, F4) == 0 and B.mx_operand_bytes(B.MX6, 128, 256, 3) == 0   # FP4: MX4 only
    assert B.mx_operand_bytes(B.MX4, 128, 256, F4) == 128 * 128 + 128 * 16            # codes + one scale byte per block
    assert B.mx_operand_bytes(B.MX4, 130, 256, F4) == 130 * 128 + 256 * 16            # scale rows padded to 128
    assert B.mx_operand_bytes(B.MX4, 128, 192, F4) == 0                               # K in multiples of 128
    qo = lambda fm=f, x=FAKE, dtype=0, rows=128, cols=128, ld=128, axis=0, image=FP6, img=FAKE: \
        L.bdr_quantize_operand(ctypes.byref(fm), x, dtype, rows, cols, ld, axis, image, 0, img, NULL)
    assert qo(fm=B.MX9) == ERR_FORMAT and qo(fm=B.fmt(32, 2, 1, 4)) == ERR_FORMAT and qo(dtype=2) == ERR_DTYPE
    assert qo(fm=B.fmt(32, 2, 1, 4), image=BF) == ERR_FORMAT and qo(image=7) == ERR_SHAPE
    assert qo(cols=96, ld=96) == ERR_SHAPE and qo(axis=3) == ERR_SHAPE and qo(ld=64) == ERR_SHAPE
    assert qo(axis=1, rows=64) == ERR_SHAPE and qo(axis=1, cols=32, ld=32) == ERR_SHAPE
    assert qo(axis=1, dtype=1, cols=64, ld=64) == ERR_SHAPE            # BF16 tiles are 128 columns wide
    assert qo(fm=B.MX6, image=F4) == ERR_FORMAT and qo(fm=B.MX4, image=F4, cols=192, ld=192) == ERR_SHAPE
    assert qo(fm=B.MX4, image=F4, axis=1, cols=64, ld=64) == ERR_SHAPE   # column blocks: operand rows in 128s
    assert qo(fm=B.MX4, image=F4, x=NULL) == ERR_NULL and qo(fm=B.MX4, image=F4, rows=0) == OK
    assert qo(x=NULL) == ERR_NULL and qo(img=NULL) == ERR_NULL
    assert qo(fm=B.MX9, image=BF, x=FAKE_ODD) == ERR_ALIGN and qo(img=FAKE_ODD) == ERR_ALIGN and qo(rows=0) == OK
    go = lambda fa=f, fb=f, a=FAKE, b=FAKE, image=FP6, M=128, N=128, K=64, C=FAKE, cd=0, ldc=128: \
        L.mx_gemm_operands(ctypes.byref(fa), ctypes.byref(fb), a, b, image, M, N, K, C, cd, ldc, NULL)
    assert go(fa=B.MX9) == ERR_FORMAT and go(fb=B.fmt(16, 16, 0, 4)) == ERR_FORMAT and go(cd=5) == ERR_DTYPE
    assert go(fa=B.fmt(16, 16, 0, 4), image=BF) == ERR_FORMAT and go(image=-1) == ERR_SHAPE
    assert go(K=48) == ERR_SHAPE and go(ldc=64) == ERR_SHAPE and go(M=-1) == ERR_SHAPE
    assert go(image=F4) == ERR_FORMAT and go(fa=B.MX4, fb=B.MX4, image=F4, K=64) == ERR_SHAPE
    assert go(fa=B.MX4, fb=B.MX4, image=F4, K=128, a=NULL) == ERR_NULL and go(fa=B.MX4, fb=B.MX6, image=F4, K=128) == ERR_FORMAT
    assert go(C=NULL) == ERR_NULL and go(a=NULL) == ERR_NULL and go(b=NULL, fa=B.MX9, image=BF) == ERR_NULL
    assert go(a=FAKE_ODD) == ERR_ALIGN and go(C=ctypes.c_void_p(0x10002)) == ERR_ALIGN and go(M=0) == OK


def test_gather_argument_checks():
    L = B.lib
    f = B.MX6
    ga = lambda fm=f, rows=100, cols=128, idx=FAKE, n=10, y=FAKE, dtype=0, codes=FAKE: L.bdr_gather_dequantize(
        ctypes.byref(fm), codes, FAKE, FAKE, rows, cols, idx, n, y, dtype, NULL)
    assert ga(fm=B.fmt(32, 2, 1, 4)) == ERR_FORMAT
    assert ga(cols=48) == ERR_SHAPE and ga(n=-1) == ERR_SHAPE and ga(rows=-1) == ERR_SHAPE
    assert ga(dtype=5) == ERR_DTYPE
    assert ga(idx=NULL) == ERR_NULL and ga(y=NULL) == ERR_NULL and ga(codes=NULL) == ERR_NULL
    assert ga(idx=FAKE_ODD) == ERR_ALIGN and ga(y=FAKE_ODD) == ERR_ALIGN
    assert ga(n=0) == OK


def test_header_is_plain_c(tmp_path):
    # the boundary is a C ABI: the header must compile as C99 on its own, and a C caller must
    # be able to name every entry point and build a format from the macros
    import subprocess
    src = tmp_path / "use_header.c"
    src.write_text(
        '#include "bdr_mx.h"\n'
        "static const bdr_format mx9 = BDR_FORMAT_MX9, mx6 = BDR_FORMAT_MX6, mx4 = BDR_FORMAT_MX4;\n"
        "int probe(void) {\n"
        "    size_t a, b, c;\n"
        "    void *fns[] = {(void *)bdr_status_string, (void *)bdr_format_validate, (void *)bdr_packed_sizes,\n"
        "                   (void *)bdr_quantize, (void *)bdr_dequantize, (void *)bdr_gather_dequantize,\n"
        "                   (void *)bdr_table_row_bytes, (void *)bdr_table_pack, (void *)bdr_table_gather_dequantize,\n"
        "                   (void *)bdr_tile_packing, (void *)bdr_quantize_dequantize,\n"
        "                   (void *)bdr_qsnr_sweep_workspace_bytes, (void *)bdr_qsnr_sweep,\n"
        "                   (void *)bdr_qsnr_sweep_static, (void *)bdr_qsnr_sweep_static_scratch_bytes,\n"
        "                   (void *)mx_gemm_workspace_bytes, (void *)mx_gemm, (void *)mx_gemm_to,\n"
        "                   (void *)mx_operand_bytes, (void *)bdr_quantize_operand, (void *)mx_gemm_operands,\n"
        "                   (void *)mx_dot_pipeline_workspace_bytes, (void *)mx_dot_pipeline};\n"
        "    (void)fns;\n"
        "    return bdr_packed_sizes(&mx9, 4, 64, BDR_AXIS_ROW, &a, &b, &c) + mx6.m + mx4.m;\n"
        "}\n")
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-Wno-pedantic", "-I",
                        os.path.join(ROOT, "include"), "-c", str(src), "-o", str(tmp_path / "use_header.o")],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
