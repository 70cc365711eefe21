"""GPU parity: column-wise (strided-axis) quantize / dequantize / fused against the oracle,
bit for bit.  Column blocks are defined as row blocks of the transposed tensor (Sec. V)."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2302_08007_amd as B
import synth_inputs as S
from gpu_util import assert_bits_equal, assert_planes_equal, ofmt, to_np

pytestmark = pytest.mark.gpu
MX = ["MX9", "MX6", "MX4"]


def _check_col(f, x, what):
    rows, cols = x.shape
    xn = to_np(x)
    want = O.quantize(ofmt(f), xn, axis=O.AXIS_COL)
    planes = B.bdr_quantize(f, x, axis=B.AXIS_COL)
    torch.cuda.synchronize()
    assert_planes_equal(planes, want, what + " quantize")
    out_dtype = np.float32 if x.dtype == torch.float32 else np.uint16
    ywant = O.dequantize(ofmt(f), *want, rows, cols, axis=O.AXIS_COL, out_dtype=out_dtype)
    y = B.bdr_dequantize(f, planes, rows, cols, axis=B.AXIS_COL, dtype=x.dtype)
    assert_bits_equal(y, ywant, what + " dequantize")
    y2 = B.bdr_quantize_dequantize(f, x, axis=B.AXIS_COL)
    assert_bits_equal(y2, ywant, what + " fused")
    return planes


@pytest.mark.parametrize("name", MX)
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
# (odd and even numbers of column tiles: the quantize kernel takes tiles in pairs when it can)
@pytest.mark.parametrize("shape", [(128, 64), (256, 192), (384, 64), (1024, 320), (256, 256), (384, 1024),
                                   (128, 128 * 17), (1024, 128 * 34)])
def test_tiled_path(name, dtype, shape):
    x = S.wide_range(*shape, device="cuda", seed=shape[0] + shape[1], dtype=dtype)
    _check_col(getattr(B, name), x, "%s %s %s" % (name, dtype, shape))


@pytest.mark.parametrize("name", MX)
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("shape", [(16, 8), (48, 24), (144, 64), (128, 72), (272, 200)])
def test_shapes_that_take_the_general_path(name, dtype, shape):
    # rows not a multiple of 128 or columns not a multiple of 64
    x = S.wide_range(*shape, device="cuda", seed=shape[0] * 7 + shape[1], dtype=dtype)
    _check_col(getattr(B, name), x, "%s %s %s" % (name, dtype, shape))


@pytest.mark.parametrize("kw", [dict(k1=8, k2=1, d2=1, m=2), dict(k1=32, k2=4, d2=2, m=3),
                                dict(k1=64, k2=64, d2=0, m=4), dict(k1=4, k2=2, d2=1, m=6),
                                dict(k1=128, k2=16, d2=3, m=5), dict(k1=16, k2=2, d2=1, m=4, rounding=1)],
                         ids=lambda kw: "-".join("%s%d" % kv for kv in kw.items()))
def test_other_formats_column_wise(kw):
    f = B.fmt(**kw)
    x = S.wide_range(256, 40, device="cuda", seed=11)
    _check_col(f, x, repr(f))


GEN_TILED = [dict(k1=8, k2=1, d2=1, m=2), dict(k1=8, k2=8, d2=1, m=4), dict(k1=32, k2=4, d2=2, m=3),
             dict(k1=32, k2=32, d2=1, m=4), dict(k1=64, k2=64, d2=0, m=4), dict(k1=64, k2=64, d2=1, m=2),
             dict(k1=64, k2=4, d2=1, m=2), dict(k1=128, k2=16, d2=3, m=5), dict(k1=128, k2=128, d2=1, m=4),
             dict(k1=16, k2=1, d2=3, m=8), dict(k1=16, k2=2, d2=1, m=4, rounding=1),
             dict(k1=16, k2=2, d2=1, m=7, rounding=2), dict(k1=16, k2=16, d2=0, m=7)]


@pytest.mark.parametrize("kw", GEN_TILED, ids=lambda kw: "-".join("%s%d" % kv for kv in kw.items()))
@pytest.mark.parametrize("shape", [(1024, 64), (2048, 192)])
def test_other_formats_on_whole_tiles(kw, shape):
    # Formats outside Table II (or rounded another way) on shapes made of whole 128-row tiles take
    # the tiled general kernel: block sizes 8 to 128, codes of 3 to 9 bits, microexponent streams
    # of 1 to 384 bits per tile column (those below a byte make a workgroup walk 2, 4 or 8 tiles).
    f = B.fmt(**kw)
    x = S.wide_range(*shape, device="cuda", seed=shape[1] + kw["k1"] + kw["m"])
    _check_col(f, x, repr(f))


@pytest.mark.parametrize("m", [2, 4])
@pytest.mark.parametrize("d2", [0, 1])
@pytest.mark.parametrize("k2", [1, 2, 4, 0])
@pytest.mark.parametrize("k1", [8, 16, 32, 64])
def test_design_space_sweep_formats_column_wise(k1, k2, d2, m):
    # the 64 formats of the design-space sweep (Sec. IV) along columns: on whole tiles the tiled
    # kernel compiled for the tuple (FP32 and BF16; one, two or four tiles per workgroup
    # depending on how many microexponent bits a tile column has), with special values in
    # some columns; the same data rounded another way goes through the run-time-tuple kernel
    f = B.fmt(k1, k1 if k2 == 0 else k2, d2, m)
    x = S.wide_range(1024, 128, device="cuda", seed=k1 + 3 * m + d2, spread=5)
    x[0, 0], x[1, 0], x[17, 0] = float("inf"), float("nan"), -float("inf")
    x[:, 1] = 0.0
    x[5, 1] = -0.0
    x[:64, 2] = 2.0 ** -140
    x[:, 3] = 1.9999999
    _check_col(f, x, "%r fp32" % f)
    _check_col(f, x.to(torch.bfloat16), "%r bf16" % f)
    _check_col(B.fmt(k1, k1 if k2 == 0 else k2, d2, m, rounding=B.RTZ), x[:512], "%r truncating" % f)


@pytest.mark.parametrize("kw", [GEN_TILED[0], GEN_TILED[2], GEN_TILED[4], GEN_TILED[6], GEN_TILED[11]],
                         ids=lambda kw: "-".join("%s%d" % kv for kv in kw.items()))
def test_other_formats_on_whole_tiles_bf16(kw):
    f = B.fmt(**kw)
    x = S.wide_range(1024, 256, device="cuda", seed=kw["k1"], dtype=torch.bfloat16)
    _check_col(f, x, repr(f) + " bf16")


def test_other_formats_on_whole_tiles_strided_in_place_and_special_values():
    f = B.fmt(32, 2, 1, 4)
    big = S.wide_range(512, 512, device="cuda", seed=33)
    x = big[:, 64:64 + 128]                        # ld > cols
    xn = np.ascontiguousarray(to_np(big)[:, 64:64 + 128])
    want = O.quantize(ofmt(f), xn, axis=O.AXIS_COL)
    assert_planes_equal(B.bdr_quantize(f, x, axis=B.AXIS_COL), want, "strided")
    ywant = O.quantize_dequantize(ofmt(f), xn, axis=O.AXIS_COL)
    z = x.clone()
    B.bdr_quantize_dequantize(f, z, axis=B.AXIS_COL, out=z)
    assert_bits_equal(z, ywant, "in place")
    y = torch.full((512, 512), 7.0, device="cuda")
    B.bdr_dequantize(f, [torch.from_numpy(p).cuda() for p in want], 512, 128, axis=B.AXIS_COL, out=y[:, 64:64 + 128])
    assert_bits_equal(y[:, 64:64 + 128].contiguous(), ywant, "strided dequantize")
    assert torch.all(y[:, :64] == 7.0) and torch.all(y[:, 192:] == 7.0)
    s = torch.zeros(128, 64, device="cuda")
    s[3, 0] = -0.0
    s[:32, 1] = 2.0 ** -140
    s[5, 1] = -3 * 2.0 ** -149
    s[:32, 2] = 2.0 ** -126
    s[0, 3], s[1, 3], s[2, 3] = 3.4e38, -1.7e38, 1e-30
    s[0, 4], s[1, 4], s[2, 4], s[3, 4] = float("inf"), -float("inf"), float("nan"), 1.0
    s[:, 6] = 1.9999999
    for kw in (dict(k1=32, k2=2, d2=1, m=4), dict(k1=8, k2=4, d2=2, m=2), dict(k1=64, k2=1, d2=1, m=6)):
        _check_col(B.fmt(**kw), s, "special %r" % (kw,))


@pytest.mark.parametrize("kw", [dict(k1=16, k2=2, d2=1, m=7), dict(k1=16, k2=2, d2=1, m=4),
                                dict(k1=16, k2=2, d2=1, m=2), dict(k1=64, k2=8, d2=2, m=4, rounding=1),
                                dict(k1=8, k2=8, d2=0, m=6), dict(k1=2, k2=1, d2=1, m=3)],
                         ids=lambda kw: "-".join("%s%d" % kv for kv in kw.items()))
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_columns_with_a_short_last_block(kw, dtype):
    """Column blocks on shapes whose column length is not a whole number of blocks, or whose
    row length is not a multiple of 8: every column is a padded row of the transpose."""
    f = B.fmt(**kw)
    if dtype == torch.bfloat16 and f.m + (1 << f.d2) - 1 > 8:
        pytest.skip("bf16 cannot hold this format exactly")
    for rows, cols in ((50, 7), (1, 1), (1000, 24), (130, 64), (16, 3), (24, 9)):
        if (-(-rows // f.k1) * f.k1) % 8:
            continue
        x = S.wide_range(rows, cols, device="cuda", seed=3 * rows + cols, dtype=dtype)
        planes = _check_col(f, x, "%r %s %s" % (f, dtype, (rows, cols)))
        want = O.quantize(ofmt(f), np.ascontiguousarray(to_np(x).T))
        assert_planes_equal(planes, want, "%r %s: rows of the transpose" % (f, (rows, cols)))
    if (-(-45 // f.k1) * f.k1) % 8:
        return
    big = S.wide_range(45, 131, device="cuda", seed=78, dtype=dtype)
    view = big[:, 5:5 + 9]
    xn = np.ascontiguousarray(to_np(big)[:, 5:5 + 9])
    want = O.quantize(ofmt(f), xn, axis=O.AXIS_COL)
    planes = B.bdr_quantize(f, view, axis=B.AXIS_COL)
    assert_planes_equal(planes, want, "%r view" % f)
    out_dtype = np.float32 if dtype == torch.float32 else np.uint16
    ywant = O.dequantize(ofmt(f), *want, 45, 9, axis=O.AXIS_COL, out_dtype=out_dtype)
    out = torch.full_like(big, 7.0)
    B.bdr_dequantize(f, planes, 45, 9, axis=B.AXIS_COL, out=out[:, 5:5 + 9])
    assert_bits_equal(out[:, 5:5 + 9].contiguous(), ywant, "%r view dequantize" % f)
    assert bool((out[:, :5] == 7).all()) and bool((out[:, 14:] == 7).all())


@pytest.mark.parametrize("name", MX)
def test_column_blocks_equal_row_blocks_of_the_transpose(name):
    f = getattr(B, name)
    x = S.wide_range(256, 128, device="cuda", seed=21)
    pc = B.bdr_quantize(f, x, axis=B.AXIS_COL)
    pr = B.bdr_quantize(f, x.t().contiguous(), axis=B.AXIS_ROW)
    for a, b in zip(pc, pr):
        assert torch.equal(a, b)
    # and differs from quantizing along rows
    pr2 = B.bdr_quantize(f, x, axis=B.AXIS_ROW)
    assert not torch.equal(pc[0], pr2[0])


def test_strided_and_in_place():
    big = S.wide_range(256, 512, device="cuda", seed=31)
    x = big[:, 128:128 + 192]                      # ld > cols
    xn = np.ascontiguousarray(to_np(big)[:, 128:128 + 192])
    for f in (B.MX9, B.MX6):
        want = O.quantize(ofmt(f), xn, axis=O.AXIS_COL)
        assert_planes_equal(B.bdr_quantize(f, x, axis=B.AXIS_COL), want, "strided")
        ywant = O.quantize_dequantize(ofmt(f), xn, axis=O.AXIS_COL)
        z = x.clone()
        B.bdr_quantize_dequantize(f, z, axis=B.AXIS_COL, out=z)
        assert_bits_equal(z, ywant, "in place")


def test_special_values_column_wise():
    x = torch.zeros(128, 64, device="cuda")
    x[3, 0] = -0.0
    x[:16, 1] = 2.0 ** -140
    x[5, 1] = -3 * 2.0 ** -149
    x[:16, 2] = 2.0 ** -126
    x[1, 2] = 2.0 ** -127
    x[0, 3], x[1, 3], x[2, 3] = 3.4e38, -1.7e38, 1e-30
    x[0, 4], x[1, 4], x[2, 4], x[3, 4] = float("inf"), -float("inf"), float("nan"), 1.0
    x[:64, 5] = torch.tensor([(-1.0) ** i * (i + 0.5) for i in range(64)], device="cuda")
    x[:, 6] = 1.9999999
    for name in MX:
        _check_col(getattr(B, name), x, name + " special")
        _check_col(getattr(B, name), x.to(torch.bfloat16), name + " special bf16")


def test_activation_config_full_size_sampled_columns():
    # 8192 x 12288 bf16, MX9, the bench configuration: the oracle checks whole column tiles
    # sampled across the tensor (each column's planes are a contiguous slice of the full planes)
    x = S.activation(device="cuda")
    rows, cols = x.shape
    f = B.MX9
    planes = B.bdr_quantize(f, x, axis=B.AXIS_COL)
    y = B.bdr_quantize_dequantize(f, x, axis=B.AXIS_COL)
    torch.cuda.synchronize()
    rng = np.random.default_rng(0)
    for c0 in sorted(set([0, cols - 64] + [int(v) * 64 for v in rng.integers(0, cols // 64, 4)])):
        sub = x[:, c0:c0 + 64].contiguous()
        want = O.quantize(ofmt(f), to_np(sub), axis=O.AXIS_COL)
        per_col = [rows * 8 // 8, rows // 16, rows // 16]
        got = [p[c0 * n:(c0 + 64) * n] for p, n in zip(planes, per_col)]
        assert_planes_equal(got, want, "columns %d.." % c0)
        ywant = O.dequantize(ofmt(f), *want, rows, 64, axis=O.AXIS_COL, out_dtype=np.uint16)
        assert_bits_equal(y[:, c0:c0 + 64].contiguous(), ywant, "fused columns %d.." % c0)
    # the outlier columns really are there, and row-wise quantization of the same tensor differs
    pr = B.bdr_quantize(f, x, axis=B.AXIS_ROW)
    assert not torch.equal(pr[1][:4096], planes[1][:4096])


@pytest.mark.parametrize("kw", [dict(k1=32, k2=2, d2=1, m=4), dict(k1=64, k2=64, d2=1, m=2)],
                         ids=lambda kw: "-".join("%s%d" % kv for kv in kw.items()))
def test_other_formats_full_size_sampled_columns(kw):
    # 8192 x 8192 fp32, the size of the bench leg for formats outside Table II blocked down the
    # columns (the second format makes a workgroup walk four tiles per microexponent byte): the
    # oracle checks whole column tiles sampled across the tensor, planes, dequantize and fused
    f = B.fmt(**kw)
    x = S.gemm_operands(8192, 8, 8192, device="cuda", seed=40)[0]
    rows, cols = x.shape
    planes = B.bdr_quantize(f, x, axis=B.AXIS_COL)
    y = B.bdr_quantize_dequantize(f, x, axis=B.AXIS_COL)
    yd = B.bdr_dequantize(f, planes, rows, cols, axis=B.AXIS_COL)
    torch.cuda.synchronize()
    assert torch.equal(y, yd)
    rng = np.random.default_rng(1)
    per_col = [rows * (f.m + 1) // 8, rows // f.k1, rows // f.k2 * f.d2 // 8]
    for c0 in sorted(set([0, cols - 64] + [int(v) * 64 for v in rng.integers(0, cols // 64, 3)])):
        sub = x[:, c0:c0 + 64].contiguous()
        want = O.quantize(ofmt(f), to_np(sub), axis=O.AXIS_COL)
        got = [p[c0 * n:(c0 + 64) * n] for p, n in zip(planes, per_col)]
        assert_planes_equal(got, want, "columns %d.." % c0)
        ywant = O.dequantize(ofmt(f), *want, rows, 64, axis=O.AXIS_COL, out_dtype=np.float32)
        assert_bits_equal(y[:, c0:c0 + 64].contiguous(), ywant, "fused columns %d.." % c0)
