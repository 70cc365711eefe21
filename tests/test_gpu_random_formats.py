"""GPU parity on seeded random BDR formats and shapes: the general kernels (row and column
blocks, FP32 and BF16, packed and fused) bit for bit against the oracle, and the sweep on random
format lists (duplicates, every rounding rule, more (m, rounding) pairs per k1 than one group
holds) within the QSNR tolerance."""
import math

import numpy as np
import pytest
import torch

import oracle as O
import paper_2302_08007_amd as B
import synth_inputs as S
from gpu_util import assert_bits_equal, assert_planes_equal, ofmt, to_np

pytestmark = pytest.mark.gpu


def _random_format(rng):
    lk1 = int(rng.integers(0, 9))                      # k1 = 1 .. 256
    lk2 = int(rng.integers(0, lk1 + 1))
    d2 = int(rng.integers(0, 4))
    m = int(rng.integers(1, 9))
    return B.fmt(1 << lk1, 1 << lk2, d2, m, rounding=int(rng.integers(0, 3)))


@pytest.mark.parametrize("seed", range(24))
def test_random_format_row_and_column(seed):
    rng = np.random.default_rng(1000 + seed)
    f = _random_format(rng)
    dtype = torch.float32 if seed % 2 == 0 or f.m + (1 << f.d2) - 1 > 8 else torch.bfloat16
    unit = max(f.k1, 8)
    for axis in (B.AXIS_ROW, B.AXIS_COL):
        # the blocked axis is a multiple of max(k1, 8); sizes straddle workgroup and wave bounds
        blocked = unit * int(rng.integers(1, max(2, 4096 // unit)))
        other = int(rng.integers(1, 40)) * (8 if axis == B.AXIS_COL else 1)
        rows, cols = (other, blocked) if axis == B.AXIS_ROW else (blocked, other)
        x = S.wide_range(rows, cols, device="cuda", seed=seed * 7 + axis, spread=10, dtype=dtype)
        xn = to_np(x)
        oaxis = O.AXIS_ROW if axis == B.AXIS_ROW else O.AXIS_COL
        want = O.quantize(ofmt(f), xn, axis=oaxis)
        what = "%r axis %d %s %dx%d" % (f, axis, dtype, rows, cols)
        planes = B.bdr_quantize(f, x, axis=axis)
        torch.cuda.synchronize()
        assert_planes_equal(planes, want, what + " quantize")
        out_dtype = np.float32 if dtype == torch.float32 else np.uint16
        ywant = O.dequantize(ofmt(f), *want, rows, cols, axis=oaxis, out_dtype=out_dtype)
        assert_bits_equal(B.bdr_dequantize(f, planes, rows, cols, axis=axis, dtype=dtype), ywant,
                          what + " dequantize")
        assert_bits_equal(B.bdr_quantize_dequantize(f, x, axis=axis), ywant, what + " fused")


@pytest.mark.parametrize("seed", range(24))
def test_random_format_on_shapes_of_any_size(seed):
    """Random formats on shapes whose blocked axis is any length (a short last block is stored
    as a whole one, its pads as code 0) and whose other axis is any length too."""
    rng = np.random.default_rng(3000 + seed)
    f = _random_format(rng)
    dtype = torch.float32 if seed % 2 == 0 or f.m + (1 << f.d2) - 1 > 8 else torch.bfloat16
    for axis in (B.AXIS_ROW, B.AXIS_COL):
        while True:
            blocked = int(rng.integers(1, 3000))
            if (-(-blocked // f.k1) * f.k1) % 8 == 0:       # only k1 < 8 can miss this
                break
        other = int(rng.integers(1, 60))
        rows, cols = (other, blocked) if axis == B.AXIS_ROW else (blocked, other)
        x = S.wide_range(rows, cols, device="cuda", seed=seed * 11 + axis, spread=10, dtype=dtype)
        oaxis = O.AXIS_ROW if axis == B.AXIS_ROW else O.AXIS_COL
        want = O.quantize(ofmt(f), to_np(x), axis=oaxis)
        what = "%r axis %d %s %dx%d" % (f, axis, dtype, rows, cols)
        planes = B.bdr_quantize(f, x, axis=axis)
        torch.cuda.synchronize()
        assert_planes_equal(planes, want, what + " quantize")
        out_dtype = np.float32 if dtype == torch.float32 else np.uint16
        ywant = O.dequantize(ofmt(f), *want, rows, cols, axis=oaxis, out_dtype=out_dtype)
        assert_bits_equal(B.bdr_dequantize(f, planes, rows, cols, axis=axis, dtype=dtype), ywant,
                          what + " dequantize")
        assert_bits_equal(B.bdr_quantize_dequantize(f, x, axis=axis), ywant, what + " fused")


@pytest.mark.parametrize("seed", range(6))
def test_random_format_lists_in_the_sweep(seed):
    rng = np.random.default_rng(2000 + seed)
    n = int(rng.integers(1, 200))
    fmts = [_random_format(rng) for _ in range(n)]
    fmts += [fmts[int(i)] for i in rng.integers(0, n, size=n // 4)]      # duplicates
    if seed % 2:
        for f in fmts:                                                     # the all-nearest-even kernel
            f.rounding = B.RNE
    kmax = max(f.k1 for f in fmts)
    rows, cols = int(rng.integers(1, 30)), max(kmax, 8) * int(rng.integers(1, 9))
    x = S.wide_range(rows, cols, device="cuda", seed=seed, spread=4)
    q, s = B.bdr_qsnr_sweep(fmts, x)
    torch.cuda.synchronize()
    q, s = q.cpu().numpy(), s.cpu().numpy()
    qw, sw = O.qsnr_sweep([ofmt(f) for f in fmts], to_np(x))
    for i, f in enumerate(fmts):
        if math.isinf(qw[i]):
            assert math.isinf(q[i]) and s[i] == 0.0, f
        else:
            assert q[i] == pytest.approx(qw[i], rel=1e-4), (f, q[i], qw[i])
            assert s[i] == pytest.approx(sw[i], rel=2e-5), f
    assert s[-1] == pytest.approx(sw[-1], rel=2e-5)
