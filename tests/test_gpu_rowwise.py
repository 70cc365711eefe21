"""GPU parity: row-wise quantize / dequantize / fused round trip against the CPU oracle,
bit for bit, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle as O
import synth_inputs as S
from gpu_util import assert_bits_equal, assert_planes_equal, ofmt, to_np

pytestmark = pytest.mark.gpu

import paper_2302_08007_amd as B  # noqa: E402

MX = ["MX9", "MX6", "MX4"]


def _fmt(name):
    return getattr(B, name)


def _roundtrip_check(f, x, what):
    rows, cols = x.shape
    xn = to_np(x)
    want = O.quantize(ofmt(f), xn)
    planes = B.bdr_quantize(f, x)
    torch.cuda.synchronize()
    assert_planes_equal(planes, want, what + " quantize")
    out_dtype = np.float32 if x.dtype == torch.float32 else np.uint16
    ywant = O.dequantize(ofmt(f), *want, rows, cols, out_dtype=out_dtype)
    y = B.bdr_dequantize(f, planes, rows, cols, dtype=x.dtype)
    assert_bits_equal(y, ywant, what + " dequantize")
    y2 = B.bdr_quantize_dequantize(f, x)
    assert_bits_equal(y2, ywant, what + " fused")


@pytest.mark.parametrize("name", MX)
def test_tiny_config(name):
    # 4096 x 256 fp32 N(0,1): codes, shared exponents, microexponents, dequantized values
    x = S.tiny(device="cuda")
    _roundtrip_check(_fmt(name), x, name)


@pytest.mark.parametrize("name", MX)
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("shape", [(2, 16), (1, 32), (3, 32), (7, 48), (5, 2064), (513, 4096 + 32)])
def test_mx_shapes_and_edge_values(name, dtype, shape):
    # several tiles plus a ragged tail; exponents over many binades, zeros, negative zeros
    x = S.wide_range(*shape, device="cuda", seed=shape[0] * 1000 + shape[1], dtype=dtype)
    _roundtrip_check(_fmt(name), x, "%s %s %s" % (name, dtype, shape))


@pytest.mark.parametrize("name", MX)
def test_special_values(name):
    f = _fmt(name)
    x = torch.zeros(8, 64, device="cuda")
    x[0, 3] = -0.0                                   # all-zero block with one negative zero
    x[1, :16] = torch.tensor(2.0 ** -140)            # all-subnormal block
    x[1, 5] = -3 * 2.0 ** -149
    x[2, :16] = torch.tensor(2.0 ** -126)            # lowest normal binade next to subnormals
    x[2, 1] = 2.0 ** -127
    x[2, 2] = 1.5 * 2.0 ** -127
    x[3, 0] = 3.4e38                                 # top binade
    x[3, 1] = -1.7e38
    x[3, 2] = 1e-30
    x[4, 0] = float("inf")
    x[4, 1] = -float("inf")
    x[4, 2] = float("nan")
    x[4, 3] = 1.0
    x[5, :] = torch.tensor([(-1.0) ** i * (i + 0.5) for i in range(64)])   # exact ties
    x[6, :] = 1.9999999                              # everything rounds up past the top code
    x[7, ::2] = 1.0
    x[7, 1::2] = 2.0 ** -20                          # far below the block maximum
    _roundtrip_check(f, x, name + " special")


GENERIC = [
    dict(k1=8, k2=1, d2=1, m=2), dict(k1=8, k2=8, d2=0, m=4), dict(k1=16, k2=4, d2=1, m=4),
    dict(k1=32, k2=2, d2=2, m=3), dict(k1=64, k2=64, d2=1, m=2), dict(k1=64, k2=1, d2=3, m=8),
    dict(k1=128, k2=16, d2=2, m=5), dict(k1=256, k2=32, d2=3, m=1), dict(k1=4, k2=2, d2=1, m=3),
    dict(k1=2, k2=1, d2=2, m=6), dict(k1=1, k2=1, d2=0, m=4), dict(k1=16, k2=2, d2=1, m=5),
    dict(k1=16, k2=2, d2=1, m=4, rounding=1), dict(k1=16, k2=2, d2=1, m=7, rounding=2),
    dict(k1=32, k2=8, d2=1, m=4, rounding=1), dict(k1=256, k2=256, d2=1, m=4),
]


@pytest.mark.parametrize("kw", GENERIC, ids=lambda kw: "-".join("%s%d" % kv for kv in kw.items()))
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_generic_formats(kw, dtype):
    f = B.fmt(**kw)
    if dtype == torch.bfloat16 and f.m + (1 << f.d2) - 1 > 8:
        pytest.skip("bf16 cannot hold this format exactly")
    for shape in ((3, 256), (9, 1024 + 256)):
        x = S.wide_range(*shape, device="cuda", seed=17 + shape[0], dtype=dtype)
        _roundtrip_check(f, x, "%r %s %s" % (f, dtype, shape))


@pytest.mark.parametrize("m", [2, 4])
@pytest.mark.parametrize("d2", [0, 1])
@pytest.mark.parametrize("k2", [1, 2, 4, 0])
@pytest.mark.parametrize("k1", [8, 16, 32, 64])
def test_design_space_sweep_formats(k1, k2, d2, m):
    # the 64 formats of the design-space sweep (Sec. IV) as storage formats: FP32 rows with
    # pitch = row length take kernels compiled for the tuple; several workgroups and a ragged
    # last one, a single block, and (pitched rows) the run-time-tuple kernels on the same data
    f = B.fmt(k1, k1 if k2 == 0 else k2, d2, m)
    for shape in ((5, 1088), (1, 64), (40, 64)):
        x = S.wide_range(*shape, device="cuda", seed=k1 + shape[1], spread=4)
        _roundtrip_check(f, x, "%r %s" % (f, shape))
        _roundtrip_check(f, x.to(torch.bfloat16), "%r %s bf16" % (f, shape))   # BF16 rows: compiled for the tuple too
    big = S.wide_range(6, 1024, device="cuda", seed=k1 + 1, spread=4)
    sub = big[:, 128:128 + 704]
    want = O.quantize(ofmt(f), to_np(sub))
    assert_planes_equal(B.bdr_quantize(f, sub), want, "%r pitched" % f)


RAGGED_FORMATS = [dict(k1=16, k2=2, d2=1, m=7), dict(k1=16, k2=2, d2=1, m=4), dict(k1=16, k2=2, d2=1, m=2),
                  dict(k1=64, k2=4, d2=1, m=4), dict(k1=32, k2=32, d2=0, m=5, rounding=2),
                  dict(k1=8, k2=1, d2=2, m=3, rounding=1), dict(k1=256, k2=16, d2=3, m=8),
                  dict(k1=4, k2=2, d2=1, m=3), dict(k1=128, k2=128, d2=1, m=1)]


@pytest.mark.parametrize("kw", RAGGED_FORMATS, ids=lambda kw: "-".join("%s%d" % kv for kv in kw.items()))
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_rows_with_a_short_last_block(kw, dtype):
    """Row lengths that are not a whole number of blocks (Sec. IX, the remark after Theorem 1:
    fewer than k1 elements are a block of their own length): planes as the oracle pads them,
    pads stored as code 0, dequantize and the fused form writing the real elements only."""
    f = B.fmt(**kw)
    if dtype == torch.bfloat16 and f.m + (1 << f.d2) - 1 > 8:
        pytest.skip("bf16 cannot hold this format exactly")
    for rows, cols in ((1, 1), (3, 24), (5, 1000), (2, 2049), (33, 40), (300, 7)):
        if (-(-cols // f.k1) * f.k1) % 8:
            with pytest.raises(B.BdrError):
                B.bdr_packed_sizes(f, rows, cols)
            continue
        x = S.wide_range(rows, cols, device="cuda", seed=rows + cols, dtype=dtype)
        _roundtrip_check(f, x, "%r %s %s" % (f, dtype, (rows, cols)))
    # inside a wider tensor (odd pitch, odd offset): nothing outside the view is touched
    big = S.wide_range(9, 131, device="cuda", seed=77, dtype=dtype)
    view = big[:, 3:3 + 45]
    xn = np.ascontiguousarray(to_np(big)[:, 3:3 + 45])
    want = O.quantize(ofmt(f), xn)
    planes = B.bdr_quantize(f, view)
    assert_planes_equal(planes, want, "%r view" % f)
    out_dtype = np.float32 if dtype == torch.float32 else np.uint16
    ywant = O.dequantize(ofmt(f), *want, 9, 45, out_dtype=out_dtype)
    out = torch.full_like(big, 7.0)
    B.bdr_dequantize(f, planes, 9, 45, out=out[:, 3:3 + 45])
    assert_bits_equal(out[:, 3:3 + 45].contiguous(), ywant, "%r view dequantize" % f)
    assert bool((out[:, :3] == 7).all()) and bool((out[:, 48:] == 7).all())
    keep = big.clone()
    B.bdr_quantize_dequantize(f, view, out=view)       # in place
    assert_bits_equal(view.contiguous(), ywant, "%r view fused in place" % f)
    assert torch.equal(big[:, :3], keep[:, :3]) and torch.equal(big[:, 48:], keep[:, 48:])


@pytest.mark.parametrize("name", MX)
def test_strided_rows(name):
    # ld > cols: a column slice of a wider tensor
    f = _fmt(name)
    big = S.wide_range(33, 512, device="cuda", seed=5)
    x = big[:, 64:64 + 256]
    xn = np.ascontiguousarray(to_np(big)[:, 64:64 + 256])
    want = O.quantize(ofmt(f), xn)
    planes = B.bdr_quantize(f, x)
    assert_planes_equal(planes, want, name + " strided")
    ywant = O.dequantize(ofmt(f), *want, 33, 256)
    out = torch.full_like(big, 7.0)
    B.bdr_dequantize(f, planes, 33, 256, out=out[:, 64:64 + 256])
    assert_bits_equal(out[:, 64:64 + 256].contiguous(), ywant, name + " strided dequantize")
    assert torch.all(out[:, :64] == 7.0) and torch.all(out[:, 320:] == 7.0)


def test_fused_in_place_and_empty():
    x = S.tiny(64, 256, device="cuda")
    want = O.quantize_dequantize(ofmt(B.MX6), to_np(x))
    B.bdr_quantize_dequantize(B.MX6, x, out=x)
    assert_bits_equal(x, want, "in place")
    e = torch.empty(0, 256, device="cuda")
    assert B.bdr_quantize_dequantize(B.MX6, e).shape == (0, 256)
    planes = B.bdr_quantize(B.MX6, e)
    assert all(p.numel() == 0 for p in planes)


def test_idempotent_on_gpu():
    x = S.tiny(256, 256, device="cuda")
    for f in (B.MX9, B.MX6, B.MX4):
        y = B.bdr_quantize_dequantize(f, x)
        y2 = B.bdr_quantize_dequantize(f, y)
        assert torch.equal(y.view(torch.int32), y2.view(torch.int32))


def test_bandwidth_config_full_size_sampled_rows():
    # 2^28 fp32 (1 GiB), heavy-tailed, MX9 / MX6 / MX4: the tensor and launch shapes the bench
    # times.  Blocks never cross rows, so the planes of a band of rows are a contiguous slice of
    # the full planes: the oracle quantizes sampled 64-row bands (first, last, four random ones)
    # and every byte and value of those bands is compared.  Then properties over the whole tensor.
    x = S.bandwidth(device="cuda")
    rows, cols = x.shape
    assert rows * cols == 1 << 28
    rng = np.random.default_rng(1)
    bands = sorted(set([0, rows - 64] + [int(v) * 64 for v in rng.integers(0, rows // 64, 4)]))
    for name in MX:
        f = _fmt(name)
        planes = B.bdr_quantize(f, x)
        y = B.bdr_dequantize(f, planes, rows, cols)
        torch.cuda.synchronize()
        per_row = [cols * (f.m + 1) // 8, cols // 16, cols // 16]
        for r0 in bands:
            sub = x[r0:r0 + 64]
            want = O.quantize(ofmt(f), to_np(sub))
            got = [p[r0 * n:(r0 + 64) * n] for p, n in zip(planes, per_row)]
            assert_planes_equal(got, want, "%s rows %d.." % (name, r0))
            ywant = O.dequantize(ofmt(f), *want, 64, cols)
            assert_bits_equal(y[r0:r0 + 64], ywant, "%s dequantize rows %d.." % (name, r0))
        # whole tensor: the fused round trip gives the same bits as quantize then dequantize,
        # and quantizing the result again changes nothing
        y2 = B.bdr_quantize_dequantize(f, x)
        assert torch.equal(y2.view(torch.int32), y.view(torch.int32)), name
        del y2
        p2 = B.bdr_quantize(f, y)
        assert all(torch.equal(a, b) for a, b in zip(planes, p2)), name
        # error bound of Sec. IX per element, wherever the magnitude did not saturate:
        # |x - Q(x)| <= 2^(E - tau - m) <= 2^(E - m), E = exponent of the block maximum
        se = planes[1].view(rows, cols // 16).to(torch.float32)
        bound = torch.exp2(se - 127 - f.m).repeat_interleave(16, dim=1)
        sat = y.abs() >= (2.0 - 2.0 ** (1 - f.m)) * torch.exp2(se - 127).repeat_interleave(16, dim=1)
        assert torch.all(((x - y).abs() <= bound) | sat), name
        del planes, y, p2, se, bound, sat


def test_activation_config_full_size_sampled_rows():
    # 8192 x 12288 bf16 with channel outliers, the activation-shaped bench configuration, along
    # rows (the forward operand layout, Sec. V): MX9 / MX6 / MX4 through the BF16 row kernels at
    # the launch shape the bench times.  The oracle quantizes sampled 64-row bands (first, last,
    # four random ones); every byte of their planes and every dequantized BF16 value is compared.
    x = S.activation(device="cuda")
    rows, cols = x.shape
    assert (rows, cols) == (8192, 12288) and x.dtype == torch.bfloat16
    rng = np.random.default_rng(2)
    bands = sorted(set([0, rows - 64] + [int(v) * 64 for v in rng.integers(0, rows // 64, 4)]))
    for name in MX:
        f = _fmt(name)
        planes = B.bdr_quantize(f, x)
        y = B.bdr_dequantize(f, planes, rows, cols, dtype=torch.bfloat16)
        y2 = B.bdr_quantize_dequantize(f, x)
        torch.cuda.synchronize()
        per_row = [cols * (f.m + 1) // 8, cols // 16, cols // 16]
        for r0 in bands:
            want = O.quantize(ofmt(f), to_np(x[r0:r0 + 64]))
            got = [p[r0 * n:(r0 + 64) * n] for p, n in zip(planes, per_row)]
            assert_planes_equal(got, want, "%s bf16 rows %d.." % (name, r0))
            ywant = O.dequantize(ofmt(f), *want, 64, cols, out_dtype=np.uint16)
            assert_bits_equal(y[r0:r0 + 64], ywant, "%s bf16 dequantize rows %d.." % (name, r0))
            assert_bits_equal(y2[r0:r0 + 64], ywant, "%s bf16 fused rows %d.." % (name, r0))
        # whole tensor: fused = quantize then dequantize, and the result is a fixed point
        assert torch.equal(y2.view(torch.int16), y.view(torch.int16)), name
        p2 = B.bdr_quantize(f, y)
        assert all(torch.equal(a, b) for a, b in zip(planes, p2)), name
        del planes, y, y2, p2


@pytest.mark.parametrize("kw", [dict(k1=32, k2=2, d2=1, m=4), dict(k1=64, k2=64, d2=1, m=2),
                                dict(k1=8, k2=1, d2=1, m=4), dict(k1=16, k2=16, d2=0, m=4)],
                         ids=lambda kw: "-".join("%s%d" % kv for kv in kw.items()))
def test_design_space_formats_on_the_activation_tensor_sampled_rows(kw):
    # BF16 8192 x 12288 through the kernels compiled for the tuple (quantize, dequantize, fused),
    # at full size: sampled 64-row bands against the oracle, the rest through identities
    f = B.fmt(**kw)
    x = S.activation(device="cuda")
    rows, cols = x.shape
    rng = np.random.default_rng(5)
    bands = sorted(set([0, rows - 64] + [int(v) * 64 for v in rng.integers(0, rows // 64, 3)]))
    planes = B.bdr_quantize(f, x)
    y = B.bdr_dequantize(f, planes, rows, cols, dtype=torch.bfloat16)
    y2 = B.bdr_quantize_dequantize(f, x)
    torch.cuda.synchronize()
    sizes = B.bdr_packed_sizes(f, rows, cols)
    per_row = [n // rows for n in sizes]
    for r0 in bands:
        want = O.quantize(ofmt(f), to_np(x[r0:r0 + 64]))
        got = [p[r0 * n:(r0 + 64) * n] for p, n in zip(planes, per_row)]
        assert_planes_equal(got, want, "%r rows %d.." % (f, r0))
        ywant = O.dequantize(ofmt(f), *want, 64, cols, out_dtype=np.uint16)
        assert_bits_equal(y[r0:r0 + 64], ywant, "%r dequantize rows %d.." % (f, r0))
        assert_bits_equal(y2[r0:r0 + 64], ywant, "%r fused rows %d.." % (f, r0))
    assert torch.equal(y2.view(torch.int16), y.view(torch.int16))
    p2 = B.bdr_quantize(f, y)
    assert all(torch.equal(a, b) for a, b in zip(planes, p2))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_rows_with_a_short_last_block_at_a_large_size(dtype):
    # 4099 x 12295: neither axis a multiple of anything; sampled rows against the oracle
    rows, cols = 4099, 12295
    x = S.wide_range(rows, cols, device="cuda", seed=91, spread=5, dtype=dtype)
    pick = np.array([0, 1, 63, 64, 2048, 4097, 4098])
    out_dtype = np.float32 if dtype == torch.float32 else np.uint16
    for f in (B.MX9, B.fmt(32, 4, 1, 4), B.fmt(128, 2, 2, 3, rounding=B.RNA)):
        planes = B.bdr_quantize(f, x)
        y = B.bdr_dequantize(f, planes, rows, cols, dtype=dtype)
        y2 = B.bdr_quantize_dequantize(f, x)
        torch.cuda.synchronize()
        per_row = [n // rows for n in B.bdr_packed_sizes(f, rows, cols)]
        for r in pick:
            want = O.quantize(ofmt(f), np.ascontiguousarray(to_np(x[r:r + 1])))
            got = [p[r * n:(r + 1) * n] for p, n in zip(planes, per_row)]
            assert_planes_equal(got, want, "%r row %d" % (f, r))
            ywant = O.dequantize(ofmt(f), *want, 1, cols, out_dtype=out_dtype)
            assert_bits_equal(y[r:r + 1], ywant, "%r dequantize row %d" % (f, r))
        assert torch.equal(y.view(torch.int32 if dtype == torch.float32 else torch.int16),
                           y2.view(torch.int32 if dtype == torch.float32 else torch.int16))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_more_than_four_gibi_elements(dtype):
    # 2^32 + 2^18 elements: every element index, byte offset and plane offset passes 2^32.
    # Row bands around the 2^31 and 2^32 element marks and at both ends go through the oracle.
    cols = 4096
    rows = (1 << 20) + 64
    g = torch.Generator(device="cuda").manual_seed(77)
    x = torch.empty(rows, cols, dtype=dtype, device="cuda")
    step = 1 << 16
    for r in range(0, rows, step):                       # filled in pieces to bound temporaries
        n = min(step, rows - r)
        x[r:r + n] = (torch.randn(n, cols, generator=g, device="cuda") * 0.3).to(dtype)
    f = B.MX6
    planes = B.bdr_quantize(f, x)
    y = B.bdr_dequantize(f, planes, rows, cols, dtype=dtype)
    y2 = B.bdr_quantize_dequantize(f, x)
    torch.cuda.synchronize()
    per_row = [cols * 5 // 8, cols // 16, cols // 16]
    out_dtype = np.float32 if dtype == torch.float32 else np.uint16
    for r0 in (0, (1 << 19) - 8, (1 << 20) - 8, rows - 16):
        sub = x[r0:r0 + 16]
        want = O.quantize(ofmt(f), to_np(sub))
        got = [p[r0 * n:(r0 + 16) * n] for p, n in zip(planes, per_row)]
        assert_planes_equal(got, want, "rows %d.." % r0)
        ywant = O.dequantize(ofmt(f), *want, 16, cols, out_dtype=out_dtype)
        assert_bits_equal(y[r0:r0 + 16], ywant, "dequantize rows %d.." % r0)
        assert_bits_equal(y2[r0:r0 + 16], ywant, "fused rows %d.." % r0)
    itype = torch.int32 if dtype == torch.float32 else torch.int16
    assert torch.equal(y.view(itype), y2.view(itype))


def test_work_goes_to_the_callers_stream():
    # the library enqueues on the stream it is handed and never synchronizes: work issued on a
    # side stream behind a long-running kernel must not have run before that stream is waited for
    f = B.MX6
    x = S.tiny(device="cuda")
    want = O.quantize(ofmt(f), to_np(x))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    big = torch.empty(1 << 28, device="cuda")
    with torch.cuda.stream(side):
        for _ in range(20):
            big.normal_()                                 # keeps the side stream busy for a while
        planes = B.bdr_quantize(f, x)
        y = B.bdr_dequantize(f, planes, *x.shape)
    side.synchronize()
    assert_planes_equal(planes, want, "side stream")
    assert_bits_equal(y, O.dequantize(ofmt(f), *want, *x.shape), "side stream dequantize")
