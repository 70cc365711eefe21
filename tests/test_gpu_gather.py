"""GPU parity of gather + dequantize from an MX-packed table: every gathered row must equal,
bit for bit, that row of the oracle's dequantization of the whole table."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2302_08007_amd as B
import synth_inputs as S
from gpu_util import assert_bits_equal, ofmt, to_np

pytestmark = pytest.mark.gpu
MX = ["MX9", "MX6", "MX4"]


def _table(rows, cols, seed):
    x = S.wide_range(rows, cols, device="cuda", seed=seed, spread=6)
    return x


@pytest.mark.parametrize("name", MX)
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("shape", [(50, 32, 7), (1000, 128, 513), (300, 416, 1031)])
def test_gather_rows(name, dtype, shape):
    rows, cols, n = shape
    f = getattr(B, name)
    x = _table(rows, cols, rows + cols)
    planes = B.bdr_quantize(f, x)
    g = torch.Generator(device="cuda").manual_seed(n)
    idx = torch.randint(0, rows, (n,), generator=g, device="cuda", dtype=torch.int64)
    idx[0], idx[-1] = rows - 1, 0                      # both ends of the table, and repeats
    if n > 4:
        idx[2] = idx[1]
    y = B.bdr_gather_dequantize(f, planes, rows, cols, idx, dtype=dtype)
    torch.cuda.synchronize()
    pn = [p.cpu().numpy() for p in planes]
    out_dtype = np.float32 if dtype == torch.float32 else np.uint16
    full = O.dequantize(ofmt(f), *pn, rows, cols, out_dtype=out_dtype)
    assert_bits_equal(y, full[idx.cpu().numpy()], "%s %s %s" % (name, dtype, shape))


def test_out_of_range_indices_give_zero_rows_and_nothing_else_is_touched():
    rows, cols = 64, 128
    f = B.MX6
    x = _table(rows, cols, 3)
    planes = B.bdr_quantize(f, x)
    idx = torch.tensor([5, -1, rows, 2 ** 40, 7, -(2 ** 50)], device="cuda", dtype=torch.int64)
    buf = torch.full((idx.numel() + 2, cols), 7.0, device="cuda")
    B.bdr_gather_dequantize(f, planes, rows, cols, idx, out=buf[1:-1])
    torch.cuda.synchronize()
    full = O.dequantize(ofmt(f), *[p.cpu().numpy() for p in planes], rows, cols)
    want = np.zeros((idx.numel(), cols), np.float32)
    want[0], want[4] = full[5], full[7]
    assert_bits_equal(buf[1:-1], want, "out of range")
    assert torch.all(buf[0] == 7.0) and torch.all(buf[-1] == 7.0)


@pytest.mark.parametrize("rounding", [B.RNA, B.RTZ])
def test_tables_rounded_another_way(rounding):
    # a lookup only decodes: a table quantized with ties-away or truncation is read like any
    # other, by the same kernels (the rounding rule is not part of the stored image)
    rows, cols = 200, 96
    f = B.fmt(16, 2, 1, 4, rounding=rounding)
    x = _table(rows, cols, 17)
    planes = B.bdr_quantize(f, x)
    idx = torch.randint(0, rows, (333,), device="cuda", dtype=torch.int64,
                        generator=torch.Generator(device="cuda").manual_seed(5))
    y = B.bdr_gather_dequantize(f, planes, rows, cols, idx)
    full = O.dequantize(ofmt(f), *[p.cpu().numpy() for p in planes], rows, cols)
    assert_bits_equal(y, full[idx.cpu().numpy()], "rounding %d" % rounding)
    # the planes themselves are the oracle's for that rounding rule, and differ from nearest-even
    want = O.quantize(ofmt(f), to_np(x))
    assert all(np.array_equal(p.cpu().numpy(), w) for p, w in zip(planes, want))
    if rounding == B.RTZ:       # ties-away differs from ties-to-even only on exact ties
        assert not torch.equal(planes[0], B.bdr_quantize(B.MX6, x)[0])
    # the row-wise dequantize of such an image takes the same path
    assert_bits_equal(B.bdr_dequantize(f, planes, rows, cols), full, "dequantize")


def test_identity_gather_equals_dequantize_and_empty():
    rows, cols = 256, 256
    f = B.MX9
    x = _table(rows, cols, 11)
    planes = B.bdr_quantize(f, x)
    idx = torch.arange(rows, device="cuda", dtype=torch.int64)
    y = B.bdr_gather_dequantize(f, planes, rows, cols, idx)
    assert torch.equal(y.view(torch.int32), B.bdr_dequantize(f, planes, rows, cols).view(torch.int32))
    e = B.bdr_gather_dequantize(f, planes, rows, cols, idx[:0])
    assert e.shape == (0, cols)


def test_embedding_table_shape_sampled():
    # a recommendation-model sized table: 2^20 rows x 128, MX6, 2^20 random lookups; the oracle
    # dequantizes the sampled source rows only (rows are independent: their planes are slices)
    rows, cols, n = 1 << 20, 128, 1 << 20
    f = B.MX6
    g = torch.Generator(device="cuda").manual_seed(12)
    x = torch.randn(rows, cols, generator=g, device="cuda") * 0.05
    planes = B.bdr_quantize(f, x)
    idx = torch.randint(0, rows, (n,), generator=g, device="cuda", dtype=torch.int64)
    y = B.bdr_gather_dequantize(f, planes, rows, cols, idx)
    torch.cuda.synchronize()
    pick = np.random.default_rng(0).choice(n, 512, replace=False)
    src = idx.cpu().numpy()[pick]
    per_row = [cols * 5 // 8, cols // 16, cols // 16]
    pn = [p.cpu().numpy() for p in planes]
    sub = [np.concatenate([p[r * k:(r + 1) * k] for r in src]) for p, k in zip(pn, per_row)]
    want = O.dequantize(ofmt(f), *sub, len(src), cols)
    assert_bits_equal(y[torch.as_tensor(pick, device="cuda")], want, "sampled lookups")


def _rows_together(f, planes, rows, cols):
    """The table image written out from the oracle-checked planes: per row, its run of each
    plane, one after the other (pure byte movement)."""
    cb = cols // 8 * (f.m + 1)
    c, s, m = (p.cpu().numpy() for p in planes)
    return np.concatenate([c.reshape(rows, cb), s.reshape(rows, cols // 16), m.reshape(rows, cols // 16)],
                          axis=1).reshape(-1)


@pytest.mark.parametrize("name", MX)
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("shape", [(50, 64, 7), (1000, 128, 513), (300, 448, 1031), (3, 2048, 100)])
def test_tables_that_keep_a_row_together(name, dtype, shape):
    rows, cols, n = shape
    f = getattr(B, name)
    x = _table(rows, cols, rows + cols)
    want = O.quantize(ofmt(f), to_np(x))
    planes = B.bdr_quantize(f, x)
    assert all(np.array_equal(p.cpu().numpy(), w) for p, w in zip(planes, want))
    table = B.bdr_table_pack(f, planes, rows, cols)
    torch.cuda.synchronize()
    assert B.bdr_table_row_bytes(f, cols) * rows == table.numel() == sum(w.size for w in want)
    assert np.array_equal(table.cpu().numpy(), _rows_together(f, planes, rows, cols))
    g = torch.Generator(device="cuda").manual_seed(n)
    idx = torch.randint(0, rows, (n,), generator=g, device="cuda", dtype=torch.int64)
    idx[0], idx[-1] = rows - 1, 0
    idx[1] = -3                                            # outside the table: a row of +0
    y = B.bdr_table_gather_dequantize(f, table, rows, cols, idx, dtype=dtype)
    torch.cuda.synchronize()
    out_dtype = np.float32 if dtype == torch.float32 else np.uint16
    full = O.dequantize(ofmt(f), *want, rows, cols, out_dtype=out_dtype)
    ref = full[idx.cpu().numpy().clip(0, rows - 1)]
    ref[1] = 0
    assert_bits_equal(y, ref, "%s %s %s" % (name, dtype, shape))
    # the same rows as the three-plane lookup gives
    assert torch.equal(y, B.bdr_gather_dequantize(f, planes, rows, cols, idx, dtype=dtype))


def test_table_image_full_size_sampled():
    """The bench's table (2^20 rows of 128, MX6): sampled rows of the image and of the lookup."""
    rows, cols, f = 1 << 20, 128, B.MX6
    x = S.wide_range(rows, cols, device="cuda", seed=41, spread=4)
    planes = B.bdr_quantize(f, x)
    table = B.bdr_table_pack(f, planes, rows, cols)
    idx = torch.randint(0, rows, (1 << 20,), device="cuda", dtype=torch.int64,
                        generator=torch.Generator(device="cuda").manual_seed(9))
    y = B.bdr_table_gather_dequantize(f, table, rows, cols, idx)
    torch.cuda.synchronize()
    rb = B.bdr_table_row_bytes(f, cols)
    pick = np.concatenate([[0, 1, (1 << 20) - 1], np.random.default_rng(4).integers(0, 1 << 20, 400)])
    ii = idx[pick].cpu().numpy()
    xs = np.ascontiguousarray(to_np(x[torch.from_numpy(ii).cuda()]))
    want = O.quantize(ofmt(f), xs)
    got = table.view(rows, rb)[torch.from_numpy(ii).cuda()].cpu().numpy()
    exp = np.concatenate([want[0].reshape(len(ii), -1), want[1].reshape(len(ii), -1),
                          want[2].reshape(len(ii), -1)], axis=1)
    assert np.array_equal(got, exp)
    assert_bits_equal(y[torch.from_numpy(pick).cuda()], O.dequantize(ofmt(f), *want, len(ii), cols), "sampled lookups")

