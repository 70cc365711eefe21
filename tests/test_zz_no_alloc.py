"""GPU test of the sweep entry point that allocates nothing (static device scratch): it must
give, bit for bit, what bdr_qsnr_sweep gives with a caller's workspace -- on two calls in a row,
the second on a smaller input (so whatever the first call left in the scratch must not matter),
then on a format list longer than one launch holds and on a BF16 tensor.  The C ABI is called
directly (ctypes), not through the package's wrapper."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2302_08007_amd as B
import synth_inputs as S

pytestmark = pytest.mark.gpu


def _raw(fn, fmts, x, workspace=None):
    n = len(fmts)
    arr = (B.Format * n)(*fmts)
    q = torch.full((n,), -1.0, dtype=torch.float64, device="cuda")
    s = torch.full((n + 1,), -1.0, dtype=torch.float64, device="cuda")
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    dt = B.F32 if x.dtype == torch.float32 else B.BF16
    args = [arr, n, ctypes.c_void_p(x.data_ptr()), dt, x.shape[0], x.shape[1], x.stride(0),
            ctypes.c_void_p(q.data_ptr()), ctypes.c_void_p(s.data_ptr())]
    if workspace is not None:
        args += [ctypes.c_void_p(workspace.data_ptr()), workspace.numel()]
    st = fn(*args, stream)
    assert st == B.OK, B.status_string(st)
    torch.cuda.synchronize()
    return q.cpu().numpy(), s.cpu().numpy()


def _both(fmts, x):
    ws = torch.empty(B.lib.bdr_qsnr_sweep_workspace_bytes(len(fmts)), dtype=torch.uint8, device="cuda")
    want = _raw(B.lib.bdr_qsnr_sweep, fmts, x, ws)
    got = _raw(B.lib.bdr_qsnr_sweep_static, fmts, x)
    assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1])
    assert np.all(np.isfinite(got[1])) and np.all(got[1] >= 0)
    return got


def test_static_scratch_sweep_matches_the_workspace_one():
    assert 0 < B.lib.bdr_qsnr_sweep_static_scratch_bytes() <= 1 << 20
    fmts = [B.fmt(k1, k1 if k2 == 0 else k2, d2, m)
            for k1 in (8, 16, 32, 64) for k2 in (1, 2, 4, 0) for d2 in (0, 1) for m in (2, 4)]
    big = S.sweep(1 << 22, device="cuda")            # 768 workgroups, several rounds each
    q1, _ = _both(fmts, big)
    small = S.tiny(24, 128, device="cuda", seed=3)   # fewer workgroups than the first call used
    q2, s2 = _both(fmts[:5] + [B.MX9, B.MX6, B.MX4], small)
    assert not np.array_equal(q1[:5], q2[:5])
    # the wrapper goes the same way
    out = (torch.empty(8, dtype=torch.float64, device="cuda"), torch.empty(9, dtype=torch.float64, device="cuda"))
    B.bdr_qsnr_sweep_static(fmts[:5] + [B.MX9, B.MX6, B.MX4], small, out)
    torch.cuda.synchronize()
    assert np.array_equal(out[0].cpu().numpy(), q2) and np.array_equal(out[1].cpu().numpy(), s2)
    # a list longer than one launch holds reuses the array chunk by chunk; BF16 input
    many = [B.fmt(k1, k2, d2, m, rounding=r) for k1 in (16, 64) for k2 in (1, 2, 8)
            for d2 in (0, 1, 2, 3) for m in range(1, 9) for r in (0, 1)]
    assert len(many) > 256
    _both(many, S.tiny(64, 256, device="cuda", seed=6))
    _both(fmts, S.wide_range(96, 1280, device="cuda", seed=3, spread=5, dtype=torch.bfloat16))
    # an empty tensor: nothing to read, sums are zero
    q0, s0 = _both([B.MX6], torch.empty(0, 64, device="cuda"))
    assert s0[0] == 0.0 and s0[1] == 0.0


def test_static_scratch_sweep_argument_checks():
    L = B.lib
    arr = (B.Format * 1)(B.MX6)
    x = torch.zeros(4, 64, device="cuda")
    q = torch.zeros(1, dtype=torch.float64, device="cuda")
    s = torch.zeros(2, dtype=torch.float64, device="cuda")
    P = ctypes.c_void_p
    call = lambda n=1, xp=x.data_ptr(), cols=64, qp=q.data_ptr(): L.bdr_qsnr_sweep_static(
        arr, n, P(xp), 0, 4, cols, cols, P(qp), P(s.data_ptr()), P(0))
    assert call(n=0) == 3 and call(n=1025) == 3          # BDR_ERR_SHAPE: the stated limit
    assert call(cols=40) == 3
    assert call(xp=0) == 1 and call(qp=0) == 1           # BDR_ERR_NULL
    assert call(xp=x.data_ptr() + 4) == 4                # BDR_ERR_ALIGN
    assert call() == 0
    torch.cuda.synchronize()
