"""GPU parity of the MX compute flow of a linear layer (forward, backward-data,
backward-weight) against the same flow composed from oracle calls: each operand quantized and
dequantized by the oracle along the reduction axis of its product, products in FP64."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2302_08007_amd as B
from paper_2302_08007_amd.training import FP32_BACKWARD, MXWeight, mx_linear, mx_linear_inference
from gpu_util import ofmt, to_np

pytestmark = pytest.mark.gpu
RTOL = 1e-4


def _qdq(f, a, axis):
    """Oracle quantize -> dequantize of a 2-D array along `axis`, as FP64."""
    if a.dtype == np.uint16:
        out_dtype = np.uint16
    else:
        out_dtype = np.float32
    rows, cols = a.shape
    planes = O.quantize(ofmt(f), a, axis=axis)
    y = O.dequantize(ofmt(f), *planes, rows, cols, axis=axis, out_dtype=out_dtype)
    if out_dtype == np.uint16:
        y = (y.astype(np.uint32) << 16).view(np.float32)
    return y.astype(np.float64)


def _close(got, want, absdot, what):
    err = np.abs(got.astype(np.float64) - want)
    assert np.all(err <= RTOL * absdot + 1e-30), (what, float((err / (absdot + 1e-30)).max()))


@pytest.mark.parametrize("names", [("MX9", "MX9"), ("MX6", "MX9"), ("MX4", "MX6"), ("MX4", "MX4")])
@pytest.mark.parametrize("shape", [(128, 128, 128), (256, 384, 128), (192, 64, 320)])
def test_linear_layer_flow_fp32(names, shape):
    T, I, Osz = shape
    ff, fb = getattr(B, names[0]), getattr(B, names[1])
    g = torch.Generator(device="cuda").manual_seed(T + I + Osz)
    x = torch.randn(T, I, generator=g, device="cuda", requires_grad=True)
    w = (torch.randn(Osz, I, generator=g, device="cuda") / I ** 0.5).requires_grad_()
    gy = torch.randn(T, Osz, generator=g, device="cuda")
    y = mx_linear(x, w, ff, fb)
    y.backward(gy)
    torch.cuda.synchronize()
    xn, wn, gn = to_np(x), to_np(w), to_np(gy)
    # forward: both blocked along I
    xa, wa = _qdq(ff, xn, O.AXIS_ROW), _qdq(ff, wn, O.AXIS_ROW)
    _close(to_np(y), xa @ wa.T, np.abs(xa) @ np.abs(wa).T, "forward")
    # backward-data: reduce over O -> g along its rows, w down its columns
    ga, wc = _qdq(fb, gn, O.AXIS_ROW), _qdq(fb, wn, O.AXIS_COL)
    _close(to_np(x.grad), ga @ wc, np.abs(ga) @ np.abs(wc), "backward-data")
    # backward-weight: reduce over T -> g and x down their columns
    gc, xc = _qdq(fb, gn, O.AXIS_COL), _qdq(fb, xn, O.AXIS_COL)
    _close(to_np(w.grad), gc.T @ xc, np.abs(gc).T @ np.abs(xc), "backward-weight")
    # the two quantized copies of w really differ (quantizing and transposing do not commute)
    assert not np.array_equal(_qdq(fb, wn, O.AXIS_ROW), wc)


def test_linear_layer_flow_bf16():
    T, I, Osz = 128, 256, 128
    f = B.MX9
    g = torch.Generator(device="cuda").manual_seed(9)
    x = torch.randn(T, I, generator=g, device="cuda").to(torch.bfloat16).requires_grad_()
    w = (torch.randn(Osz, I, generator=g, device="cuda") / 16).to(torch.bfloat16).requires_grad_()
    gy = torch.randn(T, Osz, generator=g, device="cuda").to(torch.bfloat16)
    y = mx_linear(x, w, f)
    y.backward(gy)
    torch.cuda.synchronize()
    assert y.dtype == torch.bfloat16 and x.grad.dtype == torch.bfloat16
    xn, wn, gn = to_np(x), to_np(w), to_np(gy)
    xa, wa = _qdq(f, xn, O.AXIS_ROW), _qdq(f, wn, O.AXIS_ROW)
    want = xa @ wa.T
    got = y.detach().float().cpu().numpy().astype(np.float64)
    # the product is rounded once more, to BF16 (8 significant bits), on the way out
    assert np.all(np.abs(got - want) <= 2.0 ** -8 * np.abs(want) + RTOL * (np.abs(xa) @ np.abs(wa).T))
    gc, xc = _qdq(f, gn, O.AXIS_COL), _qdq(f, xn, O.AXIS_COL)
    wantw = gc.T @ xc
    gotw = w.grad.float().cpu().numpy().astype(np.float64)
    assert np.all(np.abs(gotw - wantw) <= 2.0 ** -8 * np.abs(wantw) + RTOL * (np.abs(gc).T @ np.abs(xc)))


def test_two_streams_do_not_share_a_workspace():
    # forward products issued on two streams at once: each stream's GEMMs work in a scratch
    # buffer of their own, and both results equal what one stream alone gives
    from paper_2302_08007_amd import training
    T, I, Osz = 512, 1024, 512
    g = torch.Generator(device="cuda").manual_seed(21)
    xs = [torch.randn(T, I, generator=g, device="cuda") for _ in range(2)]
    ws = [torch.randn(Osz, I, generator=g, device="cuda") / 32 for _ in range(2)]
    want = [mx_linear(x, w, B.MX6) for x, w in zip(xs, ws)]
    torch.cuda.synchronize()
    training.release_workspaces()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    got = [None, None]
    for rep in range(4):
        for k in (0, 1):
            with torch.cuda.stream(streams[k]):
                got[k] = mx_linear(xs[k], ws[k], B.MX6)
    torch.cuda.synchronize()
    keys = list(training._workspaces)
    assert len(keys) == 2 and keys[0] != keys[1]
    assert training._workspaces[keys[0]].data_ptr() != training._workspaces[keys[1]].data_ptr()
    for k in (0, 1):
        assert torch.equal(got[k], want[k])
    training.release_workspaces()
    assert not training._workspaces


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("names", [("MX9", "MX9"), ("MX6", "MX6"), ("MX9", "MX6"), ("MX6", "MX4"), ("MX4", "MX4")])
@pytest.mark.parametrize("shape", [(128, 256, 128), (100, 192, 72), (257, 1024, 384)])
def test_direct_cast_inference(shape, names, dtype):
    """Sec. V, "Inferencing": the weight is cast once, the activations at every call; the result is
    the product of what the oracle's quantize + dequantize make of both, and calling again with
    other activations reuses the weight's image."""
    T, I, Osz = shape
    fa, fw = getattr(B, names[0]), getattr(B, names[1])      # (activations, weights)
    g = torch.Generator(device="cuda").manual_seed(T + 3 * I + Osz)
    w = (torch.randn(Osz, I, generator=g, device="cuda") / I ** 0.5).to(dtype)
    wq = MXWeight(w, fw)
    wn = to_np(w)
    wa = _qdq(fw, wn, O.AXIS_ROW)
    for rep in range(2):
        x = torch.randn(T, I, generator=g, device="cuda").to(dtype)
        y = mx_linear_inference(x, wq, fa, out_dtype=torch.float32)
        torch.cuda.synchronize()
        xa = _qdq(fa, to_np(x), O.AXIS_ROW)
        _close(to_np(y), xa @ wa.T, np.abs(xa) @ np.abs(wa).T, "inference %d" % rep)
        if rep == 0:
            wq.drop_source()
    assert len(wq._images) == 1
    with pytest.raises(ValueError):
        mx_linear_inference(torch.zeros(T, I + 64, device="cuda", dtype=dtype), wq, fa)


def test_fine_tuning_flow_keeps_the_backward_pass_unquantized():
    """Quantization-aware fine-tuning as the paper runs it: MX6 forward (checked against the oracle
    flow), gradients in FP32 on the unquantized tensors."""
    T, I, Osz = 192, 256, 128
    g = torch.Generator(device="cuda").manual_seed(5)
    x = torch.randn(T, I, generator=g, device="cuda", requires_grad=True)
    w = (torch.randn(Osz, I, generator=g, device="cuda") / 16).requires_grad_()
    gy = torch.randn(T, Osz, generator=g, device="cuda")
    y = mx_linear(x, w, B.MX6, FP32_BACKWARD)
    y.backward(gy)
    torch.cuda.synchronize()
    xn, wn, gn = to_np(x), to_np(w), to_np(gy)
    xa, wa = _qdq(B.MX6, xn, O.AXIS_ROW), _qdq(B.MX6, wn, O.AXIS_ROW)
    _close(to_np(y), xa @ wa.T, np.abs(xa) @ np.abs(wa).T, "forward")
    gx, gw = gn.astype(np.float64) @ wn.astype(np.float64), gn.astype(np.float64).T @ xn.astype(np.float64)
    _close(to_np(x.grad), gx, np.abs(gn).astype(np.float64) @ np.abs(wn).astype(np.float64), "backward-data")
    _close(to_np(w.grad), gw, np.abs(gn).astype(np.float64).T @ np.abs(xn).astype(np.float64), "backward-weight")
