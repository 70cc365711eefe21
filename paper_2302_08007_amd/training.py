"""The MX compute flow of one training iteration for a linear layer (Sec. V, "Training", and
the compute-flow figure there): the three tensor reductions -- forward, backward-data and
backward-weight -- each take BOTH operands MX-quantized along that reduction's own axis.

MX is a directional format, so a tensor that is reduced along different axes in different
passes is quantized once per axis; quantizing and transposing do not commute (Sec. V).  With
x [T, I], w [O, I] and the incoming gradient g [T, O]:

    forward          y[t, o] = sum_i x[t, i] w[o, i]    x, w blocked along I   (both row-wise)
    backward-data   gx[t, i] = sum_o g[t, o] w[o, i]    g row-wise, w column-wise (image of w^T)
    backward-weight gw[o, i] = sum_t g[t, o] x[t, i]    g and x column-wise (images of g^T, x^T)

Column-wise quantization yields the packed image of the transpose directly, which is exactly
the K-contiguous operand mx_gemm takes, so no transpose is ever materialized.  Everything that
touches tensor data runs in the library's kernels (bdr_quantize, mx_gemm); this file only
orders the calls and plugs them into autograd.  Element-wise work stays in the caller's dtype.
"""
import torch

from . import (AXIS_COL, AXIS_ROW, OPERAND_BF16, OPERAND_FP4, OPERAND_FP6, bdr_quantize, bdr_quantize_operand, mx_gemm,
               mx_gemm_operands, mx_gemm_workspace_bytes, mx_operand_bytes)

_workspaces = {}


def _workspace(device, nbytes):
    """One scratch buffer per (device, stream), grown on demand: the GEMMs that share it run one
    after the other on that stream, and work on another stream gets a buffer of its own, so two
    streams never meet in one workspace.  `release_workspaces()` drops them all."""
    key = (device, torch.cuda.current_stream(device).cuda_stream)
    ws = _workspaces.get(key)
    if ws is None or ws.numel() < nbytes:
        ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
        _workspaces[key] = ws
    return ws


def release_workspaces():
    """Forget every cached GEMM workspace (their memory goes back to torch's allocator once the
    work that uses them has run)."""
    _workspaces.clear()


def _mx_matmul(fa, fb, a, a_axis, b, b_axis, M, N, K, out_dtype):
    """C[M, N] = Q(a) Q(b)^T with a, b quantized along the K axis of the product; C comes out in
    out_dtype (FP32 sums; a BF16 C is rounded as the product kernel stores it, not in a pass of
    its own)."""
    image = OPERAND_FP6 if fa.m <= 4 and fb.m <= 4 else OPERAND_BF16
    if fa.m == 2 and fb.m == 2 and _direct(fa, a, a_axis, M, K, OPERAND_FP4) and _direct(fb, b, b_axis, N, K, OPERAND_FP4):
        image = OPERAND_FP4
    if _direct(fa, a, a_axis, M, K, image) and _direct(fb, b, b_axis, N, K, image):
        # the quantizer writes the product kernel's operand images itself (no planes, no rewriting
        # pass): FP4 images for an MX4 pair (K a multiple of 128), FP6 images when both formats have
        # m <= 4, BF16 images when MX9 takes part; the two images share the stream's scratch buffer
        na, nb = mx_operand_bytes(fa, M, K, image), mx_operand_bytes(fb, N, K, image)
        ws = _workspace(a.device, na + nb)
        ia = bdr_quantize_operand(fa, a, axis=a_axis, image=image, b_operand=False, out=ws[:na])
        ib = bdr_quantize_operand(fb, b, axis=b_axis, image=image, b_operand=True, out=ws[na:na + nb])
        return mx_gemm_operands(fa, fb, ia, ib, M, N, K, image=image, dtype=out_dtype)
    pa = bdr_quantize(fa, a, axis=a_axis)
    pb = bdr_quantize(fb, b, axis=b_axis)
    ws = _workspace(a.device, mx_gemm_workspace_bytes(M, N, K))
    return mx_gemm(fa, fb, pa, pb, M, N, K, workspace=ws, dtype=out_dtype)


def _direct(f, t, axis, op_rows, K, image):
    """Whether bdr_quantize_operand takes this operand (format, and whole tiles for column blocks)."""
    if mx_operand_bytes(f, op_rows, K, image) == 0 or t.stride(0) * t.element_size() % 16:
        return False
    if axis == AXIS_ROW:
        return True
    rows, cols = t.shape
    return rows % 128 == 0 and cols % (64 if t.dtype == torch.float32 and image != OPERAND_FP4 else 128) == 0


class _MXLinear(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, w, fmt_fwd, fmt_bwd):
        T, I = x.shape
        O = w.shape[0]
        ctx.save_for_backward(x, w)
        ctx.fmt_bwd = fmt_bwd
        return _mx_matmul(fmt_fwd, fmt_fwd, x, AXIS_ROW, w, AXIS_ROW, T, O, I, x.dtype)

    @staticmethod
    def backward(ctx, g):
        x, w = ctx.saved_tensors
        f = ctx.fmt_bwd
        T, I = x.shape
        O = w.shape[0]
        g = g.contiguous()
        gx = gw = None
        if ctx.needs_input_grad[0]:
            gx = _mx_matmul(f, f, g, AXIS_ROW, w, AXIS_COL, T, I, O, x.dtype)
        if ctx.needs_input_grad[1]:
            gw = _mx_matmul(f, f, g, AXIS_COL, x, AXIS_COL, O, I, T, w.dtype)
        return gx, gw, None, None


def mx_linear(x, w, fmt_fwd, fmt_bwd=None):
    """y = x w^T with the forward, backward-data and backward-weight products all computed on
    MX-quantized operands (formats of Table II: MX9, MX6 or MX4).  x [T, I] and w [O, I] are
    contiguous FP32 or BF16 CUDA tensors with T, I and O multiples of 64 (each is the reduction
    length of one of the three products)."""
    return _MXLinear.apply(x, w, fmt_fwd, fmt_bwd if fmt_bwd is not None else fmt_fwd)
