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
        if f is FP32_BACKWARD:
            # quantization-aware fine-tuning (Sec. VI, "Inferencing with the MX data format"): the
            # forward pass is the MX one, the backward pass is not quantized at all, so it is the
            # framework's own matrix product on the unquantized tensors
            if ctx.needs_input_grad[0]:
                gx = (g.float() @ w.float()).to(x.dtype)
            if ctx.needs_input_grad[1]:
                gw = (g.float().t() @ x.float()).to(w.dtype)
            return gx, gw, None, None
        if ctx.needs_input_grad[0]:
            gx = _mx_matmul(f, f, g, AXIS_ROW, w, AXIS_COL, T, I, O, x.dtype)
        if ctx.needs_input_grad[1]:
            gw = _mx_matmul(f, f, g, AXIS_COL, x, AXIS_COL, O, I, T, w.dtype)
        return gx, gw, None, None


FP32_BACKWARD = object()   # as fmt_bwd: leave the backward pass unquantized


def mx_linear(x, w, fmt_fwd, fmt_bwd=None):
    """y = x w^T with the forward, backward-data and backward-weight products all computed on
    MX-quantized operands (formats of Table II: MX9, MX6 or MX4).  x [T, I] and w [O, I] are
    contiguous FP32 or BF16 CUDA tensors with T, I and O multiples of 64 (each is the reduction
    length of one of the three products).  fmt_bwd = FP32_BACKWARD keeps the MX forward pass
    and computes both gradients in FP32 on the unquantized tensors (the paper's
    quantization-aware fine-tuning setting)."""
    return _MXLinear.apply(x, w, fmt_fwd, fmt_bwd if fmt_bwd is not None else fmt_fwd)


# ---- inference: direct cast (Sec. V, "Inferencing")
#
# A trained weight matrix is cast to its MX format once; every call then quantizes only the
# activations and multiplies.  Weights and activations may have different formats (the paper's
# generative-inference table pairs them freely); the pair decides the kind of operand image.

def _image_kind(fa, fb):
    if fa.m == 2 and fb.m == 2:
        return OPERAND_FP4
    return OPERAND_FP6 if fa.m <= 4 and fb.m <= 4 else OPERAND_BF16


class MXWeight:
    """w [O, I] cast to `fmt` (a Table II format), blocks along I: the B operand of y = x w^T.
    The operand image is made on first use for each image kind an activation format asks for
    and kept; the weight itself is not referenced again."""

    def __init__(self, w, fmt):
        if w.dim() != 2 or not w.is_cuda or w.dtype not in (torch.float32, torch.bfloat16):
            raise ValueError("w must be a 2-D float32 or bfloat16 CUDA tensor")
        self.fmt, self.shape, self.dtype = fmt, tuple(w.shape), w.dtype
        self._w = w.detach().contiguous()
        self._images = {}

    def image(self, kind):
        img = self._images.get(kind)
        if img is None:
            O, I = self.shape
            if mx_operand_bytes(self.fmt, O, I, kind) == 0:
                raise ValueError("weight of shape %s in this format has no operand image of kind %d "
                                 "(I must be a multiple of 64; of 128 for an MX4 x MX4 product)" % (self.shape, kind))
            img = bdr_quantize_operand(self.fmt, self._w, axis=AXIS_ROW, image=kind, b_operand=True)
            self._images[kind] = img
        return img

    def drop_source(self):
        """Forget the unquantized weight (images made so far stay)."""
        self._w = None


def mx_linear_inference(x, weight, act_fmt, out_dtype=None):
    """y [T, O] = Q_act(x) Q_w(w)^T for x [T, I] (contiguous FP32 or BF16 CUDA tensor, I as the
    weight's) and an MXWeight: the activations are quantized straight into the operand image,
    the weight's image is reused.  FP4 images and products when both formats are MX4 and I is a
    multiple of 128, FP6 when both have m <= 4, BF16 otherwise."""
    T, I = x.shape
    O, I2 = weight.shape
    if I != I2:
        raise ValueError("x [T, %d] against w [O, %d]" % (I, I2))
    kind = _image_kind(act_fmt, weight.fmt)
    if kind == OPERAND_FP4 and I % 128:
        kind = OPERAND_FP6
    na = mx_operand_bytes(act_fmt, T, I, kind)
    if na == 0 or not _direct(act_fmt, x, AXIS_ROW, T, I, kind):
        raise ValueError("activations of shape %s cannot be quantized into an operand image (I a multiple "
                         "of 64, rows 16-byte aligned)" % (tuple(x.shape),))
    ib = weight.image(kind)
    ia = bdr_quantize_operand(act_fmt, x, axis=AXIS_ROW, image=kind, b_operand=False, out=_workspace(x.device, na)[:na])
    return mx_gemm_operands(act_fmt, weight.fmt, ia, ib, T, O, I, image=kind, dtype=out_dtype or x.dtype)
