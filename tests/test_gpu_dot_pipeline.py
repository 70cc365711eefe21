"""GPU parity of mx_dot_pipeline (bit-true model of the dot-product pipeline of Sec. IV-B) against
the oracle's model of the same readings: an integer pipeline, so every entry must agree bit for
bit (results are kept inside the FP32 normal range)."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2302_08007_amd as B
import synth_inputs as S
from gpu_util import ofmt

pytestmark = pytest.mark.gpu


def _planes_np(planes):
    return [p.cpu().numpy() for p in planes]


def _operands(M, N, K, seed, spread):
    """Gaussian rows whose blocks sit at exponents spread over 2 * spread binades."""
    g = torch.Generator(device="cuda").manual_seed(seed)
    out = []
    for rows in (M, N):
        x = torch.randn(rows, K, generator=g, device="cuda")
        e = torch.randint(-spread, spread + 1, (rows, K // 16), generator=g, device="cuda")
        x = x * torch.exp2(e.float()).repeat_interleave(16, dim=1)
        x[torch.rand(rows, K, generator=g, device="cuda") < 0.03] = 0.0
        out.append(x.contiguous())
    return out


def _check(fa, fb, A, Bm, r, f_bits, what):
    M, K = A.shape
    N = Bm.shape[0]
    pa, pb = B.bdr_quantize(fa, A), B.bdr_quantize(fb, Bm)
    C = B.mx_dot_pipeline(fa, fb, pa, pb, M, N, K, r=r, f_bits=f_bits)
    torch.cuda.synchronize()
    want = O.dot_pipeline(ofmt(fa), ofmt(fb), _planes_np(pa), _planes_np(pb), M, N, K, r=r, f_bits=f_bits)
    got = C.cpu().numpy()
    if not np.array_equal(got.view(np.uint32), want.view(np.uint32)):
        bad = np.argwhere(got.view(np.uint32) != want.view(np.uint32))
        i, j = bad[0]
        raise AssertionError("%s: %d of %d entries differ, first at (%d, %d): got %r want %r"
                             % (what, len(bad), got.size, i, j, got[i, j], want[i, j]))
    return C, pa, pb


@pytest.mark.parametrize("names", [("MX9", "MX9"), ("MX6", "MX6"), ("MX4", "MX4"), ("MX9", "MX4"), ("MX6", "MX9")])
@pytest.mark.parametrize("shape,r", [((64, 128, 64), 64), ((128, 256, 256), 64), ((128, 128, 256), 256),
                                     ((64, 256, 1280), 128)])
def test_entries_equal_the_oracle(names, shape, r):
    M, N, K = shape
    fa, fb = getattr(B, names[0]), getattr(B, names[1])
    A, Bm = _operands(M, N, K, M + N + K, spread=6)
    _check(fa, fb, A, Bm, r, 25, "%s %s r=%d" % (names, shape, r))


@pytest.mark.parametrize("f_bits", [2, 5, 9, 12, 17, 20, 26])
def test_word_widths(f_bits):
    # from a word that keeps one magnitude bit of the largest block to one with room to spare;
    # wide exponent spread, so that many blocks fall partly or wholly below the word
    A, Bm = _operands(64, 128, 512, 100 + f_bits, spread=14)
    for fa, fb in ((B.MX6, B.MX6), (B.MX9, B.MX9), (B.MX4, B.MX6)):
        _check(fa, fb, A, Bm, 128, f_bits, "f=%d" % f_bits)


@pytest.mark.parametrize("shape", [(1, 1, 64), (70, 130, 128), (33, 257, 192), (200, 64, 64)])
def test_edges_of_c_and_pitched_output(shape):
    M, N, K = shape
    A, Bm = _operands(M, N, K, 7 * M + N, spread=4)
    C, pa, pb = _check(B.MX6, B.MX9, A, Bm, 64, 25, str(shape))
    big = torch.full((M + 2, N + 3), 7.0, device="cuda")
    B.mx_dot_pipeline(B.MX6, B.MX9, pa, pb, M, N, K, r=64, out=big[:M, :N])
    assert torch.equal(big[:M, :N], C) and torch.all(big[M:] == 7.0) and torch.all(big[:, N:] == 7.0)


def test_exact_when_nothing_is_dropped_and_close_to_the_fp32_path_otherwise():
    # operands whose blocks all share one exponent: every block result is aligned without a
    # shift, the word (f = 25) holds every bit, and one pass equals the FP64 product rounded once
    g = torch.Generator(device="cuda").manual_seed(3)
    M, N, K = 128, 128, 512
    A = torch.randn(M, K, generator=g, device="cuda").clamp(-3, 3)
    Bm = torch.randn(N, K, generator=g, device="cuda").clamp(-3, 3)
    A[:, ::16] = 3.5
    Bm[:, ::16] = -3.5                                  # every block's maximum is in [2, 4)
    f = B.MX6
    pa, pb = B.bdr_quantize(f, A), B.bdr_quantize(f, Bm)
    assert int(pa[1].min()) == int(pa[1].max()) == 128
    Ah, Bh = B.bdr_dequantize(f, pa, M, K).double(), B.bdr_dequantize(f, pb, N, K).double()
    C = B.mx_dot_pipeline(f, f, pa, pb, M, N, K)
    assert torch.equal(C, (Ah @ Bh.t()).float())
    # general data: the pipeline and the FP32-accumulating product agree to FP32 accuracy
    A, Bm = S.gemm_operands(256, 256, 1024, device="cuda", seed=9)
    pa, pb = B.bdr_quantize(f, A), B.bdr_quantize(f, Bm)
    C1 = B.mx_dot_pipeline(f, f, pa, pb, 256, 256, 1024, r=64)
    C2 = B.mx_gemm(f, f, pa, pb, 256, 256, 1024)
    assert ((C1 - C2).abs() <= 1e-4 * C2.abs().max()).all()


@pytest.mark.parametrize("names,r", [(("MX6", "MX6"), 64), (("MX9", "MX9"), 8192), (("MX6", "MX6"), 8192)])
def test_full_size_sampled_entries(names, r):
    # 8192^3 (the GEMM configuration of the bench): 48 x 48 sampled entries against the oracle,
    # with the unit length the paper normalizes its area to (64) and as one pass over all of K
    M = N = K = 8192
    A, Bm = S.gemm_operands(M, N, K, device="cuda")
    fa, fb = getattr(B, names[0]), getattr(B, names[1])
    pa, pb = B.bdr_quantize(fa, A), B.bdr_quantize(fb, Bm)
    C = B.mx_dot_pipeline(fa, fb, pa, pb, M, N, K, r=r, f_bits=25)
    torch.cuda.synchronize()
    rng = np.random.default_rng(6)
    ri = np.sort(np.concatenate([[0, M - 1], rng.choice(M, 46, replace=False)]))
    ci = np.sort(np.concatenate([[0, N - 1], rng.choice(N, 46, replace=False)]))
    ii, jj = [a.reshape(-1) for a in np.meshgrid(ri, ci, indexing="ij")]
    want = O.dot_pipeline_sampled(ofmt(fa), ofmt(fb), _planes_np(pa), _planes_np(pb), M, N, K, ii, jj,
                                  r=r, f_bits=25)
    got = C[torch.as_tensor(ii, device="cuda"), torch.as_tensor(jj, device="cuda")].cpu().numpy()
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_argument_checks_on_the_device():
    f = B.MX6
    A, Bm = _operands(64, 128, 128, 1, 2)
    pa, pb = B.bdr_quantize(f, A), B.bdr_quantize(f, Bm)
    for kw in (dict(r=32), dict(r=96), dict(f_bits=1), dict(f_bits=27)):
        with pytest.raises(B.BdrError) as e:
            B.mx_dot_pipeline(f, f, pa, pb, 64, 128, 128, **kw)
        assert e.value.status == 3
    with pytest.raises(ValueError):
        B.mx_dot_pipeline(f, f, pa, pb, 64, 128, 128, workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
    with pytest.raises(B.BdrError):
        B.mx_dot_pipeline(f, B.fmt(32, 2, 1, 4), pa, pb, 64, 128, 128)
