"""GPU parity: mx_gemm against the fp64 oracle.  Tolerance: |C - C_ref| <= 1e-4 * sum_k |a b|
(norm-relative, because entries of C can be near zero).  Both forms of the call are checked
against the oracle: the single kernel (no workspace, BF16 in LDS) and the two-pass form
(operands rewritten once in a caller-supplied workspace, as BF16, as block-scaled FP6 when
both formats have m <= 4, or as block-scaled FP4 for MX4 x MX4).  The BF16 forms walk K in the
same order and must agree bit for bit; the FP6 and FP4 forms round the sum at other points and
are held to the tolerance."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2302_08007_amd as B
import synth_inputs as S
from gpu_util import ofmt, to_np

pytestmark = pytest.mark.gpu
RTOL = 1e-4


def _planes_np(planes):
    return [p.cpu().numpy() for p in planes]


def _workspace(M, N, K, extra=0):
    return torch.empty(B.mx_gemm_workspace_bytes(M, N, K) + extra, dtype=torch.uint8, device="cuda")


def _check(fa, fb, A, Bm, what):
    M, K = A.shape
    N = Bm.shape[0]
    pa, pb = B.bdr_quantize(fa, A), B.bdr_quantize(fb, Bm)
    C = B.mx_gemm(fa, fb, pa, pb, M, N, K)
    C2 = B.mx_gemm(fa, fb, pa, pb, M, N, K, workspace=_workspace(M, N, K))
    torch.cuda.synchronize()
    if not _fp6_form(fa, fb, K) and M > 64:
        # the tiled BF16 kernels add the same products in the same order; with M <= 64 the two-pass
        # form streams over B's image instead and splits K over its waves
        assert torch.equal(C, C2), what
    pan, pbn = _planes_np(pa), _planes_np(pb)
    Ah = O.dequantize(ofmt(fa), *pan, M, K).astype(np.float64)
    Bh = O.dequantize(ofmt(fb), *pbn, N, K).astype(np.float64)
    Cref = O.mx_gemm(ofmt(fa), ofmt(fb), pan, pbn, M, N, K)
    assert np.allclose(Cref, Ah @ Bh.T, rtol=1e-6, atol=1e-30)       # the oracle is a plain GEMM
    bound = RTOL * (np.abs(Ah) @ np.abs(Bh).T)
    for form, got in (("single kernel", C), ("two-pass", C2)):
        err = np.abs(got.cpu().numpy().astype(np.float64) - Cref)
        assert np.all(err <= bound + 1e-30), (what, form, float((err / (bound + 1e-30)).max()))
    return C


def _fp6_form(fa, fb, K):
    return fa.m <= 4 and fb.m <= 4


@pytest.mark.parametrize("shape", [(128, 128, 64), (128, 256, 128), (384, 128, 192), (256, 256, 512)])
@pytest.mark.parametrize("names", [("MX6", "MX6"), ("MX9", "MX9"), ("MX4", "MX4"),
                                   ("MX9", "MX4"), ("MX4", "MX6"), ("MX6", "MX9")])
def test_small_full_matrix(shape, names):
    M, N, K = shape
    A, Bm = S.gemm_operands(M, N, K, device="cuda", seed=M + N + K)
    _check(getattr(B, names[0]), getattr(B, names[1]), A, Bm, "%s %s" % (shape, names))


@pytest.mark.parametrize("shape", [(1, 1, 64), (130, 70, 128), (257, 129, 64), (100, 384, 192), (33, 31, 256)])
@pytest.mark.parametrize("names", [("MX6", "MX6"), ("MX9", "MX6")])
def test_c_edges_that_are_not_tile_multiples(shape, names):
    # M and N are free: edge tiles read the last operand row again and store only what lies
    # inside C; the canary columns behind each row of a pitched C stay untouched
    M, N, K = shape
    A, Bm = S.gemm_operands(M, N, K, device="cuda", seed=3 * M + N)
    fa, fb = getattr(B, names[0]), getattr(B, names[1])
    _check(fa, fb, A, Bm, "%s %s" % (shape, names))
    pa, pb = B.bdr_quantize(fa, A), B.bdr_quantize(fb, Bm)
    for ws in (None, _workspace(M, N, K)):
        big = torch.full((M + 3, N + 5), 7.0, device="cuda")
        B.mx_gemm(fa, fb, pa, pb, M, N, K, out=big[:M, :N], workspace=ws)
        assert torch.all(big[M:] == 7.0) and torch.all(big[:, N:] == 7.0)
        assert torch.equal(big[:M, :N], B.mx_gemm(fa, fb, pa, pb, M, N, K, workspace=ws))


def test_exact_on_small_integers():
    # integers below 2^m sharing one exponent are exact in MX: the product is an integer matrix
    g = torch.Generator(device="cuda").manual_seed(5)
    M, N, K = 128, 128, 256
    A = torch.randint(-7, 8, (M, K), generator=g, device="cuda").float()
    Bm = torch.randint(-7, 8, (N, K), generator=g, device="cuda").float()
    A[:, ::16] = 8.0
    Bm[:, ::16] = -8.0
    f = B.MX6
    pa, pb = B.bdr_quantize(f, A), B.bdr_quantize(f, Bm)
    want = (A.double() @ Bm.double().t()).float()
    assert torch.equal(B.mx_gemm(f, f, pa, pb, M, N, K), want)
    assert torch.equal(B.mx_gemm(f, f, pa, pb, M, N, K, workspace=_workspace(M, N, K)), want)


@pytest.mark.parametrize("name", ["MX6", "MX4"])
@pytest.mark.parametrize("side", ["A", "B"])
def test_two_pass_fp6_form_reproduces_every_element(name, side):
    # One operand is 2^s times the identity, so every entry of C is a single product and must
    # equal 2^s times the dequantized element of the other operand, bit for bit: this walks all
    # codes (both signs, every magnitude, both microexponents) through the FP6 rewrite, over
    # block exponents from the lowest code (1, where elements move down one binade) to the top.
    f = getattr(B, name)
    rows, K = 256, 256
    g = torch.Generator(device="cuda").manual_seed(11)
    X = torch.randn(rows, K, generator=g, device="cuda")
    X = X * torch.exp2(torch.randint(-3, 4, X.shape, generator=g, device="cuda").float())
    blk_exp = torch.tensor([-126.0, -125.0, -124.0, -60.0, 0.0, 1.0, 60.0, 90.0], device="cuda")
    pick = torch.randint(0, len(blk_exp), (rows, K // 16), generator=g, device="cuda")
    X = X.view(rows, K // 16, 16)
    X = X / X.abs().amax(dim=2, keepdim=True) * 1.9           # block maxima just below 2
    X = (X * torch.exp2(blk_exp[pick]).unsqueeze(2)).view(rows, K).contiguous()
    X[:, 16:32] = 0.0                                           # and an all-zero block per row
    px = B.bdr_quantize(f, X)
    assert int(px[1].min()) == 1 and int(px[1].max()) >= 127 + 90
    Xh = B.bdr_dequantize(f, px, rows, K)
    # the scale keeps every product an FP32 normal: 2^-130 * 2^40 at the low end, 2^91 * 2^-40 ...
    for s in (40.0, 0.0, -40.0):
        keep = (Xh == 0) | ((Xh.abs() * 2.0 ** s >= 2.0 ** -126) & (Xh.abs() * 2.0 ** s < 2.0 ** 127))
        I = torch.eye(K, device="cuda") * 2.0 ** s
        pi = B.bdr_quantize(f, I)
        assert torch.equal(B.bdr_dequantize(f, pi, K, K), I)
        ws = _workspace(max(rows, K), max(rows, K), K)
        if side == "A":
            C = B.mx_gemm(f, f, px, pi, rows, K, K, workspace=ws)             # Xh * (2^s I)^T
        else:
            C = B.mx_gemm(f, f, pi, px, K, rows, K, workspace=ws).t()         # (2^s I) * Xh^T
        want = Xh * 2.0 ** s
        assert torch.equal(C[keep], want[keep]), (name, side, s)
        assert torch.equal(torch.signbit(C[keep & (Xh != 0)]), torch.signbit(want[keep & (Xh != 0)]))


@pytest.mark.parametrize("shape", [(128, 128, 256), (256, 256, 1024), (384, 130, 320), (200, 517, 832),
                                   (512, 256, 2048), (129, 128, 256), (127, 256, 512), (256, 256, 192),
                                   (256, 128, 128), (128, 384, 384), (256, 256, 640)])
def test_mx4_pair_fp4_form_shapes(shape):
    # MX4 x MX4 with M, N >= 128 and K >= 128 runs on 4-bit images with a scale image beside
    # them: one to sixteen K steps of 128 (fewer and more than the ring's four stages), K padded
    # up to a whole step (320, 832, 192), both tile shapes, edge tiles whose rows run past M or
    # N, and a shape just outside the condition (127 rows), which takes the FP6 form.  Block
    # exponents vary so that the scale bytes matter.
    M, N, K = shape
    A, Bm = S.gemm_operands(M, N, K, device="cuda", seed=M + 7 * N + K)
    g = torch.Generator(device="cuda").manual_seed(K)
    A = A * torch.exp2(torch.randint(-6, 7, (M, K // 16), generator=g, device="cuda").float()).repeat_interleave(16, 1)
    Bm = Bm * torch.exp2(torch.randint(-6, 7, (N, K // 16), generator=g, device="cuda").float()).repeat_interleave(16, 1)
    _check(B.MX4, B.MX4, A.contiguous(), Bm.contiguous(), "fp4 %s" % (shape,))


def test_random_shapes_and_format_pairs():
    # 30 seeded draws of M, N (1 .. 600, so most tiles hang over an edge and both tile shapes
    # occur), K (1 .. 12 steps of 64, fewer and more than the ring's four stages, odd counts
    # that pad the FP4 image) and a format pair: both forms against the oracle
    rng = np.random.default_rng(2302)
    names = ["MX9", "MX6", "MX4"]
    for case in range(30):
        M, N = (int(v) for v in rng.integers(1, 601, 2))
        if case % 5 == 0:
            M, N = 256 * int(rng.integers(1, 3)), 256 * int(rng.integers(1, 3))   # whole 256-tiles
        K = 64 * int(rng.integers(1, 13))
        na, nb = names[int(rng.integers(0, 3))], names[int(rng.integers(0, 3))]
        A, Bm = S.gemm_operands(M, N, K, device="cuda", seed=1000 + case)
        _check(getattr(B, na), getattr(B, nb), A, Bm, "case %d: %s x %s, %d x %d x %d" % (case, na, nb, M, N, K))


@pytest.mark.parametrize("name", ["MX9", "MX6", "MX4"])
@pytest.mark.parametrize("form", ["single kernel", "two-pass"])
def test_bf16_forms_reproduce_every_element_down_to_the_lowest_exponent(name, form):
    # The BF16 forms (single kernel for every format; two-pass for MX9 and mixed pairs) expand an
    # element to BF16.  In a block whose exponent code is small the elements are BF16 subnormals
    # (below 2^-126), which the matrix cores of this chip take as they are: one operand is 2^s
    # times the identity, so every entry of C is a single product and must equal 2^s times the
    # dequantized element of the other operand, bit for bit, for block exponents from code 1 up.
    f = getattr(B, name)
    other = B.MX9                       # keeps the pair on the BF16 path in the two-pass form too
    rows, K = 256, 256
    g = torch.Generator(device="cuda").manual_seed(13)
    X = torch.randn(rows, K, generator=g, device="cuda")
    X = X * torch.exp2(torch.randint(-3, 4, X.shape, generator=g, device="cuda").float())
    blk_exp = torch.tensor([-126.0, -125.0, -124.0, -122.0, -119.0, -60.0, 0.0, 60.0], device="cuda")
    pick = torch.randint(0, len(blk_exp), (rows, K // 16), generator=g, device="cuda")
    X = X.view(rows, K // 16, 16)
    X = X / X.abs().amax(dim=2, keepdim=True) * 1.9
    X = (X * torch.exp2(blk_exp[pick]).unsqueeze(2)).view(rows, K).contiguous()
    X[:, 16:32] = 0.0
    px = B.bdr_quantize(f, X)
    assert int(px[1].min()) == 1 and int(px[1].max()) >= 127 + 60
    Xh = B.bdr_dequantize(f, px, rows, K)
    assert int(((Xh != 0) & (Xh.abs() < 2.0 ** -126)).sum()) > 1000     # BF16 subnormals are there
    for s in (40.0, 0.0, -40.0):
        keep = (Xh == 0) | ((Xh.abs() * 2.0 ** s >= 2.0 ** -126) & (Xh.abs() * 2.0 ** s < 2.0 ** 127))
        I = torch.eye(K, device="cuda") * 2.0 ** s
        pi = B.bdr_quantize(other, I)
        ws = _workspace(max(rows, K), max(rows, K), K) if form == "two-pass" else None
        for side in ("A", "B"):
            if side == "A":
                C = B.mx_gemm(f, other, px, pi, rows, K, K, workspace=ws)
            else:
                C = B.mx_gemm(other, f, pi, px, K, rows, K, workspace=ws).t()
            want = Xh * 2.0 ** s
            assert torch.equal(C[keep], want[keep]), (name, form, side, s)
            nz = keep & (Xh != 0)
            assert torch.equal(torch.signbit(C[nz]), torch.signbit(want[nz]))


@pytest.mark.parametrize("ws", [False, True])
def test_operands_rounded_another_way_decode_the_same(ws):
    # reading a packed image never depends on the rounding rule it was made with: images
    # quantized with ties-away or truncation multiply like any other (Sec. III: the rule is
    # part of the quantizer, not of the stored format)
    M, N, K = 128, 256, 128
    A, Bm = S.gemm_operands(M, N, K, device="cuda", seed=77)
    for fa, fb in ((B.fmt(16, 2, 1, 4, rounding=B.RNA), B.fmt(16, 2, 1, 7, rounding=B.RTZ)),
                   (B.fmt(16, 2, 1, 2, rounding=B.RTZ), B.fmt(16, 2, 1, 4, rounding=B.RNA))):
        pa, pb = B.bdr_quantize(fa, A), B.bdr_quantize(fb, Bm)
        w = _workspace(M, N, K) if ws else None
        C = B.mx_gemm(fa, fb, pa, pb, M, N, K, workspace=w)
        torch.cuda.synchronize()
        pan, pbn = _planes_np(pa), _planes_np(pb)
        Cref = O.mx_gemm(ofmt(fa), ofmt(fb), pan, pbn, M, N, K)
        Ah = O.dequantize(ofmt(fa), *pan, M, K).astype(np.float64)
        Bh = O.dequantize(ofmt(fb), *pbn, N, K).astype(np.float64)
        err = np.abs(C.cpu().numpy().astype(np.float64) - Cref)
        assert np.all(err <= RTOL * (np.abs(Ah) @ np.abs(Bh).T) + 1e-30)
        # the same call with the rounding field set to nearest-even gives the same bits
        fa0, fb0 = B.fmt(16, 2, 1, fa.m), B.fmt(16, 2, 1, fb.m)
        assert torch.equal(C, B.mx_gemm(fa0, fb0, pa, pb, M, N, K, workspace=w))


@pytest.mark.parametrize("pair", [
    (dict(k1=16, k2=16, d2=0, m=7), dict(k1=16, k2=16, d2=0, m=7)),     # MSFP16-like block floating point
    (dict(k1=16, k2=16, d2=0, m=3), dict(k1=16, k2=2, d2=1, m=4)),      # MSFP12-like x MX6
    (dict(k1=32, k2=4, d2=1, m=4), dict(k1=64, k2=1, d2=2, m=5, rounding=1)),
    (dict(k1=8, k2=1, d2=1, m=7), dict(k1=128, k2=8, d2=0, m=8)),
], ids=lambda p: "%d-%d-%d-%d" % (p[0]["k1"], p[0]["m"], p[1]["k1"], p[1]["m"]))
def test_formats_outside_table_two(pair):
    # block floating point (d2 = 0, which the paper's design-space study compares against,
    # Sec. IV) and other tuples whose elements BF16 holds exactly: two-pass BF16 form
    fa, fb = B.fmt(**pair[0]), B.fmt(**pair[1])
    M, N, K = 160, 96, 384
    A = S.wide_range(M, K, device="cuda", seed=51, spread=6)
    Bm = S.wide_range(N, K, device="cuda", seed=52, spread=6)
    pa, pb = B.bdr_quantize(fa, A), B.bdr_quantize(fb, Bm)
    C = B.mx_gemm(fa, fb, pa, pb, M, N, K, workspace=_workspace(M, N, K))
    torch.cuda.synchronize()
    pan, pbn = _planes_np(pa), _planes_np(pb)
    Cref = O.mx_gemm(ofmt(fa), ofmt(fb), pan, pbn, M, N, K)
    Ah = O.dequantize(ofmt(fa), *pan, M, K).astype(np.float64)
    Bh = O.dequantize(ofmt(fb), *pbn, N, K).astype(np.float64)
    err = np.abs(C.cpu().numpy().astype(np.float64) - Cref)
    assert np.all(err <= RTOL * (np.abs(Ah) @ np.abs(Bh).T) + 1e-30)
    with pytest.raises(B.BdrError) as e:
        B.mx_gemm(fa, fb, pa, pb, M, N, K)                  # no workspace
    assert e.value.status == 7
    wide = B.fmt(16, 2, 2, 7)                                # 10 significant bits: not BF16-exact
    with pytest.raises(B.BdrError) as e:
        B.mx_gemm(wide, fb, B.bdr_quantize(wide, A), pb, M, N, K, workspace=_workspace(M, N, K))
    assert e.value.status == 2


def test_empty_k_with_many_rows():
    # K = 0 is an empty sum: C is all zeros, also when M is above what one grid axis takes
    M, N = 70000, 24
    C = torch.full((M, N + 8), 5.0, device="cuda")
    f = B.MX6
    e = torch.empty(0, dtype=torch.uint8, device="cuda")
    B.mx_gemm(f, f, (e, e, e), (e, e, e), M, N, 0, out=C[:, :N])
    assert torch.count_nonzero(C[:, :N]) == 0 and torch.all(C[:, N:] == 5.0)


def test_wide_exponent_range_and_signs():
    A = S.wide_range(128, 256, device="cuda", seed=41, spread=8)
    Bm = S.wide_range(256, 256, device="cuda", seed=42, spread=8)
    _check(B.MX6, B.MX9, A, Bm, "wide")


def test_wide_exponent_range_fp6_form():
    # the same mix (16 binades of spread, zeros, negative zeros) through the FP6 form, both roles
    A = S.wide_range(128, 256, device="cuda", seed=43, spread=8)
    Bm = S.wide_range(256, 256, device="cuda", seed=44, spread=8)
    _check(B.MX6, B.MX4, A, Bm, "wide fp6")
    _check(B.MX4, B.MX6, A, Bm, "wide fp6, roles swapped")


def test_strided_output_and_empty_k():
    M, N, K = 128, 128, 64
    A, Bm = S.gemm_operands(M, N, K, device="cuda", seed=8)
    pa, pb = B.bdr_quantize(B.MX6, A), B.bdr_quantize(B.MX6, Bm)
    big = torch.full((M, 2 * N), 3.0, device="cuda")
    B.mx_gemm(B.MX6, B.MX6, pa, pb, M, N, K, out=big[:, :N])
    ref = B.mx_gemm(B.MX6, B.MX6, pa, pb, M, N, K)
    assert torch.equal(big[:, :N], ref) and torch.all(big[:, N:] == 3.0)
    z = B.mx_gemm(B.MX6, B.MX6, pa, pb, M, N, 0)
    assert torch.count_nonzero(z) == 0
    # the same through the two-pass form; the workspace is guarded by a canary behind it
    need = B.mx_gemm_workspace_bytes(M, N, K)
    ws = torch.full((need + 256,), 0x5A, dtype=torch.uint8, device="cuda")
    big2 = torch.full((M, 2 * N), 3.0, device="cuda")
    B.mx_gemm(B.MX6, B.MX6, pa, pb, M, N, K, out=big2[:, :N], workspace=ws)
    ref2 = B.mx_gemm(B.MX6, B.MX6, pa, pb, M, N, K, workspace=ws)
    assert torch.equal(big2[:, :N], ref2) and torch.all(big2[:, N:] == 3.0)
    assert torch.allclose(ref2, ref, rtol=1e-5, atol=1e-5) and torch.all(ws[need:] == 0x5A)
    z = B.mx_gemm(B.MX6, B.MX6, pa, pb, M, N, 0, workspace=ws)
    assert torch.count_nonzero(z) == 0
    with pytest.raises(B.BdrError):
        B.mx_gemm(B.MX6, B.MX6, pa, pb, M, N, K, workspace=ws[:need - 16])


def _two_step_images(fa, fb, pa, pb, M, N, K):
    """The operand images mx_gemm's two-pass form writes into its workspace from the (oracle-checked)
    planes: A's at the start, B's after A's half (an operand's half is rows * K BF16 values,
    rounded up to 256 bytes).  One byte per element for FP6 images (both formats m <= 4), two
    for BF16 images (MX9 takes part)."""
    ws = _workspace(M, N, K)
    C = B.mx_gemm(fa, fb, pa, pb, M, N, K, workspace=ws)
    torch.cuda.synchronize()
    half = (2 * M * K + 255) // 256 * 256
    per = 1 if fa.m <= 4 and fb.m <= 4 else 2
    return ws[:per * M * K].clone(), ws[half:half + per * N * K].clone(), C


def _special(t, top=3.0e38):
    """zeros, -0, subnormals, blocks with the lowest exponent code, large values"""
    t[0, :16] = 0.0
    t[0, 5] = -0.0
    t[1, :32] = 2.0 ** -140
    t[1, 7] = -3 * 2.0 ** -149
    t[2, :16] = 2.0 ** -126
    t[2, 3] = -1.5 * 2.0 ** -126
    t[3, :16] = top
    t[3, 1] = -top / 3
    return t


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("names", [("MX6", "MX6"), ("MX4", "MX6"), ("MX6", "MX4"), ("MX9", "MX9"), ("MX9", "MX4"),
                                   ("MX6", "MX9")])
@pytest.mark.parametrize("shape", [(128, 128, 64), (256, 384, 512), (130, 70, 128), (512, 256, 1024)])
def test_operands_made_by_the_quantizer(shape, names, dtype):
    """bdr_quantize_operand writes, byte for byte, the image that mx_gemm's two-pass form makes of
    the planes bdr_quantize gives (which are the oracle's, bit for bit), for either operand role;
    mx_gemm_operands on two such images returns the same C as that call, and that C is within
    the tolerance of the oracle's product."""
    M, N, K = shape
    fa, fb = getattr(B, names[0]), getattr(B, names[1])
    A, Bm = S.gemm_operands(M, N, K, device="cuda", seed=M + 5 * N + K)
    A, Bm = _special(A, 1.0e15).to(dtype), _special(Bm, 1.0e15).to(dtype)   # (products stay inside FP32)
    pa, pb = B.bdr_quantize(fa, A), B.bdr_quantize(fb, Bm)
    for p, w in zip(pa, O.quantize(ofmt(fa), to_np(A))):
        assert np.array_equal(p.cpu().numpy(), w)
    ia, ib, C2 = _two_step_images(fa, fb, pa, pb, M, N, K)
    image = B.OPERAND_FP6 if fa.m <= 4 and fb.m <= 4 else B.OPERAND_BF16     # (with MX9: BF16 images)
    ga = B.bdr_quantize_operand(fa, A, image=image, b_operand=False)
    gb = B.bdr_quantize_operand(fb, Bm, image=image, b_operand=True)
    torch.cuda.synchronize()
    assert ga.numel() == ia.numel() == B.mx_operand_bytes(fa, M, K, image) and gb.numel() == ib.numel()
    assert torch.equal(ga, ia), "image of A"
    assert torch.equal(gb, ib), "image of B"
    for cd in (torch.float32, torch.bfloat16):
        C = B.mx_gemm_operands(fa, fb, ga, gb, M, N, K, image=image, dtype=cd)
        want = B.mx_gemm(fa, fb, pa, pb, M, N, K, workspace=_workspace(M, N, K), dtype=cd)
        assert torch.equal(C.view(torch.int32 if cd == torch.float32 else torch.int16),
                           want.view(torch.int32 if cd == torch.float32 else torch.int16))
    pan, pbn = _planes_np(pa), _planes_np(pb)
    Cref = O.mx_gemm(ofmt(fa), ofmt(fb), pan, pbn, M, N, K)
    Ah = O.dequantize(ofmt(fa), *pan, M, K).astype(np.float64)
    Bh = O.dequantize(ofmt(fb), *pbn, N, K).astype(np.float64)
    err = np.abs(B.mx_gemm_operands(fa, fb, ga, gb, M, N, K, image=image).cpu().numpy().astype(np.float64) - Cref)
    assert np.all(err <= RTOL * (np.abs(Ah) @ np.abs(Bh).T) + 1e-30)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("name", ["MX6", "MX4", "MX9 as BF16", "MX6 as BF16", "MX4 as BF16"])
@pytest.mark.parametrize("shape", [(128, 128), (384, 256), (1024, 640)])
def test_operands_of_the_transpose(shape, name, dtype):
    """Blocks down the columns: the image of the transpose of x equals the image made of the planes
    that column-wise bdr_quantize gives (those of the transposed tensor), in either role, also for
    a pitched view."""
    rows, cols = shape
    f = getattr(B, name[:3])
    image = B.OPERAND_BF16 if name.endswith("BF16") else B.OPERAND_FP6
    partner = B.MX9 if image == B.OPERAND_BF16 else B.MX6      # makes the two-pass form write that kind
    big = _special(S.wide_range(rows, cols + 256, device="cuda", seed=rows + cols, spread=8)).to(dtype)
    for x in (big[:, :cols].contiguous(), big[:, 128:128 + cols]):
        planes = B.bdr_quantize(f, x, axis=B.AXIS_COL)          # = row-wise planes of x^T [cols x rows]
        want = O.quantize(ofmt(f), np.ascontiguousarray(to_np(x.contiguous()).T))
        for p, w in zip(planes, want):
            assert np.array_equal(p.cpu().numpy(), w)
        # as operand A, then as operand B, of a product with a partner image of the same tensor (MX6:
        # FP6 images, an MX4 x MX4 pair would take the FP4 form; MX9: BF16 images): the writer's images
        other = B.bdr_quantize(partner, x, axis=B.AXIS_COL)
        ia, _, _ = _two_step_images(f, partner, planes, other, cols, cols, rows)
        _, ib, _ = _two_step_images(partner, f, other, planes, cols, cols, rows)
        assert torch.equal(B.bdr_quantize_operand(f, x, axis=B.AXIS_COL, image=image, b_operand=False), ia)
        assert torch.equal(B.bdr_quantize_operand(f, x, axis=B.AXIS_COL, image=image, b_operand=True), ib)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("name", ["MX6", "MX4", "MX9 as BF16", "MX6 as BF16", "MX4 as BF16"])
@pytest.mark.parametrize("shape", [(1, 64), (3, 192), (17, 64), (33, 320), (130, 704), (64, 2112)])
def test_operands_from_few_rows_and_pitched_views(shape, name, dtype):
    """Row blocks on shapes that leave the row-wise kernels' tiles (16 rows x 4 K steps per
    workgroup) partly empty in both directions, from a contiguous tensor and from a view whose rows
    are further apart than their length: the image equals the one made of the oracle-checked planes."""
    rows, K = shape
    f = getattr(B, name[:3])
    image = B.OPERAND_BF16 if name.endswith("BF16") else B.OPERAND_FP6
    partner = B.MX9 if image == B.OPERAND_BF16 else B.MX6
    big = _special(S.wide_range(max(rows, 4), K + 192, device="cuda", seed=rows + K, spread=8))[:rows].to(dtype)
    for x in (big[:, :K].contiguous(), big[:, 64:64 + K]):
        planes = B.bdr_quantize(f, x.contiguous())
        for p, w in zip(planes, O.quantize(ofmt(f), to_np(x.contiguous()))):
            assert np.array_equal(p.cpu().numpy(), w)
        other = B.bdr_quantize(partner, x.contiguous())
        ia, _, _ = _two_step_images(f, partner, planes, other, rows, rows, K)
        # (with few rows in A the two-pass BF16 form reads B from its planes and writes no image of
        # it: the partner in the A role gets 128 rows)
        tall = x.contiguous().repeat((127 + rows) // rows, 1)[:128].contiguous()
        _, ib, _ = _two_step_images(partner, f, B.bdr_quantize(partner, tall), planes, 128, rows, K)
        assert torch.equal(B.bdr_quantize_operand(f, x, image=image, b_operand=False), ia)
        assert torch.equal(B.bdr_quantize_operand(f, x, image=image, b_operand=True), ib)


def _bf16_rne(v):
    """float32 array -> bfloat16 bit patterns, ties to even (written out, no library cast)."""
    u = np.ascontiguousarray(v, np.float32).view(np.uint32).astype(np.uint64)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


@pytest.mark.parametrize("shape", [(128, 128, 64), (256, 256, 512), (130, 70, 128), (257, 129, 64), (512, 384, 1024)])
@pytest.mark.parametrize("names", [("MX6", "MX6"), ("MX9", "MX9"), ("MX4", "MX4"), ("MX9", "MX6")])
def test_c_in_bf16(shape, names):
    """mx_gemm_to with a BF16 C (the dtype of the tensors between tensor operations, Sec. V): every
    element is the FP32 sum of the same form rounded once more to nearest even, so it equals, bit for
    bit, the rounding of what the FP32 call returns, in every form, and lies within half a BF16
    unit (plus the FP32 tolerance) of the oracle's product."""
    M, N, K = shape
    fa, fb = getattr(B, names[0]), getattr(B, names[1])
    A, Bm = S.gemm_operands(M, N, K, device="cuda", seed=3 * M + N + K)
    pa, pb = B.bdr_quantize(fa, A), B.bdr_quantize(fb, Bm)
    pan, pbn = _planes_np(pa), _planes_np(pb)
    Cref = O.mx_gemm(ofmt(fa), ofmt(fb), pan, pbn, M, N, K)
    Ah = O.dequantize(ofmt(fa), *pan, M, K).astype(np.float64)
    Bh = O.dequantize(ofmt(fb), *pbn, N, K).astype(np.float64)
    bound = RTOL * (np.abs(Ah) @ np.abs(Bh).T) + np.abs(Cref) * 2.0 ** -8 + 1e-30
    for ws in (None, _workspace(M, N, K)):
        C32 = B.mx_gemm(fa, fb, pa, pb, M, N, K, workspace=ws)
        C16 = B.mx_gemm(fa, fb, pa, pb, M, N, K, workspace=ws, dtype=torch.bfloat16)
        torch.cuda.synchronize()
        assert C16.dtype == torch.bfloat16
        got = to_np(C16)
        assert np.array_equal(got, _bf16_rne(C32.cpu().numpy())), (shape, names, ws is not None)
        val = (got.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        assert np.all(np.abs(val - Cref) <= bound), (shape, names, ws is not None)
    # a pitched BF16 C inside a wider tensor, and the empty sum
    big = torch.full((M + 2, N + 24), 7.0, dtype=torch.bfloat16, device="cuda")
    B.mx_gemm(fa, fb, pa, pb, M, N, K, out=big[1:M + 1, 8:8 + N], workspace=_workspace(M, N, K))
    assert np.array_equal(to_np(big[1:M + 1, 8:8 + N].contiguous()), _bf16_rne(B.mx_gemm(
        fa, fb, pa, pb, M, N, K, workspace=_workspace(M, N, K)).cpu().numpy()))
    assert bool((big[0] == 7).all()) and bool((big[-1] == 7).all())
    assert bool((big[:, :8] == 7).all()) and bool((big[:, 8 + N:] == 7).all())
    z = torch.full((M, N), 3.0, dtype=torch.bfloat16, device="cuda")
    B.mx_gemm(fa, fb, pa, pb, M, N, 0, out=z)
    assert bool((z == 0).all())


@pytest.mark.parametrize("names", [("MX6", "MX6"), ("MX9", "MX9"), ("MX4", "MX4"), ("MX6", "MX4")])
def test_full_size_sampled_entries(names):
    # 8192^3, the bench configuration (MX6 x MX6) and the other instruction paths at that size:
    # 64 x 64 sampled entries against the oracle
    M = N = K = 8192
    A, Bm = S.gemm_operands(M, N, K, device="cuda")
    f, fb = getattr(B, names[0]), getattr(B, names[1])
    pa, pb = B.bdr_quantize(f, A), B.bdr_quantize(fb, Bm)
    C = B.mx_gemm(f, fb, pa, pb, M, N, K)
    C2 = B.mx_gemm(f, fb, pa, pb, M, N, K, workspace=_workspace(M, N, K))
    torch.cuda.synchronize()
    rng = np.random.default_rng(4)
    ri = np.sort(rng.choice(M, 64, replace=False))
    ci = np.sort(rng.choice(N, 64, replace=False))
    ii, jj = [a.reshape(-1) for a in np.meshgrid(ri, ci, indexing="ij")]
    want, absdot = O.mx_gemm_sampled(ofmt(f), ofmt(fb), _planes_np(pa), _planes_np(pb), M, N, K, ii, jj)
    for got_all in (C, C2):
        got = got_all[torch.as_tensor(ii, device="cuda"), torch.as_tensor(jj, device="cuda")].cpu().numpy()
        err = np.abs(got.astype(np.float64) - want.astype(np.float64))
        assert np.all(err <= RTOL * absdot), float((err / absdot).max())
    # both forms round the same exact products: they differ by a few ulps of the sum at most
    assert ((C - C2).abs() <= 1e-5 * C.abs().max()).all()
    del C2
    # fidelity against the unquantized FP32 product (library GEMM): finite and in a sane band
    Cfp = A @ Bm.t()
    q = 10 * torch.log10(Cfp.double().square().sum() / (C.double() - Cfp.double()).square().sum())
    assert 10.0 < q.item() < 50.0


# ---- operand images read back by a decoder written here, from the documented layout alone
#
# FP6 image: [K / 64][row][4 chunks of 16 bytes]; a chunk is one block of 16: its E2M3 codes in
# dwords 0-2 (element j at bits 6 j .. 6 j + 5), its scale byte in dword 3 (byte 0 for an A
# operand, byte 2 for a B operand, the other three bytes zero).  E2M3: sign, two exponent bits e,
# three fraction bits m; m / 8 for e = 0, else (1 + m / 8) 2^(e - 1).  Scale byte b: 2^(b - 127).
# BF16 image: [K / 32][row][32 BF16 values].

def _decode_fp6_image(img, rows, K, b_operand, sel):
    """values [len(sel) x K] (float64) of the image rows `sel`"""
    a = img.cpu().numpy().reshape(K // 64, rows, 4, 16)[:, sel]
    w = np.ascontiguousarray(a).view(np.uint32).astype(np.uint64)        # [q, s, chunk, 4 dwords]
    lo, hi = w[..., 0] | (w[..., 1] << np.uint64(32)), w[..., 2]
    sc = w[..., 3]
    shift = np.uint64(16 if b_operand else 0)
    assert np.all(sc & ~(np.uint64(0xff) << shift) == 0), "dword 3 holds the scale byte and nothing else"
    scale = ((sc >> shift) & np.uint64(0xff)).astype(np.int64)
    out = np.empty(a.shape[:3] + (16,), np.float64)
    for j in range(16):
        bit = 6 * j
        if bit + 6 <= 64:
            c = (lo >> np.uint64(bit)) & np.uint64(63)
        elif bit >= 64:
            c = (hi >> np.uint64(bit - 64)) & np.uint64(63)
        else:
            c = ((lo >> np.uint64(bit)) | (hi << np.uint64(64 - bit))) & np.uint64(63)
        c = c.astype(np.int64)
        e, m = (c >> 3) & 3, (c & 7).astype(np.float64)
        mag = np.where(e == 0, m / 8.0, (1.0 + m / 8.0) * np.exp2((e - 1).astype(np.float64)))
        out[..., j] = np.where(c >> 5 == 1, -mag, mag) * np.exp2((scale - 127).astype(np.float64))
    return out.transpose(1, 0, 2, 3).reshape(len(sel), K)


def _decode_bf16_image(img, rows, K, sel):
    a = img.cpu().numpy().view(np.uint16).reshape(K // 32, rows, 32)[:, sel]
    bits = a.astype(np.uint32) << np.uint32(16)
    return bits.view(np.float32).astype(np.float64).transpose(1, 0, 2).reshape(len(sel), K)


def _decode_fp4_image(img, rows, K, sel):
    """FP4 image: [K / 128][row][4 chunks of 16 bytes], a chunk = two blocks of 16 E2M1 codes
    (element j of a block at bits 4 j .. 4 j + 3 of its 8 bytes; rows with bit 4 set keep the two
    blocks of a chunk in swapped order), then the scale image [K / 128][row padded to 128][8 bytes]:
    the scales of the step's blocks 0, 2, 4, 6, then of blocks 1, 3, 5, 7.  E2M1: sign, two exponent
    bits e, one fraction bit m; m / 2 for e = 0, else (1 + m / 2) 2^(e - 1)."""
    raw = img.cpu().numpy()
    rows_pad = (rows + 127) // 128 * 128
    nchunk = rows * K // 2
    assert raw.size == nchunk + rows_pad * K // 16
    a = raw[:nchunk].reshape(K // 128, rows, 4, 2, 8)[:, sel]                 # [q, s, chunk, half, 8 bytes]
    sc_all = raw[nchunk:].reshape(K // 128, rows_pad, 8)
    assert not sc_all[:, rows:].any(), "rows that only pad the scale image hold zero scales"
    sc = sc_all[:, sel].astype(np.int64)                                       # [q, s, 8]
    out = np.empty((K // 128, len(sel), 8, 16), np.float64)
    swap = ((np.asarray(sel) >> 4) & 1)[None, :]                               # [1, s]
    for b in range(8):
        half = (b & 1) ^ swap                                                  # [1, s]
        blk = np.where(half[..., None] == 1, a[:, :, b >> 1, 1], a[:, :, b >> 1, 0])   # [q, s, 8 bytes]
        scale = np.exp2((sc[:, :, 4 * (b & 1) + (b >> 1)] - 127).astype(np.float64))
        for j in range(16):
            c = ((blk[..., j >> 1] >> (4 * (j & 1))) & 15).astype(np.int64)
            e, m = (c >> 1) & 3, (c & 1).astype(np.float64)
            mag = np.where(e == 0, m / 2.0, (1.0 + m / 2.0) * np.exp2((e - 1).astype(np.float64)))
            out[:, :, b, j] = np.where(c >> 3 == 1, -mag, mag) * scale
    return out.transpose(1, 0, 2, 3).reshape(len(sel), K)


def _oracle_values(f, x_rows):
    """what the oracle's quantizer and decoder make of the rows x_rows [s x K] (float64)"""
    x_rows = np.ascontiguousarray(x_rows)
    s, K = x_rows.shape
    return O.dequantize(ofmt(f), *O.quantize(ofmt(f), x_rows), s, K).astype(np.float64)


def _check_images_against_the_oracle(f, image, x, axis, sel):
    rows, K = (x.shape[0], x.shape[1]) if axis == B.AXIS_ROW else (x.shape[1], x.shape[0])
    src = x[torch.as_tensor(sel, device=x.device)] if axis == B.AXIS_ROW else x[:, torch.as_tensor(sel, device=x.device)].t()
    want = _oracle_values(f, to_np(src.contiguous()))
    for b_operand in (False, True):
        img = B.bdr_quantize_operand(f, x, axis=axis, image=image, b_operand=b_operand)
        torch.cuda.synchronize()
        assert img.numel() == B.mx_operand_bytes(f, rows, K, image)
        got = (_decode_fp6_image(img, rows, K, b_operand, sel) if image == B.OPERAND_FP6
               else _decode_fp4_image(img, rows, K, sel) if image == B.OPERAND_FP4
               else _decode_bf16_image(img, rows, K, sel))
        assert np.array_equal(got, want), (f, image, axis, b_operand)
        del img


def _image_kind(name):
    return B.OPERAND_BF16 if name.endswith("BF16") else B.OPERAND_FP4 if name.endswith("FP4") else B.OPERAND_FP6


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("name", ["MX6", "MX4", "MX9 as BF16", "MX6 as BF16", "MX4 as BF16", "MX4 as FP4"])
@pytest.mark.parametrize("shape", [(16, 64), (130, 192), (41, 256), (256, 1024), (384, 640)])
def test_operand_images_hold_the_oracles_values(shape, name, dtype):
    """Every element of an image made by bdr_quantize_operand, decoded here from the documented
    layout, is the value the oracle's quantize + dequantize give: row blocks on any shape, column
    blocks on whole tiles (rows a multiple of 128, columns of 128)."""
    rows, cols = shape
    f = getattr(B, name[:3])
    image = _image_kind(name)
    if image == B.OPERAND_FP4 and cols % 128:
        pytest.skip("an FP4 image takes K in multiples of 128")
    x = _special(S.wide_range(rows, cols, device="cuda", seed=7 * rows + cols, spread=8)).to(dtype)
    _check_images_against_the_oracle(f, image, x, B.AXIS_ROW, np.arange(rows))
    if rows % 128 == 0 and cols % 128 == 0:
        _check_images_against_the_oracle(f, image, x, B.AXIS_COL, np.arange(cols))


@pytest.mark.parametrize("name", ["MX6", "MX4", "MX9 as BF16", "MX4 as FP4"])
def test_operand_images_of_the_activation_tensor_at_full_size(name):
    """The bench's operand-image legs (8192 x 12288 BF16, channel outliers), both block directions:
    96 sampled image rows against the oracle, through the decoder above."""
    f = getattr(B, name[:3])
    image = _image_kind(name)
    x = S.activation(device="cuda")
    rng = np.random.default_rng(11)
    for axis, n in ((B.AXIS_ROW, x.shape[0]), (B.AXIS_COL, x.shape[1])):
        sel = np.sort(np.concatenate([[0, n - 1], rng.choice(np.arange(1, n - 1), 94, replace=False)]))
        _check_images_against_the_oracle(f, image, x, axis, sel)


def _two_step_fp4_images(pa, pb, M, N, K):
    """What mx_gemm's two-pass form writes into its workspace for an MX4 x MX4 product with M, N,
    K >= 128 and K a multiple of 128: per operand the FP4 chunks, then the scale image."""
    ws = _workspace(M, N, K)
    C = B.mx_gemm(B.MX4, B.MX4, pa, pb, M, N, K, workspace=ws)
    torch.cuda.synchronize()
    half = (2 * M * K + 255) // 256 * 256
    na, nb = B.mx_operand_bytes(B.MX4, M, K, B.OPERAND_FP4), B.mx_operand_bytes(B.MX4, N, K, B.OPERAND_FP4)
    return ws[:na].clone(), ws[half:half + nb].clone(), C


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("shape", [(128, 128, 128), (256, 384, 512), (130, 200, 256), (512, 256, 1024)])
def test_fp4_operands_made_by_the_quantizer(shape, dtype):
    """MX4 x MX4 on FP4 images: bdr_quantize_operand writes, byte for byte, the chunks and the scale
    image the two-pass form makes of the planes; mx_gemm_operands returns that form's C, which is
    within the tolerance of the oracle's product."""
    M, N, K = shape
    f = B.MX4
    A, Bm = S.gemm_operands(M, N, K, device="cuda", seed=2 * M + N + K)
    A, Bm = _special(A, 1.0e15).to(dtype), _special(Bm, 1.0e15).to(dtype)
    pa, pb = B.bdr_quantize(f, A), B.bdr_quantize(f, Bm)
    ia, ib, want = _two_step_fp4_images(pa, pb, M, N, K)
    ga = B.bdr_quantize_operand(f, A, image=B.OPERAND_FP4, b_operand=False)
    gb = B.bdr_quantize_operand(f, Bm, image=B.OPERAND_FP4, b_operand=True)
    torch.cuda.synchronize()
    assert torch.equal(ga, ia), "image of A"
    assert torch.equal(gb, ib), "image of B"
    for cd in (torch.float32, torch.bfloat16):
        C = B.mx_gemm_operands(f, f, ga, gb, M, N, K, image=B.OPERAND_FP4, dtype=cd)
        w = B.mx_gemm(f, f, pa, pb, M, N, K, workspace=_workspace(M, N, K), dtype=cd)
        assert torch.equal(C.view(torch.int32 if cd == torch.float32 else torch.int16),
                           w.view(torch.int32 if cd == torch.float32 else torch.int16))
    pan, pbn = _planes_np(pa), _planes_np(pb)
    Cref = O.mx_gemm(ofmt(f), ofmt(f), pan, pbn, M, N, K)
    Ah = O.dequantize(ofmt(f), *pan, M, K).astype(np.float64)
    Bh = O.dequantize(ofmt(f), *pbn, N, K).astype(np.float64)
    err = np.abs(B.mx_gemm_operands(f, f, ga, gb, M, N, K, image=B.OPERAND_FP4).cpu().numpy().astype(np.float64) - Cref)
    assert np.all(err <= RTOL * (np.abs(Ah) @ np.abs(Bh).T) + 1e-30)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("shape", [(128, 128), (384, 256), (1024, 640)])
def test_fp4_operands_of_the_transpose(shape, dtype):
    """Column blocks into the FP4 image: the image of the transpose equals the one the two-pass form
    makes of the column-wise planes, also from a pitched view."""
    rows, cols = shape
    f = B.MX4
    big = _special(S.wide_range(rows, cols + 256, device="cuda", seed=rows + cols, spread=8)).to(dtype)
    for x in (big[:, :cols].contiguous(), big[:, 128:128 + cols]):
        planes = B.bdr_quantize(f, x, axis=B.AXIS_COL)
        ia, _, _ = _two_step_fp4_images(planes, planes, cols, cols, rows)
        for b_operand in (False, True):
            assert torch.equal(B.bdr_quantize_operand(f, x, axis=B.AXIS_COL, image=B.OPERAND_FP4, b_operand=b_operand), ia)


@pytest.mark.parametrize("names", [("MX6", "MX6"), ("MX4", "MX6"), ("MX9", "MX9"), ("MX9", "MX4"), ("MX4", "MX4"),
                                   ("MX9", "MX6"), ("MX6", "MX9")])
@pytest.mark.parametrize("shape", [(1, 32, 64), (5, 100, 128), (16, 384, 1024), (32, 257, 2048), (31, 64, 4096 + 128),
                                   (33, 96, 256), (64, 130, 1152), (100, 320, 512), (128, 257, 2048)])
def test_few_rows_of_a(shape, names):
    """M <= 64 (a decoding step): the product streams over B's image with all of A in one or two MFMA tiles
    (the larger shapes here take the tiled kernels: the boundary is crossed on both sides).
    Both entry points against the oracle, every image kind (an MX4 pair on FP4 images through
    mx_gemm_operands), FP32 and BF16 results, edges of N that are not tile multiples, more K steps
    than waves and fewer."""
    M, N, K = shape
    fa, fb = getattr(B, names[0]), getattr(B, names[1])
    A, Bm = S.gemm_operands(M, N, K, device="cuda", seed=7 * M + N + K)
    A, Bm = _special(A.repeat(4, 1), 1.0e15)[:max(M, 4)][:M].contiguous(), _special(Bm, 1.0e15)
    pa, pb = B.bdr_quantize(fa, A), B.bdr_quantize(fb, Bm)
    pan, pbn = _planes_np(pa), _planes_np(pb)
    Cref = O.mx_gemm(ofmt(fa), ofmt(fb), pan, pbn, M, N, K)
    Ah = O.dequantize(ofmt(fa), *pan, M, K).astype(np.float64)
    Bh = O.dequantize(ofmt(fb), *pbn, N, K).astype(np.float64)
    bound = RTOL * (np.abs(Ah) @ np.abs(Bh).T) + 1e-30
    kinds = [B.OPERAND_BF16 if 7 in (fa.m, fb.m) else B.OPERAND_FP6]
    if fa.m == 2 and fb.m == 2 and K % 128 == 0:
        kinds.append(B.OPERAND_FP4)
    got = [B.mx_gemm(fa, fb, pa, pb, M, N, K, workspace=_workspace(M, N, K))]
    for kind in kinds:
        ia = B.bdr_quantize_operand(fa, A, image=kind, b_operand=False)
        ib = B.bdr_quantize_operand(fb, Bm, image=kind, b_operand=True)
        got.append(B.mx_gemm_operands(fa, fb, ia, ib, M, N, K, image=kind))
        Cb = B.mx_gemm_operands(fa, fb, ia, ib, M, N, K, image=kind, dtype=torch.bfloat16)
        assert torch.equal(Cb.view(torch.int16), got[-1].to(torch.bfloat16).view(torch.int16))
    torch.cuda.synchronize()
    for C in got:
        err = np.abs(C.cpu().numpy().astype(np.float64) - Cref)
        assert np.all(err <= bound), float((err / bound).max())
    # a pitched C keeps what lies between its rows
    big = torch.full((M, N + 40), -7.0, device="cuda")
    ia = B.bdr_quantize_operand(fa, A, image=kinds[0])
    ib = B.bdr_quantize_operand(fb, Bm, image=kinds[0], b_operand=True)
    B.mx_gemm_operands(fa, fb, ia, ib, M, N, K, image=kinds[0], out=big[:, :N])
    assert torch.equal(big[:, :N], got[1]) and bool((big[:, N:] == -7.0).all())
