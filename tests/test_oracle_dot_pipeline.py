"""Pins of the oracle's model of the paper's dot-product pipeline (Sec. IV-B, "Dot Product
Architecture").  The paper gives no worked value, so the pins are what the arithmetic fixes:
the exact integer block product (d2 = 0), the shift tau_a + tau_b per sub-block pair, equality
with the exactly rounded dot product once the fixed-point word is wide enough, the error bound
of one unit per block, scale equivariance -- plus hand-worked examples and an independent
big-integer model, which check the code against the readings it states (tests/golden)."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle as O

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "dot_pipeline_examples.txt")


# ---------------------------------------------------------------- independent plane reader

def read_planes(f, planes, rows, K):
    """(sign * M [rows, K] as Python-int array, SE [rows, K/k1], tau [rows, K/k2]) read from
    the packed planes with numpy.unpackbits (layout: include/bdr_mx.h, little-endian streams)."""
    codes, sexp, mexp = planes
    cb = f.m + 1
    bits = np.unpackbits(codes, bitorder="little")[:rows * K * cb].reshape(rows * K, cb)
    mag = (bits[:, :f.m].astype(np.int64) << np.arange(f.m)).sum(axis=1)
    sm = np.where(bits[:, f.m] == 1, -mag, mag).reshape(rows, K)
    se = sexp.astype(np.int64).reshape(rows, K // f.k1)
    if f.d2:
        tb = np.unpackbits(mexp, bitorder="little")[:rows * (K // f.k2) * f.d2]
        tau = (tb.reshape(-1, f.d2).astype(np.int64) << np.arange(f.d2)).sum(axis=1)
    else:
        tau = np.zeros(rows * (K // f.k2), np.int64)
    return sm, se, tau.reshape(rows, K // f.k2)


def fraction_to_f32(v):
    """Exactly rounded (nearest even) float32 of a Fraction; normal range only."""
    if v == 0:
        return np.float32(0.0)
    s, a = (-1 if v < 0 else 1), abs(v)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    assert Fraction(2) ** e <= a < Fraction(2) ** (e + 1) and -126 <= e <= 126
    q = a / Fraction(2) ** (e - 23)          # in [2^23, 2^24)
    n = q.numerator // q.denominator
    rem = q - n
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and n % 2 == 1):
        n += 1
    return np.float32(s * math.ldexp(n, e - 23))


def exact_dot(fa, fb, pa, pb, i, j, K, rows_a, rows_b):
    """The dot product of the dequantized rows as a Fraction (dequantize is pinned elsewhere)."""
    ah = O.dequantize(fa, *pa, rows_a, K)[i]
    bh = O.dequantize(fb, *pb, rows_b, K)[j]
    return sum(Fraction(float(x)) * Fraction(float(y)) for x, y in zip(ah, bh))


def model(fa, fb, pa, pb, M, N, K, r, f_bits):
    """The readings D1-D8 once more, in Python integers (an independent second writing of the
    same steps: it guards the C code against slips, it does not pin the readings)."""
    sa, ea, ta = read_planes(fa, pa, M, K)
    sb, eb, tb = read_planes(fb, pb, N, K)
    k1, k2 = fa.k1, fa.k2
    ba, bb = (1 << fa.d2) - 1, (1 << fb.d2) - 1
    W = fa.m + fb.m + int(math.log2(k1)) + ba + bb
    g = f_bits - 1 - W
    C = np.zeros((M, N), np.float32)
    for i in range(M):
        for j in range(N):
            acc = None
            for k0 in range(0, K, r):
                blocks = range(k0 // k1, (k0 + r) // k1)
                e = {b: int(ea[i, b] + eb[j, b]) for b in blocks}
                emax = max(e.values())
                V = 0
                for b in blocks:
                    T = 0
                    for u in range(b * (k1 // k2), (b + 1) * (k1 // k2)):
                        S = sum(int(sa[i, t]) * int(sb[j, t]) for t in range(u * k2, (u + 1) * k2))
                        T += S << (ba + bb - int(ta[i, u]) - int(tb[j, u]))
                    sh = g - (emax - e[b])
                    V += T << sh if sh >= 0 else T >> -sh          # Python's >> floors
                x = emax - 254 - (fa.m - 1) - (fb.m - 1) - ba - bb - g
                p = fraction_to_f32(Fraction(V) * Fraction(2) ** x)
                acc = p if acc is None else np.float32(acc + p)
            C[i, j] = acc
    return C


# ------------------------------------------------------------------------------- the pins

def _ab_rows():
    a = np.array([1.5, -0.75, 0.3, 0.2], np.float32)
    b = np.array([1.5, 0.5, 0.25, -0.5], np.float32)
    return a, b


def test_hand_worked_examples():
    f = O.fmt(4, 2, 1, 2)
    a, b = _ab_rows()
    rows = {
        "single": (a[None, :], b[None, :]),
        "two": (np.concatenate([a, -a / 8])[None, :], np.concatenate([b, b])[None, :]),
        "neg": (np.concatenate([-a, a / 8])[None, :], np.concatenate([b, b])[None, :]),
    }
    # the decoded blocks are the ones the golden file derives
    pa, pb = O.quantize(f, rows["single"][0]), O.quantize(f, rows["single"][1])
    sa, ea, ta = read_planes(f, pa, 1, 4)
    sb, eb, tb = read_planes(f, pb, 1, 4)
    assert sa.tolist() == [[3, -2, 1, 1]] and ta.tolist() == [[0, 1]] and ea.tolist() == [[127]]
    assert sb.tolist() == [[3, 1, 1, -2]] and tb.tolist() == [[0, 1]] and eb.tolist() == [[127]]
    n = 0
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        name, K, r, fb, want = line.split()
        A, B = rows["single" if name.startswith("single") else "neg" if name.startswith("neg") else "two"]
        K, r, fb = int(K), int(r), int(fb)
        got = O.dot_pipeline(f, f, O.quantize(f, A), O.quantize(f, B), 1, 1, K, r=r, f_bits=fb)
        assert got[0, 0] == np.float32(float(want)), (name, got, want)
        n += 1
    assert n == 8


@pytest.mark.parametrize("k1,m", [(16, 7), (8, 4), (64, 2), (1, 5), (32, 8)])
def test_without_microexponents_a_block_is_the_exact_integer_dot_product(k1, m):
    # d2 = 0 (block floating point, Sec. IV-B: "block floating-point (d2 = 0) dot product"):
    # one block per pass, so the result is sum(Ma Mb) 2^(Ea + Eb - 2 (m - 1)) with nothing dropped
    f = O.fmt(k1, k1, 0, m)
    rng = np.random.default_rng(k1 + m)
    A = (rng.standard_normal((6, k1)) * np.exp2(rng.integers(-8, 9, (6, 1)))).astype(np.float32)
    B = (rng.standard_normal((5, k1)) * np.exp2(rng.integers(-8, 9, (5, 1)))).astype(np.float32)
    pa, pb = O.quantize(f, A), O.quantize(f, B)
    sa, ea, _ = read_planes(f, pa, 6, k1)
    sb, eb, _ = read_planes(f, pb, 5, k1)
    got = O.dot_pipeline(f, f, pa, pb, 6, 5, k1, f_bits=25)
    for i in range(6):
        for j in range(5):
            dot = int(np.dot(sa[i], sb[j]))
            want = fraction_to_f32(Fraction(dot) * Fraction(2) ** int(ea[i, 0] + eb[j, 0] - 254 - 2 * (m - 1)))
            assert got[i, j] == want, (i, j)


def test_the_shift_is_tau_a_plus_tau_b_per_sub_block():
    # one block of MX6 operands in which every sub-block pair meets every combination of shifts;
    # the block result equals sum_j S_j 2^-(tau_a + tau_b) exactly (f = 25 leaves room)
    f = O.MX6
    a = np.array([8, 9, 1, 1.5, 15, 3, 0.5, 0.75, 12, -7, 0.9, -0.6, 2, 1, 3, -2.5], np.float32)
    b = np.array([1, -1, 15, 9, 0.5, 0.5, 0.9, 0.3, -14, 2, 6, 5, 1, 1, 0.25, 0.125], np.float32)
    pa, pb = O.quantize(f, a[None, :]), O.quantize(f, b[None, :])
    sa, ea, ta = read_planes(f, pa, 1, 16)
    sb, eb, tb = read_planes(f, pb, 1, 16)
    assert {(int(x), int(y)) for x, y in zip(ta[0], tb[0])} == {(0, 0), (0, 1), (1, 0), (1, 1)}
    want = Fraction(0)
    for u in range(8):
        S = int(sa[0, 2 * u] * sb[0, 2 * u] + sa[0, 2 * u + 1] * sb[0, 2 * u + 1])
        want += Fraction(S, 2 ** int(ta[0, u] + tb[0, u]))
    want *= Fraction(2) ** int(ea[0, 0] + eb[0, 0] - 254 - 6)
    got = O.dot_pipeline(f, f, pa, pb, 1, 1, 16)
    assert got[0, 0] == fraction_to_f32(want)
    assert want == exact_dot(f, f, pa, pb, 0, 0, 16, 1, 1)


@pytest.mark.parametrize("names", [("MX9", "MX9"), ("MX6", "MX6"), ("MX4", "MX9"), ("MX6", "MX4")])
@pytest.mark.parametrize("r", [16, 64, 256])
def test_a_wide_enough_word_gives_the_exactly_rounded_dot_product(names, r):
    # with f = 64 no block loses a bit as long as the exponent sums of a pass spread over fewer
    # than 63 - W binades; one pass (r = K) must then equal the dot product of the dequantized
    # operands, rounded once
    fa, fb = getattr(O, names[0]), getattr(O, names[1])
    rng = np.random.default_rng(r)
    K = r
    A = (rng.standard_normal((4, K)) * np.exp2(rng.integers(-5, 6, (4, K // 16)).repeat(16, 1))).astype(np.float32)
    B = (rng.standard_normal((3, K)) * np.exp2(rng.integers(-5, 6, (3, K // 16)).repeat(16, 1))).astype(np.float32)
    pa, pb = O.quantize(fa, A), O.quantize(fb, B)
    got = O.dot_pipeline(fa, fb, pa, pb, 4, 3, K, f_bits=64)
    for i in range(4):
        for j in range(3):
            assert got[i, j] == fraction_to_f32(exact_dot(fa, fb, pa, pb, i, j, K, 4, 3)), (i, j)


@pytest.mark.parametrize("f_bits", [12, 18, 25, 31])
def test_error_is_below_one_unit_per_block(f_bits):
    # every block drops less than one unit of the f-bit word, and only downwards
    fa = fb = O.MX6
    rng = np.random.default_rng(f_bits)
    K = 128
    A = (rng.standard_normal((5, K)) * np.exp2(rng.integers(-9, 10, (5, K // 16)).repeat(16, 1))).astype(np.float32)
    B = (rng.standard_normal((5, K)) * np.exp2(rng.integers(-9, 10, (5, K // 16)).repeat(16, 1))).astype(np.float32)
    pa, pb = O.quantize(fa, A), O.quantize(fb, B)
    got = O.dot_pipeline(fa, fb, pa, pb, 5, 5, K, f_bits=f_bits)
    _, ea, _ = read_planes(fa, pa, 5, K)
    _, eb, _ = read_planes(fb, pb, 5, K)
    W = 4 + 4 + 4 + 2
    for i in range(5):
        for j in range(5):
            exact = exact_dot(fa, fb, pa, pb, i, j, K, 5, 5)
            unit = Fraction(2) ** int((ea[i] + eb[j]).max() - 254 - 6 - 2 - (f_bits - 1 - W))
            lo = exact - (K // 16) * unit
            g = Fraction(float(got[i, j]))
            half_ulp = Fraction(2) ** (max(abs(g), abs(exact)).numerator.bit_length()
                                       - max(abs(g), abs(exact)).denominator.bit_length() - 23)
            assert lo - half_ulp <= g <= exact + half_ulp, (i, j, f_bits)


def test_power_of_two_scaling_passes_through():
    fa, fb = O.MX9, O.MX6
    rng = np.random.default_rng(3)
    A = rng.standard_normal((4, 64)).astype(np.float32)
    B = rng.standard_normal((4, 64)).astype(np.float32)
    base = O.dot_pipeline(fa, fb, O.quantize(fa, A), O.quantize(fb, B), 4, 4, 64, r=32, f_bits=20)
    for ja, jb in ((3, 0), (-7, 2), (10, -30)):
        got = O.dot_pipeline(fa, fb, O.quantize(fa, np.ldexp(A, ja)), O.quantize(fb, np.ldexp(B, jb)),
                             4, 4, 64, r=32, f_bits=20)
        assert np.array_equal(got, np.ldexp(base, ja + jb))


@pytest.mark.parametrize("case", [
    dict(fa=O.MX9, fb=O.MX9, K=128, r=64, f=25), dict(fa=O.MX6, fb=O.MX6, K=128, r=128, f=25),
    dict(fa=O.MX4, fb=O.MX4, K=64, r=16, f=14), dict(fa=O.MX9, fb=O.MX4, K=64, r=32, f=17),
    dict(fa=O.fmt(8, 4, 2, 3), fb=O.fmt(8, 4, 1, 5), K=64, r=16, f=20),
    dict(fa=O.fmt(1, 1, 0, 4), fb=O.fmt(1, 1, 0, 4), K=32, r=32, f=25),     # scalar: k1 = k2 = 1
    dict(fa=O.fmt(32, 1, 3, 2), fb=O.fmt(32, 1, 0, 6), K=64, r=64, f=9),
    dict(fa=O.MX6, fb=O.MX6, K=64, r=64, f=5), dict(fa=O.MX6, fb=O.MX6, K=64, r=16, f=40),
], ids=lambda c: "%d-%d-%d" % (c["K"], c["r"], c["f"]))
def test_against_the_big_integer_model(case):
    fa, fb, K, r, fbits = case["fa"], case["fb"], case["K"], case["r"], case["f"]
    rng = np.random.default_rng(K + r + fbits)
    nb = K // fa.k1
    A = (rng.standard_normal((4, K)) * np.exp2(rng.integers(-12, 13, (4, nb)).repeat(fa.k1, 1))).astype(np.float32)
    B = (rng.standard_normal((5, K)) * np.exp2(rng.integers(-12, 13, (5, nb)).repeat(fa.k1, 1))).astype(np.float32)
    A[0, :fa.k1] = 0.0                    # an all-zero block
    B[1] = 0.0                            # and an all-zero row
    pa, pb = O.quantize(fa, A), O.quantize(fb, B)
    got = O.dot_pipeline(fa, fb, pa, pb, 4, 5, K, r=r, f_bits=fbits)
    want = model(fa, fb, pa, pb, 4, 5, K, r, fbits)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_arguments():
    f = O.MX6
    A = np.ones((2, 32), np.float32)
    p = O.quantize(f, A)
    idx = np.zeros(1, np.int64)
    with pytest.raises(O.OracleError):
        O.dot_pipeline_sampled(f, O.fmt(32, 2, 1, 4), p, p, 2, 2, 32, idx, idx)      # different k1
    with pytest.raises(O.OracleError):
        O.dot_pipeline_sampled(f, f, p, p, 2, 2, 32, idx, idx, r=24)                 # r % k1
    with pytest.raises(O.OracleError):
        O.dot_pipeline_sampled(f, f, p, p, 2, 2, 32, idx, idx, f_bits=1)
    with pytest.raises(O.OracleError):
        O.dot_pipeline_sampled(f, f, p, p, 2, 2, 32, idx + 2, idx)
    assert O.dot_pipeline(f, f, p, p, 2, 2, 32)[0, 0] == 32.0
