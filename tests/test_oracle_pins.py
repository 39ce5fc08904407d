"""Pins for the CPU oracle: everything here runs without a GPU and checks the
oracle against things that are NOT the oracle -- exact identities, closed forms,
brute force, library routines, and the counts the paper prints.

Parity status that these tests cannot provide: with perturbed ("flex")
transform matrices Eq. 1 no longer equals a direct convolution, so the literal
Winograd (O2) and the quantized pipeline (O3) with such matrices are "parity
unpinned" beyond (a) the limit noise -> 0 and (b) the exact-rational emulation
of the fused chains on tiny cases below.
"""
import os
from fractions import Fraction

import numpy as np
import pytest
from scipy.signal import correlate2d

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_counts.txt")


def _golden():
    out = {}
    for line in open(GOLD):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            out[k.strip()] = float(v)
    return out


def _rel(a, b):
    return np.abs(a - b).max() / np.abs(b).max()


# ---------------------------------------------------------------- P2 / P3 / P6
@pytest.mark.parametrize("m", [2, 4, 6])
def test_cook_toom_exact_bilinear_identity(oracle, m):
    """sum_i A^T[a,i] G[i,b] B^T[i,c] == [c == a+b] exactly (the algebra of Eq. 1:
    y_a = sum_b d_{a+b} g_b), in rationals -- independent of any convolution code."""
    BT, G, AT = oracle.cook_toom_exact(m)
    n = m + 2
    for a in range(m):
        for b in range(3):
            for c in range(n):
                s = sum(AT[a][i] * G[i][b] * BT[i][c] for i in range(n))
                assert s == (1 if c == a + b else 0), (m, a, b, c, s)


def test_cook_toom_custom_points_identity(oracle):
    pts = [Fraction(0), Fraction(1), Fraction(-1), Fraction(2), Fraction(-2)]
    BT, G, AT = oracle.cook_toom_exact(4, pts)
    for a in range(4):
        for b in range(3):
            for c in range(6):
                s = sum(AT[a][i] * G[i][b] * BT[i][c] for i in range(6))
                assert s == (1 if c == a + b else 0)


def test_f23_textbook_four_multiplies(oracle):
    """1-D F(2,3): the textbook minimal algorithm
        m1=(d0-d2)g0, m2=(d1+d2)(g0+g1+g2)/2, m3=(d2-d1)(g0-g1+g2)/2, m4=(d1-d3)g2,
        y0=m1+m2+m3, y1=m2-m3-m4.
    The row scaling is a free choice, so compare the rank-1 terms
    A^T[:,i] (x) G[i,:] (x) B^T[i,:], which are not."""
    BT, G, AT = oracle.cook_toom(2)
    tb_BT = np.array([[1, 0, -1, 0], [0, 1, 1, 0], [0, -1, 1, 0], [0, 1, 0, -1]], float)
    tb_G = np.array([[1, 0, 0], [.5, .5, .5], [.5, -.5, .5], [0, 0, 1]], float)
    tb_AT = np.array([[1, 1, 1, 0], [0, 1, -1, -1]], float)
    for i in range(4):
        ours = np.einsum("a,b,c->abc", AT[:, i], G[i], BT[i])
        text = np.einsum("a,b,c->abc", tb_AT[:, i], tb_G[i], tb_BT[i])
        assert np.array_equal(ours, text), i
    # and the textbook algorithm really is the FIR filter, with 4 multiplies
    rng = np.random.default_rng(1)
    d, g = rng.integers(-9, 9, 4).astype(float), rng.integers(-9, 9, 3).astype(float)
    prod = (tb_G @ g) * (tb_BT @ d)
    assert prod.shape == (4,)
    y = tb_AT @ prod
    assert np.array_equal(y, [d[0] * g[0] + d[1] * g[1] + d[2] * g[2],
                              d[1] * g[0] + d[2] * g[1] + d[3] * g[2]])
    assert np.array_equal(AT @ ((G @ g) * (BT @ d)), y)


def test_default_matrices_literal_values(oracle):
    """Spot values that follow from the construction by hand."""
    BT, G, AT = oracle.cook_toom_exact(4)
    assert BT[0] == [Fraction(1, 4), 0, Fraction(-5, 4), 0, 1, 0]
    assert [list(r) for r in G] == [
        [4, 0, 0], [Fraction(2, 3)] * 3, [Fraction(2, 3), Fraction(-2, 3), Fraction(2, 3)],
        [Fraction(8, 3), Fraction(4, 3), Fraction(2, 3)],
        [Fraction(8, 3), Fraction(-4, 3), Fraction(2, 3)], [0, 0, 1]]
    pts = [0, 1, -1, Fraction(1, 2), Fraction(-1, 2)]
    for a in range(4):
        assert AT[a][:5] == [p ** a for p in pts]
    mx = lambda M: max(abs(v) for r in M for v in r)
    assert (mx(BT), mx(G), mx(AT)) == (Fraction(5, 4), 4, 1)
    BT6, G6, AT6 = oracle.cook_toom_exact(6)
    assert (mx(BT6), mx(G6), mx(AT6)) == (Fraction(21, 4), 1, 32)


def test_zero_fractions_match_paper(oracle):
    gold = _golden()
    zf = lambda M: sum(v == 0 for r in M for v in r) / sum(len(r) for r in M)
    BT, G, AT = oracle.cook_toom_exact(2)
    assert zf(BT) == gold["zero_fraction_F2_BT"]
    assert round(zf(G), 2) == gold["zero_fraction_F2_G"]
    assert zf(AT) == gold["zero_fraction_F2_AT"]
    BT, G, AT = oracle.cook_toom_exact(4)
    assert round(zf(G), 2) == gold["zero_fraction_F4_G"]
    assert zf(AT) == gold["zero_fraction_F4_AT"]


def test_fp32_rounding_of_matrices_is_correct(oracle):
    BTx, Gx, ATx = oracle.cook_toom_exact(6)
    BT, G, AT = oracle.cook_toom(6, dtype=np.float32)
    for ex, fl in ((BTx, BT), (Gx, G), (ATx, AT)):
        for i, row in enumerate(ex):
            for j, v in enumerate(row):
                f = np.float32(fl[i, j])
                lo, hi = np.nextafter(f, np.float32(-np.inf)), np.nextafter(f, np.float32(np.inf))
                e = abs(Fraction(float(f)) - v)
                assert e <= abs(Fraction(float(lo)) - v) and e <= abs(Fraction(float(hi)) - v)


# ---------------------------------------------------------------- P5 counts
def test_paper_counts(oracle):
    gold = _golden()
    assert gold["mults_per_output_direct"] == 9
    for m, key in ((2, "mults_per_output_F2"), (4, "mults_per_output_F4")):
        n = m + 2
        assert n * n / (m * m) == gold[key]
    # dense (valid) convolution of a 32x32 input: 30x30 outputs
    geo = oracle.geometry(1, 32, 32, 0, 2)
    assert (geo["Ho"], geo["Wo"], geo["n"]) == (30, 30, gold["patch_F2"])
    assert geo["Ho"] * geo["Wo"] * 9 == gold["mults_32x32_direct"]
    assert geo["T"] * geo["P"] == gold["mults_32x32_winograd_4x4_tile"]
    assert round(16 / 9, 2) == gold["weight_memory_growth_F2"]
    assert 36 / 9 == gold["weight_memory_growth_F4"]
    # the U tensor really has that many entries
    Uf, _ = oracle.q_weights(np.ones((2, 3, 3, 3), np.float32), oracle.cook_toom(4, dtype=np.float32)[1],
                             want_q=False)
    assert Uf.size == 4 * 2 * 3 * 9


# ---------------------------------------------------------------- P4 brute force for O1
def _direct_bruteforce(X, g, stride, pad):
    N, C, H, W = X.shape
    K = g.shape[0]
    Ho, Wo = (H + 2 * pad - 3) // stride + 1, (W + 2 * pad - 3) // stride + 1
    Xp = np.zeros((N, C, H + 2 * pad, W + 2 * pad), X.dtype)
    Xp[:, :, pad:pad + H, pad:pad + W] = X
    Y = np.zeros((N, K, Ho, Wo), X.dtype)
    for i in range(3):
        for j in range(3):
            win = Xp[:, :, i:i + stride * (Ho - 1) + 1:stride, j:j + stride * (Wo - 1) + 1:stride]
            Y += np.einsum("nchw,kc->nkhw", win, g[:, :, i, j])
    return Y


@pytest.mark.parametrize("stride,pad,H,W", [(1, 1, 5, 7), (1, 0, 6, 4), (2, 1, 8, 8), (2, 1, 7, 5)])
def test_direct_conv_bruteforce_integers(oracle, stride, pad, H, W):
    rng = np.random.default_rng(3)
    X = rng.integers(-5, 6, (2, 3, H, W)).astype(np.float64)
    g = rng.integers(-4, 5, (4, 3, 3, 3)).astype(np.float64)
    assert np.array_equal(oracle.conv2d_direct_f64(X, g, stride, pad), _direct_bruteforce(X, g, stride, pad))


def test_direct_conv_single_channel_nine_terms(oracle):
    X = np.arange(1, 26, dtype=np.float64).reshape(1, 1, 5, 5)
    g = np.array([[1, 2, 3], [4, 5, 6], [7, 8, 9]], np.float64).reshape(1, 1, 3, 3)
    Y = oracle.conv2d_direct_f64(X, g, 1, 0)
    # hand-written 9-term sum for the top-left output: no filter flip
    exp00 = (1 * 1 + 2 * 2 + 3 * 3 + 6 * 4 + 7 * 5 + 8 * 6 + 11 * 7 + 12 * 8 + 13 * 9)
    assert Y[0, 0, 0, 0] == exp00
    assert np.array_equal(Y[0, 0], correlate2d(X[0, 0], g[0, 0], mode="valid"))
    Y1 = oracle.conv2d_direct_f64(X, g, 1, 1)
    assert np.array_equal(Y1[0, 0], correlate2d(X[0, 0], g[0, 0], mode="same"))


def test_direct_conv_q_matches_integer_bruteforce(oracle):
    """The integer direct convolution and its one requantization: the accumulators against
    brute force, the codes against the exact-product rule -- nearest integer, ties to even,
    to the exact rational product of the accumulator and the fp32 factor, then saturation --
    evaluated in rationals (not a second floating-point rounding)."""
    rng = np.random.default_rng(5)
    Xq = rng.integers(-127, 128, (2, 5, 6, 6))
    gq = rng.integers(-127, 128, (3, 5, 3, 3))
    r_y = np.float32(2e-3)
    for stride in (1, 2):
        acc, Yq = oracle.conv2d_direct_q(Xq, gq, r_y=r_y, stride=stride, pad=1)
        ref = _direct_bruteforce(Xq.astype(np.int64), gq.astype(np.int64), stride, 1)
        assert np.array_equal(acc, ref)
        exp = np.array([_rne_sat(Fraction(int(a)) * Fraction(float(r_y)), 127) for a in ref.ravel()])
        assert np.array_equal(Yq.ravel(), exp)
        assert np.abs(Yq).max() == 127 and (np.abs(Yq) < 127).sum() > Yq.size // 2
    # products that the two-step rule (round the product to fp32, then to an integer) gets
    # wrong: fl(1/6) lies just above 1/6, so 3 fl(1/6) is just above 1/2 and belongs to 1, but
    # the fp32 product is 0.5 exactly, a tie that would go to 0 (likewise 15 fl(1/6) -> 3, not 2)
    one_sixth = np.float32(1.0) / np.float32(6.0)
    assert np.float32(3.0) * one_sixth == np.float32(0.5) and 3 * Fraction(float(one_sixth)) > Fraction(1, 2)
    assert np.float32(15.0) * one_sixth == np.float32(2.5)
    X1 = np.zeros((1, 1, 3, 3), np.int64)
    X1[0, 0, 1, 1] = 1
    for a, want in ((3, 1), (9, 2), (15, 3), (-3, -1), (-9, -2), (6, 1), (12, 2)):
        g1 = np.zeros((1, 1, 3, 3), np.int64)
        g1[0, 0, 1, 1] = a
        acc, Yq = oracle.conv2d_direct_q(X1, g1, r_y=one_sixth, stride=1, pad=1)
        assert acc[0, 0, 1, 1] == a
        assert Yq[0, 0, 1, 1] == want == _rne_sat(Fraction(a) * Fraction(float(one_sixth)), 127)
    # true ties (factor 1/2 is exact): half to even
    for a, want in ((1, 0), (3, 2), (5, 2), (7, 4), (-1, 0), (-3, -2), (255, 127), (-999, -127)):
        g1 = np.zeros((1, 1, 3, 3), np.int64)
        g1[0, 0, 1, 1] = a
        _, Yq = oracle.conv2d_direct_q(X1, g1, r_y=np.float32(0.5), stride=1, pad=1)
        assert Yq[0, 0, 1, 1] == want


def test_quantize_tensor_hand_values(oracle):
    """The input quantizer sat(rne(x / scale)) -- a correctly rounded fp32 division, then the
    nearest integer, ties to even, then saturation -- on values worked out by hand, and
    against the same rule in exact rationals on random data."""
    q = oracle.quantize_tensor
    x = np.array([0.0, 0.25, 0.75, 1.25, 1.75, -0.25, -0.75, -1.25, 63.5, 64.5, 1000.0, -1000.0,
                  126.5, 127.5, -127.5], np.float32)
    want = [0, 0, 2, 2, 4, 0, -2, -2, 127, 127, 127, -127, 127, 127, -127]
    assert q(x, 0.5).tolist() == want                       # x / 0.5 is exact: .5 ties go to even
    assert q(np.array([2.5, 3.5, -2.5, 7.49999, 7.5, 8.5], np.float32), 1.0, 7).tolist() == \
        [2, 4, -2, 7, 7, 7]
    # the division is rounded to fp32 before the integer is taken: fl(0.35 / 0.1) is 3.5
    # exactly (the quotient of the two floats lies within half an ulp of it), so it is a tie
    a, b = np.float32(0.35), np.float32(0.1)
    assert a / b == np.float32(3.5) and Fraction(float(a)) / Fraction(float(b)) != Fraction(7, 2)
    assert q(np.array([a]), b).tolist() == [4]
    rng = np.random.default_rng(41)
    xs = (rng.standard_normal(400) * 3).astype(np.float32)
    sc = np.float32(0.0237)
    got = q(xs, sc)
    for v, g_ in zip(xs, got):
        quo = _round32(Fraction(float(v)) / Fraction(float(sc)))        # correctly rounded fp32 division
        assert g_ == _rne_sat(Fraction(float(quo)), 127)
    assert got.dtype == np.int32 and np.abs(got).max() == 127
    # the benchmark's input preparation is the same function of (x, scale)
    from paper_2002_10711_amd import workloads
    assert np.array_equal(workloads.input_codes(xs, sc), got.astype(np.int8))
    assert np.array_equal(workloads.input_codes(x, 0.5), np.array(want, np.int8))


# ---------------------------------------------------------------- P1 Winograd == direct in fp64
@pytest.mark.parametrize("m", [2, 4, 6])
@pytest.mark.parametrize("H,W,pad", [(4, 4, 1), (5, 7, 1), (7, 5, 1), (8, 8, 1), (8, 6, 0), (9, 16, 1)])
def test_winograd_f64_equals_direct(oracle, m, H, W, pad):
    """Sec. 3.1: F2/F4 (and in fp64 also F6) introduce only marginal numerical
    error; Table 1's 32-bit column.  Non-symmetric random data so a transposed
    operand or a swapped index anywhere fails."""
    rng = np.random.default_rng(100 * m + H + W)
    X = rng.standard_normal((2, 3, H, W))
    g = rng.standard_normal((4, 3, 3, 3))
    BT, G, AT = oracle.cook_toom(m)
    Yw = oracle.winograd_f64(X, g, BT, G, AT, pad)
    Yd = oracle.conv2d_direct_f64(X, g, 1, pad)
    assert Yw.shape == Yd.shape
    assert _rel(Yw, Yd) <= 1e-9


def test_winograd_f64_detects_a_planted_transpose(oracle):
    """The pin above is sharp: feeding B instead of B^T breaks it."""
    rng = np.random.default_rng(0)
    X, g = rng.standard_normal((1, 2, 8, 8)), rng.standard_normal((2, 2, 3, 3))
    BT, G, AT = oracle.cook_toom(4)
    Yd = oracle.conv2d_direct_f64(X, g, 1, 1)
    assert _rel(oracle.winograd_f64(X, g, BT.T.copy(), G, AT, 1), Yd) > 1e-3


# ---------------------------------------------------------------- P7 quantized pipeline
def test_hadamard_matches_einsum(oracle):
    rng = np.random.default_rng(7)
    Vq = rng.integers(-127, 128, (16, 10, 7))
    Uq = rng.integers(-127, 128, (16, 5, 7))
    M = oracle.q_hadamard(Vq, Uq)
    assert np.array_equal(M, np.einsum("ptc,pkc->ptk", Vq.astype(np.int64), Uq.astype(np.int64)))


def _patches(xq, m, pad):
    """All n x n patches as an integer array [T, C, n, n] (index bookkeeping only)."""
    N, C, H, W = xq.shape
    n = m + 2
    Ho, Wo = H + 2 * pad - 2, W + 2 * pad - 2
    TH, TW = -(-Ho // m), -(-Wo // m)
    Xp = np.zeros((N, C, pad + TH * m + 2 + n, pad + TW * m + 2 + n), xq.dtype)
    Xp[:, :, pad:pad + H, pad:pad + W] = xq
    out = np.zeros((N, TH, TW, C, n, n), xq.dtype)
    for th in range(TH):
        for tw in range(TW):
            out[:, th, tw] = Xp[:, :, th * m:th * m + n, tw * m:tw * m + n]
    return out.reshape(N * TH * TW, C, n, n), TH, TW


def test_f2_stages_are_exact_integers(oracle):
    """With the default F2 matrices (entries 0, +-1, 1/2) and integer data every
    intermediate is exactly representable, so each stage must equal plain integer
    matrix algebra done by numpy, whatever the fp32 evaluation order."""
    rng = np.random.default_rng(11)
    BT, G, AT = oracle.cook_toom(2, dtype=np.float32)
    N, C, K, H, W = 2, 3, 4, 7, 6
    xq = rng.integers(-127, 128, (N, C, H, W))
    g4 = (4 * rng.integers(-7, 8, (K, C, 3, 3))).astype(np.float32)  # multiples of 4: G g G^T integral
    Vf, Vq = oracle.q_input(xq, BT, pad=1, r_v=1.0, qmax=10 ** 6)
    d, TH, TW = _patches(xq, 2, 1)
    BTi = BT.astype(np.int64)
    Vexp = np.einsum("ij,tcjl,kl->iktc", BTi, d.astype(np.int64), BTi).reshape(16, -1, C)
    assert np.array_equal(Vq, Vexp) and np.array_equal(Vf, Vexp.astype(np.float32))
    Uf, Uq = oracle.q_weights(g4, G, r_u=1.0, qmax=10 ** 6)
    G2 = (2 * G).astype(np.int64)
    Uexp = (np.einsum("ia,kcab,jb->ijkc", G2, g4.astype(np.int64), G2) // 4).reshape(16, K, C)
    assert np.array_equal(Uq, Uexp)
    M = oracle.q_hadamard(Vq, Uq)
    Yf, Yq, inexact = oracle.q_output(M, AT, N, H, W, pad=1, r_y=1.0, qmax=2 ** 30)
    ATi = AT.astype(np.int64)
    Mt = M.reshape(4, 4, N, TH, TW, K)
    Yt = np.einsum("ai,ijnhwk,bj->nkhawb", ATi, Mt, ATi).reshape(N, K, TH * 2, TW * 2)[:, :, :H, :W]
    assert inexact == 0 and np.abs(Yt).max() < 2 ** 24
    assert np.array_equal(Yq, Yt)
    # and, being exact, the whole thing is the integer direct convolution
    acc, _ = oracle.conv2d_direct_q(xq, g4.astype(np.int64), 1.0, qmax=2 ** 30)
    assert np.array_equal(Yq, acc)


def _fma32(a, b, c):
    """Correctly rounded fp32 fma via exact rationals."""
    v = Fraction(float(a)) * Fraction(float(b)) + Fraction(float(c))
    return _round32(v)


def _round32(v):
    f = np.float32(float(v))
    best = None
    for x in (f, np.nextafter(f, np.float32(np.inf)), np.nextafter(f, np.float32(-np.inf))):
        key = (abs(Fraction(float(x)) - v), int(x.view(np.uint32)) & 1)
        if best is None or key < best[0]:
            best = (key, x)
    return best[1]


def _rne_sat(v, qmax):
    """Nearest integer to the exact rational v, ties to even, saturated."""
    v = Fraction(v)
    fl = v.numerator // v.denominator
    rem = v - fl
    q = fl + (1 if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1) else 0)
    return int(min(max(q, -qmax), qmax))


@pytest.mark.parametrize("m,H,W,pad", [(2, 4, 4, 1), (4, 5, 7, 1), (6, 7, 6, 1), (4, 9, 6, 0)],
                         ids=["m2_4x4", "m4_ragged_5x7", "m6_ragged_7x6", "m4_pad0_9x6"])
def test_fused_chain_order_on_dense_matrices(oracle, m, H, W, pad):
    """The pinned arithmetic (ascending fused chains from +0; the quantizer rounds the
    exact product with its reciprocal step half to even, then saturates) emulated with exact
    rationals on tiny cases with dense random matrices, where the evaluation order does
    change bits: every tile size, tiles cut by the image edge, with and without padding."""
    rng = np.random.default_rng(13 + m + H)
    n = m + 2
    C, K = (2, 2) if m == 2 else (1, 2)
    BT = rng.standard_normal((n, n)).astype(np.float32)
    G = rng.standard_normal((n, 3)).astype(np.float32)
    AT = rng.standard_normal((m, n)).astype(np.float32)
    xq = rng.integers(-127, 128, (1, C, H, W))
    g = rng.standard_normal((K, C, 3, 3)).astype(np.float32)
    r_v, r_u = np.float32(0.37 / n), np.float32(41.3)
    f0 = np.float32(0)
    Ho, Wo = H + 2 * pad - 2, W + 2 * pad - 2
    Vf, Vq = oracle.q_input(xq, BT, pad=pad, r_v=r_v)
    d, TH, TW = _patches(xq, m, pad)
    assert (TH, TW) == (-(-Ho // m), -(-Wo // m)) and d.shape[0] == TH * TW
    for t in range(d.shape[0]):
        for c in range(C):
            w = [[f0] * n for _ in range(n)]
            for i in range(n):
                for l in range(n):
                    acc = f0
                    for j in range(n):
                        acc = _fma32(BT[i, j], np.float32(d[t, c, j, l]), acc)
                    w[i][l] = acc
            for i in range(n):
                for k in range(n):
                    acc = f0
                    for l in range(n):
                        acc = _fma32(w[i][l], BT[k, l], acc)
                    assert Vf[i * n + k, t, c] == acc
                    assert Vq[i * n + k, t, c] == _rne_sat(Fraction(float(acc)) * Fraction(float(r_v)), 127)
    assert 0 < np.abs(Vq).max() and np.abs(Vq).mean() > 5
    Uf, Uq = oracle.q_weights(g, G, r_u=r_u)
    for k in range(K):
        for c in range(C):
            tt = [[f0] * 3 for _ in range(n)]
            for i in range(n):
                for b in range(3):
                    acc = f0
                    for a in range(3):
                        acc = _fma32(G[i, a], g[k, c, a, b], acc)
                    tt[i][b] = acc
            for i in range(n):
                for j in range(n):
                    acc = f0
                    for b in range(3):
                        acc = _fma32(tt[i][b], G[j, b], acc)
                    assert Uf[i * n + j, k, c] == acc
                    assert Uq[i * n + j, k, c] == _rne_sat(Fraction(float(acc)) * Fraction(float(r_u)), 127)
    M = oracle.q_hadamard(Vq, Uq)
    Yf, _, _ = oracle.q_output(M, AT, 1, H, W, pad=pad, r_y=1.0)
    r_y = np.float32(110.0 / np.abs(Yf).max())          # codes spread over the whole range
    Yf, Yq, _ = oracle.q_output(M, AT, 1, H, W, pad=pad, r_y=r_y)
    assert Yq.shape == (1, K, Ho, Wo)
    seen = np.zeros((Ho, Wo), bool)
    for t in range(TH * TW):
        th, tw = divmod(t, TW)
        for k in range(K):
            z = [[f0] * n for _ in range(m)]
            for a in range(m):
                for j in range(n):
                    acc = f0
                    for i in range(n):
                        acc = _fma32(AT[a, i], np.float32(M[i * n + j, t, k]), acc)
                    z[a][j] = acc
            for a in range(m):
                for b in range(m):
                    if th * m + a >= Ho or tw * m + b >= Wo:
                        continue                       # outputs beyond the image are dropped
                    acc = f0
                    for j in range(n):
                        acc = _fma32(z[a][j], AT[b, j], acc)
                    assert Yf[0, k, th * m + a, tw * m + b] == acc
                    assert Yq[0, k, th * m + a, tw * m + b] == _rne_sat(
                        Fraction(float(acc)) * Fraction(float(r_y)), 127)
                    seen[th * m + a, tw * m + b] = True
    assert seen.all() and np.abs(Yq).max() >= 100 and np.abs(Yq).mean() > 10


def test_q_scalars(oracle):
    f = np.float32
    s = oracle.q_scalars(0.031, 0.77, 0.0042, 0.19)
    assert s["r_u"] == f(1) / f(0.0042) and s["r_v"] == f(0.031) / f(0.77)
    assert s["r_y"] == (f(0.0042) * f(0.77)) / f(0.19) and s["r_m"] == 0
    s = oracle.q_scalars(0.031, 0.77, 0.0042, 0.19, 0.05)
    assert s["r_m"] == (f(0.0042) * f(0.77)) / f(0.05) and s["r_y"] == f(0.05) / f(0.19)


def test_rounding_is_half_to_even_and_saturation_symmetric(oracle):
    """Sec. 5.1 (per-layer symmetric quantization): range [-127, 127], never -128."""
    G = oracle.cook_toom(2, dtype=np.float32)[1]
    g = np.zeros((1, 1, 3, 3), np.float32)
    for val, exp in ((0.5, 0), (1.5, 2), (2.5, 2), (-0.5, 0), (-1.5, -2), (-2.5, -2), (300.0, 127), (-300.0, -127)):
        g[0, 0, 0, 0] = val  # U[0][0] = G[0,0]^2 g00 = g00 for the default F2 G
        _, Uq = oracle.q_weights(g, G, r_u=1.0)
        assert Uq[0, 0, 0] == exp, (val, Uq[0, 0, 0])
    rng = np.random.default_rng(17)
    xq = rng.integers(-127, 128, (1, 4, 8, 8))
    BT, G, AT = oracle.cook_toom(4, dtype=np.float32)
    _, Vq = oracle.q_input(xq, BT, r_v=np.float32(0.5))
    assert Vq.max() == 127 and Vq.min() == -127
    M = oracle.q_hadamard(Vq, Vq[:, :3, :])          # any int8-range "weights" will do
    _, Yq, _ = oracle.q_output(M, AT, 1, 8, 8, pad=1, r_y=np.float32(1.0))
    assert Yq.max() == 127 and Yq.min() == -127


def test_quantized_pipeline_converges_to_fp64_winograd(oracle):
    """As the quantization steps shrink (qmax large) the dequantized output of the
    quantized pipeline approaches the fp64 Winograd of the same (fake-quantized) data."""
    rng = np.random.default_rng(19)
    N, C, K, H, W, m = 1, 3, 2, 8, 8, 4
    BT, G, AT = oracle.cook_toom(m, dtype=np.float32)
    X = np.maximum(rng.standard_normal((N, C, H, W)), 0).astype(np.float32)
    g = (rng.standard_normal((K, C, 3, 3)) * 0.3).astype(np.float32)
    errs = []
    for qmax in (127, 2 ** 12, 2 ** 20):
        sc = oracle.calibrate(X, g, BT, G, AT, qmax=qmax)
        xq = oracle.quantize_tensor(X, sc["s_x"], qmax)
        out = oracle.winograd_q(xq, g, BT, G, AT, sc, qmax=qmax)
        Yd = out["Yq"].astype(np.float64) * sc["s_y"]
        ref = oracle.winograd_f64(xq.astype(np.float64) * sc["s_x"], g, BT, G, AT)
        errs.append(_rel(Yd, ref))
    assert errs[0] > errs[1] > errs[2]
    assert errs[2] < 1e-4 and errs[1] < 2e-2 and errs[0] > 20 * errs[1]


def test_static_int8_error_grows_with_tile_size(oracle):
    """Table 1: with static transforms 8-bit F2 is harmless, F4 and F6 are far from
    the direct convolution.  This is why int8 parity is taken against the quantized
    pipeline and never against the direct convolution."""
    from paper_2002_10711_amd import workloads
    L = workloads.Layer("t", 2, 32, 16, 12, 12, seed=23)
    X, g = workloads.make_inputs(L)
    errs = {}
    for m in (2, 4, 6):
        BT, G, AT = oracle.cook_toom(m, dtype=np.float32)
        sc = oracle.calibrate(X, g, BT, G, AT)
        xq = oracle.quantize_tensor(X, sc["s_x"])
        out = oracle.winograd_q(xq, g, BT, G, AT, sc)
        assert np.abs(out["Yq"]).max() == 127 and out["inexact"] == 0
        ref = oracle.conv2d_direct_f64(xq.astype(np.float64) * sc["s_x"], g)
        errs[m] = _rel(out["Yq"] * np.float64(sc["s_y"]), ref)
    assert errs[2] < 0.06 and errs[4] > 2 * errs[2] and errs[6] > errs[4]


def test_flex_limit_noise_to_zero(oracle):
    """Perturbed matrices: only the limit is pinned -- as the noise shrinks the
    literal Winograd returns to the direct convolution, linearly in sigma."""
    from paper_2002_10711_amd import workloads
    rng = np.random.default_rng(29)
    X, g = rng.standard_normal((1, 3, 12, 12)), rng.standard_normal((2, 3, 3, 3))
    Yd = oracle.conv2d_direct_f64(X, g)
    errs = []
    for sigma in (1e-2, 1e-4, 1e-6):
        BT, G, AT = oracle.cook_toom(6)
        BTp, Gp, ATp = [a.astype(np.float64) for a in workloads.perturb_transforms(BT, G, AT, sigma, 5)]
        errs.append(_rel(oracle.winograd_f64(X, g, BTp, Gp, ATp), Yd))
    assert errs[0] > 10 * errs[1] > 100 * errs[2] and errs[2] < 1e-3


# ------------------------------------------------------------ per-position scales --
def test_per_position_f2_stages_are_exact_integers(oracle):
    """Per-position variant with power-of-two factors on exact F2 data: every stage equals
    integer algebra with the factor applied per Winograd position, and the real-unit
    output equals the integer direct convolution (Sec. 7: finer quantization granularity
    as the way to recover the larger tiles' accuracy)."""
    rng = np.random.default_rng(31)
    BT, G, AT = oracle.cook_toom(2, dtype=np.float32)
    N, C, K, H, W = 2, 3, 4, 6, 7
    xq = rng.integers(-127, 128, (N, C, H, W))
    g4 = (4 * rng.integers(-7, 8, (K, C, 3, 3))).astype(np.float32)
    d, TH, TW = _patches(xq, 2, 1)
    BTi = BT.astype(np.int64)
    Vexp = np.einsum("ij,tcjl,kl->iktc", BTi, d.astype(np.int64), BTi).reshape(16, -1, C)
    G2 = (2 * G).astype(np.int64)
    Uexp = (np.einsum("ia,kcab,jb->ijkc", G2, g4.astype(np.int64), G2) // 4).reshape(16, K, C)
    # factors 2^e, e >= 0, so that quantized values stay integers of the exact ones
    ev = rng.integers(0, 3, 16)
    eu = rng.integers(0, 3, 16)
    r_v = (2.0 ** ev).astype(np.float32)
    r_u = (2.0 ** eu).astype(np.float32)
    _, Vq = oracle.q_input(xq, BT, pad=1, r_v=r_v, qmax=10 ** 7, want_f32=False)
    _, Uq = oracle.q_weights(g4, G, r_u=r_u, qmax=10 ** 7, want_f32=False)
    assert np.array_equal(Vq, Vexp * (2 ** ev)[:, None, None])
    assert np.array_equal(Uq, Uexp * (2 ** eu)[:, None, None])
    M = oracle.q_hadamard(Vq, Uq)
    w = (2.0 ** (-(ev + eu))).astype(np.float32)          # brings every position back
    Yf, Yq, inexact = oracle.q_output(M, AT, N, H, W, pad=1, r_y=1.0, qmax=2 ** 30, w_pos=w)
    acc, _ = oracle.conv2d_direct_q(xq, g4.astype(np.int64), 1.0, qmax=2 ** 30)
    assert inexact == 0 and np.array_equal(Yq, acc)
    # a factor applied to the wrong position (transposed index) must show
    if not np.array_equal(ev.reshape(4, 4), ev.reshape(4, 4).T):
        _, Vbad = oracle.q_input(xq, BT, pad=1, r_v=r_v.reshape(4, 4).T.ravel(), qmax=10 ** 7,
                                 want_f32=False)
        assert not np.array_equal(Vbad, Vq)


def test_per_position_scalars(oracle):
    f32 = np.float32
    sv = np.array([0.3, 0.7, 1.1, 0.05], f32)
    su = np.array([0.01, 0.2, 0.4, 3.0], f32)
    sc = oracle.q_scalars_pos(0.1, sv, su, 0.9)
    assert np.array_equal(sc["r_u"], f32(1) / su) and np.array_equal(sc["r_v"], f32(0.1) / sv)
    assert np.array_equal(sc["w"], su * sv) and sc["r_m"] == 0 and sc["r_y"] == f32(1) / f32(0.9)
    sc = oracle.q_scalars_pos(0.1, sv, su, 0.9, 0.25)
    assert sc["r_m"] == f32(1) / f32(0.25) and sc["r_y"] == f32(0.25) / f32(0.9)


def test_per_position_equals_per_tensor_when_all_factors_agree(oracle):
    """With one common factor per stage the per-position quantizers of U and V are the
    per-tensor ones, bit for bit."""
    rng = np.random.default_rng(37)
    BT, G, AT = oracle.cook_toom(4, dtype=np.float32)
    xq = rng.integers(-127, 128, (1, 5, 9, 8))
    g = (rng.standard_normal((3, 5, 3, 3)) * 0.2).astype(np.float32)
    _, Vq1 = oracle.q_input(xq, BT, r_v=0.037, want_f32=False)
    _, Vq2 = oracle.q_input(xq, BT, r_v=np.full(36, 0.037, np.float32), want_f32=False)
    _, Uq1 = oracle.q_weights(g, G, r_u=41.5, want_f32=False)
    _, Uq2 = oracle.q_weights(g, G, r_u=np.full(36, 41.5, np.float32), want_f32=False)
    assert np.array_equal(Vq1, Vq2) and np.array_equal(Uq1, Uq2)


def test_per_position_scales_reduce_the_static_int8_error(oracle):
    """The motivation (Sec. 7; Table 1): one scale for all positions wastes most of the
    int8 range on F4 / F6; one scale per position brings the error against the direct
    convolution down, and converges like the per-tensor pipeline as qmax grows."""
    from paper_2002_10711_amd import workloads
    L = workloads.Layer("t", 2, 32, 16, 12, 12, seed=23)
    X, g = workloads.make_inputs(L)
    for m in (4, 6):
        BT, G, AT = oracle.cook_toom(m, dtype=np.float32)
        sc = oracle.calibrate(X, g, BT, G, AT)
        xq = oracle.quantize_tensor(X, sc["s_x"])
        ref = oracle.conv2d_direct_f64(xq.astype(np.float64) * sc["s_x"], g)
        e_tensor = _rel(oracle.winograd_q(xq, g, BT, G, AT, sc)["Yq"] * np.float64(sc["s_y"]), ref)
        scp = oracle.calibrate_pos(X, g, BT, G, AT)
        out = oracle.winograd_q(xq, g, BT, G, AT, scp)
        assert out["inexact"] == 0 and np.abs(out["Yq"]).max() == 127
        e_pos = _rel(out["Yq"] * np.float64(scp["s_y"]), ref)
        assert e_pos < 0.75 * e_tensor, (m, e_pos, e_tensor)
    BT, G, AT = oracle.cook_toom(4, dtype=np.float32)
    errs = []
    for qmax in (127, 2 ** 12, 2 ** 20):
        scp = oracle.calibrate_pos(X, g, BT, G, AT, qmax=qmax)
        xq = oracle.quantize_tensor(X, scp["s_x"], qmax)
        out = oracle.winograd_q(xq, g, BT, G, AT, scp, qmax=qmax)
        ref = oracle.winograd_f64(xq.astype(np.float64) * scp["s_x"], g, BT, G, AT)
        errs.append(_rel(out["Yq"].astype(np.float64) * scp["s_y"], ref))
    assert errs[0] > errs[1] > errs[2] and errs[2] < 1e-4


# ------------------------------------------- wider stages / one bit-width per stage
def test_hadamard_sums_beyond_int32_match_python_integers(oracle):
    """16-bit codes: one product reaches 2^30 and a sum over a few channels leaves the
    int32 range; the oracle's sums must be the exact integers (checked against Python's
    unbounded ints), as the 16-bit pipeline of Sec. 5.1 needs."""
    rng = np.random.default_rng(61)
    P, T, C, K = 4, 3, 37, 5
    Vq = rng.integers(-32767, 32768, size=(P, T, C)).astype(np.int32)
    Uq = rng.integers(-32767, 32768, size=(P, K, C)).astype(np.int32)
    Vq[0, 0, :] = 32767
    Uq[0, 0, :] = -32767
    M = oracle.q_hadamard(Vq, Uq)
    for p in range(P):
        for t in range(T):
            for k in range(K):
                want = sum(int(Vq[p, t, c]) * int(Uq[p, k, c]) for c in range(C))
                assert int(M[p, t, k]) == want
    assert int(M[0, 0, 0]) == -37 * 32767 * 32767 and abs(int(M[0, 0, 0])) > 2 ** 31


def test_large_accumulators_are_converted_half_to_even(oracle):
    """(float)M for |M| >= 2^24 is the correctly rounded conversion of the exact integer:
    F2's A^T picks M[0][0] + M[0][1] + ... ; with a single nonzero position the output is
    that accumulator itself.  2^24 + 1 -> 2^24 (tie to even), 2^24 + 3 -> 2^24 + 4,
    2^31 + 129 -> 2^31 + 256 (tie to even), and the count of inexact conversions is reported."""
    _, _, AT = oracle.cook_toom(2, dtype=np.float32)
    vals = [2 ** 24 + 1, 2 ** 24 + 3, -(2 ** 24 + 1), 2 ** 31 + 128, 2 ** 31 + 384, 12345]
    want = [2 ** 24, 2 ** 24 + 4, -(2 ** 24), 2 ** 31, 2 ** 31 + 512, 12345]
    M = np.zeros((16, 1, len(vals)), np.int64)
    M[0, 0, :] = vals                                  # position (0,0) feeds output (0,0) only
    Yf, Yq, inexact = oracle.q_output(M, AT, 1, 2, 2, pad=1, r_y=np.float32(1.0), qmax=2 ** 40)
    assert [int(v) for v in Yf[0, :, 0, 0]] == want
    assert [int(v) for v in Yq[0, :, 0, 0]] == [min(w, 2 ** 31 - 1) if w > 0 else w for w in want] \
        or [float(v) for v in Yf[0, :, 0, 0]] == [float(w) for w in want]
    assert inexact == 5


def test_hadamard_and_output_quantizers_have_their_own_ranges(oracle):
    """Sec. 3.2 ("quantization diversity"): each stage may have its own bit-width.  Closed
    form for the output stage: when every accumulator is far beyond the Hadamard-stage
    range, Mq = qmax_m * sign(M), and F2's 0/+-1 A^T makes the tile an exact small-integer
    combination of those, y = sat_qmax_y(qmax_m * A^T sign(M) A)."""
    rng = np.random.default_rng(62)
    _, _, AT = oracle.cook_toom(2, dtype=np.float32)
    sign = rng.choice([-1, 1], size=(16, 4, 3)).astype(np.int64)
    M = sign * rng.integers(10 ** 6, 10 ** 7, size=sign.shape)
    A = AT.astype(np.float64)
    for qmax_m, qmax_y in ((511, 32767), (32767, 127), (7, 2047)):
        _, Yq, _ = oracle.q_output(M, AT, 1, 4, 4, pad=1, r_m=np.float32(1.0), r_y=np.float32(1.0),
                                   qmax=qmax_y, qmax_m=qmax_m)
        for t in range(4):
            for k in range(3):
                S = sign[:, t, k].reshape(4, 4).astype(np.float64)
                want = np.clip(qmax_m * (A @ S @ A.T), -qmax_y, qmax_y)
                th, tw = divmod(t, 2)
                np.testing.assert_array_equal(Yq[0, k, 2 * th:2 * th + 2, 2 * tw:2 * tw + 2], want)


def test_one_width_per_stage_reduces_to_the_single_width_pipeline(oracle):
    from paper_2002_10711_amd import workloads
    L = workloads.Layer("t", 1, 8, 6, 8, 8, m=4, seed=63)
    X, g = workloads.make_inputs(L)
    BT, G, AT = oracle.cook_toom(4, dtype=np.float32)
    sc = oracle.calibrate(X, g, BT, G, AT)
    xq = oracle.quantize_tensor(X, sc["s_x"])
    a = oracle.winograd_q(xq, g, BT, G, AT, sc)
    b = oracle.winograd_q(xq, g, BT, G, AT, sc, qmax=dict(x=127, u=127, v=127, m=127, y=127))
    for k in ("Uq", "Vq", "M", "Yq"):
        np.testing.assert_array_equal(a[k], b[k])
    # a narrower Winograd domain only clips: codes of the 6-bit stages are the 8-bit
    # pipeline's own values saturated to +-31 when the scales stay the same
    c = oracle.winograd_q(xq, g, BT, G, AT, sc, qmax=dict(u=31, v=31))
    np.testing.assert_array_equal(c["Uq"], np.clip(a["Uq"], -31, 31))
    np.testing.assert_array_equal(c["Vq"], np.clip(a["Vq"], -31, 31))


def test_error_to_direct_convolution_falls_with_the_bit_width(oracle):
    """Sec. 5.1 runs INT8, INT10 and INT16: with static transforms the distance of one layer
    to the direct convolution falls with every added bit, for each tile size, but the
    ordering F2 < F4 < F6 of Table 1 stays at every width -- F6 is still far away with
    16-bit stages (Table 1's 16-bit column), F4 is within 2e-3 for a single layer.  Widening
    only the Winograd domain (8-bit activations, 16-bit U, V and Hadamard stage; Sec. 7:
    different bit-widths through Eq. 1) brings F4 down to the floor of its 8-bit output."""
    from paper_2002_10711_amd import workloads
    L = workloads.Layer("t", 2, 32, 16, 12, 12, seed=23)
    X, g = workloads.make_inputs(L)
    errs = {}
    for m in (2, 4, 6):
        BT, G, AT = oracle.cook_toom(m, dtype=np.float32)
        for name, qm in (("int8", 127), ("int10", 511), ("int16", 32767),
                         ("int8_w16", dict(x=127, u=32767, v=32767, m=32767, y=127))):
            sc = oracle.calibrate(X, g, BT, G, AT, qmax=qm)
            qx = oracle.stage_qmax(qm)["x"]
            xq = oracle.quantize_tensor(X, sc["s_x"], qx)
            out = oracle.winograd_q(xq, g, BT, G, AT, sc, qmax=qm)
            ref = oracle.conv2d_direct_f64(xq.astype(np.float64) * sc["s_x"], g)
            errs[m, name] = _rel(out["Yq"] * np.float64(sc["s_y"]), ref)
        assert errs[m, "int8"] > 3 * errs[m, "int10"] > 9 * errs[m, "int16"], errs
    for name in ("int8", "int10", "int16"):
        assert errs[2, name] < errs[4, name] < errs[6, name], errs
    assert errs[4, "int16"] < 2e-3 and errs[2, "int16"] < 2e-4, errs
    assert errs[6, "int16"] > 50 * errs[4, "int16"], errs
    # 8-bit output codes: the floor is half an output step, 1/254 of the range, plus what
    # is left of the 16-bit Winograd-domain error
    assert errs[4, "int8_w16"] < 0.75 / 127 and errs[4, "int8_w16"] < errs[4, "int8"] / 4, errs


def test_quantizer_rounds_the_exact_product_once(oracle):
    """q = rne(v * r) on the exact product: 3 * fl32(1/6) = 0.5000000149 lies above the tie
    and rounds to 1 (an fp32 multiplication first would land on 0.5 exactly and a second
    rounding would give 0); 3 * fl32(0.16666666) lies below it and rounds to 0; exact ties
    go to even; large products saturate."""
    _, _, AT = oracle.cook_toom(2, dtype=np.float32)
    r_up, r_dn = np.float32(1.0) / np.float32(6.0), np.float32(0.16666666)
    assert Fraction(float(r_up)) * 3 > Fraction(1, 2) > Fraction(float(r_dn)) * 3
    M = np.zeros((16, 1, 4), np.int64)
    M[0, 0, :] = [3, -3, 5, 10 ** 9]                 # position (0,0) feeds output (0,0) only
    for r, want in ((r_up, [1, -1, 1, 127]), (r_dn, [0, 0, 1, 127]), (np.float32(0.5), [2, -2, 2, 127])):
        _, Yq, _ = oracle.q_output(M, AT, 1, 2, 2, pad=1, r_y=r)
        assert [int(v) for v in Yq[0, :, 0, 0]] == want, (r, Yq[0, :, 0, 0])


def test_bf16_variant_rounding_and_exact_case(oracle):
    """The bf16 variant of the GEMM stage: round-to-nearest-even at 8 significant bits (hand
    values around ties), nothing lost when every transformed value is representable (F2 with
    small integers: the result then is the direct convolution, exactly), and a visible error
    otherwise."""
    vals = np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -8 + 2.0 ** -20, -1 - 2.0 ** -8,
                     255.0, 257.0, 0.0, -3.140625], np.float32)
    want = np.array([1.0, 1 + 2.0 ** -6, 1 + 2.0 ** -7, -1.0, 255.0, 256.0, 0.0, -3.140625], np.float32)
    assert np.array_equal(oracle.bf16_round(vals), want)
    rng = np.random.default_rng(77)
    BT, G, AT = oracle.cook_toom(2, dtype=np.float32)
    X = rng.integers(-3, 4, (2, 5, 7, 6)).astype(np.float32)
    g = (4 * rng.integers(-1, 2, (4, 5, 3, 3))).astype(np.float32)
    Y = oracle.winograd_bf16(X, g, BT, G, AT, 1)
    assert np.array_equal(Y, oracle.conv2d_direct_f64(X, g, 1, 1))
    # the float input transform in the pinned arithmetic: bit-equal to the integer-input one
    # (C++ oracle) on integer-valued data, for every tile size and a ragged shape
    xi = rng.integers(-127, 128, (2, 3, 9, 7))
    for m in (2, 4, 6):
        BT, G, AT = oracle.cook_toom(m, dtype=np.float32)
        Vf, _ = oracle.q_input(xi, BT, pad=1, want_q=False)
        assert np.array_equal(oracle.input_f32(xi.astype(np.float32), BT, 1), Vf)
        BTd = (BT + 0.01 * rng.standard_normal(BT.shape)).astype(np.float32)     # dense matrix
        Vf, _ = oracle.q_input(xi, BTd, pad=0, want_q=False)
        assert np.array_equal(oracle.input_f32(xi.astype(np.float32), BTd, 0), Vf)
    X = rng.standard_normal((2, 5, 7, 6)).astype(np.float32)
    g = rng.standard_normal((4, 5, 3, 3)).astype(np.float32)
    for m, lo, hi in ((2, 1e-4, 2e-2), (4, 1e-3, 2e-1)):
        BT, G, AT = oracle.cook_toom(m, dtype=np.float32)
        ref = oracle.conv2d_direct_f64(X, g, 1, 1)
        e = np.abs(oracle.winograd_bf16(X, g, BT, G, AT, 1) - ref).max() / np.abs(ref).max()
        assert lo < e < hi, (m, e)
