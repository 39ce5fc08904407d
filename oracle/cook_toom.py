"""Cook-Toom construction of the Winograd transform matrices (oracle side).

TEST INFRASTRUCTURE.  This file belongs to the CPU oracle: it is imported only by
the tests, by the smoke check and by the CPU-baseline leg of the benchmark.  It
shares no code with the HIP library and never imports it.

What it follows.  Section 3.1 of the paper states the matrix form (Eq. 1)

    Y = A^T [ (G g G^T) (.) (B^T d B) ] A

and says the three matrices are built by the Cook-Toom algorithm from a set of
polynomial points (it points to Blahut, Sec. 5.2, for the recipe; it prints no
matrices).  The construction below is the Lagrange-interpolation derivation of a
minimal FIR algorithm F(m, r), r = 3, n = m + r - 1 evaluation points of which the
last is the point at infinity:

  * the filter g(x) = g0 + g1 x + g2 x^2 and the wanted outputs
    y_a = sum_b d_{a+b} g_b are the middle coefficients of a polynomial product;
    evaluating at n points, multiplying point-wise and interpolating back is exact;
  * for a finite point p_i let M_i(x) = prod_{j != i} (x - p_j) over the finite
    points and N_i = M_i(p_i).  Row i of the three matrices is
        B^T[i, :] = sign(N_i) * coefficients of M_i(x), ascending powers
        G[i, b]   = p_i^b / |N_i|
        A^T[a, i] = p_i^a
  * the point at infinity gives the row
        B^T[n-1, :] = coefficients of M(x) = prod_j (x - p_j)
        G[n-1, :]   = (0, 0, 1)
        A^T[:, n-1] = unit vector e_{m-1}.

The scaling of a row (where the 1/N_i goes, and its sign) is a free choice: any
rescaling (B^T_i, G_i, A^T_{.i}) -> (a B^T_i, b G_i, A^T_{.i}/(ab)) is again a
Winograd algorithm.  The choice here puts every denominator into G and makes the
leading entry of every G row positive.

Everything is computed in exact rational arithmetic (fractions.Fraction) and only
rounded at the very end, so the fp64 / fp32 matrices are the correctly rounded
values of the exact ones.
"""
from fractions import Fraction

import numpy as np

# Polynomial points used by the workloads, in the order the rows are laid out.
# The paper says there is a consensus for small tiles but lists none; these are
# the sets the workload definitions name (0, +-1, +-1/2, +-2), infinity implied.
DEFAULT_POINTS = {
    2: (Fraction(0), Fraction(1), Fraction(-1)),
    4: (Fraction(0), Fraction(1), Fraction(-1), Fraction(1, 2), Fraction(-1, 2)),
    6: (Fraction(0), Fraction(1), Fraction(-1), Fraction(1, 2), Fraction(-1, 2),
        Fraction(2), Fraction(-2)),
}


def _poly_mul_linear(coeffs, root):
    """coeffs(x) * (x - root); coefficients in ascending powers."""
    out = [Fraction(0)] * (len(coeffs) + 1)
    for k, c in enumerate(coeffs):
        out[k + 1] += c
        out[k] -= c * root
    return out


def cook_toom_exact(m, points=None, r=3):
    """Exact (Fraction) matrices B^T (n x n), G (n x r), A^T (m x n), n = m + r - 1."""
    n = m + r - 1
    if points is None:
        points = DEFAULT_POINTS[m]
    pts = [Fraction(p) for p in points]
    if len(pts) != n - 1:
        raise ValueError("F(%d,%d) needs %d finite points" % (m, r, n - 1))
    if len(set(pts)) != len(pts):
        raise ValueError("polynomial points must be distinct")

    BT = [[Fraction(0)] * n for _ in range(n)]
    G = [[Fraction(0)] * r for _ in range(n)]
    AT = [[Fraction(0)] * n for _ in range(m)]

    for i, p in enumerate(pts):
        Mi = [Fraction(1)]
        for j, q in enumerate(pts):
            if j != i:
                Mi = _poly_mul_linear(Mi, q)
        Ni = sum(c * p ** k for k, c in enumerate(Mi))
        sgn = 1 if Ni > 0 else -1
        for k, c in enumerate(Mi):
            BT[i][k] = sgn * c
        for b in range(r):
            G[i][b] = p ** b / abs(Ni)
        for a in range(m):
            AT[a][i] = p ** a

    Mfull = [Fraction(1)]
    for q in pts:
        Mfull = _poly_mul_linear(Mfull, q)
    for k, c in enumerate(Mfull):
        BT[n - 1][k] = c
    G[n - 1][r - 1] = Fraction(1)
    AT[m - 1][n - 1] = Fraction(1)
    return BT, G, AT


def _to_array(rows, dtype):
    # Fraction -> float is correctly rounded (CPython converts the exact ratio);
    # fp32 values are obtained by rounding the exact value once, not the fp64 one
    # twice: go through a float64 only when that is exact enough to be harmless,
    # which it is not in general, so round explicitly.
    out = np.empty((len(rows), len(rows[0])), dtype=dtype)
    for i, row in enumerate(rows):
        for j, v in enumerate(row):
            out[i, j] = _round_fraction(v, dtype)
    return out


def _round_fraction(v, dtype):
    if dtype == np.float64:
        return float(v)
    # fp32: nearest-even rounding of the exact rational.  Compare the two fp32
    # neighbours of the fp64 approximation against the exact value.
    f64 = float(v)
    c = np.float32(f64)
    cands = {float(c), float(np.nextafter(c, np.float32(np.inf))),
             float(np.nextafter(c, np.float32(-np.inf)))}
    best = None
    for x in cands:
        err = abs(Fraction(x) - v)
        mant_even = (np.float32(x).view(np.uint32) & 1) == 0
        key = (err, 0 if mant_even else 1)
        if best is None or key < best[0]:
            best = (key, x)
    return np.float32(best[1])


def cook_toom(m, points=None, dtype=np.float64):
    """B^T, G, A^T as numpy arrays of the requested floating type."""
    BT, G, AT = cook_toom_exact(m, points)
    return _to_array(BT, dtype), _to_array(G, dtype), _to_array(AT, dtype)
