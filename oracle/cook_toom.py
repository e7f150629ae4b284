"""Exact Cook-Toom construction of the Winograd transforms (test oracle).

Test infrastructure only; see the package docstring.

Everything in this module works on `fractions.Fraction` so that no rounding
takes place before the caller asks for floating-point tables.

Conventions (Sec. 2.1 "Winograd Convolution via Cook-Toom"):
    F(m, r) computes m outputs  y_i = sum_k g_k x_{i+k}  (a correlation, no
    kernel flip) from n = m + r - 1 inputs with n multiplications,
        y = A^T [ (G g) * (B^T x) ],
    using n - 1 finite interpolation points alpha_0 .. alpha_{n-2} and the point
    at infinity.  Row p of A (n x m), B^T (n x n) and G (n x r) belongs to
    alpha_p; the last row belongs to infinity.
"""
from fractions import Fraction

import numpy as np


def _as_fractions(points):
    return [Fraction(p) for p in points]


def poly_from_roots(roots):
    """Coefficients (ascending powers) of prod_j (t - root_j), exactly."""
    coeffs = [Fraction(1)]
    for root in roots:
        nxt = [Fraction(0)] * (len(coeffs) + 1)
        for power, c in enumerate(coeffs):
            nxt[power + 1] += c          # t * c t^power
            nxt[power] -= root * c       # -root * c t^power
        coeffs = nxt
    return coeffs


def cook_toom(points, m, r=3):
    """A (n x m), B^T (n x n), G (n x r) as nested lists of Fractions.

    Alg. "Symbolic Cook-Toom Construction": Vandermonde rows alpha_p^j for the
    finite points, the row [0 .. 0 1] for infinity, Lagrange factors
    F_p = prod_{j != p}(alpha_p - alpha_j); A is the Vandermonde basis truncated
    to m columns, G the r-column Vandermonde basis scaled by 1/F_p, and B^T holds
    the Lagrange numerator polynomials.

    The algorithm box leaves the construction of B^T ("Lagrange x shift") and the
    split of the 1/F_p factor between the three matrices unstated.  The reading
    used here: row p of B^T = coefficients (ascending) of
    N_p(t) = prod_{j != p}(t - alpha_j), a trailing zero appended; the infinity
    row = coefficients of M(t) = prod_j (t - alpha_j); all of 1/F_p sits in G.
    It follows from Lagrange interpolation of t^(i+k) on the finite points
    (exact for i + k <= n - 2, and off by exactly M(t) for i + k = n - 1), it
    satisfies the tensor identity of Sec. 2.4 exactly, and it is the only split
    found that reproduces the printed kappa_2(A), kappa_2(B), kappa_2(G) of
    Table "Condition numbers of transform matrices".
    """
    alphas = _as_fractions(points)
    n = m + r - 1
    if len(alphas) != n - 1:
        raise ValueError(f"F({m},{r}) needs {n - 1} finite points, got {len(alphas)}")
    if len(set(alphas)) != len(alphas):
        raise ValueError("interpolation points must be distinct")

    A = [[alpha ** i for i in range(m)] for alpha in alphas]
    A.append([Fraction(0)] * (m - 1) + [Fraction(1)])

    G = []
    for p, alpha in enumerate(alphas):
        F_p = Fraction(1)
        for j, other in enumerate(alphas):
            if j != p:
                F_p *= alpha - other
        G.append([alpha ** k / F_p for k in range(r)])
    G.append([Fraction(0)] * (r - 1) + [Fraction(1)])

    BT = []
    for p in range(n - 1):
        N_p = poly_from_roots(alphas[:p] + alphas[p + 1:])   # degree n - 2
        BT.append(N_p + [Fraction(0)])
    BT.append(poly_from_roots(alphas))                        # degree n - 1
    return A, BT, G


def tensor_identity_holds(A, BT, G):
    """Exact check of sum_p A[p][i] B^T[p][j] G[p][k] == 1[j == i + k]
    (Sec. 2.4, the convolution tensor T_{ijk} of the correlation)."""
    n = len(A)
    m = len(A[0])
    r = len(G[0])
    for i in range(m):
        for j in range(n):
            for k in range(r):
                total = Fraction(0)
                for p in range(n):
                    total += A[p][i] * BT[p][j] * G[p][k]
                if total != (1 if j == i + k else 0):
                    return False
    return True


def rank_one_terms(A, BT, G):
    """The n rank-one tensors A[p][i] B^T[p][j] G[p][k]; these, unlike the three
    matrices, do not depend on how a per-row scale is split between them."""
    terms = []
    for p in range(len(A)):
        terms.append([[[a * b * g for g in G[p]] for b in BT[p]] for a in A[p]])
    return terms


def scale_rows(A, BT, G, log2_b, log2_g):
    """Diagonal rescaling of the three matrices by powers of two, exactly.

    The "learned diagonal scales" form discussed with the related work,
        Y = D_A A^T [ (D_G G g) * (D_B B^T d) ],
    restricted to the case that keeps the algorithm exact: row p of B^T is
    multiplied by 2**log2_b[p], row p of G by 2**log2_g[p], and row p of A by
    2**-(log2_b[p] + log2_g[p]), so the three factors of every row multiply to
    one and the rank-one terms (hence the bilinear identity) are unchanged.
    Only the range of the intermediate tensors U and V moves.
    """
    n = len(A)
    if len(log2_b) != n or len(log2_g) != n:
        raise ValueError("one exponent per row of B^T and of G is needed")
    two = Fraction(2)
    A2 = [[entry * two ** -(int(log2_b[p]) + int(log2_g[p])) for entry in A[p]] for p in range(n)]
    BT2 = [[entry * two ** int(log2_b[p]) for entry in BT[p]] for p in range(n)]
    G2 = [[entry * two ** int(log2_g[p]) for entry in G[p]] for p in range(n)]
    return A2, BT2, G2


def _balancing_exponent(row):
    """The integer e with 1 <= 2**e * sum|row| < 2, found by exact comparisons."""
    norm = sum(abs(entry) for entry in row)
    if norm == 0:
        raise ValueError("a transform row cannot vanish")
    e = 0
    while norm * Fraction(2) ** e >= 2:
        e -= 1
    while norm * Fraction(2) ** e < 1:
        e += 1
    return e


def balanced_row_exponents(BT, G):
    """Exponents (log2_b, log2_g) for `scale_rows` that bring the absolute row
    sums of B^T and of G into [1, 2).

    With them |V[(i,j)]| <= 4 max|d| and |U[(i,j)]| <= 4 max|g| for every
    position (i, j) of the 2D transforms, whatever the points: the dynamic range
    of the stored tensors no longer depends on the magnitude of the Lagrange
    factors.  (The paper's comparison uses learned scales; this fixed rule is
    the exact, data-free member of the same family.)
    """
    return [_balancing_exponent(row) for row in BT], [_balancing_exponent(row) for row in G]


def quantize_int8(matrix):
    """Symmetric per-tensor INT8 quantisation of a matrix, exactly (Sec. "INT8 Convolution
    Error Validation", Setup): scale s = max|entry| / 127, code = entry / s rounded to nearest
    with ties to even and saturated to [-128, 127], value = code * s.
    Returns (values, codes, s): the de-quantised matrix (Fractions), the integer codes and the
    scale.  (With this scale the largest entry gets code +-127, so nothing saturates; the clamp
    is part of the stated scheme.)"""
    top = max(abs(entry) for row in matrix for entry in row)
    if top == 0:
        raise ValueError("cannot quantise a zero matrix")
    s = top / 127
    codes = []
    for row in matrix:
        out = []
        for entry in row:
            scaled = entry / s
            lo = scaled.numerator // scaled.denominator          # floor
            rem = scaled - lo
            if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and lo % 2 != 0):
                lo += 1
            out.append(max(-128, min(127, lo)))
        codes.append(out)
    values = [[code * s for code in row] for row in codes]
    return values, codes, s


def vandermonde(points):
    """Square Vandermonde matrix of the finite points, V[i][j] = alpha_i^j
    (Sec. 2.2; the point at infinity does not enter)."""
    alphas = _as_fractions(points)
    return [[alpha ** j for j in range(len(alphas))] for alpha in alphas]


def to_f64(matrix):
    """Nearest fp64 of every entry (int / int true division is correctly rounded)."""
    return np.array([[entry.numerator / entry.denominator for entry in row] for row in matrix],
                    dtype=np.float64)


def _round_fraction(value, mant_bits, min_exp):
    """Nearest (ties to even) binary float with `mant_bits` significand bits and
    smallest normal exponent `min_exp`, returned as an exact Fraction.  No
    overflow handling: transform entries are far from any format's range."""
    if value == 0:
        return Fraction(0)
    sign = -1 if value < 0 else 1
    mag = abs(value)
    e = mag.numerator.bit_length() - mag.denominator.bit_length()
    if Fraction(2) ** e > mag:
        e -= 1
    if Fraction(2) ** (e + 1) <= mag:
        e += 1
    e = max(e, min_exp)
    quantum = Fraction(2) ** (e - (mant_bits - 1))
    scaled = mag / quantum
    lo = scaled.numerator // scaled.denominator
    rem = scaled - lo
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and lo % 2 == 1):
        lo += 1
    return sign * lo * quantum


def to_f32(matrix):
    """Nearest fp32 of every exact entry, rounded once from the rational."""
    out = np.empty((len(matrix), len(matrix[0])), dtype=np.float32)
    for i, row in enumerate(matrix):
        for j, entry in enumerate(row):
            rounded = _round_fraction(entry, 24, -126)
            out[i, j] = np.float32(rounded.numerator / rounded.denominator)  # exact in fp64 and fp32
    return out


def to_f16(matrix):
    """Nearest fp16 of every exact entry, rounded once from the rational."""
    out = np.empty((len(matrix), len(matrix[0])), dtype=np.float16)
    for i, row in enumerate(matrix):
        for j, entry in enumerate(row):
            rounded = _round_fraction(entry, 11, -14)
            out[i, j] = np.float16(rounded.numerator / rounded.denominator)
    return out


def kappa(matrix, norm=2):
    """Condition number of a Fraction or float matrix.  norm: 2 (sigma_max/sigma_min of the
    fp64 SVD, also for rectangular matrices), 1, inf or 'fro' (square only:
    ||M|| ||M^-1||) -- Sec. 2.2 "Condition Number Definition" and the norm
    sensitivity paragraph."""
    mat = to_f64(matrix) if isinstance(matrix[0][0], Fraction) else np.asarray(matrix, dtype=np.float64)
    if norm == 2:
        sv = np.linalg.svd(mat, compute_uv=False)
        return float(sv[0] / sv[-1])
    inv = np.linalg.inv(mat)
    return float(np.linalg.norm(mat, norm) * np.linalg.norm(inv, norm))


def kappa_V(points):
    """kappa_2 of the finite-point Vandermonde matrix."""
    return kappa(vandermonde(points))


def kron(matrix_a, matrix_b):
    """Exact Kronecker product (App. "2D Extension via Kronecker Products")."""
    out = []
    for row_a in matrix_a:
        for row_b in matrix_b:
            out.append([a * b for a in row_a for b in row_b])
    return out
