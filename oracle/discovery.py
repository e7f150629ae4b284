"""Point discovery by symmetric search and snap-to-rational (test oracle).

Test infrastructure only; see the package docstring.

Two of the steps of the paper's discovery pipeline (Sec. "Complete Pipeline"), the ones
that are deterministic: the enumeration of symmetric configurations
(Sec. "Symmetric Search", Alg. "Symmetric Search") and the conversion of a real
number to a simple fraction (Sec. "Snap-to-Rational", Alg. "Snap-to-Rational").
"""
import itertools
from fractions import Fraction

import numpy as np

from . import cook_toom as ct


def positive_rationals(d_max, bound=5):
    """The candidate magnitudes: all distinct a/b with 1 <= b <= d_max and 1 <= a <= bound*b,
    ascending ("positive rationals up to d_max", with the numerator range of the snapping
    definition, |a| <= 5b)."""
    values = {Fraction(a, b) for b in range(1, d_max + 1) for a in range(1, bound * b + 1)}
    return sorted(values)


def symmetric_points(magnitudes, with_zero):
    """Finite points of a symmetric configuration in the order 0, +p1, -p1, +p2, -p2, ..."""
    points = [Fraction(0)] if with_zero else []
    for p in magnitudes:
        points += [p, -p]
    return points


def symmetric_search(m, r=3, d_max=6, bound=5, chunk=20000):
    """Best symmetric configuration {0, +-p1, +-p2, ..} for F(m, r) by exhaustive enumeration.

    n - 1 finite points are needed (n = m + r - 1): zero plus (n - 2) / 2 pairs when n - 1 is
    odd, (n - 1) / 2 pairs when it is even.  Every combination of that many candidate
    magnitudes (ascending) is tried in lexicographic order, its quality is the spectral
    condition number of the Vandermonde matrix of its finite points (Sec. 2.2), and the first
    combination with the lowest value wins.  Any set of distinct points is a valid
    algorithm, so only the winner is verified symbolically (exact tensor identity).

    Returns (points, kappa): the finite points as Fractions in canonical order."""
    n = m + r - 1
    finite = n - 1
    with_zero = finite % 2 == 1
    n_pairs = (finite - 1) // 2 if with_zero else finite // 2
    cands = positive_rationals(d_max, bound)
    values = np.array([c.numerator / c.denominator for c in cands], dtype=np.float64)
    best_kappa, best_combo = np.inf, None
    combos = itertools.combinations(range(len(cands)), n_pairs)
    while True:
        block = list(itertools.islice(combos, chunk))
        if not block:
            break
        mags = values[np.array(block, dtype=np.int64)]                     # [count, n_pairs]
        pairs = np.stack([mags, -mags], axis=2).reshape(len(block), -1)     # +p1, -p1, +p2, ...
        pts = np.concatenate([np.zeros((len(block), 1)), pairs], axis=1) if with_zero else pairs
        vander = pts[:, :, None] ** np.arange(finite)[None, None, :]        # V[i][j] = alpha_i^j
        sv = np.linalg.svd(vander, compute_uv=False)
        kappas = sv[:, 0] / sv[:, -1]
        i = int(np.argmin(kappas))                                          # first minimum of the block
        if kappas[i] < best_kappa:
            best_kappa, best_combo = float(kappas[i]), block[i]
    points = symmetric_points([cands[i] for i in best_combo], with_zero)
    A, BT, G = ct.cook_toom(points, m, r)
    if not ct.tensor_identity_holds(A, BT, G):
        raise AssertionError("symbolic verification failed")
    return points, best_kappa


def snap_to_rational(x, d_max=10, bound=5):
    """The simple fraction nearest to x: denominators 1..d_max ascending, numerators
    -bound*d .. bound*d ascending, a candidate replaces the best so far only if it is
    strictly nearer (so among equally near fractions the first in that order is kept).
    Distances are compared exactly (x is taken as the rational the float represents)."""
    target = Fraction(x)
    best, best_dist = None, None
    for d in range(1, d_max + 1):
        for a in range(-bound * d, bound * d + 1):
            f = Fraction(a, d)
            dist = abs(target - f)
            if best is None or dist < best_dist:
                best, best_dist = f, dist
    return best
