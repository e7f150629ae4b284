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


# ---------------------------------------------------------------------------------------------
# Evolution strategy (Sec. "Evolution Strategy", Alg. "Evolution Strategy for Winograd Point
# Discovery", Table "Evolution Strategy hyperparameters", Table "Fitness function weights").
#
# The random numbers are an input: `normals` is a sequence of independent standard normal draws
# that is consumed in the order the algorithm needs them (per restart: n - 1 for the initial mean,
# then per generation population * (n - 1) for the offspring, candidate by candidate).
#
# Readings where the text leaves a choice: mu ~ N(0, 0.5 I) is taken as covariance 0.5 I (standard
# deviation sqrt(0.5)); the "success rate" of the 1/5 rule is the fraction of offspring that are
# fitter than the mean they were sampled around; the elite is the best floor(0.25 * population)
# (at least one), ties in fitness broken by sample index; sigma is clamped to [0.01, 2.0] after
# every adaptation; a configuration whose fitness is not finite (coinciding points) ranks last.

ES_LAMBDA_MAGNITUDE = 1e-3
ES_LAMBDA_CONDITION = 1e-4


def float_cook_toom(p, m, r):
    """A (n x m), B^T (n x n), G (n x r) from finite points given as floats, in binary64: the
    construction of cook_toom.cook_toom with every operation rounded."""
    n = m + r - 1
    p = [float(v) for v in p]
    assert len(p) == n - 1
    A = np.zeros((n, m))
    BT = np.zeros((n, n))
    G = np.zeros((n, r))
    full = [1.0]                                   # coefficients of prod_j (t - p_j), ascending
    for j in range(n - 1):
        full = [(full[k - 1] if k > 0 else 0.0) - p[j] * (full[k] if k < len(full) else 0.0) for k in range(len(full) + 1)]
    for q in range(n - 1):
        lag = [1.0]                                # coefficients of prod_{j != q} (t - p_j)
        f = 1.0
        for j in range(n - 1):
            if j == q:
                continue
            lag = [(lag[k - 1] if k > 0 else 0.0) - p[j] * (lag[k] if k < len(lag) else 0.0) for k in range(len(lag) + 1)]
            f *= p[q] - p[j]
        BT[q, :n - 1] = lag
        pw = 1.0
        for i in range(max(m, r)):
            if i < m:
                A[q, i] = pw
            if i < r:
                G[q, i] = pw / f if f != 0.0 else np.inf
            pw *= p[q]
    A[n - 1, m - 1] = 1.0
    G[n - 1, r - 1] = 1.0
    BT[n - 1, :] = full
    return A, BT, G


def es_fitness(p, m, r=3):
    """f(p) = tensor error + 0.001 |p|^2 / (n - 1) + 0.0001 log10(kappa(V) + 1)  (Sec. "Evolution
    Strategy", "Fitness Function").  Returns (f, tensor error, magnitude term, kappa)."""
    n = m + r - 1
    with np.errstate(all="ignore"):
        A, BT, G = float_cook_toom(p, m, r)
        rec = np.einsum("qi,qj,qk->ijk", A, BT, G)
        target = np.zeros((m, n, r))
        for i in range(m):
            for k in range(r):
                target[i, i + k, k] = 1.0
        err = float(np.sqrt(np.sum((rec - target) ** 2)))
        mag = float(sum(float(v) ** 2 for v in p) / (n - 1))
        vander = np.array([[float(v) ** j for j in range(n - 1)] for v in p])
        sv = np.linalg.svd(vander, compute_uv=False)
        kappa = float(sv[0] / sv[-1]) if sv[-1] > 0 else np.inf
        f = err + ES_LAMBDA_MAGNITUDE * mag + ES_LAMBDA_CONDITION * np.log10(kappa + 1.0)
    if not np.isfinite(f):
        f = np.inf
    return float(f), err, mag, kappa


def es_normals_needed(m, r=3, generations=100, population=50, restarts=3):
    return restarts * (m + r - 2) * (1 + generations * population)


def evolution_strategy(m, r, normals, generations=100, population=50, restarts=3):
    """Alg. "Evolution Strategy for Winograd Point Discovery".  Returns (best points, best fitness)."""
    dim = m + r - 2
    z = iter(np.asarray(normals, dtype=np.float64).tolist())
    elite_count = max(1, population // 4)
    best_p, best_f = None, np.inf
    for _ in range(restarts):
        mu = [np.sqrt(0.5) * next(z) for _ in range(dim)]
        sigma = 0.5
        for _ in range(generations):
            f_parent = es_fitness(mu, m, r)[0]
            cands = [[mu[d] + sigma * next(z) for d in range(dim)] for _ in range(population)]
            fits = [es_fitness(c, m, r)[0] for c in cands]
            order = sorted(range(population), key=lambda i: (fits[i], i))
            elite = order[:elite_count]
            new_mu = []
            for d in range(dim):
                acc = 0.0
                for i in elite:
                    acc += cands[i][d]
                new_mu.append(acc / elite_count)
            mu = new_mu
            success = sum(1 for v in fits if v < f_parent) / population
            sigma = sigma * 1.1 if success > 0.2 else sigma * 0.9
            sigma = min(2.0, max(0.01, sigma))
            if fits[order[0]] < best_f:
                best_f, best_p = fits[order[0]], list(cands[order[0]])
    return best_p, best_f


def snap_points(x, m, r=3, d_max=10, bound=5, radius=Fraction(6, 5), budget=10 ** 5):
    """Sec. "Snap-to-Rational" and "Neighborhood Search": every coordinate goes to its nearest simple
    fraction; if two of them coincide (the one way a set of points can be invalid), every point gets
    the candidates a/b (b <= d_max, |a| <= bound * b) within `radius` of its snapped value, nearest to
    its continuous value first -- as many per point as keep the number of combinations within
    `budget` (a deterministic stand-in for the sampling the text mentions) -- and the combination of
    distinct points with the lowest kappa(V) wins (first in enumeration order, last point varying
    fastest, among those within a relative 1e-9 of each other).
    The result is verified exactly.  Returns (points as Fractions, kappa)."""
    dim = m + r - 2
    assert len(x) == dim
    snapped = [snap_to_rational(v, d_max, bound) for v in x]
    points = snapped
    if len(set(snapped)) < dim:
        per_point = max(1, int(np.floor(budget ** (1.0 / dim) + 1e-9)))
        every = sorted({Fraction(a, b) for b in range(1, d_max + 1) for a in range(-bound * b, bound * b + 1)})
        choices = []
        for v, s in zip(x, snapped):
            near = [c for c in every if abs(c - s) <= radius]
            near.sort(key=lambda c: (abs(c - Fraction(v)), c))
            choices.append(near[:per_point])
        best, best_kappa = None, np.inf
        for combo in itertools.product(*choices):
            if len(set(combo)) < dim:
                continue
            kappa = ct.kappa_V(list(combo))
            if kappa < best_kappa * (1.0 - 1e-9):      # (permutations of one set differ in the last bits only)
                best, best_kappa = list(combo), kappa
        if best is None:
            raise ValueError("no valid configuration near the snapped points")
        points = best
    A, BT, G = ct.cook_toom(points, m, r)
    if not ct.tensor_identity_holds(A, BT, G):
        raise AssertionError("symbolic verification failed")
    return points, ct.kappa_V(points)
