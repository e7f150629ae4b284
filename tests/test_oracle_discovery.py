"""Pins for the oracle's point discovery (CPU only): the exhaustive symmetric search must land on
the point sets the paper prints, and snapping must follow the printed algorithm."""
import os
from fractions import Fraction as Fr

import numpy as np
import pytest

from oracle import cook_toom as ct
from oracle import discovery


def printed_sets(golden_dir):
    out = {}
    for ln in open(os.path.join(golden_dir, "discovered_points_printed.txt")):
        if ln.strip() and not ln.startswith("#"):
            parts = ln.split()
            out[int(parts[0][1:])] = ([Fr(v) for v in parts[1:-1]], float(parts[-1]))
    return out


@pytest.mark.parametrize("m", [4, 6, 8])
def test_symmetric_search_finds_the_printed_point_sets(golden_dir, m):
    mags, printed_kappa = printed_sets(golden_dir)[m]
    points, kappa = discovery.symmetric_search(m, 3, d_max=6)
    assert points == discovery.symmetric_points(mags, True)
    assert abs(kappa - printed_kappa) <= 0.007 * printed_kappa
    assert kappa == pytest.approx(ct.kappa_V(points), rel=1e-12)


def test_symmetric_search_small_cases_by_brute_force():
    # F(2,3): one pair; the winner must be the candidate magnitude with the smallest kappa of
    # [[1,0,0],[1,p,p^2],[1,-p,p^2]], found here one candidate at a time
    cands = discovery.positive_rationals(4)
    assert cands[0] == Fr(1, 4) and cands[-1] == Fr(5) and len(cands) == len(set(cands))
    assert all(c.denominator <= 4 and c <= 5 for c in cands) and Fr(7, 3) in cands and Fr(11, 2) not in cands
    kappas = [ct.kappa_V([Fr(0), c, -c]) for c in cands]
    points, kappa = discovery.symmetric_search(2, 3, d_max=4)
    assert points == [Fr(0), cands[int(np.argmin(kappas))], -cands[int(np.argmin(kappas))]]
    assert kappa == pytest.approx(min(kappas), rel=1e-12)
    # even number of finite points (F(3,3): n - 1 = 4): two pairs, no zero
    points, kappa = discovery.symmetric_search(3, 3, d_max=3)
    assert len(points) == 4 and Fr(0) not in points and points[0] == -points[1] and points[2] == -points[3]
    best = min((ct.kappa_V([a, -a, b, -b]), a, b) for i, a in enumerate(discovery.positive_rationals(3))
               for b in discovery.positive_rationals(3)[i + 1:])
    assert (points[0], points[2]) == (best[1], best[2]) and kappa == pytest.approx(best[0], rel=1e-12)


def test_discovered_sets_beat_the_integer_points_by_the_printed_factors():
    # Table "Complete discovered configurations": improvements 2.9x, 27x, 415x
    for m, factor in ((4, 2.9), (6, 27.0), (8, 415.0)):
        _, kappa = discovery.symmetric_search(m, 3, d_max=6)
        std = ct.kappa_V([Fr(0)] + [s * Fr(k) for k in range(1, m // 2 + 1) for s in (1, -1)])
        assert std / kappa == pytest.approx(factor, rel=0.02)


def test_snap_to_rational():
    assert discovery.snap_to_rational(0.8333) == Fr(5, 6)
    assert discovery.snap_to_rational(1.1666) == Fr(7, 6)
    assert discovery.snap_to_rational(0.6001) == Fr(3, 5)
    assert discovery.snap_to_rational(-0.4) == Fr(-2, 5)
    assert discovery.snap_to_rational(0.0) == Fr(0)
    assert discovery.snap_to_rational(3.14159, d_max=10) == Fr(22, 7)
    assert discovery.snap_to_rational(7.3) == Fr(5)                     # numerators stop at 5 * denominator
    assert discovery.snap_to_rational(-9.0, d_max=3) == Fr(-5)
    # exactly half-way between 0 and 1 with d_max = 1: the first candidate in enumeration order stays
    assert discovery.snap_to_rational(0.5, d_max=1) == Fr(0)
    # the nearest fraction, by exhaustive comparison
    rng = np.random.default_rng(3)
    for x in rng.uniform(-5, 5, 50):
        want = min((abs(Fr(x) - Fr(a, d)), d, a) for d in range(1, 8) for a in range(-5 * d, 5 * d + 1))
        assert abs(Fr(x) - discovery.snap_to_rational(x, d_max=7)) == want[0]


# ---- evolution strategy (Sec. "Evolution Strategy")

def test_es_fitness_at_the_printed_point_sets(golden_dir):
    # tensor error zero (to rounding), kappa the printed one, magnitude term by hand
    for m, (mags, printed_kappa) in printed_sets(golden_dir).items():
        points = discovery.symmetric_points(mags, True)
        f, err, mag, kappa = discovery.es_fitness([float(p) for p in points], m, 3)
        assert err < 1e-12
        assert abs(kappa - printed_kappa) <= 0.007 * printed_kappa
        assert mag == pytest.approx(float(sum(p * p for p in points)) / (m + 1), rel=1e-14)
        assert f == pytest.approx(err + 1e-3 * mag + 1e-4 * np.log10(kappa + 1.0), rel=1e-14)


def test_float_cook_toom_is_the_exact_construction_rounded():
    points = [Fr(0), Fr(5, 6), Fr(-5, 6), Fr(7, 6), Fr(-7, 6)]
    A, BT, G = discovery.float_cook_toom([float(p) for p in points], 4, 3)
    Ae, BTe, Ge = ct.cook_toom(points, 4, 3)
    for got, want in ((A, Ae), (BT, BTe), (G, Ge)):
        assert np.allclose(got, ct.to_f64(want), rtol=1e-13, atol=1e-15)
    # coinciding points: no finite fitness
    assert discovery.es_fitness([0.5, 0.5, 1.0, -1.0, 0.0], 4, 3)[0] == np.inf


def test_es_fitness_tensor_error_sees_a_wrong_matrix():
    # planted mistake: the tensor error is what tells a valid algorithm from an invalid one
    p = [0.0, 0.8, -0.8, 1.2, -1.2]
    A, BT, G = discovery.float_cook_toom(p, 4, 3)
    target = np.zeros((4, 6, 3))
    for i in range(4):
        for k in range(3):
            target[i, i + k, k] = 1.0
    assert np.sqrt(np.sum((np.einsum("qi,qj,qk->ijk", A, BT, G) - target) ** 2)) < 1e-13
    G[1, 2] *= 1.01
    assert np.sqrt(np.sum((np.einsum("qi,qj,qk->ijk", A, BT, G) - target) ** 2)) > 1e-3


def test_evolution_strategy_small_run_by_hand():
    # one restart, one generation, four candidates in one dimension less than nothing: F(2,3) has n - 1 = 3
    m, r, dim = 2, 3, 3
    z = np.array([0.2, -1.0, 0.7,                 # mu = sqrt(0.5) z
                  1.0, 0.0, 0.0,  0.0, 1.0, 0.0,  0.0, 0.0, 1.0,  -1.0, -1.0, 0.5])
    best_p, best_f = discovery.evolution_strategy(m, r, z, generations=1, population=4, restarts=1)
    mu = np.sqrt(0.5) * z[:3]
    cands = [mu + 0.5 * z[3 + 3 * i:6 + 3 * i] for i in range(4)]
    fits = [discovery.es_fitness(c, m, r)[0] for c in cands]
    assert best_f == min(fits) and np.array_equal(best_p, cands[int(np.argmin(fits))])
    assert discovery.es_normals_needed(m, r, 1, 4, 1) == len(z)
    # two generations: the second samples around the mean of the elite (one of four) with the adapted step
    z2 = np.concatenate([z, np.linspace(-1, 1, 12)])
    best_p2, best_f2 = discovery.evolution_strategy(m, r, z2, generations=2, population=4, restarts=1)
    elite = cands[int(np.argmin(fits))]
    f_parent = discovery.es_fitness(mu, m, r)[0]
    sigma = 0.5 * (1.1 if sum(f < f_parent for f in fits) / 4 > 0.2 else 0.9)
    cands2 = [elite + sigma * z2[15 + 3 * i:18 + 3 * i] for i in range(4)]
    fits2 = [discovery.es_fitness(c, m, r)[0] for c in cands2]
    assert best_f2 == min(fits + fits2)


def test_snap_points_and_neighbourhood_search():
    # distinct after snapping: nothing else happens
    pts, kappa = discovery.snap_points([0.0, 0.8334, -0.8331, 1.1669, -1.16], 4, 3, d_max=6)
    assert pts == [Fr(0), Fr(5, 6), Fr(-5, 6), Fr(7, 6), Fr(-7, 6)]
    assert kappa == pytest.approx(14.5456, rel=1e-4)
    # two coordinates snap to the same fraction: the neighbourhood search separates them, and among the
    # combinations it may try (10 nearest candidates per point) the winner has the lowest kappa
    x = [0.3301, 0.3302, -0.5, 0.0, 1.0]
    pts, kappa = discovery.snap_points(x, 4, 3)
    assert len(set(pts)) == 5 and kappa == pytest.approx(ct.kappa_V(pts), rel=1e-12)
    every = sorted({Fr(a, b) for b in range(1, 11) for a in range(-5 * b, 5 * b + 1)})
    snapped = [discovery.snap_to_rational(v) for v in x]
    choices = []
    for v, s in zip(x, snapped):
        near = sorted((c for c in every if abs(c - s) <= Fr(6, 5)), key=lambda c: (abs(c - Fr(v)), c))[:10]
        choices.append(near)
    import itertools
    best = min(ct.kappa_V(list(c)) for c in itertools.product(*choices) if len(set(c)) == 5)
    assert kappa == pytest.approx(best, rel=1e-9)
