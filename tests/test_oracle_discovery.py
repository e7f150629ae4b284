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
