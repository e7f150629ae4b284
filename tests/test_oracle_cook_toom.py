"""Pins for the oracle's exact Cook-Toom construction (CPU only).

Each test ties oracle/cook_toom.py to something the paper or the mathematics fixes:
printed condition numbers, the textbook F(2,3)/F(4,3) algorithms, the exact bilinear
identity, brute-force correlation.  The last tests plant plausible mistakes in a copy
of the construction and check that the pins reject them.
"""
import os
import random
from fractions import Fraction as Fr

import numpy as np
import pytest

from oracle import cook_toom as ct
from oracle import exact
from paper_2512_18453_amd import synth


def pts(pairs):
    return [Fr(a, b) for a, b in pairs]


SETS = {("std", m): pts(synth.STANDARD[m]) for m in (2, 4, 6, 8)}
SETS.update({("disc", m): pts(synth.NOVA[m]) for m in (2, 4, 6, 8)})


def read_rows(path):
    with open(path) as fh:
        return [ln.split() for ln in fh if ln.strip() and not ln.startswith("#")]


# ---------------------------------------------------------------- exact identity


@pytest.mark.parametrize("key", sorted(SETS))
def test_tensor_identity_exact(key):
    A, BT, G = ct.cook_toom(SETS[key], key[1], 3)
    assert ct.tensor_identity_holds(A, BT, G)


def test_tensor_identity_random_rational_points_and_other_r():
    rnd = random.Random(7)
    for m, r in [(2, 3), (3, 2), (4, 3), (4, 5), (5, 3), (6, 3), (2, 5), (8, 3), (1, 3), (3, 1)]:
        n = m + r - 1
        chosen = set()
        while len(chosen) < n - 1:
            chosen.add(Fr(rnd.randint(-12, 12), rnd.randint(1, 7)))
        points = list(chosen)
        rnd.shuffle(points)
        A, BT, G = ct.cook_toom(points, m, r)
        assert len(A) == n and len(A[0]) == m and len(BT[0]) == n and len(G[0]) == r
        assert ct.tensor_identity_holds(A, BT, G)


def test_identity_check_detects_a_wrong_entry():
    A, BT, G = ct.cook_toom(SETS[("disc", 4)], 4, 3)
    BT[2][3] += Fr(1, 1000)
    assert not ct.tensor_identity_holds(A, BT, G)


def test_rejects_bad_point_sets():
    with pytest.raises(ValueError):
        ct.cook_toom([0, 1, -1, 1, 2], 4, 3)     # duplicate
    with pytest.raises(ValueError):
        ct.cook_toom([0, 1, -1], 4, 3)            # wrong count


@pytest.mark.parametrize("key", sorted(SETS))
def test_1d_algorithm_equals_brute_force_correlation(key):
    m = key[1]
    A, BT, G = ct.cook_toom(SETS[key], m, 3)
    rnd = random.Random(m)
    for _ in range(5):
        x = [rnd.randint(-9, 9) for _ in range(m + 2)]
        g = [rnd.randint(-9, 9) for _ in range(3)]
        want = [sum(g[k] * x[i + k] for k in range(3)) for i in range(m)]   # y_i = sum_k g_k x_{i+k}
        assert exact.winograd_1d(x, g, A, BT, G) == want


# ---------------------------------------------------------------- printed values


def test_printed_condition_numbers(golden_dir):
    rows = read_rows(os.path.join(golden_dir, "kappa_printed.txt"))
    assert len(rows) == 35
    for table, m, which, matrix, printed, tol in rows:
        m, printed, tol = int(m), float(printed), float(tol)
        points = SETS[(which, m)]
        if matrix == "V":
            got = ct.kappa_V(points)
        elif matrix == "V2D":
            got = ct.kappa_V(points) ** 2
        else:
            A, BT, G = ct.cook_toom(points, m, 3)
            got = ct.kappa({"A": A, "B": BT, "G": G}[matrix])
        assert abs(got - printed) <= tol * printed, (table, m, which, matrix, got, printed)


def test_printed_improvement_ratios():
    # abstract / Table "Complete discovered configurations": 2.9x, 27x, 415x; 2D: 8.5x, 733x, 172k x
    for m, ratio, ratio2d in [(4, 2.9, 8.5), (6, 27, 733), (8, 415, 172e3)]:
        got = ct.kappa_V(SETS[("std", m)]) / ct.kappa_V(SETS[("disc", m)])
        assert abs(got - ratio) / ratio < 0.02
        assert abs(got * got - ratio2d) / ratio2d < 0.01


def test_printed_norm_sensitivity(golden_dir):
    for m, k1, k2, kinf, kf in read_rows(os.path.join(golden_dir, "norm_sensitivity_printed.txt")):
        m = int(m)
        Vs, Vd = ct.vandermonde(SETS[("std", m)]), ct.vandermonde(SETS[("disc", m)])
        for norm, printed in [(1, k1), (2, k2), (np.inf, kinf), ("fro", kf)]:
            got = ct.kappa(Vs, norm) / ct.kappa(Vd, norm)
            assert abs(got - float(printed)) / float(printed) < 0.012, (m, norm, got, printed)


def test_kronecker_condition_number_squares():
    # Fact "Kronecker Condition Number": kappa_2(A (x) A) = kappa_2(A)^2
    for key in [("std", 4), ("disc", 4), ("disc", 6)]:
        A, BT, G = ct.cook_toom(SETS[key], key[1], 3)
        for mat in (A, BT, G):
            k1 = ct.kappa(mat)
            assert ct.kappa(ct.kron(mat, mat)) == pytest.approx(k1 * k1, rel=1e-8)


def test_printed_max_coefficient():
    # "Coefficient Magnitude Reduction": F(4,3) 8.0 -> 1.6, F(6,3) 243 -> 2.2 (the entries of A)
    for key, printed in [(("std", 4), 8.0), (("disc", 4), 1.6), (("std", 6), 243), (("disc", 6), 2.2)]:
        A, _, _ = ct.cook_toom(SETS[key], key[1], 3)
        got = float(max(abs(e) for row in A for e in row))
        assert abs(got - printed) <= 0.05 * max(1.0, printed / 100)


def test_printed_entry_vocabulary_f43():
    # "Structural Sparsity Analysis": standard F(4,3) entries come from
    # {0, +-1, +-2, +-4, +-8, 1/4, 1/6, 1/12, 1/24} (5 also occurs in B^T, as in the textbook matrices)
    A, BT, G = ct.cook_toom(SETS[("std", 4)], 4, 3)
    vocab = {Fr(0), Fr(1), Fr(2), Fr(4), Fr(8), Fr(1, 4), Fr(1, 6), Fr(1, 12), Fr(1, 24), Fr(5)}
    seen = {abs(e) for mat in (A, BT, G) for row in mat for e in row}
    assert seen <= vocab
    assert {Fr(8), Fr(1, 24), Fr(1, 12), Fr(1, 6), Fr(1, 4)} <= seen


# ---------------------------------------------------------------- textbook algorithms


def parse_textbook(path):
    out, cur = {}, None
    for ln in open(path):
        ln = ln.strip()
        if not ln or ln.startswith("#"):
            continue
        tag, rest = ln.split(None, 1)
        if tag == "F":
            cur = int(rest)
            out[cur] = {}
        else:
            out[cur][tag] = [[Fr(tok) for tok in row.split()] for row in rest.split(";")]
    return out


@pytest.mark.parametrize("m", [2, 4])
def test_matches_textbook_rank_one_terms(golden_dir, m):
    book = parse_textbook(os.path.join(golden_dir, "textbook_transforms.txt"))[m]
    A, BT, G = ct.cook_toom(SETS[("std", m)], m, 3)
    assert ct.rank_one_terms(A, BT, G) == ct.rank_one_terms(book["A"], book["BT"], book["G"])


def test_f43_matrices_equal_textbook_entrywise(golden_dir):
    # for F(4,3) even the split of the scale agrees with the textbook matrices
    book = parse_textbook(os.path.join(golden_dir, "textbook_transforms.txt"))[4]
    A, BT, G = ct.cook_toom(SETS[("std", 4)], 4, 3)
    assert (A, BT, G) == (book["A"], book["BT"], book["G"])


# ---------------------------------------------------------------- power-of-two row scaling


def test_row_scaling_leaves_the_algorithm_unchanged():
    # any integer exponents: rank-one terms, identity and the exact 1D result stay what they were
    rng = random.Random(11)
    for key in sorted(SETS):
        m = key[1]
        A, BT, G = ct.cook_toom(SETS[key], m, 3)
        n = m + 2
        log2_b = [rng.randint(-9, 9) for _ in range(n)]
        log2_g = [rng.randint(-9, 9) for _ in range(n)]
        A2, BT2, G2 = ct.scale_rows(A, BT, G, log2_b, log2_g)
        assert ct.rank_one_terms(A2, BT2, G2) == ct.rank_one_terms(A, BT, G)
        assert ct.tensor_identity_holds(A2, BT2, G2)
        x = [Fr(rng.randint(-50, 50), rng.randint(1, 7)) for _ in range(n)]
        g = [Fr(rng.randint(-50, 50), rng.randint(1, 7)) for _ in range(3)]
        assert exact.winograd_1d(x, g, A2, BT2, G2) == [sum(g[k] * x[i + k] for k in range(3)) for i in range(m)]
        # and the scale really sits where it was asked for
        for p in range(n):
            assert BT2[p] == [e * Fr(2) ** log2_b[p] for e in BT[p]]
            assert G2[p] == [e * Fr(2) ** log2_g[p] for e in G[p]]


def test_balanced_rows_hand_worked_f43(golden_dir):
    rows = read_rows(os.path.join(golden_dir, "balanced_rows_f43_textbook.txt"))
    want = {}
    for row in rows:
        if row[0] in ("log2_b", "log2_g"):
            want[row[0]] = [int(v) for v in row[1:]]
        else:
            want[row[0]] = [[Fr(v) for v in part.split()] for part in " ".join(row[1:]).split(";")]
    A, BT, G = ct.cook_toom(SETS[("std", 4)], 4, 3)
    log2_b, log2_g = ct.balanced_row_exponents(BT, G)
    assert (log2_b, log2_g) == (want["log2_b"], want["log2_g"])
    assert ct.scale_rows(A, BT, G, log2_b, log2_g) == (want["A"], want["BT"], want["G"])


@pytest.mark.parametrize("key", sorted(SETS))
def test_balanced_rows_bound_the_row_sums(key):
    m = key[1]
    A, BT, G = ct.cook_toom(SETS[key], m, 3)
    log2_b, log2_g = ct.balanced_row_exponents(BT, G)
    _, BT2, G2 = ct.scale_rows(A, BT, G, log2_b, log2_g)
    for row in BT2 + G2:
        assert 1 <= sum(abs(e) for e in row) < 2
    # rows of +a and -a get the same exponent (their entries differ in sign only)
    for p in range(1, m + 1, 2):
        assert log2_b[p] == log2_b[p + 1] and log2_g[p] == log2_g[p + 1]


def test_scale_rows_rejects_wrong_lengths():
    A, BT, G = ct.cook_toom(SETS[("std", 2)], 2, 3)
    with pytest.raises(ValueError):
        ct.scale_rows(A, BT, G, [0, 0, 0], [0, 0, 0, 0])


# ---------------------------------------------------------------- float tables


def test_float_tables_are_single_roundings():
    vals = [[Fr(5, 6), Fr(-7, 6), Fr(1, 3)], [Fr(2, 5), Fr(1, 24), Fr(-16384)],
            [Fr(1, 3) * Fr(1, 2 ** 130), Fr(0), Fr(16777217, 16777216)]]
    f64 = ct.to_f64(vals)
    f32 = ct.to_f32(vals)
    f16 = ct.to_f16(vals[:2])
    assert f64[0, 0] == 5 / 6 and f64[1, 1] == 1 / 24
    # library roundings as the yardstick (numpy rounds fp64 -> fp32 / fp16 to nearest even)
    assert f32[0, 0] == np.float32(5 / 6) and f32[0, 1] == np.float32(-7 / 6)
    assert f32[1, 0] == np.float32(0.4) and f32[1, 2] == np.float32(-16384)
    assert f32[2, 0] == np.float32(float(vals[2][0]))           # binary32 sub-normal
    assert f32[2, 2] == np.float32(1.0)                         # 1 + 2^-24: tie, rounds to even
    assert f16[0, 0] == np.float16(5 / 6) and f16[1, 1] == np.float16(1 / 24)
    # nearest: no other representable value is closer
    for fr, got in [(Fr(5, 6), f32[0, 0]), (Fr(2, 5), f32[1, 0])]:
        got_fr = Fr(float(got))
        for nb in (np.nextafter(got, np.float32(2)), np.nextafter(got, np.float32(-2))):
            assert abs(got_fr - fr) <= abs(Fr(float(nb)) - fr)


# ---------------------------------------------------------------- planted mistakes


def _variant(points, m, mistake):
    """cook_toom with one plausible slip planted."""
    A, BT, G = ct.cook_toom(points, m, 3)
    n = m + 2
    if mistake == "scale_in_BT":           # 1/F_p moved from G to B^T: still a valid algorithm
        for p in range(n - 1):
            f = G[p][0]                     # alpha^0 / F_p
            G[p] = [g / f for g in G[p]]
            BT[p] = [b * f for b in BT[p]]
    elif mistake == "transposed_BT":
        BT = [list(col) for col in zip(*BT)]
    elif mistake == "descending_powers":
        BT = [row[::-1] for row in BT]
    elif mistake == "no_infinity_fix":      # infinity row of B^T taken as e_{n-1}
        BT[n - 1] = [Fr(0)] * (n - 1) + [Fr(1)]
    elif mistake == "wrong_sign_F":
        G = [[-g for g in row] for row in G[:-1]] + [G[-1]]
    return A, BT, G


def test_pins_reject_planted_mistakes():
    points, m = SETS[("std", 4)], 4
    # a different split of the scale keeps the identity but not the printed kappa(B) = 20.1
    A, BT, G = _variant(points, m, "scale_in_BT")
    assert ct.tensor_identity_holds(A, BT, G)
    assert abs(ct.kappa(BT) - 20.1) > 1.0
    for mistake in ["transposed_BT", "descending_powers", "no_infinity_fix", "wrong_sign_F"]:
        A, BT, G = _variant(points, m, mistake)
        assert not ct.tensor_identity_holds(A, BT, G), mistake
