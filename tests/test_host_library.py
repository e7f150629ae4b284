"""CPU-only checks of libnova's host side: the library loads, exports every symbol the header
declares, and its exact Cook-Toom construction agrees entry by entry with the oracle's (two
independent implementations of the same construction).  No device call is made here."""
import ctypes
import os
import re
from fractions import Fraction as Fr

import numpy as np
import pytest

from oracle import cook_toom as ct
from oracle import discovery
from paper_2512_18453_amd import nova, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

ALL_SETS = [("standard", 2), ("standard", 4), ("standard", 6), ("standard", 8), ("nova", 4), ("nova", 6),
            ("nova", 8), ("classic_half", 6), ("dyadic", 4)]


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "nova.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(nova_[a-z0-9_]+)\s*\(", header))
    assert declared == set(nova.EXPORTS), declared ^ set(nova.EXPORTS)
    L = nova.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert "gfx950" in nova.nova_version()


@pytest.mark.parametrize("name,m", ALL_SETS)
def test_matrices_equal_oracle_exactly(name, m):
    points = synth.point_set(name, m)
    t = nova.nova_make_transforms(points, m, 3)
    assert (t.m, t.r, t.n, t.symmetric) == (m, 3, m + 2, True)
    A, BT, G = ct.cook_toom([Fr(a, b) for a, b in points], m, 3)
    assert nova.nova_get_matrix(t, nova.NOVA_MATRIX_A) == A
    assert nova.nova_get_matrix(t, nova.NOVA_MATRIX_BT) == BT
    assert nova.nova_get_matrix(t, nova.NOVA_MATRIX_G) == G
    for which, mat in [(nova.NOVA_MATRIX_A, A), (nova.NOVA_MATRIX_BT, BT), (nova.NOVA_MATRIX_G, G)]:
        assert np.array_equal(np.array(nova.nova_get_matrix_f64(t, which)), ct.to_f64(mat))
        assert np.array_equal(np.array(nova.nova_get_matrix_f32(t, which), dtype=np.float32), ct.to_f32(mat))


@pytest.mark.parametrize("name,m", ALL_SETS)
def test_row_scaling_and_fp16_matrices_equal_oracle(name, m):
    points = synth.point_set(name, m)
    A, BT, G = ct.cook_toom([Fr(a, b) for a, b in points], m, 3)
    log2_b, log2_g = ct.balanced_row_exponents(BT, G)
    t = nova.nova_make_transforms(points, m, 3, row_scaling="balanced")
    assert nova.nova_get_row_scaling(t) == (log2_b, log2_g)
    assert t.symmetric
    A2, BT2, G2 = ct.scale_rows(A, BT, G, log2_b, log2_g)
    got = [nova.nova_get_matrix(t, w) for w in (nova.NOVA_MATRIX_A, nova.NOVA_MATRIX_BT, nova.NOVA_MATRIX_G)]
    assert got == [A2, BT2, G2]
    assert np.array_equal(np.array(nova.nova_get_matrix_f32(t, nova.NOVA_MATRIX_BT), dtype=np.float32), ct.to_f32(BT2))
    # explicit exponents, different for the rows of +a and -a: exact, but no longer paired
    rng = np.random.default_rng(m)
    eb, eg = [int(v) for v in rng.integers(-5, 6, m + 2)], [int(v) for v in rng.integers(-5, 6, m + 2)]
    if m >= 2:
        eb[2] = eb[1] + 1
    tg = nova.nova_make_transforms(points, m, 3, row_scaling=(eb, eg))
    assert nova.nova_get_row_scaling(tg) == (eb, eg)
    assert [nova.nova_get_matrix(tg, w) for w in (0, 1, 2)] == list(ct.scale_rows(A, BT, G, eb, eg))
    assert not tg.symmetric
    # plain handle reports zero exponents
    assert nova.nova_get_row_scaling(nova.nova_make_transforms(points, m, 3)) == ([0] * (m + 2), [0] * (m + 2))
    # matrices stored in binary16: every table holds the nearest binary16 of the exact entry
    t16 = nova.nova_make_transforms(points, m, 3, matrix_dtype="f16")
    for which, mat in [(nova.NOVA_MATRIX_A, A), (nova.NOVA_MATRIX_BT, BT), (nova.NOVA_MATRIX_G, G)]:
        want = ct.to_f16(mat)
        assert np.array_equal(np.array(nova.nova_get_matrix_f32(t16, which), dtype=np.float32), want.astype(np.float32))
        assert np.array_equal(np.array(nova.nova_get_matrix_f64(t16, which)), want.astype(np.float64))
        assert nova.nova_get_matrix(t16, which) == mat           # the exact matrices are untouched


@pytest.mark.parametrize("name,m", ALL_SETS)
def test_int8_matrices_equal_oracle(name, m):
    points = synth.point_set(name, m)
    exact_mats = ct.cook_toom([Fr(a, b) for a, b in points], m, 3)
    t = nova.nova_make_transforms(points, m, 3, matrix_dtype="int8")
    assert t.symmetric
    for which, mat in zip((nova.NOVA_MATRIX_A, nova.NOVA_MATRIX_BT, nova.NOVA_MATRIX_G), exact_mats):
        vals, codes, s = ct.quantize_int8(mat)
        got_codes, got_scale = nova.nova_get_matrix_int8(t, which)
        assert got_codes == codes
        assert got_scale == s.numerator / s.denominator
        assert np.array_equal(np.array(nova.nova_get_matrix_f32(t, which), dtype=np.float32), ct.to_f32(vals))
        assert np.array_equal(np.array(nova.nova_get_matrix_f64(t, which)), ct.to_f64(vals))
        assert nova.nova_get_matrix(t, which) == mat
    with pytest.raises(nova.NovaError):
        nova.nova_get_matrix_int8(nova.nova_make_transforms(points, m, 3), nova.NOVA_MATRIX_A)


def test_fp16_matrix_rounding_covers_subnormals():
    # G entries of wide integer point sets fall below 2^-14: 1/F_p = 1/40320 for F(8,3)
    pts = synth.point_set("standard", 8)
    G = ct.cook_toom([Fr(a, b) for a, b in pts], 8, 3)[2]
    assert min(abs(e) for row in G for e in row if e != 0) < Fr(1, 2 ** 14)
    t16 = nova.nova_make_transforms(pts, 8, 3, matrix_dtype="f16")
    assert np.array_equal(np.array(nova.nova_get_matrix_f64(t16, nova.NOVA_MATRIX_G)), ct.to_f16(G).astype(np.float64))


def test_other_shapes_and_orders():
    # r = 5 and unordered, non-symmetric points: accepted by the host construction
    pts = [Fr(1, 3), Fr(-2), Fr(0), Fr(5, 7), Fr(1), Fr(-1, 2), Fr(3, 2)]
    t = nova.nova_make_transforms(pts, 4, 5)
    assert (t.n, t.symmetric) == (8, False)
    A, BT, G = ct.cook_toom(pts, 4, 5)
    assert nova.nova_get_matrix(t, nova.NOVA_MATRIX_BT) == BT and nova.nova_get_matrix(t, nova.NOVA_MATRIX_G) == G
    # symmetric set in a non-canonical order is not flagged symmetric
    t2 = nova.nova_make_transforms([1, -1, 0, 2, -2], 4, 3)
    assert not t2.symmetric
    assert nova.nova_get_matrix(t2, nova.NOVA_MATRIX_A) == ct.cook_toom([1, -1, 0, 2, -2], 4, 3)[0]


@pytest.mark.parametrize("name,m", ALL_SETS)
def test_kappa_matches_oracle(name, m):
    points = [Fr(a, b) for a, b in synth.point_set(name, m)]
    t = nova.nova_make_transforms(points, m, 3)
    got = nova.nova_kappa(t)
    A, BT, G = ct.cook_toom(points, m, 3)
    want = dict(V=ct.kappa_V(points), A=ct.kappa(A), B=ct.kappa(BT), G=ct.kappa(G))
    for key in want:
        assert got[key] == pytest.approx(want[key], rel=1e-7), key


def test_error_codes():
    L = nova.lib()
    handle = ctypes.c_void_p()

    def make(pairs, m, r=3, n_points=None):
        arr = (nova.nova_rational * max(len(pairs), 1))()
        for i, (a, b) in enumerate(pairs):
            arr[i].num, arr[i].den = a, b
        return L.nova_make_transforms(arr, len(pairs) if n_points is None else n_points, m, r, ctypes.byref(handle))

    std4 = synth.STANDARD[4]
    assert make(std4, 4) == 0
    L.nova_free_transforms(handle)
    assert make(std4[:-1], 4) == -1                         # wrong count
    assert make(std4, 0) == -1 and make(std4, 4, 0) == -1   # bad m / r
    assert make([(0, 1), (1, 0), (-1, 1), (2, 1), (-2, 1)], 4) == -1      # zero denominator
    assert make([(0, 1), (1, 1), (2, 2), (2, 1), (-2, 1)], 4) == -2       # 1 == 2/2
    assert handle.value is None
    big = [(0, 1)] + [(s * (10 ** 9 + 7 * i), 10 ** 9 + 9 + i) for i in range(4) for s in (1, -1)]
    assert make(big, 8) == -3                               # exact entries exceed 64 bits
    assert L.nova_make_transforms(None, 5, 4, 3, ctypes.byref(handle)) == -1
    assert make([(i, 1) for i in range(20)], 18, 3) == -1   # n > 16
    assert L.nova_get_matrix(None, 0, None) == -1
    assert L.nova_strerror(-2).decode().startswith("duplicate")
    # device entry points reject bad arguments before touching the GPU
    t = nova.nova_make_transforms(synth.STANDARD[4], 4, 3)
    assert L.nova_winograd_conv2d(t.handle, None, None, None, 1, 1, 1, 1, 1, 0, 0, None, 0, None) == -1
    t7 = nova.nova_make_transforms([0, 1, -1, 2, -2, 3, -3], 2, 7)
    assert L.nova_filter_transform(t7.handle, 1, 1, 1, 0, 1, None) == -6      # r = 7: host only
    t85 = nova.nova_make_transforms([0, 1, -1, 2, -2, 3, -3, 4, -4, 5, -5], 8, 5)
    assert L.nova_filter_transform(t85.handle, 1, 1, 1, 0, 1, None) == -6     # F(8,5): n = 12, host only
    assert L.nova_conv2d_workspace_bytes(1, 1, 1, 1, 1, 5, 3, 0, 0, 0) == 0   # m = 5
    assert L.nova_conv2d_workspace_bytes(1, 1, 1, 1, 1, 8, 5, 0, 0, 0) == 0   # F(8,5)
    assert L.nova_conv2d_workspace_bytes(1, 1, 1, 1, 1, 6, 5, 0, 0, 0) > 0    # F(6,5): n = 10


def test_extended_constructor_rejects_bad_options():
    arr = nova._points_array(synth.point_set("standard", 4))
    h = ctypes.c_void_p()
    L = nova.lib()
    ok_b = (ctypes.c_int * 6)(0, 0, 0, 0, 0, 0)
    assert L.nova_make_transforms_ex(arr, 5, 4, 3, 7, None, None, 0, ctypes.byref(h)) == -1        # unknown scaling
    assert L.nova_make_transforms_ex(arr, 5, 4, 3, 0, None, None, 9, ctypes.byref(h)) == -1        # unknown dtype
    assert L.nova_make_transforms_ex(arr, 5, 4, 3, 2, None, ok_b, 0, ctypes.byref(h)) == -1        # exponents missing
    big = (ctypes.c_int * 6)(0, 61, 0, 0, 0, 0)
    assert L.nova_make_transforms_ex(arr, 5, 4, 3, 2, big, ok_b, 0, ctypes.byref(h)) == -1         # out of range
    assert h.value is None
    assert L.nova_make_transforms_ex(arr, 5, 4, 3, 2, ok_b, ok_b, 0, ctypes.byref(h)) == 0
    assert L.nova_get_row_scaling(None, None, None) == -1
    L.nova_free_transforms(h)


def test_sizes_follow_documented_layouts():
    # U [n*n][ceil(C/32)][Kp][32], V [n*n][ceil(C/32)][T][32], M [n*n][ceil(K/32)][Tp][32], Tp = 128*ceil(T/128)
    assert nova.nova_filter_bytes(256, 256, 8, nova.NOVA_F16) == 100 * 8 * 256 * 32 * 2
    assert nova.nova_filter_bytes(20, 3, 4, nova.NOVA_F32) == 36 * 1 * 32 * 32 * 4
    assert nova.nova_input_bytes(32, 256, 56, 56, 8, nova.NOVA_F16) == 100 * 8 * (32 * 49) * 32 * 2
    assert nova.nova_product_bytes(2, 40, 9, 13, 6, nova.NOVA_F16) == 64 * 2 * 128 * 32 * 4          # T = 12
    assert nova.nova_product_bytes(2, 40, 9, 13, 6, nova.NOVA_F16, nova.NOVA_FLAG_M_F16) == 64 * 2 * 128 * 32 * 2
    whole = nova.nova_conv2d_workspace_bytes(32, 256, 56, 56, 256, 8, nova.NOVA_F16, 0, 32)
    assert whole == 100 * 8 * 1568 * 32 * 2 + 100 * 8 * 1664 * 32 * 4          # T = 1568, Tp = 1664
    one = nova.nova_conv2d_workspace_bytes(32, 256, 56, 56, 256, 8, nova.NOVA_F16, 0, 1)
    assert one == 100 * 8 * 49 * 32 * 2 + 100 * 8 * 128 * 32 * 4
    default = nova.nova_conv2d_workspace_bytes(32, 256, 56, 56, 256, 8, nova.NOVA_F16, 0, 0)
    assert default == whole
    # at most 4 input channels: V compact [n*n][T][4], packed filters [n*n][Kp][4], no M (each part 256-byte aligned)
    few = nova.nova_conv2d_workspace_bytes(32, 3, 224, 224, 64, 8, nova.NOVA_F16, 0, 32)
    assert few == 100 * (32 * 28 * 28) * 4 * 2 + 100 * 64 * 4 * 2
    few32 = nova.nova_conv2d_workspace_bytes(2, 4, 9, 13, 40, 6, nova.NOVA_F32, 0, 2)                 # T = 12, Kp = 64
    assert few32 == 64 * 12 * 4 * 4 + 64 * 64 * 4 * 4
    assert nova.nova_conv2d_workspace_bytes(2, 5, 9, 13, 40, 6, nova.NOVA_F32, 0, 2) == 64 * 1 * 12 * 32 * 4 + 64 * 2 * 128 * 32 * 4
    # 5 x 5 kernels: n = m + 4, tiles still at stride m
    assert nova.nova_filter_bytes(64, 64, 4, nova.NOVA_F16, r=5) == 64 * 2 * 64 * 32 * 2
    assert nova.nova_input_bytes(2, 64, 9, 13, 6, nova.NOVA_F16, r=5) == 100 * 2 * 12 * 32 * 2       # T = 2*2*3
    assert nova.nova_product_bytes(2, 40, 9, 13, 6, nova.NOVA_F16, r=5) == 100 * 2 * 128 * 32 * 4


@pytest.mark.parametrize("m,r,d_max", [(2, 3, 3), (2, 3, 10), (3, 3, 4), (4, 3, 6), (4, 3, 10), (5, 3, 5), (6, 3, 6),
                                       (8, 3, 6), (2, 5, 6), (4, 5, 5)])
def test_symmetric_search_equals_oracle(m, r, d_max):
    points, kappa = nova.nova_symmetric_search(m, r, d_max)
    want_points, want_kappa = discovery.symmetric_search(m, r, d_max)
    assert points == want_points
    assert kappa == pytest.approx(want_kappa, rel=1e-9)
    # the result is ready for the constructor, and is the paired order the device kernels exploit
    t = nova.nova_make_transforms(points, m, r)
    assert t.symmetric == ((m + r) % 2 == 1)           # zero is part of the set only for an odd number of points


def test_symmetric_search_rejects_bad_arguments():
    L = nova.lib()
    buf, kappa = (nova.nova_rational * 16)(), ctypes.c_double()
    assert L.nova_symmetric_search(0, 3, 6, buf, ctypes.byref(kappa)) == -1
    assert L.nova_symmetric_search(4, 3, 0, buf, ctypes.byref(kappa)) == -1
    assert L.nova_symmetric_search(4, 3, 65, buf, ctypes.byref(kappa)) == -1
    assert L.nova_symmetric_search(4, 3, 6, None, ctypes.byref(kappa)) == -1
    assert L.nova_symmetric_search(14, 3, 6, buf, ctypes.byref(kappa)) == -6      # too many combinations
    assert L.nova_symmetric_search(1, 1, 6, buf, ctypes.byref(kappa)) == -1       # fewer than two finite points


def test_snap_to_rational_equals_oracle():
    rng = np.random.default_rng(12)
    xs = list(rng.uniform(-6.5, 6.5, 300)) + [0.0, 0.5, -0.5, 1e-13, -1e-300, 5.0, 5.5, -5.999, 6.0, 123.0, 0.8333, 1 / 3,
                                               2 / 7, 0.1 + 0.2, 1.25, -4.95]
    for d_max in (1, 2, 6, 10, 37):
        for x in xs:
            assert nova.nova_snap_to_rational(x, d_max) == discovery.snap_to_rational(x, d_max), (x, d_max)
    L = nova.lib()
    out = nova.nova_rational()
    assert L.nova_snap_to_rational(float("nan"), 10, ctypes.byref(out)) == -1
    assert L.nova_snap_to_rational(0.5, 0, ctypes.byref(out)) == -1
    assert L.nova_snap_to_rational(0.5, 10, None) == -1


def test_evolution_strategy_equals_oracle_for_fixed_draws():
    # Alg. "Evolution Strategy for Winograd Point Discovery": the same standard normal draws go to both
    # implementations; fitness values agree to rounding and the runs pick the same candidates
    from oracle import discovery
    for m in (2, 4, 6):
        p = [a / b for a, b in synth.NOVA[m]]
        got, want = nova.nova_es_fitness(m, 3, p), discovery.es_fitness(p, m, 3)
        assert got[0] == pytest.approx(want[0], rel=1e-12) and got[3] == pytest.approx(want[3], rel=1e-10)
        assert got[1] < 1e-12 and got[2] == pytest.approx(want[2], rel=1e-15)
    assert nova.nova_es_fitness(4, 3, [0.5, 0.5, 1.0, -1.0, 0.0])[0] == np.inf
    for m, seed, gens, pop, restarts in ((4, 0, 12, 20, 2), (6, 1, 6, 16, 1), (2, 2, 10, 8, 3)):
        count = discovery.es_normals_needed(m, 3, gens, pop, restarts)
        assert nova.nova_es_normals_needed(m, 3, gens, pop, restarts) == count
        z = np.random.default_rng(seed).standard_normal(count)
        p_o, f_o = discovery.evolution_strategy(m, 3, z, gens, pop, restarts)
        p_l, f_l = nova.nova_evolution_strategy(m, 3, z, gens, pop, restarts)
        assert f_l == pytest.approx(f_o, rel=1e-9)
        assert np.allclose(p_l, p_o, rtol=0, atol=1e-9)
    with pytest.raises(nova.NovaError):
        nova.nova_evolution_strategy(4, 3, np.zeros(10), 12, 20, 2)          # too few draws


def test_snap_points_equals_oracle():
    from oracle import discovery
    for x in ([0.0, 0.8334, -0.8331, 1.1669, -1.16], [0.3301, 0.3302, -0.5, 0.0, 1.0], [0.04, -0.21, 0.35, 0.28, -0.36]):
        want, kappa_o = discovery.snap_points(x, 4, 3)
        got, kappa_l = nova.nova_snap_points(4, 3, x)
        assert got == want and kappa_l == pytest.approx(kappa_o, rel=1e-10)
    want, _ = discovery.snap_points([0.1, 0.1001, -0.7], 2, 3, d_max=4)
    assert nova.nova_snap_points(2, 3, [0.1, 0.1001, -0.7], d_max=4)[0] == want


def test_conv2d_path_names_the_kernels_of_a_layer_shape():
    # host-side decision only: which kernels nova_winograd_conv2d would launch
    t8 = nova.nova_make_transforms(synth.point_set("nova", 8), 8, 3)
    t6 = nova.nova_make_transforms(synth.point_set("nova", 6), 6, 3)
    t4 = nova.nova_make_transforms(synth.point_set("nova", 4), 4, 3)
    F16, F32 = nova.NOVA_F16, nova.NOVA_F32
    assert nova.nova_conv2d_path(t8, 3, 224, 224, 64, F16) == nova.NOVA_PATH_FEW_CHANNELS
    assert nova.nova_conv2d_path(t8, 64, 224, 224, 64, F16) == nova.NOVA_PATH_FUSED_OUTPUT
    assert nova.nova_conv2d_path(t8, 64, 17, 23, 192, F16) == nova.NOVA_PATH_FUSED_OUTPUT
    assert nova.nova_conv2d_path(t6, 64, 56, 56, 64, F16) == nova.NOVA_PATH_FUSED_OUTPUT
    assert nova.nova_conv2d_path(t6, 64, 112, 112, 128, F16) == nova.NOVA_PATH_FUSED_OUTPUT
    for (t, C, K, dt, flags) in ((t8, 128, 128, F16, 0), (t8, 64, 80, F16, 0), (t8, 64, 64, F32, 0),
                                 (t8, 64, 64, F16, nova.NOVA_FLAG_M_F16), (t4, 64, 64, F16, 0), (t8, 256, 256, F16, 0)):
        assert nova.nova_conv2d_path(t, C, 56, 56, K, dt, flags) == nova.NOVA_PATH_STAGES
    with pytest.raises(nova.NovaError):
        nova.nova_conv2d_path(t8, 0, 56, 56, 64, F16)
