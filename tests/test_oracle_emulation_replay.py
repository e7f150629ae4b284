"""Pin of the reduced-precision emulation's general (inexact) case: an exact replay.

oracle.conv.winograd_conv2d_emulated is C code on hardware floats.  Here the same contract
(Sec. "Float16 Precision Analysis" set-up: binary16 storage, binary32 transforms) is evaluated a
second time in exact rational arithmetic: every product, sum and fused multiply-add is formed
exactly on Fractions and then rounded to the format the contract names for that step with
cook_toom._round_fraction, which has pins of its own (against numpy's conversions).  The two must
agree bit for bit in U, V, M and y for every combination of the options.  A rounding that is
skipped, done in the wrong format or at the wrong place, an option that is ignored or takes the
wrong branch, a transposed matrix or a wrong tile offset all change some bit: the test also checks
that each rounding step it replays is not the identity on this data.

The contract, step by step (all roundings to nearest, ties to even):
  matrices  exact entry -> binary32 (A, B^T) / binary64 (G); transform_dtype "f16": -> binary16 first
  U         G g G^T in binary64 arithmetic (products and sums rounded one by one, index ascending,
            first G g, then . G^T), then one rounding to the storage format
  V         binary32: a 1D transform row is E + O, E / O fused-multiply-add chains from 0 over the
            even / odd indices in ascending order, coefficients that are exactly zero skipped;
            columns of the tile first, then rows; then one rounding to the storage format.
            v_exact: B^T d B in binary64 arithmetic instead, then the one rounding
  M         sum over channels of U * V in binary64 arithmetic, channel ascending, then one rounding
            to binary32 or binary16 (m_storage)
  y         A^T M A in binary64 arithmetic, optional ReLU, one rounding to the storage format; the
            image is zero-extended to whole tiles and the result cropped
"""
from fractions import Fraction as Fr

import numpy as np
import pytest

from oracle import conv
from oracle import cook_toom as ct
from paper_2512_18453_amd import synth

F16 = (11, -14)
F32 = (24, -126)
F64 = (53, -1022)


def rnd(value, fmt):
    return ct._round_fraction(value, *fmt)


def fr(x):
    return Fr(float(x))                  # exact: every float is a rational


class Replay:
    """Counts, per rounding step, how often the rounding changed the value."""

    def __init__(self):
        self.changed = {}

    def round(self, value, fmt, step):
        out = rnd(value, fmt)
        assert abs(out) < 65504 or fmt != F16, "replay has no overflow handling; keep the data in range"
        self.changed[step] = self.changed.get(step, 0) + (out != value)
        return out

    def dot64(self, left, right, step):
        """sum_k left[k] * right[k] as binary64 multiplications and additions, k ascending, from 0."""
        acc = Fr(0)
        for a, b in zip(left, right):
            acc = self.round(acc + self.round(a * b, F64, step + ".mul64"), F64, step + ".add64")
        return acc

    def sandwich64(self, L, mid, R):
        """L mid R^T in binary64 arithmetic: first L mid, then (.) R^T."""
        inner, inner2 = len(mid), len(mid[0])
        tmp = [[self.dot64(L[i], [mid[a][b] for a in range(inner)], "sandwich") for b in range(inner2)]
               for i in range(len(L))]
        return [[self.dot64(tmp[i], R[j], "sandwich") for j in range(len(R))] for i in range(len(L))]

    def transform32(self, BT, v):
        """One 1D input transform in binary32 (E + O, fused multiply-add chains)."""
        n = len(BT)
        out = []
        for p in range(n):
            even = odd = Fr(0)
            for a in range(0, n, 2):
                if BT[p][a] != 0:
                    even = self.round(BT[p][a] * v[a] + even, F32, "V.fma32")
            for a in range(1, n, 2):
                if BT[p][a] != 0:
                    odd = self.round(BT[p][a] * v[a] + odd, F32, "V.fma32")
            out.append(self.round(even + odd, F32, "V.add32"))
        return out


def replay(x, g, points, m, storage, m_storage, v_exact, transform_dtype, relu):
    """x [N][C][H][W], g [K][C][r][r] numpy arrays of values exact in the storage format.
    Returns (y, U, V, M) as numpy fp64 arrays in the oracle's layouts, and the Replay counters."""
    rp = Replay()
    N, C, H, W = x.shape
    K, r = g.shape[0], g.shape[-1]
    n, pad = m + r - 1, (r - 1) // 2
    st = F16 if storage == 16 else F32
    mst = F16 if m_storage == 16 else F32
    A, BT, G = ct.cook_toom(points, m, r)
    if transform_dtype == "f16":
        A = [[rnd(e, F16) for e in row] for row in A]
        BT = [[rnd(e, F16) for e in row] for row in BT]
        G = [[rnd(e, F16) for e in row] for row in G]
    A32 = [[rnd(e, F32) for e in row] for row in A]
    BT32 = [[rnd(e, F32) for e in row] for row in BT]
    G64 = [[rnd(e, F64) for e in row] for row in G]
    AT = [[A32[p][i] for p in range(n)] for i in range(m)]

    th, tw = -(-H // m), -(-W // m)
    T = N * th * tw
    U = np.empty((n * n, K, C))
    V = np.empty((n * n, T, C))
    M = np.empty((n * n, T, K))
    y = np.empty((N, K, H, W))
    Uq = {}
    for k in range(K):
        for c in range(C):
            gk = [[fr(g[k, c, a, b]) for b in range(r)] for a in range(r)]
            u = rp.sandwich64(G64, gk, G64)
            for i in range(n):
                for j in range(n):
                    Uq[i * n + j, k, c] = rp.round(u[i][j], st, "U.store")
                    U[i * n + j, k, c] = float(Uq[i * n + j, k, c])
    for img in range(N):
        for tr in range(th):
            for tc in range(tw):
                t = (img * th + tr) * tw + tc
                Vq = {}
                for c in range(C):
                    d = [[Fr(0)] * n for _ in range(n)]
                    for a in range(n):
                        for b in range(n):
                            hh, ww = tr * m - pad + a, tc * m - pad + b
                            if 0 <= hh < H and 0 <= ww < W:
                                d[a][b] = fr(x[img, c, hh, ww])
                    if v_exact:
                        v = rp.sandwich64(BT32, d, BT32)
                    else:
                        cols = [rp.transform32(BT32, [d[a][b] for a in range(n)]) for b in range(n)]   # cols[b][i]
                        v = [rp.transform32(BT32, [cols[b][i] for b in range(n)]) for i in range(n)]
                    for i in range(n):
                        for j in range(n):
                            Vq[i * n + j, c] = rp.round(v[i][j], st, "V.store")
                            V[i * n + j, t, c] = float(Vq[i * n + j, c])
                for k in range(K):
                    Mk = [[None] * n for _ in range(n)]
                    for xi in range(n * n):
                        s = rp.dot64([Uq[xi, k, c] for c in range(C)], [Vq[xi, c] for c in range(C)], "M")
                        Mk[xi // n][xi % n] = rp.round(s, mst, "M.store")
                        M[xi, t, k] = float(Mk[xi // n][xi % n])
                    Y = rp.sandwich64(AT, Mk, AT)
                    for p in range(m):
                        for q in range(m):
                            h, w = tr * m + p, tc * m + q
                            if h < H and w < W:
                                out = Y[p][q]
                                if relu and out < 0:
                                    out = Fr(0)
                                y[img, k, h, w] = float(rp.round(out, st, "y.store"))
    return y, U, V, M, rp


def layer(m, storage, seed):
    """Two tiles, the second ragged (3 of its m columns lie in the image), 3 channels, 2 filters."""
    x, g = synth.make_layer(1, 3, 2, m, m + 3, seed=seed, dtype="f16" if storage == 16 else "f32", x_dist="normal")
    return x.astype(np.float64), g.astype(np.float64)


def first_difference(got, want, what):
    bad = np.argwhere(got != want)
    assert len(bad) == 0, f"{what}: {len(bad)} of {got.size} differ, first at {tuple(bad[0])}: " \
                          f"oracle {got[tuple(bad[0])]!r} replay {want[tuple(bad[0])]!r}"


@pytest.mark.parametrize("storage", [16, 32])
@pytest.mark.parametrize("m_storage", [16, 32])
@pytest.mark.parametrize("transform_dtype", ["f32", "f16"])
@pytest.mark.parametrize("v_exact", [False, True])
def test_emulation_equals_exact_replay_f83_discovered_points(storage, m_storage, transform_dtype, v_exact):
    m = 8
    points = [Fr(a, b) for a, b in synth.NOVA[m]]
    x, g = layer(m, storage, seed=811)
    relu = not v_exact                            # both settings of the flag are visited
    y_r, U_r, V_r, M_r, rp = replay(x, g, points, m, storage, m_storage, v_exact, transform_dtype, relu)
    y_o, U_o, V_o, M_o = conv.winograd_conv2d_emulated(x, g, points, m, storage=storage, m_storage=m_storage,
                                                      v_exact=v_exact, relu=relu, transform_dtype=transform_dtype,
                                                      want_intermediates=True)
    first_difference(U_o, U_r, "U")
    first_difference(V_o, V_r, "V")
    first_difference(M_o, M_r, "M")
    first_difference(y_o, y_r, "y")
    # every rounding the contract names did change values on this data, so leaving one out cannot pass
    for step in ("U.store", "V.store", "M.store", "y.store", "sandwich.mul64", "sandwich.add64"):
        if step == "V.store" and storage == 32 and not v_exact:
            continue                              # binary32 chain stored as binary32: nothing to round
        if step.startswith("sandwich") and transform_dtype == "f16":
            continue                              # binary16 matrix entries: the binary64 products are exact
        assert rp.changed.get(step, 0) > 0, step
    if not v_exact:
        assert rp.changed["V.fma32"] > 0 and rp.changed["V.add32"] > 0
    if relu:
        assert (y_o == 0).any() and (y_o > 0).any()
    if storage == 16:
        # products of binary16 numbers and sums of three of them are exact in binary64 here, so M is
        # the exact channel sum rounded once
        assert rp.changed.get("M.mul64", 0) == 0 and rp.changed.get("M.add64", 0) == 0


@pytest.mark.parametrize("m,name", [(4, "standard"), (6, "nova"), (6, "classic_half")])
def test_emulation_equals_exact_replay_other_tiles(m, name):
    points = [Fr(a, b) for a, b in synth.point_set(name, m)]
    x, g = layer(m, 16, seed=400 + m)
    y_r, U_r, V_r, M_r, _ = replay(x, g, points, m, 16, 32, False, "f32", False)
    y_o, U_o, V_o, M_o = conv.winograd_conv2d_emulated(x, g, points, m, storage=16, want_intermediates=True)
    first_difference(U_o, U_r, "U")
    first_difference(V_o, V_r, "V")
    first_difference(M_o, M_r, "M")
    first_difference(y_o, y_r, "y")


def test_emulation_equals_exact_replay_with_row_scaling_and_5x5():
    # balanced power-of-two rows (F(4,3), integer points) and a 5 x 5 kernel (F(2,5), border 2)
    points = [Fr(a, b) for a, b in synth.STANDARD[4]]
    x, g = layer(4, 16, seed=77)
    A, BT, G = ct.cook_toom(points, 4, 3)
    log2_b, log2_g = ct.balanced_row_exponents(BT, G)
    y_o, U_o, V_o, M_o = conv.winograd_conv2d_emulated(x, g, points, 4, storage=16, row_scaling="balanced",
                                                      want_intermediates=True)
    y_p, U_p, V_p, _ = conv.winograd_conv2d_emulated(x, g, points, 4, storage=16, want_intermediates=True)
    # scaling a row by 2^e scales what it produces by 2^e exactly (no sub-normals or overflow on this data)
    fb = np.array([2.0 ** (log2_b[i] + log2_b[j]) for i in range(6) for j in range(6)])
    fg = np.array([2.0 ** (log2_g[i] + log2_g[j]) for i in range(6) for j in range(6)])
    assert np.array_equal(V_o, V_p * fb[:, None, None]) and np.array_equal(U_o, U_p * fg[:, None, None])
    rng = np.random.default_rng(5)
    x5 = rng.standard_normal((1, 2, 5, 4)).astype(np.float16).astype(np.float64)
    g5 = (rng.standard_normal((2, 2, 5, 5)) * 0.2).astype(np.float16).astype(np.float64)
    pts5 = [Fr(a, b) for a, b in synth.NOVA[4]]              # n = 6 = 2 + 5 - 1
    y_r, U_r, V_r, M_r, _ = replay(x5, g5, pts5, 2, 16, 32, False, "f32", False)
    y_o, U_o, V_o, M_o = conv.winograd_conv2d_emulated(x5, g5, pts5, 2, storage=16, want_intermediates=True)
    first_difference(U_o, U_r, "U")
    first_difference(V_o, V_r, "V")
    first_difference(M_o, M_r, "M")
    first_difference(y_o, y_r, "y")


def test_stored_tensors_are_fixed_points_of_their_rounding():
    m = 8
    points = [Fr(a, b) for a, b in synth.NOVA[m]]
    x, g = synth.make_layer(2, 5, 3, 13, 19, seed=3, dtype="f16")
    x, g = x.astype(np.float64), g.astype(np.float64)
    y, U, V, M = conv.winograd_conv2d_emulated(x, g, points, m, storage=16, m_storage=16, want_intermediates=True)
    for name, tensor in (("U", U), ("V", V), ("M", M), ("y", y)):
        assert np.array_equal(tensor.astype(np.float16).astype(np.float64), tensor), name
    y, U, V, M = conv.winograd_conv2d_emulated(x, g, points, m, storage=16, m_storage=32, want_intermediates=True)
    assert np.array_equal(M.astype(np.float32).astype(np.float64), M)
    assert not np.array_equal(M.astype(np.float16).astype(np.float64), M)     # binary32 M really is kept wider
    y, U, V, M = conv.winograd_conv2d_emulated(x, g, points, m, storage=32, want_intermediates=True)
    for name, tensor in (("U", U), ("V", V), ("M", M), ("y", y)):
        assert np.array_equal(tensor.astype(np.float32).astype(np.float64), tensor), name
        assert not np.array_equal(tensor.astype(np.float16).astype(np.float64), tensor), name
