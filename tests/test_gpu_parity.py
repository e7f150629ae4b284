"""GPU parity: every stage of the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.

Bars
  U (filter transform)   bit-exact (fp64 evaluation, one rounding, on both sides)
  V (input transform)    bit-exact (both sides follow the same binary32 operation order)
  M, y in fp16 storage   rel-L2 <= 5e-3 against the oracle's fp16-storage emulation
  y in fp32 storage      F(4,3) small layer: rel-L2 <= 1e-5 and max-abs <= 1e-4 against the fp64
                         definition; other tiles: within 4x the emulation's own distance from the
                         fp64 definition (the GPU adds fp32 accumulation and an fp32 output
                         transform on top of what the emulation rounds)
"""
import os
import sys
from fractions import Fraction as Fr

import numpy as np
import pytest
import torch

from oracle import conv, int8
from oracle import cook_toom as ct
from paper_2512_18453_amd import nova, synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def pts(pairs):
    return [Fr(a, b) for a, b in pairs]


def rel_l2(a, b):
    return float(np.linalg.norm((a - b).ravel()) / max(np.linalg.norm(b.ravel()), 1e-300))


def ulp16(v):
    """Spacing of binary16 numbers at |v| (the sub-normal spacing 2^-24 below 2^-14)."""
    a = np.maximum(np.abs(v), 2.0 ** -14)
    return 2.0 ** (np.floor(np.log2(a)) - 10)


def elementwise_fp16(got, emu, points, m, want_intermediates, C, what="y"):
    """Element-by-element bars for a binary16 output against the emulation, beside the rel-L2 bar.

    The two sides start from bit-identical U and V.  They differ in (i) the channel sum -- the matrix
    unit adds C exact products in binary32 in an order of its own, the emulation in binary64: at most
    C u |U||V| summed over c per entry of M in the standard model, u = 2^-24; (ii) one rounding of M
    to binary32 on each side: 2 u |M|; (iii) the output transform, two nested sums of n terms in
    binary32 against binary64: 2 n u |A|^T |M| |A|; (iv) the final rounding to binary16, which moves
    two neighbouring values at most one binary16 spacing further apart.  With
    P[xi] = sum_c |U[xi]| |V[xi]| >= |M[xi]| and w[xi] = |A[i][p]| |A[j][q]|:

      worst case    |y_gpu - y_emu| <= ulp16(y) + 2 (C + 2 n + 2) u  sum_xi w P
                    (every rounding error at its maximum and of the same sign; the factor 2 allows
                    for intermediate sums of the matrix unit that are truncated, not rounded);
      statistical   |y_gpu - y_emu| <= ulp16(y) + 8 sqrt(C + 2 n + 2) u  sqrt(sum_xi (w P)^2)
                    (the C + 2 n + 2 rounding errors per position modelled as independent, zero
                    mean, each below u times its position's term: the second summand is about
                    8 sqrt(3) = 14 standard deviations of their sum, and 3 to 40 times narrower
                    than the worst case, narrow enough that a single misplaced or stale output
                    element -- wrong by about rms(y) -- fails it on every shape here).

    Both must hold for every element, and non-finite values must sit at the same places.
    Returns max |diff| / statistical bound and the median statistical bound relative to rms(y)."""
    y_o, U_o, V_o, M_o = want_intermediates
    n = int(round(np.sqrt(U_o.shape[0])))
    r = n - m + 1
    A = np.abs(ct.to_f32(ct.cook_toom(pts(points), m, r)[0]).astype(np.float64))      # n x m
    N, K, H, W = emu.shape
    th, tw = -(-H // m), -(-W // m)
    P = np.matmul(np.abs(V_o), np.abs(U_o).transpose(0, 2, 1)).reshape(n, n, N * th * tw, K)

    def to_image(per_tile):
        return per_tile.reshape(N, th, tw, K, m, m).transpose(0, 3, 1, 4, 2, 5).reshape(N, K, th * m, tw * m)[:, :, :H, :W]

    lin = to_image(np.einsum("ip,jq,ijtk->tkpq", A, A, P, optimize=True))
    rss = to_image(np.sqrt(np.einsum("ip,jq,ijtk->tkpq", A * A, A * A, P * P, optimize=True)))
    fin = np.isfinite(emu)
    assert np.array_equal(np.isfinite(got), fin), f"{what}: non-finite values at different places"
    spacing = ulp16(np.where(fin, np.maximum(np.abs(emu), np.abs(got)), 0.0))
    terms = C + 2 * n + 2
    worst = spacing + 2.0 * terms * 2.0 ** -24 * lin
    stat = spacing + 8.0 * np.sqrt(terms) * 2.0 ** -24 * rss
    diff = np.abs(np.where(fin, got - emu, 0.0))
    for name, bound in (("worst-case", worst), ("statistical", stat)):
        if (diff > bound).any():
            idx = np.unravel_index(np.argmax(diff / bound), diff.shape)
            raise AssertionError(f"{what}: element {idx} gpu {got[idx]!r} emulation {emu[idx]!r} "
                                 f"{name} bound {bound[idx]:.3e}")
    return float((diff / stat).max()), float(np.median(stat[fin]) / max(np.sqrt(np.mean(emu[fin] ** 2)), 1e-300))


def same(got, want, what):
    """Bit-for-bit comparison with a readable failure."""
    if np.array_equal(got, want, equal_nan=True):
        return
    bad = np.argwhere(~((got == want) | (np.isnan(got) & np.isnan(want))))
    lines = [f"{what}: {len(bad)} of {got.size} entries differ; first:"]
    for idx in bad[:12]:
        idx = tuple(idx)
        lines.append(f"  {idx}: gpu {got[idx]!r} oracle {want[idx]!r}")
    raise AssertionError("\n".join(lines))


def takes_fused_path(t, C, K, dtype, flags=0, H=56, W=56):
    """Whether nova_winograd_conv2d runs contraction and output transform as one kernel for this shape."""
    code = nova.NOVA_F16 if dtype == np.float16 else nova.NOVA_F32
    return nova.nova_conv2d_path(t, C, H, W, K, code, flags) == nova.NOVA_PATH_FUSED_OUTPUT


def single_call_agrees(got, C, storage, fused=False):
    """nova_winograd_conv2d against the three stage calls.  They run the same kernels, so the results
    are equal bit for bit -- except with at most 4 input channels, where the single call forms the
    products inside the output transform (a binary32 multiply-add chain over the channels instead of
    the matrix unit's summation order): then the two agree to rounding."""
    a, b = got["y"], got["y_conv"]
    if C > 4 and not fused:
        assert np.array_equal(a, b, equal_nan=True)
        return
    if fused:
        # one kernel instead of two: another shape of matrix instruction, hence another summation order
        # over the channels; the callers check the single call's result against the emulation element by
        # element, here only that the two are close
        assert np.array_equal(np.isfinite(a), np.isfinite(b)) and rel_l2(a, b) < 1e-3
        return
    fin = np.isfinite(a) & np.isfinite(b)
    assert (np.isfinite(a) == np.isfinite(b)).mean() > 0.99
    if fin.all():
        # (the same bar as against the emulation in binary16 storage, where products rounded to binary16
        # may fall either way; binary32: two summation orders of at most 4 exact products)
        assert rel_l2(a, b) < (5e-3 if storage == 16 else 1e-4), rel_l2(a, b)


def unblock(flat, n2, rows, chans):
    """[n2][ceil(chans/32)][rows][32] flat device tensor -> numpy [n2][rows][chans] (fp64)."""
    blocks = -(-chans // 32)
    a = flat.detach().cpu().numpy().astype(np.float64).reshape(n2, blocks, rows, 32)
    return a.transpose(0, 2, 1, 3).reshape(n2, rows, blocks * 32)[:, :, :chans]


def run_stages(t, x, w, flags=0):
    """All stages through the C ABI; returns numpy U, V, M (logical layouts) and y."""
    N, C, H, W = x.shape
    K = w.shape[0]
    m, n2 = t.m, t.n * t.n
    T = N * (-(-H // m)) * (-(-W // m))
    xd, wd = torch.from_numpy(x).to(DEV), torch.from_numpy(w).to(DEV)
    U = nova.nova_filter_transform(t, wd)
    V = nova.nova_input_transform(t, xd)
    M = nova.nova_contract(t, U, V, N, C, H, W, K, flags)
    y = nova.nova_output_transform(t, M, N, K, H, W, xd.dtype, flags)
    y2 = nova.nova_winograd_conv2d(t, xd, U, K, flags=flags, images_per_slab=1)
    torch.cuda.synchronize()
    fused = takes_fused_path(t, C, K, x.dtype, flags, H=H, W=W)
    Kp = -(-K // 32) * 32
    Ul = unblock(U, n2, Kp, C)
    assert not Ul[:, K:, :].any()                       # padding rows are zero
    Tp = -(-T // 128) * 128                             # M has Tp rows per block; rows >= T are scratch
    out = dict(U=Ul[:, :K, :], V=unblock(V, n2, T, C), M=unblock(M, n2, Tp, K)[:, :T, :],
               y=y.cpu().numpy().astype(np.float64), y_conv=y2.cpu().numpy().astype(np.float64), fused=fused)
    return out


SMALL_FP16 = [
    # name, m, N, C, K, H, W
    ("standard", 2, 2, 8, 8, 7, 9),
    ("standard", 4, 2, 40, 48, 19, 14),
    ("nova", 4, 3, 33, 70, 30, 41),
    ("classic_half", 6, 2, 64, 32, 23, 56),
    ("nova", 6, 2, 40, 130, 56, 56),
    ("nova", 8, 3, 72, 96, 56, 56),
    ("nova", 8, 1, 3, 5, 17, 70),
    # narrow images of odd size: strips staged from unaligned runs, x not a whole number of 16-byte pieces
    ("nova", 4, 1, 3, 5, 7, 9),
    ("nova", 6, 3, 35, 40, 13, 21),
    # shapes that take the weight-stationary contraction (C in {64,128,256}, K a multiple of 64),
    # one per (waves along K, channel blocks) variant, with ragged last stages
    ("nova", 4, 2, 64, 64, 20, 20),
    ("nova", 6, 3, 128, 128, 30, 27),
    ("nova", 8, 2, 256, 256, 33, 40),
    ("nova", 8, 5, 64, 256, 56, 56),
    ("nova", 6, 2, 256, 128, 24, 24),
    ("nova", 4, 1, 128, 64, 64, 64),
    ("standard", 4, 1, 256, 512, 16, 16),
    ("nova", 8, 1, 128, 256, 17, 17),
    # C = 512 (tiled contraction), K = 512 / 128 / 64
    ("nova", 8, 5, 512, 512, 24, 24),
    ("nova", 6, 2, 512, 128, 13, 13),
    ("nova", 4, 1, 512, 64, 12, 20),
]


@pytest.mark.parametrize("name,m,N,C,K,H,W", SMALL_FP16)
def test_fp16_stages_against_emulation(name, m, N, C, K, H, W):
    say(f"[case] fp16 stages {name} F({m},3) N={N} C={C} K={K} H={H} W={W}")
    points = synth.point_set(name, m)
    x, w = synth.make_layer(N, C, K, H, W, seed=100 * m + C, dtype="f16")
    t = nova.nova_make_transforms(points, m, 3)
    got = run_stages(t, x, w)
    x64, w64 = x.astype(np.float64), w.astype(np.float64)
    emu = conv.winograd_conv2d_emulated(x64, w64, pts(points), m, storage=16, want_intermediates=True)
    y_o, U_o, V_o, M_o = emu
    same(got["U"], U_o, "U")
    same(got["V"], V_o, "V")
    assert rel_l2(got["M"], M_o) < 1e-5
    single_call_agrees(got, x.shape[1], 16 if x.dtype == np.float16 else 32, got["fused"])
    err = rel_l2(got["y"], y_o)
    say(f"  rel-L2 vs emulation {err:.3e}; vs fp64 definition {rel_l2(got['y'], conv.direct_conv2d(x64, w64)):.3e}")
    assert err < 5e-3
    ratio, width = elementwise_fp16(got["y"], y_o, points, m, emu, C)
    ratio2, _ = elementwise_fp16(got["y_conv"], y_o, points, m, emu, C, "y (single call)")
    say(f"  element-wise: max |diff| / bound {ratio:.3f} (single call {ratio2:.3f}); median bound / rms(y) {width:.2e}")


def test_fp32_small_layer_against_definition():
    cfg = synth.LAYER_CONFIGS["small_f43_fp32"]
    say(f"[case] fp32 small layer {cfg}")
    x, w = synth.make_layer(cfg["N"], cfg["C"], cfg["K"], cfg["H"], cfg["W"], seed=cfg["seed"],
                            dtype="f32", x_dist=cfg["x_dist"])
    points = synth.point_set("standard", 4)
    t = nova.nova_make_transforms(points, 4, 3)
    got = run_stages(t, x, w)
    want = conv.direct_conv2d(x.astype(np.float64), w.astype(np.float64))
    err, mx = rel_l2(got["y"], want), float(np.abs(got["y"] - want).max())
    say(f"  rel-L2 {err:.3e} max-abs {mx:.3e}")
    assert err <= 1e-5 and mx <= 1e-4
    single_call_agrees(got, x.shape[1], 16 if x.dtype == np.float16 else 32, got["fused"])
    _, U_o, V_o, _ = conv.winograd_conv2d_emulated(x.astype(np.float64), w.astype(np.float64), pts(points), 4,
                                                   storage=32, want_intermediates=True)
    same(got["U"], U_o, "U")
    same(got["V"], V_o, "V")


@pytest.mark.parametrize("name,m", [("nova", 4), ("nova", 6), ("classic_half", 6), ("nova", 8), ("standard", 8)])
def test_fp32_other_tiles(name, m):
    say(f"[case] fp32 {name} F({m},3)")
    points = synth.point_set(name, m)
    x, w = synth.make_layer(2, 40, 36, 3 * m + 2, 5 * m - 1, seed=7 + m, dtype="f32", x_dist="normal")
    t = nova.nova_make_transforms(points, m, 3)
    got = run_stages(t, x, w)
    x64, w64 = x.astype(np.float64), w.astype(np.float64)
    want = conv.direct_conv2d(x64, w64)
    y_o, U_o, V_o, M_o = conv.winograd_conv2d_emulated(x64, w64, pts(points), m, storage=32, want_intermediates=True)
    same(got["U"], U_o, "U")
    same(got["V"], V_o, "V")
    own = rel_l2(y_o, want)
    err = rel_l2(got["y"], y_o)
    say(f"  emulation vs definition {own:.3e}; gpu vs emulation {err:.3e}; gpu vs definition {rel_l2(got['y'], want):.3e}")
    assert err <= max(1e-5, 4 * own)


@pytest.mark.parametrize("m", [4, 6, 8])
def test_fp32_narrow_images(m):
    # few tiles per tile row: workgroups take several tile rows, strips come from unaligned runs
    say(f"[case] fp32 narrow image F({m},3)")
    points = synth.point_set("nova", m)
    x, w = synth.make_layer(3, 9, 33, 2 * m + 3, 2 * m + 1, seed=70 + m, dtype="f32", x_dist="normal")
    t = nova.nova_make_transforms(points, m, 3)
    got = run_stages(t, x, w)
    x64, w64 = x.astype(np.float64), w.astype(np.float64)
    y_o, U_o, V_o, M_o = conv.winograd_conv2d_emulated(x64, w64, pts(points), m, storage=32, want_intermediates=True)
    same(got["U"], U_o, "U")
    same(got["V"], V_o, "V")
    own = rel_l2(y_o, conv.direct_conv2d(x64, w64))
    err = rel_l2(got["y"], y_o)
    say(f"  emulation vs definition {own:.3e}; gpu vs emulation {err:.3e}")
    assert err <= max(1e-5, 4 * own)
    single_call_agrees(got, x.shape[1], 16 if x.dtype == np.float16 else 32, got["fused"])


def test_generic_point_order_uses_the_same_contract():
    # the same F(4,3) points in a non-canonical order run through the generic (non-paired) kernels
    say("[case] generic path, permuted and asymmetric points")
    for points in ([(1, 1), (0, 1), (-1, 1), (-2, 1), (2, 1)], [(1, 3), (0, 1), (-1, 1), (5, 4), (-2, 3)]):
        t = nova.nova_make_transforms(points, 4, 3)
        assert not t.symmetric
        x, w = synth.make_layer(2, 20, 12, 11, 18, seed=3, dtype="f16")
        got = run_stages(t, x, w)
        emu = conv.winograd_conv2d_emulated(x.astype(np.float64), w.astype(np.float64), pts(points), 4,
                                            storage=16, want_intermediates=True)
        y_o, U_o, V_o, M_o = emu
        same(got["U"], U_o, "U")
        same(got["V"], V_o, "V")
        assert rel_l2(got["y"], y_o) < 5e-3
        elementwise_fp16(got["y"], y_o, points, 4, emu, 20)
        elementwise_fp16(got["y_conv"], y_o, points, 4, emu, 20, "y (single call)")


def test_flags_relu_and_fp16_products():
    say("[case] flags: relu, fp16 M")
    points = synth.point_set("nova", 6)
    x, w = synth.make_layer(2, 48, 40, 20, 31, seed=21, dtype="f16", x_dist="normal")
    t = nova.nova_make_transforms(points, 6, 3)
    x64, w64 = x.astype(np.float64), w.astype(np.float64)
    got = run_stages(t, x, w, flags=nova.NOVA_FLAG_RELU)
    emu = conv.winograd_conv2d_emulated(x64, w64, pts(points), 6, storage=16, relu=True, want_intermediates=True)
    y_o = emu[0]
    assert (got["y"] >= 0).all() and rel_l2(got["y"], y_o) < 5e-3
    elementwise_fp16(got["y"], y_o, points, 6, emu, 48)          # (ReLU does not widen a difference)
    elementwise_fp16(got["y_conv"], y_o, points, 6, emu, 48, "y (single call)")
    assert ((got["y"] == 0) == (y_o == 0)).mean() > 0.999
    got = run_stages(t, x, w, flags=nova.NOVA_FLAG_M_F16)
    y_o, _, _, M_o = conv.winograd_conv2d_emulated(x64, w64, pts(points), 6, storage=16, m_storage=16,
                                                  want_intermediates=True)
    assert rel_l2(got["M"], M_o) < 2e-4          # fp32 vs fp64 accumulation flips few binary16 roundings
    assert rel_l2(got["y"], y_o) < 5e-3


@pytest.mark.parametrize("m,C,K,H,W", [(8, 3, 64, 40, 48), (6, 4, 40, 23, 31), (4, 1, 33, 18, 18), (8, 2, 5, 9, 70)])
def test_few_input_channels_single_call(m, C, K, H, W):
    # the first layer of an image network: with C <= 4 the single call forms the products inside the
    # output transform and keeps no M.  Checked against the emulation like every other layer, in both
    # storage formats, with ReLU, binary16 products and the fused pooling.
    points = synth.point_set("nova", m)
    t = nova.nova_make_transforms(points, m, 3)
    rng = np.random.default_rng(4000 + 10 * m + C)
    assert nova.nova_conv2d_workspace_bytes(2, C, H, W, K, m, nova.NOVA_F16) < \
        nova.nova_conv2d_workspace_bytes(2, 5, H, W, K, m, nova.NOVA_F16)
    for dtype, storage in ((np.float16, 16), (np.float32, 32)):
        for flags in (0, nova.NOVA_FLAG_RELU, nova.NOVA_FLAG_M_F16 | nova.NOVA_FLAG_RELU):
            if storage == 32 and flags & nova.NOVA_FLAG_M_F16:
                continue
            say(f"[case] few channels F({m},3) {np.dtype(dtype).name} C={C} K={K} H={H} W={W} flags={flags}")
            x = rng.standard_normal((2, C, H, W)).astype(dtype)
            w = (rng.standard_normal((K, C, 3, 3)) * np.sqrt(2.0 / (9 * C))).astype(dtype)
            xd, wd = torch.from_numpy(x).to(DEV), torch.from_numpy(w).to(DEV)
            U = nova.nova_filter_transform(t, wd)
            y = nova.nova_winograd_conv2d(t, xd, U, K, flags=flags)
            x64, w64 = x.astype(np.float64), w.astype(np.float64)
            relu = bool(flags & nova.NOVA_FLAG_RELU)
            emu = conv.winograd_conv2d_emulated(x64, w64, pts(points), m, storage=storage, relu=relu,
                                                m_storage=16 if flags & nova.NOVA_FLAG_M_F16 else 32,
                                                want_intermediates=True)
            y_o = emu[0]
            want = conv.direct_conv2d(x64, w64)
            own = rel_l2(y_o, np.maximum(want, 0.0) if relu else want)
            err = rel_l2(y.cpu().numpy().astype(np.float64), y_o)
            say(f"  rel-L2 vs emulation {err:.3e} (emulation vs definition {own:.3e})")
            assert err < (5e-3 if storage == 16 else max(1e-5, 8 * own))
            if storage == 16 and not flags & nova.NOVA_FLAG_M_F16:
                elementwise_fp16(y.cpu().numpy().astype(np.float64), y_o, points, m, emu, C)
            if H % 2 == 0 and W % 2 == 0:
                pooled = nova.nova_winograd_conv2d(t, xd, U, K, flags=flags | nova.NOVA_FLAG_POOL2)
                assert torch.equal(pooled.float(), torch.nn.functional.max_pool2d(y.float(), 2))


def test_integer_point_f83_blows_up_identically():
    say("[case] integer-point F(8,3) in fp16: non-finite agreement")
    points = synth.point_set("standard", 8)
    x, w = synth.make_layer(1, 32, 8, 24, 24, seed=5, dtype="f16")
    t = nova.nova_make_transforms(points, 8, 3)
    got = run_stages(t, x, w)
    y_o, U_o, V_o, M_o = conv.winograd_conv2d_emulated(x.astype(np.float64), w.astype(np.float64), pts(points), 8,
                                                      storage=16, want_intermediates=True)
    assert np.array_equal(np.isinf(got["V"]), np.isinf(V_o))
    assert np.array_equal(got["V"][np.isfinite(V_o)], V_o[np.isfinite(V_o)])
    assert np.array_equal(got["U"], U_o)
    assert (np.isfinite(got["M"]) == np.isfinite(M_o)).mean() > 0.999
    bad_gpu, bad_o = ~np.isfinite(got["y"]), ~np.isfinite(y_o)
    say(f"  non-finite outputs: gpu {bad_gpu.mean():.3f} oracle {bad_o.mean():.3f}")
    assert bad_o.mean() > 0.9 and (bad_gpu == bad_o).mean() > 0.99


def test_balanced_rows_make_integer_point_f83_finite():
    # same data as above, rows of B^T and G scaled by powers of two into [1, 2) (exact): nothing
    # overflows any more, U and V agree bit for bit, the result is finite (and as inaccurate as the
    # conditioning of the integer points makes it)
    say("[case] integer-point F(8,3) with balanced power-of-two rows")
    points = synth.point_set("standard", 8)
    x, w = synth.make_layer(1, 32, 8, 24, 24, seed=5, dtype="f16")
    t = nova.nova_make_transforms(points, 8, 3, row_scaling="balanced")
    assert t.symmetric
    got = run_stages(t, x, w)
    x64, w64 = x.astype(np.float64), w.astype(np.float64)
    y_o, U_o, V_o, M_o = conv.winograd_conv2d_emulated(x64, w64, pts(points), 8, storage=16, row_scaling="balanced",
                                                      want_intermediates=True)
    same(got["U"], U_o, "U")
    same(got["V"], V_o, "V")
    assert np.isfinite(got["V"]).all() and np.abs(got["V"]).max() <= 4 * np.abs(x64).max()
    assert rel_l2(got["M"], M_o) < 1e-5
    # the output itself is so wrong (conditioning) that a few entries leave the binary16 range at
    # the final store; those must be the same few on both sides
    fin = np.isfinite(y_o)
    assert fin.mean() > 0.99 and (np.isfinite(got["y"]) == fin).mean() > 0.999
    both = fin & np.isfinite(got["y"])
    err = rel_l2(got["y"][both], y_o[both])
    want = conv.direct_conv2d(x64, w64)
    say(f"  rel-L2 vs emulation {err:.3e}; vs fp64 definition {rel_l2(got['y'][both], want[both]):.3e}")
    assert err < 5e-3


def test_row_scaling_and_fp16_matrices_follow_the_emulation():
    x, w = synth.make_layer(2, 24, 20, 17, 22, seed=31, dtype="f16")
    x64, w64 = x.astype(np.float64), w.astype(np.float64)
    # discovered points, balanced rows: paired kernels
    for name, m in (("nova", 4), ("nova", 6), ("nova", 8)):
        say(f"[case] balanced rows, {name} F({m},3)")
        points = synth.point_set(name, m)
        t = nova.nova_make_transforms(points, m, 3, row_scaling="balanced")
        got = run_stages(t, x, w)
        y_o, U_o, V_o, _ = conv.winograd_conv2d_emulated(x64, w64, pts(points), m, storage=16, row_scaling="balanced",
                                                        want_intermediates=True)
        same(got["U"], U_o, "U")
        same(got["V"], V_o, "V")
        assert rel_l2(got["y"], y_o) < 5e-3
    # exponents that differ between the rows of +a and -a: general kernels
    say("[case] unpaired row exponents, nova F(4,3)")
    points = synth.point_set("nova", 4)
    scaling = ([1, -2, 0, 3, 3, -1], [0, 2, 1, -3, 0, 2])
    t = nova.nova_make_transforms(points, 4, 3, row_scaling=scaling)
    assert not t.symmetric
    got = run_stages(t, x, w)
    y_o, U_o, V_o, _ = conv.winograd_conv2d_emulated(x64, w64, pts(points), 4, storage=16, row_scaling=scaling,
                                                    want_intermediates=True)
    same(got["U"], U_o, "U")
    same(got["V"], V_o, "V")
    assert rel_l2(got["y"], y_o) < 5e-3
    # matrices stored in binary16 (Table "FP16 storage"), dyadic and discovered points
    for name, m in (("dyadic", 4), ("nova", 6)):
        say(f"[case] binary16 matrices, {name} F({m},3)")
        points = synth.point_set(name, m)
        t = nova.nova_make_transforms(points, m, 3, matrix_dtype="f16")
        got = run_stages(t, x, w)
        y_o, U_o, V_o, _ = conv.winograd_conv2d_emulated(x64, w64, pts(points), m, storage=16, transform_dtype="f16",
                                                        want_intermediates=True)
        same(got["U"], U_o, "U")
        same(got["V"], V_o, "V")
        assert rel_l2(got["y"], y_o) < 5e-3


def test_int8_matrices_follow_the_emulation_and_the_printed_ordering():
    # A, B^T, G quantised to INT8 per tensor (Sec. "INT8 Convolution Error Validation"), inputs and
    # kernels uniform in [-1, 1] as there, binary32 storage so that the matrix quantisation is the
    # only coarse rounding: the layer error against the fp64 definition must sit where the printed
    # tile errors sit (standard F(4,3) 7.1e-2, discovered 2.1e-2 / 1.2e-1 / 5.9e-1)
    rng = np.random.default_rng(44)
    x = rng.uniform(-1.0, 1.0, (2, 16, 20, 27)).astype(np.float32)
    w = rng.uniform(-1.0, 1.0, (12, 16, 3, 3)).astype(np.float32)
    x64, w64 = x.astype(np.float64), w.astype(np.float64)
    want = conv.direct_conv2d(x64, w64)
    errs = {}
    for name, m in (("standard", 4), ("nova", 4), ("nova", 6), ("nova", 8)):
        say(f"[case] INT8 matrices, {name} F({m},3)")
        points = synth.point_set(name, m)
        t = nova.nova_make_transforms(points, m, 3, matrix_dtype="int8")
        got = run_stages(t, x, w)
        y_o, U_o, V_o, _ = conv.winograd_conv2d_emulated(x64, w64, pts(points), m, storage=32, transform_dtype="int8",
                                                        want_intermediates=True)
        same(got["U"], U_o, "U")
        same(got["V"], V_o, "V")
        errs[(name, m)] = rel_l2(got["y"], want)
        gap = rel_l2(got["y"], y_o)
        say(f"  rel-L2 vs fp64 definition {errs[(name, m)]:.3e}; vs emulation {gap:.3e}")
        # binary32 accumulation order (device) against fp64 accumulation (emulation): three orders of
        # magnitude below the effect of the quantised matrices
        assert gap < 1e-3 * errs[(name, m)]
    assert 0.5 * 7.1e-2 < errs[("standard", 4)] < 2 * 7.1e-2
    assert 0.5 * 2.1e-2 < errs[("nova", 4)] < 2 * 2.1e-2
    assert 0.5 * 1.24e-1 < errs[("nova", 6)] < 2 * 1.24e-1
    assert 0.5 * 5.92e-1 < errs[("nova", 8)] < 2 * 5.92e-1


def test_fp16_error_per_tile_size_and_point_set():
    # the accuracy half of the metric: relative L2 error of the fp16 device path against the fp64
    # definition, per tile size and point set, on the mid-size layer shape (N=8, C=K=64, 56x56,
    # half-normal inputs, He-normal weights).  Orderings the paper reports: discovered points beat
    # integer points from F(4,3) on; integer-point F(8,3) leaves the binary16 range; discovered
    # F(8,3) stays finite.  The table is printed, and written to $NOVA_REPORT_DIR if that is set.
    cfg = synth.LAYER_CONFIGS["mid_f63_fp16"]
    x, w = synth.make_layer(cfg["N"], cfg["C"], cfg["K"], cfg["H"], cfg["W"], seed=cfg["seed"], dtype="f16",
                            x_dist=cfg["x_dist"])
    xd, wd = torch.from_numpy(x).to(DEV), torch.from_numpy(w).to(DEV)
    want = conv.direct_conv2d(x.astype(np.float64), w.astype(np.float64))
    rows, err = [], {}
    for m, name, kw in [(2, "standard", {}), (4, "standard", {}), (4, "nova", {}), (4, "dyadic", {}),
                        (6, "standard", {}), (6, "classic_half", {}), (6, "nova", {}),
                        (8, "standard", {}), (8, "standard", {"row_scaling": "balanced"}), (8, "nova", {}),
                        (8, "nova", {"row_scaling": "balanced"})]:
        t = nova.nova_make_transforms(synth.point_set(name, m), m, 3, **kw)
        for flags, label in ((0, "fp32 M"), (nova.NOVA_FLAG_M_F16, "fp16 M")):
            y = nova.nova_winograd_conv2d(t, xd, nova.nova_filter_transform(t, wd), cfg["K"], flags=flags)
            y = y.cpu().numpy().astype(np.float64)
            bad = float((~np.isfinite(y)).mean())
            e = rel_l2(y, want) if bad == 0 else float("nan")
            key = (m, name + ("+balanced" if kw else ""), label)
            err[key] = (e, bad)
            rows.append(f"F({m},3) {key[1]:22s} {label}  rel-L2 {e:10.3e}  non-finite {bad:6.3f}")
            say("  " + rows[-1])
    report_dir = os.environ.get("NOVA_REPORT_DIR")
    if report_dir:
        os.makedirs(report_dir, exist_ok=True)
        with open(os.path.join(report_dir, "fp16_error_table.txt"), "w") as fh:
            fh.write("\n".join(rows) + "\n")
    e = lambda m, name: err[(m, name, "fp32 M")][0]
    # F(4,3): all point sets are fine in fp16 (a few 1e-3); F(6,3): the integer points {0,+-1,+-2,+-3}
    # lose more than an order of magnitude against the discovered ones.  (The classic set with +-1/2
    # is *not* worse than the discovered set on this data -- reported, not asserted either way.)
    assert max(e(4, "nova"), e(4, "standard"), e(4, "dyadic")) < 5e-3
    assert e(6, "nova") < 0.1 * e(6, "standard") and e(6, "classic_half") < e(6, "standard")
    assert err[(8, "standard", "fp32 M")][1] > 0.9                  # blow-up
    assert err[(8, "nova", "fp32 M")][1] == 0 and e(8, "nova") < 1.0          # recovery
    assert err[(8, "standard+balanced", "fp32 M")][1] < 0.01        # range fixed, conditioning not
    assert abs(e(8, "nova+balanced") - e(8, "nova")) < 0.05 * e(8, "nova")
    assert e(2, "standard") < e(4, "standard") < e(6, "standard")


def test_slabs_and_workspace_errors():
    say("[case] slab loop and workspace checks")
    points = synth.point_set("nova", 4)
    x, w = synth.make_layer(5, 32, 32, 12, 12, seed=2, dtype="f16")
    t = nova.nova_make_transforms(points, 4, 3)
    xd, wd = torch.from_numpy(x).to(DEV), torch.from_numpy(w).to(DEV)
    U = nova.nova_filter_transform(t, wd)
    ys = [nova.nova_winograd_conv2d(t, xd, U, 32, images_per_slab=s).cpu() for s in (1, 2, 5, 0)]
    for y in ys[1:]:
        assert torch.equal(ys[0], y)
    one = nova.nova_conv2d_workspace_bytes(5, 32, 12, 12, 32, 4, nova.NOVA_F16, 0, 1)
    small = torch.empty(one - 256, dtype=torch.uint8, device=DEV)
    with pytest.raises(nova.NovaError) as exc:
        nova.nova_winograd_conv2d(t, xd, U, 32, workspace=small)
    assert exc.value.code == -5
    torch.cuda.synchronize()


def test_relu_maxpool():
    say("[case] relu + 2x2 max-pool")
    rng = np.random.default_rng(4)
    for dtype in (np.float16, np.float32):
        a = rng.standard_normal((3, 5, 9, 14)).astype(dtype)
        got = nova.nova_relu_maxpool2x2(torch.from_numpy(a).to(DEV)).cpu().numpy().astype(np.float64)
        assert np.array_equal(got, conv.relu_maxpool2x2(a.astype(np.float64)))


def test_mid_layer_full_size():
    cfg = synth.LAYER_CONFIGS["mid_f63_fp16"]
    x, w = synth.make_layer(cfg["N"], cfg["C"], cfg["K"], cfg["H"], cfg["W"], seed=cfg["seed"], dtype="f16")
    x64, w64 = x.astype(np.float64), w.astype(np.float64)
    want = conv.direct_conv2d(x64, w64)
    xd, wd = torch.from_numpy(x).to(DEV), torch.from_numpy(w).to(DEV)
    for name in ("classic_half", "nova"):
        say(f"[case] mid layer F(6,3) {name} full size {cfg}")
        points = synth.point_set(name, 6)
        t = nova.nova_make_transforms(points, 6, 3)
        U = nova.nova_filter_transform(t, wd)
        y = nova.nova_winograd_conv2d(t, xd, U, cfg["K"]).cpu().numpy().astype(np.float64)
        emu = conv.winograd_conv2d_emulated(x64, w64, pts(points), 6, storage=16, want_intermediates=True)
        y_o = emu[0]
        e_emu, e_def = rel_l2(y, y_o), rel_l2(y, want)
        say(f"  rel-L2 vs emulation {e_emu:.3e}; vs fp64 definition {e_def:.3e}")
        assert e_emu < 5e-3
        ratio, width = elementwise_fp16(y, y_o, points, 6, emu, cfg["C"])
        say(f"  element-wise: max |diff| / bound {ratio:.3f}; median bound / rms(y) {width:.2e}")


def test_vgg_conv3_full_size_sampled_images():
    # the benchmark workload at full size, in the launch configuration bench.py times; the oracle
    # evaluates whole sampled images (outputs of different images are independent)
    cfg = synth.LAYER_CONFIGS["vgg_conv3_f83_fp16"]
    x, w = synth.make_layer(cfg["N"], cfg["C"], cfg["K"], cfg["H"], cfg["W"], seed=cfg["seed"], dtype="f16")
    xd, wd = torch.from_numpy(x).to(DEV), torch.from_numpy(w).to(DEV)
    sample = [0, 17, 31]
    x64, w64 = x[sample].astype(np.float64), w.astype(np.float64)
    want = conv.direct_conv2d(x64, w64)
    for name in ("nova", "standard"):
        say(f"[case] VGG conv3 F(8,3) {name} full size, images {sample}")
        points = synth.point_set(name, 8)
        t = nova.nova_make_transforms(points, 8, 3)
        U = nova.nova_filter_transform(t, wd)
        y = nova.nova_winograd_conv2d(t, xd, U, cfg["K"])
        torch.cuda.synchronize()
        y = y[sample].cpu().numpy().astype(np.float64)
        emu = conv.winograd_conv2d_emulated(x64, w64, pts(points), 8, storage=16, want_intermediates=(name == "nova"))
        y_o = emu[0] if name == "nova" else emu
        if name == "nova":
            e_emu, e_def = rel_l2(y, y_o), rel_l2(y, want)
            say(f"  rel-L2 vs emulation {e_emu:.3e}; vs fp64 definition {e_def:.3e}")
            assert np.isfinite(y).all() and e_emu < 5e-3
            ratio, width = elementwise_fp16(y, y_o, points, 8, emu, cfg["C"])
            say(f"  element-wise: max |diff| / bound {ratio:.3f}; median bound / rms(y) {width:.2e}")
        else:
            bad, bad_o = ~np.isfinite(y), ~np.isfinite(y_o)
            say(f"  non-finite outputs: gpu {bad.mean():.3f} oracle {bad_o.mean():.3f}")
            assert bad_o.mean() > 0.9 and (bad == bad_o).mean() > 0.99


def test_resnet_shapes_reduced_batch():
    # the four ResNet-50-style stride-1 3x3 shapes (C = K = 64 @56, 128 @28, 256 @14, 512 @7), F(8,3)
    # with NOVA points, at batch 4 instead of 256; 14x14 and 7x7 need cropped (padded) tiles
    points = synth.point_set("nova", 8)
    t = nova.nova_make_transforms(points, 8, 3)
    for idx, (ch, hw) in enumerate(synth.RESNET_SHAPES):
        say(f"[case] ResNet-style shape C=K={ch} H=W={hw}, batch 4")
        x, w = synth.make_layer(4, ch, ch, hw, hw, seed=5000 + idx, dtype="f16")
        xd, wd = torch.from_numpy(x).to(DEV), torch.from_numpy(w).to(DEV)
        U = nova.nova_filter_transform(t, wd)
        y = nova.nova_winograd_conv2d(t, xd, U, ch).cpu().numpy().astype(np.float64)
        emu = conv.winograd_conv2d_emulated(x.astype(np.float64), w.astype(np.float64), pts(points), 8, storage=16,
                                            want_intermediates=True)
        y_o = emu[0]
        err = rel_l2(y, y_o)
        say(f"  rel-L2 vs emulation {err:.3e}")
        assert np.isfinite(y).all() and err < 5e-3
        elementwise_fp16(y, y_o, points, 8, emu, ch)


@pytest.mark.parametrize("m", [6, 8])
def test_vgg_stack_reduced_size(m):
    # the 13-layer VGG-16 conv stack (ReLU fused, 2x2 max-pool after layers 2, 4, 7, 10, 13) on a
    # 2 x 3 x 32 x 32 input; every layer is checked on its own: the oracle is fed the GPU's input to
    # that layer, so rounding differences do not accumulate through the stack
    points = synth.point_set("nova", m)
    t = nova.nova_make_transforms(points, m, 3)
    rng = np.random.default_rng(4000 + m)
    act = torch.from_numpy(rng.standard_normal((2, 3, 32, 32)).astype(np.float16)).to(DEV)
    for layer, (cin, cout) in enumerate(synth.VGG16_LAYERS, start=1):
        w = (rng.standard_normal((cout, cin, 3, 3)) * np.sqrt(2.0 / (9.0 * cin))).astype(np.float16)
        say(f"[case] VGG stack F({m},3) layer {layer}: {cin}->{cout} @ {act.shape[2]}x{act.shape[3]}")
        U = nova.nova_filter_transform(t, torch.from_numpy(w).to(DEV))
        y = nova.nova_winograd_conv2d(t, act, U, cout, flags=nova.NOVA_FLAG_RELU)
        x64 = act.cpu().numpy().astype(np.float64)
        emu = conv.winograd_conv2d_emulated(x64, w.astype(np.float64), pts(points), m, storage=16, relu=True,
                                            want_intermediates=True)
        y_o = emu[0]
        got = y.cpu().numpy().astype(np.float64)
        err = rel_l2(got, y_o)
        say(f"  rel-L2 vs emulation {err:.3e}")
        assert np.isfinite(got).all() and err < 5e-3
        elementwise_fp16(got, y_o, points, m, emu, cin)
        if layer in synth.VGG16_POOL_AFTER:
            pooled = nova.nova_relu_maxpool2x2(y)
            assert np.array_equal(pooled.cpu().numpy().astype(np.float64), conv.relu_maxpool2x2(got))
            act = pooled
        else:
            act = y


def test_resnet_shapes_full_batch_sampled_images():
    # the same four shapes at the full batch of 256; the oracle evaluates three sampled images
    points = synth.point_set("nova", 8)
    t = nova.nova_make_transforms(points, 8, 3)
    sample = [0, 101, 255]
    for idx, (ch, hw) in enumerate(synth.RESNET_SHAPES):
        say(f"[case] ResNet-style shape C=K={ch} H=W={hw}, batch 256, images {sample}")
        x, w = synth.make_layer(256, ch, ch, hw, hw, seed=5100 + idx, dtype="f16")
        xd, wd = torch.from_numpy(x).to(DEV), torch.from_numpy(w).to(DEV)
        U = nova.nova_filter_transform(t, wd)
        y = nova.nova_winograd_conv2d(t, xd, U, ch)
        torch.cuda.synchronize()
        got = y[sample].cpu().numpy().astype(np.float64)
        emu = conv.winograd_conv2d_emulated(x[sample].astype(np.float64), w.astype(np.float64), pts(points), 8,
                                            storage=16, want_intermediates=True)
        y_o = emu[0]
        err = rel_l2(got, y_o)
        say(f"  rel-L2 vs emulation {err:.3e}")
        assert np.isfinite(got).all() and err < 5e-3
        ratio, width = elementwise_fp16(got, y_o, points, 8, emu, ch)
        say(f"  element-wise: max |diff| / bound {ratio:.3f}; median bound / rms(y) {width:.2e}")
        del xd, y


@pytest.mark.parametrize("m", [6, 8])
def test_vgg_stack_full_size_sampled_images(m):
    # the 13-layer stack at its full size (32 x 3 x 224 x 224; the library's default slabs), each
    # layer checked on two sampled images against the emulation fed with the GPU's input to that layer
    points = synth.point_set("nova", m)
    t = nova.nova_make_transforms(points, m, 3)
    rng = np.random.default_rng(4100 + m)
    sample = [0, 31]
    act = torch.from_numpy(rng.standard_normal((32, 3, 224, 224)).astype(np.float16)).to(DEV)
    for layer, (cin, cout) in enumerate(synth.VGG16_LAYERS, start=1):
        w = (rng.standard_normal((cout, cin, 3, 3)) * np.sqrt(2.0 / (9.0 * cin))).astype(np.float16)
        say(f"[case] full VGG stack F({m},3) layer {layer}: {cin}->{cout} @ {act.shape[2]}x{act.shape[3]}")
        U = nova.nova_filter_transform(t, torch.from_numpy(w).to(DEV))
        y = nova.nova_winograd_conv2d(t, act, U, cout, flags=nova.NOVA_FLAG_RELU)
        torch.cuda.synchronize()
        x64 = act[sample].cpu().numpy().astype(np.float64)
        emu = conv.winograd_conv2d_emulated(x64, w.astype(np.float64), pts(points), m, storage=16, relu=True,
                                            want_intermediates=True)
        y_o = emu[0]
        got = y[sample].cpu().numpy().astype(np.float64)
        err = rel_l2(got, y_o)
        say(f"  rel-L2 vs emulation {err:.3e}")
        assert np.isfinite(got).all() and err < 5e-3
        ratio, width = elementwise_fp16(got, y_o, points, m, emu, cin)
        say(f"  element-wise: max |diff| / bound {ratio:.3f}; median bound / rms(y) {width:.2e}")
        del emu
        if layer in synth.VGG16_POOL_AFTER:
            pooled = nova.nova_relu_maxpool2x2(y)
            assert np.array_equal(pooled[sample].cpu().numpy().astype(np.float64), conv.relu_maxpool2x2(got))
            act = pooled
        else:
            act = y
        del y


# 5 x 5 kernels (Sec. "Extension to 5 x 5 Kernels"): F(m, 5) needs m + 3 finite points -- the same
# sets as F(m + 2, 3)
R5_CASES = [
    # m, points (name, size they are listed under), N, C, K, H, W
    (2, ("standard", 4), 2, 8, 8, 7, 9),
    (2, ("nova", 4), 1, 40, 33, 16, 24),
    (4, ("standard", 6), 2, 24, 40, 19, 14),
    (4, ("nova", 6), 2, 64, 64, 24, 32),
    (4, ("nova", 6), 1, 5, 3, 13, 70),
    (6, ("nova", 8), 2, 64, 128, 36, 48),
    (6, ("nova", 8), 3, 33, 20, 17, 23),
]


def make_layer_r5(N, C, K, H, W, seed, dtype):
    rng = np.random.default_rng(seed)
    x = np.abs(rng.standard_normal((N, C, H, W))).astype(dtype)
    w = (rng.standard_normal((K, C, 5, 5)) * np.sqrt(2.0 / (25.0 * C))).astype(dtype)
    return x, w


@pytest.mark.parametrize("m,pset,N,C,K,H,W", R5_CASES)
def test_r5_fp16_stages_against_emulation(m, pset, N, C, K, H, W):
    say(f"[case] fp16 stages F({m},5) points {pset} N={N} C={C} K={K} H={H} W={W}")
    points = synth.point_set(*pset)
    x, w = make_layer_r5(N, C, K, H, W, 900 + 10 * m + C, np.float16)
    t = nova.nova_make_transforms(points, m, 5)
    assert (t.n, t.r, t.symmetric) == (m + 4, 5, True)
    got = run_stages(t, x, w)
    x64, w64 = x.astype(np.float64), w.astype(np.float64)
    emu = conv.winograd_conv2d_emulated(x64, w64, pts(points), m, storage=16, want_intermediates=True)
    y_o, U_o, V_o, M_o = emu
    same(got["U"], U_o, "U")
    same(got["V"], V_o, "V")
    assert rel_l2(got["M"], M_o) < 1e-5
    single_call_agrees(got, x.shape[1], 16 if x.dtype == np.float16 else 32, got["fused"])
    err = rel_l2(got["y"], y_o)
    say(f"  rel-L2 vs emulation {err:.3e}; vs fp64 definition {rel_l2(got['y'], conv.direct_conv2d(x64, w64)):.3e}")
    assert err < 5e-3
    elementwise_fp16(got["y"], y_o, points, m, emu, C)
    elementwise_fp16(got["y_conv"], y_o, points, m, emu, C, "y (single call)")


@pytest.mark.parametrize("m,pset", [(2, ("standard", 4)), (4, ("nova", 6)), (6, ("nova", 8))])
def test_r5_fp32_against_definition(m, pset):
    say(f"[case] fp32 F({m},5) points {pset}")
    points = synth.point_set(*pset)
    x, w = make_layer_r5(2, 20, 12, 3 * m + 2, 5 * m - 1, 950 + m, np.float32)
    x = (x * np.sign(np.random.default_rng(m).standard_normal(x.shape))).astype(np.float32)
    t = nova.nova_make_transforms(points, m, 5)
    got = run_stages(t, x, w)
    x64, w64 = x.astype(np.float64), w.astype(np.float64)
    want = conv.direct_conv2d(x64, w64)
    y_o, U_o, V_o, _ = conv.winograd_conv2d_emulated(x64, w64, pts(points), m, storage=32, want_intermediates=True)
    same(got["U"], U_o, "U")
    same(got["V"], V_o, "V")
    own, err = rel_l2(y_o, want), rel_l2(got["y"], y_o)
    say(f"  emulation vs definition {own:.3e}; gpu vs emulation {err:.3e}; gpu vs definition {rel_l2(got['y'], want):.3e}")
    assert err <= max(1e-5, 4 * own)
    if m == 2:
        assert rel_l2(got["y"], want) <= 1e-5 and np.abs(got["y"] - want).max() <= 1e-4


FUSED_CASES = [
    # m, N, C, K, H, W: wide rows (two groups of tiles), one group, narrow images (several tile rows per group),
    # ragged edges, several groups of 64 output channels
    (8, 2, 64, 64, 224, 224),
    (8, 2, 64, 128, 112, 112),
    (8, 3, 64, 128, 56, 56),
    (8, 2, 64, 96, 50, 61),         # K a multiple of 32 only
    (8, 5, 64, 64, 17, 23),
    (8, 7, 64, 64, 9, 8),
    (6, 2, 64, 128, 56, 56),
    (6, 3, 64, 64, 45, 100),
    (6, 2, 64, 64, 13, 13),
    (6, 1, 64, 64, 112, 112),       # 19 x 19 tiles in 4 x 4 blocks
    (6, 1, 64, 64, 224, 224),       # 38 x 38 tiles in 2 x 8 blocks
    (8, 2, 64, 64, 100, 36),        # widths that are no whole number of 16-byte pieces
    (8, 1, 64, 32, 1, 1),           # one pixel, one group of 32 output channels
    (6, 3, 64, 32, 5, 64),          # a single tile row, images smaller than a tile high
]


@pytest.mark.parametrize("m,N,C,K,H,W", FUSED_CASES)
def test_fused_contraction_and_output_transform(m, N, C, K, H, W):
    # steps 3 and 4 in one kernel (no M): against the emulation, element by element, with ReLU and the
    # fused max-pool; and nova_winograd_conv2d takes this path where it is the faster one
    say(f"[case] fused contraction + output transform F({m},3) N={N} C={C} K={K} H={H} W={W}")
    points = synth.point_set("nova", m)
    t = nova.nova_make_transforms(points, m, 3)
    x, w = synth.make_layer(N, C, K, H, W, seed=800 + m + C + H, dtype="f16", x_dist="normal")
    xd, wd = torch.from_numpy(x).to(DEV), torch.from_numpy(w).to(DEV)
    U = nova.nova_filter_transform(t, wd)
    V = nova.nova_input_transform(t, xd)
    y = nova.nova_contract_output_fused(t, U, V, N, C, H, W, K)
    y_relu = nova.nova_contract_output_fused(t, U, V, N, C, H, W, K, flags=nova.NOVA_FLAG_RELU)
    y_call = nova.nova_winograd_conv2d(t, xd, U, K, images_per_slab=1)
    torch.cuda.synchronize()
    if takes_fused_path(t, C, K, x.dtype, H=H, W=W):
        assert torch.equal(y, y_call)
    else:        # the single call keeps the separate kernels for this shape: another summation order
        assert rel_l2(y.cpu().numpy().astype(np.float64), y_call.cpu().numpy().astype(np.float64)) < 2e-3
    assert torch.equal(y_relu, torch.clamp(y, min=0))
    sample = [0, N - 1] if H * W > 10000 else list(range(N))
    x64, w64 = x[sample].astype(np.float64), w.astype(np.float64)
    emu = conv.winograd_conv2d_emulated(x64, w64, pts(points), m, storage=16, want_intermediates=True)
    got = y[sample].cpu().numpy().astype(np.float64)
    err = rel_l2(got, emu[0])
    ratio, width = elementwise_fp16(got, emu[0], points, m, emu, C)
    say(f"  rel-L2 vs emulation {err:.3e}; element-wise: max |diff| / bound {ratio:.3f}; median bound / rms(y) {width:.2e}")
    assert err < 5e-3
    if H % 2 == 0 and W % 2 == 0:
        pooled = nova.nova_contract_output_fused(t, U, V, N, C, H, W, K, flags=nova.NOVA_FLAG_RELU | nova.NOVA_FLAG_POOL2)
        assert torch.equal(pooled.float(), torch.nn.functional.max_pool2d(y_relu.float(), 2))
    with pytest.raises(nova.NovaError) as exc:
        nova.nova_contract_output_fused(t, U, V, N, C, H, W, K, flags=nova.NOVA_FLAG_M_F16)
    assert exc.value.code == -6


INT8_CASES = [
    # name, m, N, C, K, H, W, dtype
    ("standard", 2, 2, 8, 8, 7, 9, "f16"),
    ("nova", 4, 3, 33, 70, 30, 41, "f16"),
    ("nova", 4, 2, 64, 64, 20, 20, "f32"),
    ("nova", 6, 2, 40, 130, 24, 56, "f16"),
    ("nova", 8, 2, 72, 96, 33, 40, "f16"),
    ("nova", 8, 1, 256, 256, 28, 28, "f16"),
    ("standard", 4, 1, 3, 5, 17, 22, "f32"),
]


@pytest.mark.parametrize("name,m,N,C,K,H,W,dtype", INT8_CASES)
def test_int8_winograd_domain_against_the_oracle(name, m, N, C, K, H, W, dtype):
    # Codes, scales and the 32-bit channel sums are integers (or binary32 numbers decided by the same
    # correctly rounded binary32 steps on both sides): bit-exact.  The output goes through the binary32
    # output transform: within its rounding of the oracle's binary64 evaluation, element by element.
    points = synth.point_set(name, m)
    t = nova.nova_make_transforms(points, m, 3)
    x, w = synth.make_layer(N, C, K, H, W, seed=700 + m + C, dtype=dtype, x_dist="normal")
    xd, wd = torch.from_numpy(x).to(DEV), torch.from_numpy(w).to(DEV)
    x64, w64 = x.astype(np.float64), w.astype(np.float64)
    storage = 16 if dtype == "f16" else 32
    n2 = t.n * t.n
    T = N * (-(-H // m)) * (-(-W // m))
    Tp, Kp = -(-T // 128) * 128, -(-K // 32) * 32
    U = nova.nova_filter_transform(t, wd)
    V = nova.nova_input_transform(t, xd)
    A = np.abs(ct.to_f32(ct.cook_toom(pts(points), m, 3)[0]).astype(np.float64))
    th, tw = -(-H // m), -(-W // m)
    for mode, mode_name in ((nova.NOVA_INT8_PER_TENSOR, "per_tensor"), (nova.NOVA_INT8_PER_CHANNEL, "per_channel"),
                            (nova.NOVA_INT8_PER_POSITION, "per_position")):
        say(f"[case] int8 {mode_name} {name} F({m},3) {dtype} N={N} C={C} K={K} H={H} W={W}")
        y_o, Uq_o, su_o, Vq_o, sv_o, Mi_o, M_o = int8.winograd_conv2d_int8(x64, w64, pts(points), m, storage=storage,
                                                                         mode=mode_name, want_intermediates=True)
        Uq, su = nova.nova_quantize_filter_int8(t, U, K, C, mode)
        Vq, sv = nova.nova_quantize_input_int8(t, V, N, C, H, W, mode)
        Mi = nova.nova_contract_int8(t, Uq, Vq, None, None, mode, N, C, H, W, K, dequantise=False)
        Mf = nova.nova_contract_int8(t, Uq, Vq, su, sv, mode, N, C, H, W, K, dequantise=True)
        y = nova.nova_output_transform(t, Mf, N, K, H, W, xd.dtype)
        y2 = nova.nova_winograd_conv2d_int8(t, xd, Uq, su, mode, K)
        torch.cuda.synchronize()
        assert np.array_equal(su.cpu().numpy(), su_o) and np.array_equal(sv.cpu().numpy(), sv_o)
        Uq_l = unblock(Uq, n2, Kp, C)
        assert not Uq_l[:, K:, :].any()
        same(Uq_l[:, :K, :], Uq_o.astype(np.float64), "Uq")
        same(unblock(Vq, n2, T, C), Vq_o.astype(np.float64), "Vq")
        same(unblock(Mi, n2, Tp, K)[:, :T, :], Mi_o.astype(np.float64), "Mi")
        same(unblock(Mf, n2, Tp, K)[:, :T, :], M_o.astype(np.float64), "M (de-quantised)")
        assert torch.equal(y, y2)
        got = y.cpu().numpy().astype(np.float64)
        # |y_gpu - y_oracle| <= rounding of the storage format + (2 n + 2) u |A|^T |M| |A|, u = 2^-24
        S = np.einsum("ip,jq,ijtk->tkpq", A, A, np.abs(M_o.astype(np.float64)).reshape(t.n, t.n, T, K), optimize=True)
        S = S.reshape(N, th, tw, K, m, m).transpose(0, 3, 1, 4, 2, 5).reshape(N, K, th * m, tw * m)[:, :, :H, :W]
        spacing = ulp16(np.maximum(np.abs(got), np.abs(y_o))) if storage == 16 else 2.0 ** -23 * np.maximum(np.abs(got), np.abs(y_o))
        bound = spacing + (2 * t.n + 2) * 2.0 ** -24 * S
        assert np.isfinite(got).all() and (np.abs(got - y_o) <= bound).all(), float((np.abs(got - y_o) / bound).max())
        want = conv.direct_conv2d(x64, w64)
        say(f"  bit-exact codes, scales, sums; y: max |diff| / bound {float((np.abs(got - y_o) / bound).max()):.3f}; "
            f"rel-L2 vs fp64 definition {rel_l2(got, want):.3e}")


def test_int8_single_call_flags_and_errors():
    m = 4
    points = synth.point_set("nova", m)
    t = nova.nova_make_transforms(points, m, 3)
    x, w = synth.make_layer(2, 24, 40, 18, 20, seed=77, dtype="f16", x_dist="normal")
    xd, wd = torch.from_numpy(x).to(DEV), torch.from_numpy(w).to(DEV)
    U = nova.nova_filter_transform(t, wd)
    Uq, su = nova.nova_quantize_filter_int8(t, U, 40, 24, nova.NOVA_INT8_PER_CHANNEL)
    y = nova.nova_winograd_conv2d_int8(t, xd, Uq, su, nova.NOVA_INT8_PER_CHANNEL, 40)
    y_relu = nova.nova_winograd_conv2d_int8(t, xd, Uq, su, nova.NOVA_INT8_PER_CHANNEL, 40, flags=nova.NOVA_FLAG_RELU)
    y_pool = nova.nova_winograd_conv2d_int8(t, xd, Uq, su, nova.NOVA_INT8_PER_CHANNEL, 40,
                                            flags=nova.NOVA_FLAG_RELU | nova.NOVA_FLAG_POOL2)
    assert torch.equal(y_relu, torch.clamp(y, min=0))
    assert torch.equal(y_pool.float(), torch.nn.functional.max_pool2d(y_relu.float(), 2))
    with pytest.raises(nova.NovaError) as exc:
        nova.nova_winograd_conv2d_int8(t, xd, Uq, su, nova.NOVA_INT8_PER_CHANNEL, 40, flags=nova.NOVA_FLAG_M_F16)
    assert exc.value.code == -1
    small = torch.empty(nova.nova_conv2d_int8_workspace_bytes(2, 24, 18, 20, 40, m, nova.NOVA_F16) - 256,
                        dtype=torch.uint8, device=DEV)
    with pytest.raises(nova.NovaError) as exc:
        nova.nova_winograd_conv2d_int8(t, xd, Uq, su, nova.NOVA_INT8_PER_CHANNEL, 40, workspace=small)
    assert exc.value.code == -5
    with pytest.raises(nova.NovaError) as exc:
        nova.nova_quantize_filter_int8(t, U, 40, 24, 7)
    assert exc.value.code == -1
    torch.cuda.synchronize()


POISON_CASES = [
    # m, N, C, K, H, W, dtype: T not a multiple of 128, K not a multiple of 32, C <= 4 and C > 4
    (8, 3, 40, 33, 17, 23, "f16"),
    (8, 2, 3, 5, 30, 41, "f16"),
    (6, 5, 64, 70, 27, 56, "f16"),
    (4, 3, 4, 20, 13, 9, "f32"),
    (4, 2, 33, 50, 19, 22, "f32"),
    (8, 7, 128, 64, 28, 28, "f16"),          # streaming contraction with a ragged last stage
    (8, 3, 64, 64, 17, 23, "f16"),           # contraction + output transform in one kernel, ragged tile block
    (6, 2, 64, 128, 112, 100, "f16"),        # ... in 4 x 4 tile blocks with ragged last blocks both ways
]


@pytest.mark.parametrize("m,N,C,K,H,W,dtype", POISON_CASES)
def test_poisoned_workspace_and_output_do_not_leak(m, N, C, K, H, W, dtype):
    # The workspace (V, M, their padding rows and channels) and y are filled with NaN bit patterns
    # before the call: whatever the kernels read they must have written first, and cropped regions
    # (tile padding, channel padding, rows of M beyond T) must not reach y.  Two slab sizes.
    say(f"[case] poisoned workspace F({m},3) {dtype} N={N} C={C} K={K} H={H} W={W}")
    points = synth.point_set("nova", m)
    t = nova.nova_make_transforms(points, m, 3)
    x, w = synth.make_layer(N, C, K, H, W, seed=600 + m + C, dtype=dtype, x_dist="normal")
    xd, wd = torch.from_numpy(x).to(DEV), torch.from_numpy(w).to(DEV)
    U = nova.nova_filter_transform(t, wd)
    dt = nova.NOVA_F16 if dtype == "f16" else nova.NOVA_F32
    for flags in (0, nova.NOVA_FLAG_RELU | (nova.NOVA_FLAG_M_F16 if dtype == "f16" else 0)):
        for per_slab in (N, 1):
            nbytes = nova.nova_conv2d_workspace_bytes(N, C, H, W, K, m, dt, flags, per_slab)
            clean = torch.zeros(nbytes, dtype=torch.uint8, device=DEV)
            want = nova.nova_winograd_conv2d(t, xd, U, K, flags=flags, workspace=clean)
            dirty = torch.full((nbytes,), 0xFF, dtype=torch.uint8, device=DEV)     # 0xFFFF / 0xFFFFFFFF: NaN
            got = torch.full_like(want, float("nan"))
            nova.nova_winograd_conv2d(t, xd, U, K, y=got, flags=flags, workspace=dirty)
            torch.cuda.synchronize()
            assert torch.isfinite(got).all(), f"flags {flags}, {per_slab} images per slab"
            assert torch.equal(got, want)


def test_graph_capture_replays_match_eager():
    # the conv call enqueues kernels only (no allocation, no memset, no synchronisation), so it can be
    # captured in a graph; every replay, with eager work and synchronisation in between, must give
    # what the eager call gives for the input that is in the buffer at that time
    say("[case] graph capture of nova_winograd_conv2d")
    points = synth.point_set("nova", 6)
    t = nova.nova_make_transforms(points, 6, 3)
    N, C, K, H, W = 3, 64, 64, 30, 36
    rng = np.random.default_rng(77)
    w = (rng.standard_normal((K, C, 3, 3)) * np.sqrt(2.0 / (9.0 * C))).astype(np.float16)
    U = nova.nova_filter_transform(t, torch.from_numpy(w).to(DEV))
    x = torch.zeros((N, C, H, W), dtype=torch.float16, device=DEV)
    y = torch.empty((N, K, H, W), dtype=torch.float16, device=DEV)
    ws = torch.empty(nova.nova_conv2d_workspace_bytes(N, C, H, W, K, 6, nova.NOVA_F16), dtype=torch.uint8, device=DEV)
    nova.nova_winograd_conv2d(t, x, U, K, y=y, workspace=ws)           # warm up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        nova.nova_winograd_conv2d(t, x, U, K, y=y, workspace=ws, flags=nova.NOVA_FLAG_RELU)
    for rep in range(4):
        fresh = torch.from_numpy(rng.standard_normal((N, C, H, W)).astype(np.float16)).to(DEV)
        x.copy_(fresh)
        y.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = y.clone()
        want = nova.nova_winograd_conv2d(t, fresh, U, K, flags=nova.NOVA_FLAG_RELU)
        torch.cuda.synchronize()
        assert torch.equal(got, want), f"replay {rep} differs from the eager result"
        assert torch.isfinite(got).all()


DEGENERATE = [(1, 1, 1, 1, 1), (1, 1, 1, 1, 37), (2, 3, 2, 40, 1), (1, 2, 2, 8, 8), (1, 33, 1, 16, 16),
              (1, 1, 65, 5, 64), (1, 4, 4, 3, 130), (5, 2, 3, 2, 2)]


@pytest.mark.parametrize("m,r", [(2, 3), (4, 3), (6, 3), (8, 3), (2, 5), (6, 5)])
def test_degenerate_shapes(m, r):
    # single pixels, single rows and columns, one channel, images smaller than a tile, rows wider than
    # one group: every staging / store variant at its smallest and at its ragged edge
    n_points = m + r - 2
    points = synth.point_set("nova", n_points - 1) if n_points - 1 in (4, 6, 8) else synth.point_set("standard", n_points - 1)
    t = nova.nova_make_transforms(points, m, r)
    rng = np.random.default_rng(1000 + 10 * m + r)
    for (N, C, K, H, W) in DEGENERATE:
        for dtype, storage in ((np.float16, 16), (np.float32, 32)):
            say(f"[case] degenerate F({m},{r}) {np.dtype(dtype).name} N={N} C={C} K={K} H={H} W={W}")
            x = rng.standard_normal((N, C, H, W)).astype(dtype)
            w = (rng.standard_normal((K, C, r, r)) * np.sqrt(2.0 / (r * r * C))).astype(dtype)
            got = run_stages(t, x, w)
            x64, w64 = x.astype(np.float64), w.astype(np.float64)
            y_o, U_o, V_o, _ = conv.winograd_conv2d_emulated(x64, w64, pts(points), m, storage=storage,
                                                            want_intermediates=True)
            same(got["U"], U_o, "U")
            same(got["V"], V_o, "V")
            single_call_agrees(got, x.shape[1], 16 if x.dtype == np.float16 else 32, got["fused"])
            scale = max(np.abs(y_o).max(), 1e-30)
            assert np.abs(got["y"] - y_o).max() <= (4e-2 if storage == 16 else 1e-3) * scale


def test_random_shapes_sweep():
    # a fixed pseudo-random sample of small layers over every supported (m, r), both storage formats,
    # with and without ReLU / binary16 products: U and V bit for bit, y against the emulation
    sweep_random_shapes(20251127, 70)
    sweep_random_shapes(20251128, 30, max_hw=300, max_ch=9)          # wide / tall images: several tile groups
    sweep_random_shapes(20251129, 30, max_hw=120, max_ch=4)          # first-layer path: at most 4 channels either way


def sweep_random_shapes(seed, count, max_hw=70, max_ch=70):
    rng = np.random.default_rng(seed)
    combos = [(2, 3), (4, 3), (6, 3), (8, 3), (2, 5), (4, 5), (6, 5)]
    handles = {}
    for case in range(count):
        m, r = combos[case % len(combos)]
        n_fin = m + r - 2
        # integer points only where they are well conditioned (n <= 6); beyond that the summation order of
        # the contraction decides more digits of y than any fixed tolerance allows
        name = "standard" if n_fin - 1 == 2 or (n_fin - 1 == 4 and case % 3 == 0) else "nova"
        points = synth.point_set(name, n_fin - 1)
        key = (m, r, name)
        if key not in handles:
            handles[key] = nova.nova_make_transforms(points, m, r)
        t = handles[key]
        N, C, K = int(rng.integers(1, 4)), int(rng.integers(1, max_ch + 1)), int(rng.integers(1, max_ch + 1))
        H, W = int(rng.integers(1, max_hw + 1)), int(rng.integers(1, max_hw + 1))
        if case % 4 == 1:
            W = (W + 7) // 8 * 8                                                        # 16-byte rows
        if case % 10 == 0:
            C, K = int(rng.choice([64, 128])), int(rng.choice([64, 128, 256]))          # streaming contraction
        f16 = case % 4 != 3
        flags = 0
        if case % 5 == 1:
            flags |= nova.NOVA_FLAG_RELU
        if f16 and case % 7 == 2:
            flags |= nova.NOVA_FLAG_M_F16
        dtype = np.float16 if f16 else np.float32
        say(f"[case] sweep {case}: F({m},{r}) {name} {np.dtype(dtype).name} N={N} C={C} K={K} H={H} W={W} flags={flags}")
        x = rng.standard_normal((N, C, H, W)).astype(dtype)
        w = (rng.standard_normal((K, C, r, r)) * np.sqrt(2.0 / (r * r * C))).astype(dtype)
        got = run_stages(t, x, w, flags=flags)
        x64, w64 = x.astype(np.float64), w.astype(np.float64)
        y_o, U_o, V_o, _ = conv.winograd_conv2d_emulated(
            x64, w64, pts(points), m, storage=16 if f16 else 32, relu=bool(flags & nova.NOVA_FLAG_RELU),
            m_storage=16 if flags & nova.NOVA_FLAG_M_F16 else 32, want_intermediates=True)
        same(got["U"], U_o, "U")
        same(got["V"], V_o, "V")
        single_call_agrees(got, x.shape[1], 16 if x.dtype == np.float16 else 32, got["fused"])
        if H % 2 == 0 and W % 2 == 0 and case % 2 == 0:
            # pooling fused into the store phase against pooling the unfused result of the same call
            xd, wd = torch.from_numpy(x).to(DEV), torch.from_numpy(w).to(DEV)
            pooled = nova.nova_winograd_conv2d(t, xd, nova.nova_filter_transform(t, wd), K, flags=flags | nova.NOVA_FLAG_POOL2)
            ref = torch.nn.functional.max_pool2d(torch.from_numpy(got["y_conv"]).to(DEV).float(), 2)
            assert torch.equal(pooled.float().nan_to_num(nan=-7.0), ref.nan_to_num(nan=-7.0))
        fin = np.isfinite(y_o)
        assert (np.isfinite(got["y"]) == fin).mean() > 0.99
        if fin.all() and np.isfinite(got["y"]).all():
            want = conv.direct_conv2d(x64, w64)
            own = rel_l2(y_o, np.maximum(want, 0.0) if flags & nova.NOVA_FLAG_RELU else want)
            # binary32: the device accumulates the channel sum in binary32, the emulation in fp64; both
            # carry the conditioning of the points, which `own` measures
            tol = 5e-3 if f16 else max(1e-5, 8 * own)
            assert rel_l2(got["y"], y_o) < tol, (rel_l2(got["y"], y_o), tol)
            assert rel_l2(got["y_conv"], y_o) < tol, (rel_l2(got["y_conv"], y_o), tol)


POOL_CASES = [(8, 2, 40, 36, 24, 32), (8, 1, 33, 20, 14, 14), (4, 2, 16, 16, 12, 260), (2, 1, 8, 8, 6, 10),
              (6, 2, 24, 40, 18, 30), (8, 3, 64, 64, 56, 56), (6, 1, 5, 3, 2, 2), (4, 1, 7, 9, 22, 6)]


@pytest.mark.parametrize("m,N,C,K,H,W", POOL_CASES)
def test_fused_maxpool_equals_pooling_the_unfused_output(m, N, C, K, H, W):
    # rounding to the storage format is monotonic, so pooling before or after the final rounding gives
    # the same numbers: the fused result must equal the pooled unfused result bit for bit
    points = synth.point_set("nova", m) if m > 2 else synth.point_set("standard", 2)
    t = nova.nova_make_transforms(points, m, 3)
    rng = np.random.default_rng(300 + m + W)
    for dtype in (np.float16, np.float32):
        say(f"[case] fused 2x2 max-pool F({m},3) {np.dtype(dtype).name} N={N} C={C} K={K} H={H} W={W}")
        x = torch.from_numpy(rng.standard_normal((N, C, H, W)).astype(dtype)).to(DEV)
        w = torch.from_numpy((rng.standard_normal((K, C, 3, 3)) * np.sqrt(2.0 / (9.0 * C))).astype(dtype)).to(DEV)
        U = nova.nova_filter_transform(t, w)
        for relu in (0, nova.NOVA_FLAG_RELU):
            plain = nova.nova_winograd_conv2d(t, x, U, K, flags=relu)
            fused = nova.nova_winograd_conv2d(t, x, U, K, flags=relu | nova.NOVA_FLAG_POOL2)
            fused_slabs = nova.nova_winograd_conv2d(t, x, U, K, flags=relu | nova.NOVA_FLAG_POOL2, images_per_slab=1)
            torch.cuda.synchronize()
            assert fused.shape == (N, K, H // 2, W // 2)
            want = torch.nn.functional.max_pool2d(plain.float(), 2).to(plain.dtype)
            assert torch.equal(fused, want) and torch.equal(fused_slabs, want)
            if relu:
                assert torch.equal(fused, nova.nova_relu_maxpool2x2(plain))
    # against the oracle, end to end
    x64, w64 = x.cpu().numpy().astype(np.float64), w.cpu().numpy().astype(np.float64)
    y_o = conv.relu_maxpool2x2(conv.winograd_conv2d_emulated(x64, w64, pts(points), m, storage=32))
    assert rel_l2(fused.cpu().numpy().astype(np.float64), y_o) < 1e-3


def test_fused_maxpool_rejects_odd_sizes():
    t = nova.nova_make_transforms(synth.point_set("nova", 4), 4, 3)
    x = torch.zeros((1, 4, 7, 8), dtype=torch.float16, device=DEV)
    U = nova.nova_filter_transform(t, torch.zeros((4, 4, 3, 3), dtype=torch.float16, device=DEV))
    with pytest.raises(nova.NovaError) as err:
        nova.nova_winograd_conv2d(t, x, U, 4, flags=nova.NOVA_FLAG_POOL2)
    assert err.value.code == -1
