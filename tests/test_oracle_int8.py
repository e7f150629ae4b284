"""Pins of the oracle's INT8 Winograd-domain path (oracle/int8.py).

quantize_symmetric is checked against a replay of the stated scheme (Sec. 4.1 "INT8 Setup":
s = max|.| / 127, round to nearest even, saturate) in exact rational arithmetic, with every
binary32 rounding applied by cook_toom._round_fraction, and against hand-worked codes.
winograd_conv2d_int8 is checked (i) on data for which every step is exact, so that the result must
equal the direct convolution bit for bit; (ii) against the plain definition evaluated on the
de-quantised operands, Y = A^T [ sum_c (s_U Uq) * (s_V Vq) ] A; (iii) for the direction of the
effect the paper reports: per-channel scales do not do worse than one scale per tensor, and the
discovered points do better than the integer points.
"""
from fractions import Fraction as Fr

import numpy as np

from oracle import conv, int8
from oracle import cook_toom as ct
from paper_2512_18453_amd import synth

F32 = (24, -126)


def pts(pairs):
    return [Fr(a, b) for a, b in pairs]


def replay_codes(values):
    """codes and scale of one tensor, every binary32 step rounded explicitly."""
    vals = [Fr(float(v)) for v in values]
    top = max(abs(v) for v in vals)
    s = ct._round_fraction(top / 127, *F32) if top > 0 else Fr(1)
    codes = []
    for v in vals:
        scaled = ct._round_fraction(v / s, *F32)
        lo = scaled.numerator // scaled.denominator
        rem = scaled - lo
        if rem > Fr(1, 2) or (rem == Fr(1, 2) and lo % 2 != 0):
            lo += 1
        codes.append(max(-128, min(127, lo)))
    return codes, s


def test_quantize_hand_worked():
    # largest magnitude 127 -> s = 1: the codes are the values rounded to nearest, ties to even
    v = np.array([127.0, -63.5, 62.5, 0.4999, -127.0, 1.5, 2.5, -0.5], dtype=np.float32)
    codes, s = int8.quantize_symmetric(v)
    assert s.tolist() == [1.0]
    assert codes.tolist() == [127, -64, 62, 0, -127, 2, 2, 0]
    # an all-zero tensor keeps scale 1
    codes, s = int8.quantize_symmetric(np.zeros(5, dtype=np.float32))
    assert s.tolist() == [1.0] and not codes.any()
    # the largest magnitude always gets code +-127, nothing saturates
    codes, s = int8.quantize_symmetric(np.array([0.3, -7.77, 7.0], dtype=np.float32))
    assert codes.tolist()[1] == -127 and abs(float(s[0]) - 7.77 / 127) < 1e-8


def test_quantize_equals_exact_replay():
    rng = np.random.default_rng(11)
    for scale in (1e-3, 1.0, 37.0):
        v = (rng.standard_normal(400) * scale).astype(np.float32)
        v[7] = 0.0
        codes, s = int8.quantize_symmetric(v)
        want, s_want = replay_codes(v)
        assert Fr(float(s[0])) == s_want
        assert codes.tolist() == want
    # binary16 data (the storage format of the fp16 path)
    v = rng.standard_normal(300).astype(np.float16).astype(np.float32)
    codes, s = int8.quantize_symmetric(v)
    assert codes.tolist() == replay_codes(v)[0]


def test_quantize_per_channel_is_per_tensor_on_each_slice():
    rng = np.random.default_rng(12)
    u = (rng.standard_normal((9, 5, 7)) * np.array([1, 10, 0.1, 0, 3]).reshape(1, 5, 1)).astype(np.float32)
    codes, s = int8.quantize_symmetric(u, axis=1)
    assert s.shape == (5,) and s[3] == 1.0
    for k in range(5):
        ck, sk = int8.quantize_symmetric(u[:, k, :])
        assert np.array_equal(codes[:, k, :], ck) and s[k] == sk[0]


def test_int8_convolution_is_exact_when_every_step_is_exact():
    # F(2,3), integer points (B^T and A have entries 0, +-1; G has halves).  Filters that are multiples of 4
    # make U integral; one filter whose entries add up to 4 * 127 puts the largest |U| at exactly 127
    # (the centre position is a quarter of the sum), one image channel with a single pixel of 127 among
    # small integers elsewhere puts the largest |V| at exactly 127.  Both scales are then 1, the codes
    # are U and V themselves, and the result is the direct convolution, exactly (binary32 storage).
    m = 2
    points = pts(synth.STANDARD[m])
    rng = np.random.default_rng(3)
    g = 4.0 * rng.integers(-3, 4, size=(3, 2, 3, 3)).astype(np.float64)
    g[1, 0] = 4.0 * np.array([[14, 14, 14], [14, 15, 14], [14, 14, 14]])
    x = rng.integers(-3, 4, size=(2, 2, 5, 6)).astype(np.float64)
    x[1, 1] = 0.0
    x[1, 1, 2, 3] = 127.0
    y, Uq, s_u, Vq, s_v, Mi, M = int8.winograd_conv2d_int8(x, g, points, m, storage=32, want_intermediates=True)
    assert s_u.tolist() == [1.0] and s_v.tolist() == [1.0]
    assert np.abs(Uq).max() == 127 and np.abs(Vq).max() == 127
    want = conv.direct_conv2d(x, g)
    assert np.array_equal(y, want)
    # per-channel scales: channel 1 keeps scale 1; the others get scales that are not powers of two, so
    # the result is no longer exact, but close
    y_pc, _, s_pc, *_ = int8.winograd_conv2d_int8(x, g, points, m, storage=32, mode="per_channel", want_intermediates=True)
    assert s_pc.shape == (3,) and s_pc[1] == 1.0
    assert np.array_equal(y_pc[:, 1], want[:, 1])
    assert np.abs(y_pc - want).max() < 0.02 * np.abs(want).max()


def test_int8_convolution_equals_the_definition_on_dequantised_operands():
    m = 4
    points = pts(synth.NOVA[m])
    x, g = synth.make_layer(2, 5, 4, 9, 11, seed=8, dtype="f16", x_dist="normal")
    x, g = x.astype(np.float64), g.astype(np.float64)
    for mode in ("per_tensor", "per_channel", "per_position"):
        y, Uq, s_u, Vq, s_v, Mi, M = int8.winograd_conv2d_int8(x, g, points, m, storage=32, mode=mode,
                                                              want_intermediates=True)
        n, T, K, C = 6, Vq.shape[1], 4, 5
        # scale of the product at (position, output channel)
        if mode == "per_position":
            assert s_u.shape == (n * n,) and s_v.shape == (n * n,)
            scale = np.outer(s_u.astype(np.float64) * s_v.astype(np.float64), np.ones(K))
        elif mode == "per_channel":
            scale = np.outer(np.ones(n * n), s_u.astype(np.float64) * float(s_v[0]))
        else:
            scale = np.full((n * n, K), float(s_u[0]) * float(s_v[0]))
        A = ct.to_f32(ct.cook_toom(points, m, 3)[0]).astype(np.float64)
        th, tw = 3, 3
        for img in range(2):
            for k in range(K):
                for tr in range(th):
                    for tc in range(tw):
                        t = (img * th + tr) * tw + tc
                        Mk = np.zeros((n, n))
                        for xi in range(n * n):
                            acc = 0
                            for c in range(C):
                                acc += int(Uq[xi, k, c]) * int(Vq[xi, t, c])
                            assert acc == Mi[xi, t, k]
                            Mk[xi // n, xi % n] = acc * scale[xi, k]
                        Y = A.T @ Mk @ A
                        for p in range(m):
                            for q in range(m):
                                h, w = tr * m + p, tc * m + q
                                if h < 9 and w < 11:
                                    assert abs(y[img, k, h, w] - Y[p, q]) <= 1e-5 * max(1.0, abs(Y[p, q]))
        # the de-quantised products are binary32 numbers: fl(fl(Mi) * fl(s_U s_V))
        if mode == "per_position":
            both = (s_u * s_v).astype(np.float32).reshape(-1, 1, 1)
        else:
            both = (s_u * s_v[0]).astype(np.float32).reshape(1, 1, -1)
        assert np.array_equal(M, (Mi.astype(np.float32) * both).astype(np.float32))


def test_int8_error_follows_the_direction_the_paper_reports():
    # uniform [-1, 1] inputs and kernels as in Sec. "INT8 Convolution Error Validation"; relative L2 error
    # against the fp64 definition.  Table "Per-tensor vs per-channel INT8 quantization error": the
    # discovered points do better than the integer points, per-channel scales no worse than per-tensor.
    rng = np.random.default_rng(21)
    x = rng.uniform(-1, 1, (2, 16, 24, 24)).astype(np.float32).astype(np.float64)
    g = (rng.uniform(-1, 1, (8, 16, 3, 3)) * np.linspace(0.1, 1.0, 8).reshape(8, 1, 1, 1)).astype(np.float32).astype(np.float64)
    want = conv.direct_conv2d(x, g)

    def err(points, m, mode):
        y = int8.winograd_conv2d_int8(x, g, pts(points), m, storage=32, mode=mode)
        return float(np.linalg.norm(y - want) / np.linalg.norm(want))

    for m in (4, 6):
        e_std, e_nova = err(synth.STANDARD[m], m, "per_tensor"), err(synth.NOVA[m], m, "per_tensor")
        e_std_pc, e_nova_pc = err(synth.STANDARD[m], m, "per_channel"), err(synth.NOVA[m], m, "per_channel")
        assert e_nova < e_std and e_nova_pc < e_std_pc
        assert e_nova_pc < 1.05 * e_nova and e_std_pc < 1.05 * e_std
    assert err(synth.STANDARD[2], 2, "per_tensor") < 0.05
    # a scale per position follows the spread of magnitudes between positions that one scale cannot
    for m in (4, 6, 8):
        assert err(synth.NOVA[m], m, "per_position") < 0.8 * err(synth.NOVA[m], m, "per_tensor")
        assert err(synth.STANDARD[m], m, "per_position") < 0.2 * err(synth.STANDARD[m], m, "per_tensor")
