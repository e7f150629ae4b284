"""Seeded synthetic workloads and the interpolation-point sets they are run with.

This module holds inputs only -- no transform arithmetic -- so that the HIP path and
the CPU checker can both be fed from it.  Point sets are written as (numerator,
denominator) pairs, finite points only (the point at infinity is implicit), in the
canonical order 0, +a1, -a1, +a2, -a2, ... by increasing |a|.

STANDARD: the small-integer sets of Table "Vandermonde condition numbers for standard
integer points".  NOVA: the discovered sets of Table "Complete discovered
configurations".  CLASSIC_HALF_F63 is the {0, +-1, +-2, +-1/2} set widely used for
F(6,3) outside the paper.  DYADIC_F43 is the fp16-representable set of Table
"Dtype-aware discovery for F(4,3)".
"""
import numpy as np


def _sym(*mags):
    pts = [(0, 1)]
    for num, den in mags:
        pts += [(num, den), (-num, den)]
    return pts


STANDARD = {
    2: _sym((1, 1)),
    4: _sym((1, 1), (2, 1)),
    6: _sym((1, 1), (2, 1), (3, 1)),
    8: _sym((1, 1), (2, 1), (3, 1), (4, 1)),
}
NOVA = {
    2: _sym((1, 1)),
    4: _sym((5, 6), (7, 6)),
    6: _sym((3, 5), (1, 1), (7, 6)),
    8: _sym((2, 5), (5, 6), (1, 1), (7, 6)),
}
CLASSIC_HALF_F63 = _sym((1, 2), (1, 1), (2, 1))
DYADIC_F43 = _sym((3, 4), (5, 4))


def point_set(name, m):
    """'standard' | 'nova' | 'classic_half' (m = 6 only) | 'dyadic' (m = 4 only)."""
    if name == "standard":
        return STANDARD[m]
    if name == "nova":
        return NOVA[m]
    if name == "classic_half" and m == 6:
        return CLASSIC_HALF_F63
    if name == "dyadic" and m == 4:
        return DYADIC_F43
    raise KeyError((name, m))


def make_layer(N, C, K, H, W, *, seed, dtype="f16", x_dist="half_normal"):
    """One 3x3 conv layer's tensors: x [N,C,H,W] i.i.d. N(0,1) ('normal') or |N(0,1)|
    ('half_normal', post-ReLU-like); w [K,C,3,3] i.i.d. N(0, 2/(9 C)) (He-normal); both
    drawn in fp64 from numpy's default_rng(seed) and rounded once to the storage dtype."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((N, C, H, W))
    if x_dist == "half_normal":
        np.abs(x, out=x)
    elif x_dist != "normal":
        raise ValueError(x_dist)
    w = rng.standard_normal((K, C, 3, 3)) * np.sqrt(2.0 / (9.0 * C))
    np_dtype = {"f16": np.float16, "f32": np.float32}[dtype]
    return x.astype(np_dtype), w.astype(np_dtype)


# The single-layer workloads (shape, tile size, storage dtype, input distribution).
LAYER_CONFIGS = {
    "small_f43_fp32": dict(N=1, C=16, K=16, H=32, W=32, m=4, dtype="f32", x_dist="normal", seed=1000),
    "mid_f63_fp16": dict(N=8, C=64, K=64, H=56, W=56, m=6, dtype="f16", x_dist="half_normal", seed=2000),
    "vgg_conv3_f83_fp16": dict(N=32, C=256, K=256, H=56, W=56, m=8, dtype="f16", x_dist="half_normal", seed=3000),
}

# ResNet-50-style stride-1 3x3 bottleneck shapes at batch 256, F(8,3).
RESNET_SHAPES = [(64, 56), (128, 28), (256, 14), (512, 7)]
for _idx, (_ch, _hw) in enumerate(RESNET_SHAPES):
    LAYER_CONFIGS[f"resnet_c{_ch}_{_hw}_f83_fp16"] = dict(N=256, C=_ch, K=_ch, H=_hw, W=_hw, m=8, dtype="f16",
                                                         x_dist="half_normal", seed=5100 + _idx)
# the point set each single-layer workload is quoted on (others can be asked for)
DEFAULT_POINTS = {"small_f43_fp32": "standard", "mid_f63_fp16": "nova"}

# VGG-16 conv stack: (C_in, C_out) per layer, 2x2 max-pool after layers 2, 4, 7, 10, 13.
VGG16_LAYERS = [(3, 64), (64, 64), (64, 128), (128, 128), (128, 256), (256, 256), (256, 256),
                (256, 512), (512, 512), (512, 512), (512, 512), (512, 512), (512, 512)]
VGG16_POOL_AFTER = (2, 4, 7, 10, 13)
