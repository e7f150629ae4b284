"""INT8 quantisation in the Winograd domain (test oracle).

Test infrastructure only; see the package docstring.

The scheme is the symmetric one of Sec. 4.1 "INT8 Setup" and of the "CNN Quantization Setup"
paragraph: no zero point, scale s = max|.| / 127 -- one per tensor ("per-tensor") or, for the
weights, one per output channel ("per-channel") -- code = value / s rounded to nearest with ties to
even and saturated to [-128, 127]; the transform matrices stay in floating point and what is
quantised are the operands of the element-wise (channel) products: the transformed weights
U = G g G^T and the transformed input tiles V = B^T d B.  The products are then exact integers.

A third mode, "per-position", gives every Winograd-domain position xi a scale of its own, for U and
for V (the tap-wise scaling the paper's related-work section discusses as the complementary remedy):
the positions differ in magnitude by the products of the row norms of the transform matrices, which
one scale per tensor cannot follow.

Reading taken where the paper leaves a choice (it describes the scheme for weights w and for "the
Winograd intermediate"): the scale of U is taken over U (all positions and input channels of the
tensor, or of one output channel), the scale of V over the whole tensor V -- a scale that varied
with the input channel could not be pulled out of the channel sum.  Every floating-point step that
decides a code is binary32: s = fl(max / 127), code = rint(fl(value / s)); a tensor (or channel)
that is all zero gets s = 1.
"""
import numpy as np

from . import conv
from . import cook_toom as ct


def quantize_symmetric(values, axis=None):
    """values: array of binary32-representable numbers.  axis=None: one scale for the tensor;
    axis=k: one scale per index along that axis.  Returns (codes int8, scales float32)."""
    v = np.asarray(values, dtype=np.float32)
    if axis is None:
        top = np.float32(np.max(np.abs(v))) if v.size else np.float32(0)
        s = np.float32(top / np.float32(127.0)) if top > 0 else np.float32(1.0)
        scaled = (v / s).astype(np.float32)
        scales = np.array([s], dtype=np.float32)
    else:
        other = tuple(i for i in range(v.ndim) if i != axis)
        top = np.max(np.abs(v), axis=other).astype(np.float32)
        s = np.where(top > 0, (top / np.float32(127.0)).astype(np.float32), np.float32(1.0)).astype(np.float32)
        shape = [1] * v.ndim
        shape[axis] = -1
        scaled = (v / s.reshape(shape)).astype(np.float32)
        scales = s
    codes = np.clip(np.rint(scaled), -128, 127).astype(np.int8)       # rint: ties to even
    return codes, scales


def winograd_conv2d_int8(x, g, points, m, storage=16, mode="per_tensor", relu=False, want_intermediates=False):
    """F(m x m, r x r) convolution with INT8 operands in the Winograd domain.

    x, g: exact in the storage format (16: binary16, 32: binary32).  U and V are formed as in
    conv.winograd_conv2d_emulated (same arithmetic contract, rounded to the storage format), then
    quantised (U per tensor or per output channel, V per tensor; "per_position": both per position);
    the channel sum is taken on the integer codes, exactly; M = fl32(fl32(sum) * fl32(s_U * s_V)); Y = A^T M A in binary64 with the
    binary32 matrix A, optional ReLU, one rounding to the storage format.
    Returns y, or (y, Uq [n*n,K,C] int8, s_U, Vq [n*n,T,C] int8, s_V, Mi [n*n,T,K] int64, M float32)."""
    if mode not in ("per_tensor", "per_channel", "per_position"):
        raise ValueError(mode)
    x = np.asarray(x, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    N, C, H, W = x.shape
    K, r = g.shape[0], g.shape[-1]
    n = m + r - 1
    _, U, V, _ = conv.winograd_conv2d_emulated(x, g, points, m, storage=storage, want_intermediates=True)
    if mode == "per_position":
        Uq, s_u = quantize_symmetric(U, axis=0)
        Vq, s_v = quantize_symmetric(V, axis=0)
        both = (s_u * s_v).astype(np.float32).reshape(-1, 1, 1)                       # [n*n]
    else:
        Uq, s_u = quantize_symmetric(U, axis=1 if mode == "per_channel" else None)
        Vq, s_v = quantize_symmetric(V, axis=None)
        both = (s_u * s_v[0]).astype(np.float32).reshape(1, 1, -1)                    # [K] or [1]
    Mi = np.matmul(Vq.astype(np.int64), Uq.astype(np.int64).transpose(0, 2, 1))        # [n*n][T][K], exact
    M = (Mi.astype(np.float32) * both).astype(np.float32)
    A = ct.to_f32(ct.cook_toom(points, m, r)[0]).astype(np.float64)                    # n x m
    th, tw = -(-H // m), -(-W // m)
    Y = np.einsum("ip,jq,ijtk->tkpq", A, A, M.astype(np.float64).reshape(n, n, N * th * tw, K))
    y = Y.reshape(N, th, tw, K, m, m).transpose(0, 3, 1, 4, 2, 5).reshape(N, K, th * m, tw * m)[:, :, :H, :W]
    if relu:
        y = np.maximum(y, 0.0)
    y = conv.round_f16(y) if storage == 16 else y.astype(np.float32).astype(np.float64)
    if want_intermediates:
        return y, Uq, s_u, Vq, s_v, Mi, M
    return y
