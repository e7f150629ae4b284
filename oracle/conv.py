"""fp64 direct / Winograd convolution and reduced-precision emulation (test oracle).

Test infrastructure only; see the package docstring.  The loops live in
conv_oracle.c (plain C, OpenMP over images / tile rows); this module compiles
that file with gcc on first use and marshals numpy arrays.
"""
import ctypes
import os
import subprocess

import numpy as np

from . import cook_toom as ct

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_conv.so")
_lib = None


def build(force=False):
    """Compile conv_oracle.c.  -ffp-contract=off: the binary32 input-transform chain must
    not be re-fused or re-associated by the compiler."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fopenmp", "-fPIC",
                               "-shared", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        dp = ctypes.POINTER(ctypes.c_double)
        fp = ctypes.POINTER(ctypes.c_float)
        i = ctypes.c_int
        lib.nova_oracle_threads.restype = i
        lib.nova_oracle_round_f16.argtypes = [dp, dp, ctypes.c_long]
        lib.nova_oracle_round_f16.restype = None
        lib.nova_oracle_direct_conv2d.argtypes = [dp, dp, dp, i, i, i, i, i, i]
        lib.nova_oracle_direct_conv2d.restype = i
        lib.nova_oracle_winograd_conv2d_f64.argtypes = [dp, dp, dp, i, i, i, i, i, i, i, dp, dp, dp]
        lib.nova_oracle_winograd_conv2d_f64.restype = i
        lib.nova_oracle_winograd_conv2d_emulated.argtypes = (
            [dp, dp, dp, i, i, i, i, i, i, i, fp, fp, dp, i, i, i, i, dp, dp, dp])
        lib.nova_oracle_winograd_conv2d_emulated.restype = i
        _lib = lib
    return _lib


def _d(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _f(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _c64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def threads():
    """Number of OpenMP threads the C loops run on."""
    return int(_load().nova_oracle_threads())


def round_f16(values):
    """Nearest binary16 (as fp64) of fp64 values, by the oracle's own rounding routine."""
    src = _c64(values)
    out = np.empty_like(src)
    _load().nova_oracle_round_f16(_d(src), _d(out), src.size)
    return out


def direct_conv2d(x, g):
    """fp64 r x r convolution (r odd), stride 1, pad (r-1)/2, no flip, no bias (Sec. 2.1
    definition; 3 x 3 is the paper's case).  x [N,C,H,W], g [K,C,r,r] -> y [N,K,H,W] fp64."""
    x, g = _c64(x), _c64(g)
    N, C, H, W = x.shape
    K, r = g.shape[0], g.shape[-1]
    assert g.shape == (K, C, r, r) and r % 2 == 1
    y = np.empty((N, K, H, W), dtype=np.float64)
    rc = _load().nova_oracle_direct_conv2d(_d(x), _d(g), _d(y), N, C, H, W, K, r)
    if rc:
        raise RuntimeError(f"oracle direct conv failed ({rc})")
    return y


def winograd_conv2d_f64(x, g, points, m):
    """fp64 Winograd F(m x m, r x r), r = g.shape[-1], with the matrices of
    cook_toom(points, m, r) rounded once to fp64."""
    x, g = _c64(x), _c64(g)
    N, C, H, W = x.shape
    K, r = g.shape[0], g.shape[-1]
    A, BT, G = ct.cook_toom(points, m, r)
    y = np.empty((N, K, H, W), dtype=np.float64)
    A64, BT64, G64 = ct.to_f64(A), ct.to_f64(BT), ct.to_f64(G)
    rc = _load().nova_oracle_winograd_conv2d_f64(_d(x), _d(g), _d(y), N, C, H, W, K, m, r,
                                                 _d(A64), _d(BT64), _d(G64))
    if rc:
        raise RuntimeError(f"oracle winograd conv failed ({rc})")
    return y


def int8_matrix_tile_error(points, m, trials=100, seed=0):
    """Mean relative L2 error of one F(m x m, 3 x 3) tile computed in fp64 with A, B^T and G each
    quantised to INT8 per tensor (cook_toom.quantize_int8), against the directly computed
    m x m correlation, over `trials` input tiles and kernels drawn uniformly from [-1, 1]
    (Sec. "INT8 Convolution Error Validation": setup and Table "INT8 convolution error")."""
    A, BT, G = ct.cook_toom(points, m, 3)
    Aq, BTq, Gq = (ct.to_f64(ct.quantize_int8(mat)[0]) for mat in (A, BT, G))
    rng = np.random.default_rng(seed)
    n = m + 2
    total = 0.0
    for _ in range(trials):
        d = rng.uniform(-1.0, 1.0, (n, n))
        g = rng.uniform(-1.0, 1.0, (3, 3))
        ref = np.zeros((m, m))
        for a in range(3):
            for b in range(3):
                ref += g[a, b] * d[a:a + m, b:b + m]
        y = Aq.T @ ((Gq @ g @ Gq.T) * (BTq @ d @ BTq.T)) @ Aq
        total += np.linalg.norm(y - ref) / np.linalg.norm(ref)
    return total / trials


def _matrices(points, m, row_scaling, r=3):
    A, BT, G = ct.cook_toom(points, m, r)
    if row_scaling is None:
        return A, BT, G
    if isinstance(row_scaling, str):
        if row_scaling != "balanced":
            raise ValueError(row_scaling)
        log2_b, log2_g = ct.balanced_row_exponents(BT, G)
    else:
        log2_b, log2_g = row_scaling
    return ct.scale_rows(A, BT, G, log2_b, log2_g)


def winograd_conv2d_emulated(x, g, points, m, storage=16, m_storage=32, v_exact=False,
                             relu=False, transform_dtype="f32", want_intermediates=False,
                             row_scaling=None):
    """Winograd with the intermediate tensors rounded as the fp16 (storage=16) or fp32
    (storage=32) device path rounds them.  x and g must already be exact in the storage
    format.  transform_dtype 'f32' keeps A and B^T as binary32 constants, 'f16' first rounds
    every matrix entry to binary16 (the variant of Sec. "Float16 Precision Analysis"), 'int8' first quantises each
    matrix to INT8 per tensor (cook_toom.quantize_int8; the de-quantised values are then held as
    binary32 / binary64 constants).
    row_scaling: None, "balanced", or (log2_b, log2_g) -- power-of-two row scales applied to
    the exact matrices before any rounding (cook_toom.scale_rows).
    Returns y, or (y, U, V, M) with U [n*n,K,C], V [n*n,T,C], M [n*n,T,K] as fp64."""
    r = np.shape(g)[-1]
    A, BT, G = _matrices(points, m, row_scaling, r)
    if transform_dtype == "f32":
        A32, BT32, G64 = ct.to_f32(A), ct.to_f32(BT), ct.to_f64(G)
    elif transform_dtype == "f16":
        A32 = ct.to_f16(A).astype(np.float32)
        BT32 = ct.to_f16(BT).astype(np.float32)
        G64 = ct.to_f16(G).astype(np.float64)
    elif transform_dtype == "int8":
        A32 = ct.to_f32(ct.quantize_int8(A)[0])
        BT32 = ct.to_f32(ct.quantize_int8(BT)[0])
        G64 = ct.to_f64(ct.quantize_int8(G)[0])
    else:
        raise ValueError(transform_dtype)
    x, g = _c64(x), _c64(g)
    N, C, H, W = x.shape
    K = g.shape[0]
    n = m + r - 1
    T = N * (-(-H // m)) * (-(-W // m))
    y = np.empty((N, K, H, W), dtype=np.float64)
    null = ctypes.POINTER(ctypes.c_double)()
    U = V = M = None
    if want_intermediates:
        U = np.empty((n * n, K, C), dtype=np.float64)
        V = np.empty((n * n, T, C), dtype=np.float64)
        M = np.empty((n * n, T, K), dtype=np.float64)
    A32, BT32 = np.ascontiguousarray(A32), np.ascontiguousarray(BT32)
    rc = _load().nova_oracle_winograd_conv2d_emulated(
        _d(x), _d(g), _d(y), N, C, H, W, K, m, r, _f(A32), _f(BT32), _d(G64),
        storage, m_storage, int(bool(v_exact)), int(bool(relu)),
        _d(U) if want_intermediates else null,
        _d(V) if want_intermediates else null,
        _d(M) if want_intermediates else null)
    if rc:
        raise RuntimeError(f"oracle emulated winograd conv failed ({rc})")
    return (y, U, V, M) if want_intermediates else y


def relu_maxpool2x2(y):
    """max(y, 0) followed by a 2x2, stride-2 max-pool (the step between VGG blocks)."""
    y = np.maximum(np.asarray(y, dtype=np.float64), 0.0)
    N, K, H, W = y.shape
    return y[:, :, :H // 2 * 2, :W // 2 * 2].reshape(N, K, H // 2, 2, W // 2, 2).max(axis=(3, 5))
