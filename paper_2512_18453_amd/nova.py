"""Thin binding over libnova.so (include/nova.h): argument marshalling only.

Every function has the name of the C entry point it calls.  Torch tensors are used as
device-memory handles (`data_ptr()`) and for the current stream; all arithmetic runs in the
library's kernels.  There is no fallback: if the library is missing the import of this module
succeeds but the first call raises.
"""
import ctypes
import os
from fractions import Fraction

import torch

NOVA_F32, NOVA_F16 = 0, 1
NOVA_MATRIX_A, NOVA_MATRIX_BT, NOVA_MATRIX_G = 0, 1, 2
NOVA_ROWS_PLAIN, NOVA_ROWS_BALANCED, NOVA_ROWS_GIVEN = 0, 1, 2
NOVA_MATRIX_F32, NOVA_MATRIX_F16, NOVA_MATRIX_INT8 = 0, 1, 2
NOVA_FLAG_RELU, NOVA_FLAG_M_F16, NOVA_FLAG_POOL2 = 1, 2, 4
NOVA_INT8_PER_TENSOR, NOVA_INT8_PER_CHANNEL, NOVA_INT8_PER_POSITION = 0, 1, 2
NOVA_PATH_STAGES, NOVA_PATH_FEW_CHANNELS, NOVA_PATH_FUSED_OUTPUT = 0, 1, 2

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libnova.so")
_lib = None

EXPORTS = [
    "nova_make_transforms", "nova_make_transforms_ex", "nova_get_row_scaling", "nova_get_matrix_int8", "nova_free_transforms", "nova_symmetric_search", "nova_snap_to_rational", "nova_transforms_shape", "nova_get_matrix",
    "nova_get_matrix_f64", "nova_get_matrix_f32", "nova_kappa", "nova_filter_bytes", "nova_input_bytes",
    "nova_product_bytes", "nova_filter_transform", "nova_conv2d_workspace_bytes", "nova_winograd_conv2d",
    "nova_winograd_conv2d_static", "nova_static_workspace_bytes",
    "nova_contract_output_fused", "nova_conv2d_path", "nova_es_fitness", "nova_es_normals_needed", "nova_evolution_strategy", "nova_snap_points",
    "nova_filter_int8_bytes", "nova_input_int8_bytes", "nova_quantize_filter_int8", "nova_quantize_input_int8",
    "nova_contract_int8", "nova_conv2d_int8_workspace_bytes", "nova_winograd_conv2d_int8",
    "nova_input_transform", "nova_contract", "nova_output_transform", "nova_relu_maxpool2x2",
    "nova_strerror", "nova_last_hip_error", "nova_version",
]


class nova_rational(ctypes.Structure):
    _fields_ = [("num", ctypes.c_int64), ("den", ctypes.c_int64)]


class NovaError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        detail = lib().nova_strerror(code).decode()
        if code == -7:
            detail += f" [hipError {lib().nova_last_hip_error()}]"
        super().__init__(f"{where}: {detail} ({code})")


def lib():
    """The loaded library; raises if it has not been built (python -m paper_2512_18453_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} not found: build it with `python -m paper_2512_18453_amd.build`")
        L = ctypes.CDLL(_LIB_PATH)
        vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        ip = ctypes.POINTER(ctypes.c_int)
        L.nova_make_transforms.argtypes = [ctypes.POINTER(nova_rational), i, i, i, ctypes.POINTER(vp)]
        L.nova_make_transforms_ex.argtypes = [ctypes.POINTER(nova_rational), i, i, i, i, ip, ip, i, ctypes.POINTER(vp)]
        L.nova_get_row_scaling.argtypes = [vp, ip, ip]
        L.nova_get_matrix_int8.argtypes = [vp, i, ctypes.POINTER(ctypes.c_int8), ctypes.POINTER(ctypes.c_double)]
        L.nova_free_transforms.argtypes = [vp]
        L.nova_symmetric_search.argtypes = [i, i, i, ctypes.POINTER(nova_rational), ctypes.POINTER(ctypes.c_double)]
        L.nova_snap_to_rational.argtypes = [ctypes.c_double, i, ctypes.POINTER(nova_rational)]
        dp = ctypes.POINTER(ctypes.c_double)
        L.nova_es_fitness.argtypes = [i, i, dp, dp, dp]
        L.nova_es_normals_needed.argtypes = [i] * 5
        L.nova_es_normals_needed.restype = sz
        L.nova_evolution_strategy.argtypes = [i, i, i, i, i, dp, sz, dp, dp]
        L.nova_snap_points.argtypes = [i, i, dp, i, ctypes.POINTER(nova_rational), dp]
        L.nova_free_transforms.restype = None
        L.nova_transforms_shape.argtypes = [vp, ip, ip, ip, ip]
        L.nova_get_matrix.argtypes = [vp, i, ctypes.POINTER(nova_rational)]
        L.nova_get_matrix_f64.argtypes = [vp, i, ctypes.POINTER(ctypes.c_double)]
        L.nova_get_matrix_f32.argtypes = [vp, i, ctypes.POINTER(ctypes.c_float)]
        L.nova_kappa.argtypes = [vp, ctypes.POINTER(ctypes.c_double)]
        L.nova_filter_bytes.argtypes = [i] * 5
        L.nova_filter_bytes.restype = sz
        L.nova_input_bytes.argtypes = [i] * 7
        L.nova_input_bytes.restype = sz
        L.nova_product_bytes.argtypes = [i] * 8
        L.nova_product_bytes.restype = sz
        L.nova_conv2d_workspace_bytes.argtypes = [i] * 10
        L.nova_conv2d_workspace_bytes.restype = sz
        L.nova_filter_transform.argtypes = [vp, vp, i, i, i, vp, vp]
        L.nova_winograd_conv2d.argtypes = [vp, vp, vp, vp, i, i, i, i, i, i, i, vp, sz, vp]
        L.nova_winograd_conv2d_static.argtypes = [vp, vp, vp, vp, i, i, i, i, i, i, i, vp]
        L.nova_static_workspace_bytes.argtypes = []
        L.nova_static_workspace_bytes.restype = sz
        L.nova_filter_int8_bytes.argtypes = [i] * 4
        L.nova_filter_int8_bytes.restype = sz
        L.nova_input_int8_bytes.argtypes = [i] * 6
        L.nova_input_int8_bytes.restype = sz
        L.nova_quantize_filter_int8.argtypes = [vp, vp, i, i, i, i, vp, vp, vp]
        L.nova_quantize_input_int8.argtypes = [vp, vp, i, i, i, i, i, i, vp, vp, vp]
        L.nova_contract_int8.argtypes = [vp, vp, vp, vp, vp, i, vp, sz, i, i, i, i, i, i, vp]
        L.nova_conv2d_int8_workspace_bytes.argtypes = [i] * 8
        L.nova_conv2d_int8_workspace_bytes.restype = sz
        L.nova_winograd_conv2d_int8.argtypes = [vp, vp, vp, vp, i, vp, i, i, i, i, i, i, i, vp, sz, vp]
        L.nova_contract_output_fused.argtypes = [vp, vp, vp, vp, i, i, i, i, i, i, i, vp]
        L.nova_conv2d_path.argtypes = [vp, i, i, i, i, i, i]
        L.nova_input_transform.argtypes = [vp, vp, vp, sz, i, i, i, i, i, vp]
        L.nova_contract.argtypes = [vp, vp, vp, vp, sz, i, i, i, i, i, i, i, vp]
        L.nova_output_transform.argtypes = [vp, vp, sz, vp, i, i, i, i, i, i, vp]
        L.nova_relu_maxpool2x2.argtypes = [vp, vp, i, i, i, i, i, vp]
        L.nova_strerror.argtypes = [i]
        L.nova_strerror.restype = ctypes.c_char_p
        L.nova_last_hip_error.restype = i
        L.nova_version.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _check(code, where):
    if code != 0:
        raise NovaError(code, where)


def _dtype_code(t):
    if t.dtype == torch.float16:
        return NOVA_F16
    if t.dtype == torch.float32:
        return NOVA_F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t):
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    return ctypes.c_void_p(t.data_ptr())


class Transforms:
    """Owner of a nova_transforms handle."""

    def __init__(self, handle, m, r, n, symmetric):
        self.handle, self.m, self.r, self.n, self.symmetric = handle, m, r, n, symmetric

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.nova_free_transforms(self.handle)
            self.handle = None


def _points_array(points):
    arr = (nova_rational * max(len(points), 1))()
    for idx, p in enumerate(points):
        if isinstance(p, tuple):
            arr[idx].num, arr[idx].den = p
        else:
            fr = Fraction(p)
            arr[idx].num, arr[idx].den = fr.numerator, fr.denominator
    return arr


def nova_make_transforms(points, m, r=3, row_scaling=None, matrix_dtype="f32"):
    """points: finite interpolation points as ints, Fractions or (num, den) pairs.
    row_scaling: None, "balanced" or (log2_b, log2_g); matrix_dtype: "f32", "f16" or "int8"
    (nova_make_transforms_ex)."""
    arr = _points_array(points)
    handle = ctypes.c_void_p()
    if row_scaling is None and matrix_dtype == "f32":
        _check(lib().nova_make_transforms(arr, len(points), m, r, ctypes.byref(handle)), "nova_make_transforms")
    else:
        n = m + r - 1
        mode, b_arr, g_arr = NOVA_ROWS_PLAIN, None, None
        if isinstance(row_scaling, str):
            if row_scaling != "balanced":
                raise ValueError(row_scaling)
            mode = NOVA_ROWS_BALANCED
        elif row_scaling is not None:
            log2_b, log2_g = row_scaling
            if len(log2_b) != n or len(log2_g) != n:
                raise ValueError("row_scaling needs one exponent per matrix row")
            mode = NOVA_ROWS_GIVEN
            b_arr, g_arr = (ctypes.c_int * n)(*log2_b), (ctypes.c_int * n)(*log2_g)
        md = {"f32": NOVA_MATRIX_F32, "f16": NOVA_MATRIX_F16, "int8": NOVA_MATRIX_INT8}[matrix_dtype]
        _check(lib().nova_make_transforms_ex(arr, len(points), m, r, mode, b_arr, g_arr, md, ctypes.byref(handle)),
               "nova_make_transforms_ex")
    mm, rr, nn, sym = ctypes.c_int(), ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    _check(lib().nova_transforms_shape(handle, mm, rr, nn, sym), "nova_transforms_shape")
    return Transforms(handle, mm.value, rr.value, nn.value, bool(sym.value))


def nova_symmetric_search(m, r=3, d_max=6):
    """(points, kappa): best symmetric configuration as Fractions in canonical order."""
    count = m + r - 2
    buf = (nova_rational * max(count, 1))()
    kappa = ctypes.c_double()
    _check(lib().nova_symmetric_search(m, r, d_max, buf, ctypes.byref(kappa)), "nova_symmetric_search")
    return [Fraction(buf[idx].num, buf[idx].den) for idx in range(count)], kappa.value


def nova_snap_to_rational(x, d_max=10):
    out = nova_rational()
    _check(lib().nova_snap_to_rational(float(x), d_max, ctypes.byref(out)), "nova_snap_to_rational")
    return Fraction(out.num, out.den)


def nova_es_fitness(m, r, points):
    """(f, tensor error, |p|^2 / (n - 1), kappa(V)) of finite points given as floats."""
    pts = (ctypes.c_double * len(points))(*[float(v) for v in points])
    f, parts = ctypes.c_double(), (ctypes.c_double * 3)()
    _check(lib().nova_es_fitness(m, r, pts, ctypes.byref(f), parts), "nova_es_fitness")
    return f.value, parts[0], parts[1], parts[2]


def nova_es_normals_needed(m, r=3, generations=100, population=50, restarts=3):
    return int(lib().nova_es_normals_needed(m, r, generations, population, restarts))


def nova_evolution_strategy(m, r, normals, generations=100, population=50, restarts=3):
    """normals: sequence of standard normal draws (at least nova_es_normals_needed).  -> (points, fitness)."""
    z = (ctypes.c_double * len(normals))(*[float(v) for v in normals])
    out = (ctypes.c_double * (m + r - 2))()
    f = ctypes.c_double()
    _check(lib().nova_evolution_strategy(m, r, generations, population, restarts, z, len(normals), out, ctypes.byref(f)),
           "nova_evolution_strategy")
    return list(out), f.value


def nova_snap_points(m, r, x, d_max=10):
    pts = (ctypes.c_double * len(x))(*[float(v) for v in x])
    out = (nova_rational * (m + r - 2))()
    kappa = ctypes.c_double()
    _check(lib().nova_snap_points(m, r, pts, d_max, out, ctypes.byref(kappa)), "nova_snap_points")
    return [Fraction(p.num, p.den) for p in out], kappa.value


def nova_get_row_scaling(t):
    """(log2_b, log2_g): the power-of-two row exponents in effect."""
    b, g = (ctypes.c_int * t.n)(), (ctypes.c_int * t.n)()
    _check(lib().nova_get_row_scaling(t.handle, b, g), "nova_get_row_scaling")
    return list(b), list(g)


def nova_get_matrix_int8(t, which):
    """(codes as nested lists, scale) of one matrix of a handle made with matrix_dtype='int8'."""
    rows, cols = _matrix_shape(t, which)
    buf = (ctypes.c_int8 * (rows * cols))()
    scale = ctypes.c_double()
    _check(lib().nova_get_matrix_int8(t.handle, which, buf, ctypes.byref(scale)), "nova_get_matrix_int8")
    return [[buf[i * cols + j] for j in range(cols)] for i in range(rows)], scale.value


def _matrix_shape(t, which):
    return (t.n, {NOVA_MATRIX_A: t.m, NOVA_MATRIX_BT: t.n, NOVA_MATRIX_G: t.r}[which])


def nova_get_matrix(t, which):
    rows, cols = _matrix_shape(t, which)
    buf = (nova_rational * (rows * cols))()
    _check(lib().nova_get_matrix(t.handle, which, buf), "nova_get_matrix")
    return [[Fraction(buf[i * cols + j].num, buf[i * cols + j].den) for j in range(cols)] for i in range(rows)]


def nova_get_matrix_f64(t, which):
    rows, cols = _matrix_shape(t, which)
    buf = (ctypes.c_double * (rows * cols))()
    _check(lib().nova_get_matrix_f64(t.handle, which, buf), "nova_get_matrix_f64")
    return [[buf[i * cols + j] for j in range(cols)] for i in range(rows)]


def nova_get_matrix_f32(t, which):
    rows, cols = _matrix_shape(t, which)
    buf = (ctypes.c_float * (rows * cols))()
    _check(lib().nova_get_matrix_f32(t.handle, which, buf), "nova_get_matrix_f32")
    return [[buf[i * cols + j] for j in range(cols)] for i in range(rows)]


def nova_kappa(t):
    out = (ctypes.c_double * 4)()
    _check(lib().nova_kappa(t.handle, out), "nova_kappa")
    return dict(V=out[0], A=out[1], B=out[2], G=out[3])


def nova_filter_bytes(K, C, m, dtype, r=3):
    return lib().nova_filter_bytes(K, C, m, r, dtype)


def nova_input_bytes(N, C, H, W, m, dtype, r=3):
    return lib().nova_input_bytes(N, C, H, W, m, r, dtype)


def nova_product_bytes(N, K, H, W, m, dtype, flags=0, r=3):
    return lib().nova_product_bytes(N, K, H, W, m, r, dtype, flags)


def nova_conv2d_workspace_bytes(N, C, H, W, K, m, dtype, flags=0, images_per_slab=0, r=3):
    return lib().nova_conv2d_workspace_bytes(N, C, H, W, K, m, r, dtype, flags, images_per_slab)


def nova_filter_transform(t, w, U=None):
    """w [K,C,r,r] device tensor -> U (flat device tensor of the same dtype)."""
    K, C = w.shape[0], w.shape[1]
    if tuple(w.shape[2:]) != (t.r, t.r):
        raise ValueError(f"filter is {tuple(w.shape[2:])}, the transforms are for {t.r} x {t.r}")
    dt = _dtype_code(w)
    if U is None:
        U = torch.empty(nova_filter_bytes(K, C, t.m, dt, t.r) // w.element_size(), dtype=w.dtype, device=w.device)
    _check(lib().nova_filter_transform(t.handle, _dev(w), K, C, dt, _dev(U), _stream()), "nova_filter_transform")
    return U


def nova_winograd_conv2d(t, x, U, K, y=None, flags=0, workspace=None, images_per_slab=0):
    """x [N,C,H,W] -> y [N,K,H,W]; workspace: uint8 device tensor (allocated here if None)."""
    N, C, H, W = x.shape
    dt = _dtype_code(x)
    if y is None:
        out_hw = (H // 2, W // 2) if flags & NOVA_FLAG_POOL2 else (H, W)
        y = torch.empty((N, K) + out_hw, dtype=x.dtype, device=x.device)
    if workspace is None:
        workspace = torch.empty(nova_conv2d_workspace_bytes(N, C, H, W, K, t.m, dt, flags, images_per_slab, t.r),
                                dtype=torch.uint8, device=x.device)
    _check(lib().nova_winograd_conv2d(t.handle, _dev(x), _dev(U), _dev(y), N, C, H, W, K, dt, flags,
                                      _dev(workspace), workspace.numel(), _stream()), "nova_winograd_conv2d")
    return y


def nova_static_workspace_bytes():
    return int(lib().nova_static_workspace_bytes())


def nova_winograd_conv2d_static(t, x, U, K, y, flags=0):
    """The call that allocates nothing: y must be passed in."""
    N, C, H, W = x.shape
    _check(lib().nova_winograd_conv2d_static(t.handle, _dev(x), _dev(U), _dev(y), N, C, H, W, K, _dtype_code(x),
                                             flags, _stream()), "nova_winograd_conv2d_static")
    return y


def nova_input_transform(t, x, V=None):
    N, C, H, W = x.shape
    dt = _dtype_code(x)
    if V is None:
        V = torch.empty(nova_input_bytes(N, C, H, W, t.m, dt, t.r) // x.element_size(), dtype=x.dtype, device=x.device)
    _check(lib().nova_input_transform(t.handle, _dev(x), _dev(V), V.numel() * V.element_size(), N, C, H, W, dt,
                                      _stream()), "nova_input_transform")
    return V


def nova_contract(t, U, V, N, C, H, W, K, flags=0, M=None):
    dt = _dtype_code(V)
    if M is None:
        m_dtype = torch.float16 if (dt == NOVA_F16 and flags & NOVA_FLAG_M_F16) else torch.float32
        nbytes = nova_product_bytes(N, K, H, W, t.m, dt, flags, t.r)
        M = torch.empty(nbytes // (2 if m_dtype == torch.float16 else 4), dtype=m_dtype, device=V.device)
    _check(lib().nova_contract(t.handle, _dev(U), _dev(V), _dev(M), M.numel() * M.element_size(), N, C, H, W, K, dt,
                               flags, _stream()), "nova_contract")
    return M


def nova_output_transform(t, M, N, K, H, W, dtype, flags=0, y=None):
    """dtype: torch dtype of y (the storage format of the layer)."""
    dt = NOVA_F16 if dtype == torch.float16 else NOVA_F32
    if y is None:
        out_hw = (H // 2, W // 2) if flags & NOVA_FLAG_POOL2 else (H, W)
        y = torch.empty((N, K) + out_hw, dtype=dtype, device=M.device)
    _check(lib().nova_output_transform(t.handle, _dev(M), M.numel() * M.element_size(), _dev(y), N, K, H, W, dt,
                                       flags, _stream()), "nova_output_transform")
    return y


def nova_quantize_filter_int8(t, U, K, C, mode=NOVA_INT8_PER_TENSOR):
    """U (flat, from nova_filter_transform) -> (Uq int8 flat, u_scales float32 [1] or [K])."""
    Uq = torch.empty(lib().nova_filter_int8_bytes(K, C, t.m, t.r), dtype=torch.int8, device=U.device)
    count = K if mode == NOVA_INT8_PER_CHANNEL else t.n * t.n if mode == NOVA_INT8_PER_POSITION else 1
    scales = torch.empty(count, dtype=torch.float32, device=U.device)
    _check(lib().nova_quantize_filter_int8(t.handle, _dev(U), K, C, _dtype_code(U), mode, _dev(Uq), _dev(scales), _stream()),
           "nova_quantize_filter_int8")
    return Uq, scales


def nova_quantize_input_int8(t, V, N, C, H, W, mode=NOVA_INT8_PER_TENSOR):
    Vq = torch.empty(lib().nova_input_int8_bytes(N, C, H, W, t.m, t.r), dtype=torch.int8, device=V.device)
    scale = torch.empty(t.n * t.n if mode == NOVA_INT8_PER_POSITION else 1, dtype=torch.float32, device=V.device)
    _check(lib().nova_quantize_input_int8(t.handle, _dev(V), N, C, H, W, _dtype_code(V), mode, _dev(Vq), _dev(scale),
                                          _stream()), "nova_quantize_input_int8")
    return Vq, scale


def nova_contract_int8(t, Uq, Vq, u_scales, v_scale, mode, N, C, H, W, K, dequantise, M=None):
    if M is None:
        nbytes = nova_product_bytes(N, K, H, W, t.m, NOVA_F32, 0, t.r)
        M = torch.empty(nbytes // 4, dtype=torch.float32 if dequantise else torch.int32, device=Vq.device)
    us = _dev(u_scales) if u_scales is not None else None
    vs = _dev(v_scale) if v_scale is not None else None
    _check(lib().nova_contract_int8(t.handle, _dev(Uq), _dev(Vq), us, vs, mode, _dev(M), M.numel() * 4, N, C, H, W, K,
                                    1 if dequantise else 0, _stream()), "nova_contract_int8")
    return M


def nova_conv2d_int8_workspace_bytes(N, C, H, W, K, m, dtype, r=3):
    return lib().nova_conv2d_int8_workspace_bytes(N, C, H, W, K, m, r, dtype)


def nova_winograd_conv2d_int8(t, x, Uq, u_scales, mode, K, y=None, flags=0, workspace=None):
    N, C, H, W = x.shape
    dt = _dtype_code(x)
    if y is None:
        out_hw = (H // 2, W // 2) if flags & NOVA_FLAG_POOL2 else (H, W)
        y = torch.empty((N, K) + out_hw, dtype=x.dtype, device=x.device)
    if workspace is None:
        workspace = torch.empty(nova_conv2d_int8_workspace_bytes(N, C, H, W, K, t.m, dt, t.r), dtype=torch.uint8,
                                device=x.device)
    _check(lib().nova_winograd_conv2d_int8(t.handle, _dev(x), _dev(Uq), _dev(u_scales), mode, _dev(y), N, C, H, W, K, dt,
                                           flags, _dev(workspace), workspace.numel(), _stream()),
           "nova_winograd_conv2d_int8")
    return y


def nova_contract_output_fused(t, U, V, N, C, H, W, K, flags=0, y=None):
    if y is None:
        out_hw = (H // 2, W // 2) if flags & NOVA_FLAG_POOL2 else (H, W)
        y = torch.empty((N, K) + out_hw, dtype=V.dtype, device=V.device)
    _check(lib().nova_contract_output_fused(t.handle, _dev(U), _dev(V), _dev(y), N, C, H, W, K, _dtype_code(V), flags,
                                            _stream()), "nova_contract_output_fused")
    return y


def nova_conv2d_path(t, C, H, W, K, dtype_code, flags=0):
    """Which kernels nova_winograd_conv2d runs for this layer shape (NOVA_PATH_*).  dtype_code: NOVA_F16 / NOVA_F32."""
    rc = lib().nova_conv2d_path(t.handle, C, H, W, K, dtype_code, flags)
    _check(min(rc, 0), "nova_conv2d_path")
    return rc


def nova_relu_maxpool2x2(x, out=None):
    N, C, H, W = x.shape
    if out is None:
        out = torch.empty((N, C, H // 2, W // 2), dtype=x.dtype, device=x.device)
    _check(lib().nova_relu_maxpool2x2(_dev(x), _dev(out), N, C, H, W, _dtype_code(x), _stream()), "nova_relu_maxpool2x2")
    return out


def nova_version():
    return lib().nova_version().decode()
