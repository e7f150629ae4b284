// The device-facing entry points of libnova: argument checks, tensor geometry, the slab loop of
// nova_winograd_conv2d.  All device work is done by the launchers in the .hip files.
#include <cstring>

#include "internal.hpp"

namespace nova {

static thread_local int g_last_hip_error = 0;
void set_last_hip_error(int err) { g_last_hip_error = err; }

static int hip_result(int err)
{
    if (err == 0) return NOVA_OK;
    g_last_hip_error = err;
    return NOVA_EHIP;
}

// tile / kernel sizes the device kernels are instantiated for: n = m + r - 1 in {4, 6, 8, 10}
static bool device_tile_ok(int m, int r)
{
    if (r == 3) return m == 2 || m == 4 || m == 6 || m == 8;
    if (r == 5) return m == 2 || m == 4 || m == 6;
    return false;
}
static bool dtype_ok(int dtype) { return dtype == NOVA_F16 || dtype == NOVA_F32; }

static int check_handle(const nova_transforms *t)
{
    if (!t) return NOVA_EINVAL;
    if (!device_tile_ok(t->m, t->r)) return NOVA_EUNSUPPORTED;
    return NOVA_OK;
}

static bool dims_ok(int N, int C, int H, int W, int K)
{
    return N >= 1 && C >= 1 && H >= 1 && W >= 1 && K >= 1 && N <= (1 << 20) && C <= (1 << 20) &&
           K <= (1 << 20) && H <= (1 << 16) && W <= (1 << 16);
}

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

static size_t v_bytes(const Geometry &g, int dtype)
{
    return (size_t)g.n * g.n * g.c_blocks * (size_t)g.T * kChanBlock * dtype_size(dtype);
}
static size_t m_bytes(const Geometry &g, int dtype, int flags)
{
    const size_t es = (dtype == NOVA_F16 && (flags & NOVA_FLAG_M_F16)) ? 2 : 4;
    return (size_t)g.n * g.n * g.k_blocks * (size_t)g.Tp * kChanBlock * es;
}

// What follows V in the workspace of nova_winograd_conv2d: the products M, or, with so few input
// channels that the output transform forms the products itself, the packed filters.
static bool few_channels(int C) { return C <= few_channels_limit(); }
static size_t first_part_bytes(const Geometry &g, int dtype)
{
    return few_channels(g.C) ? few_channels_input_bytes(g, dtype) : v_bytes(g, dtype);
}
static size_t second_part_bytes(const Geometry &g, int dtype, int flags)
{
    return few_channels(g.C) ? few_channels_filter_bytes(g, dtype) : m_bytes(g, dtype, flags);
}

// V and M of a slab together: the size of the last-level cache (256 MB), so that what one stage
// writes is still there when the next reads it.  Measured on 224 x 224 and 112 x 112 VGG layers
// (batch 32): 7-10 % faster than the whole batch in one pass, and faster than smaller slabs.
constexpr size_t kDefaultSlabBytes = (size_t)256 << 20;

}  // namespace nova

using namespace nova;

extern "C" size_t nova_filter_bytes(int K, int C, int m, int r, int dtype)
{
    if (K < 1 || C < 1 || m < 1 || r < 1 || !dtype_ok(dtype)) return 0;
    const size_t n = (size_t)m + r - 1;
    return n * n * ceil_div(C, kChanBlock) * ((size_t)ceil_div(K, kChanBlock) * kChanBlock) * kChanBlock *
           dtype_size(dtype);
}

extern "C" size_t nova_input_bytes(int N, int C, int H, int W, int m, int r, int dtype)
{
    if (!dims_ok(N, C, H, W, 1) || m < 1 || r < 1 || !dtype_ok(dtype)) return 0;
    return v_bytes(make_geometry(N, C, H, W, 1, m, r), dtype);
}

extern "C" size_t nova_product_bytes(int N, int K, int H, int W, int m, int r, int dtype, int flags)
{
    if (!dims_ok(N, 1, H, W, K) || m < 1 || r < 1 || !dtype_ok(dtype)) return 0;
    return m_bytes(make_geometry(N, 1, H, W, K, m, r), dtype, flags);
}

extern "C" size_t nova_conv2d_workspace_bytes(int N, int C, int H, int W, int K, int m, int r, int dtype,
                                              int flags, int images_per_slab)
{
    if (!dims_ok(N, C, H, W, K) || !device_tile_ok(m, r) || !dtype_ok(dtype) || images_per_slab < 0) return 0;
    auto slab_bytes = [&](long long count) {
        const Geometry sg = make_geometry((int)count, C, H, W, K, m, r);
        return align256(first_part_bytes(sg, dtype)) + align256(second_part_bytes(sg, dtype, flags));
    };
    long long imgs = images_per_slab;
    if (imgs == 0) {                             // as many images as fit the default budget
        long long lo = 1, hi = N;
        while (lo < hi) {
            const long long mid = (lo + hi + 1) / 2;
            if (slab_bytes(mid) <= kDefaultSlabBytes) lo = mid; else hi = mid - 1;
        }
        imgs = lo;
    }
    if (imgs > N) imgs = N;
    return slab_bytes(imgs);
}

extern "C" int nova_filter_transform(const nova_transforms *t, const void *w, int K, int C, int dtype,
                                     void *U, void *stream)
{
    if (int rc = check_handle(t)) return rc;
    if (!w || !U || K < 1 || C < 1 || !dtype_ok(dtype)) return NOVA_EINVAL;
    return hip_result(launch_filter_transform(t, w, K, C, dtype, U, stream));
}

extern "C" int nova_input_transform(const nova_transforms *t, const void *x, void *V, size_t V_bytes, int N,
                                    int C, int H, int W, int dtype, void *stream)
{
    if (int rc = check_handle(t)) return rc;
    if (!x || !V || !dims_ok(N, C, H, W, 1) || !dtype_ok(dtype)) return NOVA_EINVAL;
    const Geometry g = make_geometry(N, C, H, W, 1, t->m, t->r);
    if (V_bytes < v_bytes(g, dtype)) return NOVA_ENOSPC;
    return hip_result(launch_input_transform(t, x, V, g, dtype, stream));
}

extern "C" int nova_contract(const nova_transforms *t, const void *U, const void *V, void *M, size_t M_bytes,
                             int N, int C, int H, int W, int K, int dtype, int flags, void *stream)
{
    if (int rc = check_handle(t)) return rc;
    if (!U || !V || !M || !dims_ok(N, C, H, W, K) || !dtype_ok(dtype)) return NOVA_EINVAL;
    const Geometry g = make_geometry(N, C, H, W, K, t->m, t->r);
    if (M_bytes < m_bytes(g, dtype, flags)) return NOVA_ENOSPC;
    return hip_result(launch_contract(t, U, V, M, g, dtype, flags, stream));
}

extern "C" int nova_output_transform(const nova_transforms *t, const void *M, size_t M_bytes, void *y, int N,
                                     int K, int H, int W, int dtype, int flags, void *stream)
{
    if (int rc = check_handle(t)) return rc;
    if (!M || !y || !dims_ok(N, 1, H, W, K) || !dtype_ok(dtype)) return NOVA_EINVAL;
    if ((flags & NOVA_FLAG_POOL2) && (H % 2 != 0 || W % 2 != 0)) return NOVA_EINVAL;
    const Geometry g = make_geometry(N, 1, H, W, K, t->m, t->r);
    if (M_bytes < m_bytes(g, dtype, flags)) return NOVA_ENOSPC;
    return hip_result(launch_output_transform(t, M, y, g, dtype, flags, stream));
}

extern "C" int nova_contract_output_fused(const nova_transforms *t, const void *U, const void *V, void *y, int N, int C,
                                          int H, int W, int K, int dtype, int flags, void *stream)
{
    if (int rc = check_handle(t)) return rc;
    if (!U || !V || !y || !dims_ok(N, C, H, W, K) || !dtype_ok(dtype)) return NOVA_EINVAL;
    if ((flags & NOVA_FLAG_POOL2) && (H % 2 != 0 || W % 2 != 0)) return NOVA_EINVAL;
    const Geometry g = make_geometry(N, C, H, W, K, t->m, t->r);
    if (!fused_contract_output_applies(t, g, dtype, flags)) return NOVA_EUNSUPPORTED;
    return hip_result(launch_fused_contract_output(t, U, V, y, g, dtype, flags, stream));
}

extern "C" int nova_conv2d_path(const nova_transforms *t, int C, int H, int W, int K, int dtype, int flags)
{
    if (int rc = check_handle(t)) return rc;
    if (!dims_ok(1, C, H, W, K) || !dtype_ok(dtype)) return NOVA_EINVAL;
    if (few_channels(C)) return NOVA_PATH_FEW_CHANNELS;
    return fused_contract_output_preferred(t, make_geometry(1, C, H, W, K, t->m, t->r), dtype, flags) ? NOVA_PATH_FUSED_OUTPUT
                                                                                                      : NOVA_PATH_STAGES;
}

// The slab loop behind nova_winograd_conv2d and nova_winograd_conv2d_static.
int nova::conv2d_with_workspace(const nova_transforms *t, const void *x, const void *U, void *y, int N,
                                int C, int H, int W, int K, int dtype, int flags, void *workspace,
                                size_t workspace_bytes, void *stream)
{
    if (int rc = check_handle(t)) return rc;
    if (!x || !U || !y || !workspace || !dims_ok(N, C, H, W, K) || !dtype_ok(dtype)) return NOVA_EINVAL;
    if (((uintptr_t)workspace & 255) != 0) return NOVA_EINVAL;
    if ((flags & NOVA_FLAG_POOL2) && (H % 2 != 0 || W % 2 != 0)) return NOVA_EINVAL;
    const int m = t->m, r = t->r;

    // (64 input channels: contraction and output transform run as one kernel and keep no M, where that is faster)
    const bool fused = fused_contract_output_preferred(t, make_geometry(1, C, H, W, K, m, r), dtype, flags);
    // largest slab (whole images) whose V and M fit the workspace; slab_bytes grows with the count
    auto slab_bytes = [&](long long count, size_t *v_part) {
        const Geometry sg = make_geometry((int)count, C, H, W, K, m, r);
        const size_t vb = align256(first_part_bytes(sg, dtype));
        if (v_part) *v_part = vb;
        return vb + (fused ? 0 : align256(second_part_bytes(sg, dtype, flags)));
    };
    if (slab_bytes(1, nullptr) > workspace_bytes) return NOVA_ENOSPC;
    long long lo = 1, hi = N;                    // invariant: lo fits
    while (lo < hi) {
        const long long mid = (lo + hi + 1) / 2;
        if (slab_bytes(mid, nullptr) <= workspace_bytes) lo = mid; else hi = mid - 1;
    }
    // (as many slabs as that size needs, but of equal size: 20 + 12 images run slower than 16 + 16)
    const long long slab_count = (N + lo - 1) / lo;
    const long long imgs = (N + slab_count - 1) / slab_count;
    size_t v_part = 0;
    (void)slab_bytes(imgs, &v_part);

    const size_t es = dtype_size(dtype);
    char *Vbuf = (char *)workspace;
    char *Mbuf = Vbuf + v_part;
    const bool few = few_channels(C);
    if (few)
        if (int err = launch_pack_few_channels(U, Mbuf, make_geometry(1, C, H, W, K, m, r), dtype, stream)) return hip_result(err);
    for (int n0 = 0; n0 < N; n0 += (int)imgs) {
        const int nb = (N - n0 < imgs) ? N - n0 : (int)imgs;
        const Geometry g = make_geometry(nb, C, H, W, K, m, r);
        const char *xs = (const char *)x + (size_t)n0 * C * H * W * es;
        const size_t y_image = (flags & NOVA_FLAG_POOL2) ? (size_t)K * (H / 2) * (W / 2) : (size_t)K * H * W;
        char *ys = (char *)y + (size_t)n0 * y_image * es;
        if (few) {
            if (int err = launch_input_transform_few(t, xs, Vbuf, g, dtype, stream)) return hip_result(err);
            if (int err = launch_output_transform_few(t, Vbuf, Mbuf, ys, g, dtype, flags, stream)) return hip_result(err);
            continue;
        }
        if (int err = launch_input_transform(t, xs, Vbuf, g, dtype, stream)) return hip_result(err);
        if (fused) {
            if (int err = launch_fused_contract_output(t, U, Vbuf, ys, g, dtype, flags, stream)) return hip_result(err);
            continue;
        }
        if (int err = launch_contract(t, U, Vbuf, Mbuf, g, dtype, flags, stream)) return hip_result(err);
        if (int err = launch_output_transform(t, Mbuf, ys, g, dtype, flags, stream)) return hip_result(err);
    }
    return NOVA_OK;
}

extern "C" int nova_winograd_conv2d(const nova_transforms *t, const void *x, const void *U, void *y, int N,
                                    int C, int H, int W, int K, int dtype, int flags, void *workspace,
                                    size_t workspace_bytes, void *stream)
{
    return conv2d_with_workspace(t, x, U, y, N, C, H, W, K, dtype, flags, workspace, workspace_bytes, stream);
}

// ---- INT8 operands in the Winograd domain

static bool int8_mode_ok(int mode)
{
    return mode == NOVA_INT8_PER_TENSOR || mode == NOVA_INT8_PER_CHANNEL || mode == NOVA_INT8_PER_POSITION;
}

extern "C" size_t nova_filter_int8_bytes(int K, int C, int m, int r)
{
    return nova_filter_bytes(K, C, m, r, NOVA_F16) / 2;
}

extern "C" size_t nova_input_int8_bytes(int N, int C, int H, int W, int m, int r)
{
    return nova_input_bytes(N, C, H, W, m, r, NOVA_F16) / 2;
}

extern "C" int nova_quantize_filter_int8(const nova_transforms *t, const void *U, int K, int C, int dtype, int mode,
                                         void *Uq, float *u_scales, void *stream)
{
    if (int rc = check_handle(t)) return rc;
    if (!U || !Uq || !u_scales || K < 1 || C < 1 || !dtype_ok(dtype) || !int8_mode_ok(mode)) return NOVA_EINVAL;
    const Geometry g = make_geometry(1, C, 1, 1, K, t->m, t->r);
    const long long elements = (long long)g.n * g.n * g.c_blocks * g.Kp * kChanBlock;
    const int count = mode == NOVA_INT8_PER_CHANNEL ? K : mode == NOVA_INT8_PER_POSITION ? g.n * g.n : 1;
    return hip_result(launch_quantize_int8(U, Uq, u_scales, elements, g.n * g.n, g.Kp, count, mode, dtype, stream));
}

extern "C" int nova_quantize_input_int8(const nova_transforms *t, const void *V, int N, int C, int H, int W, int dtype,
                                        int mode, void *Vq, float *v_scale, void *stream)
{
    if (int rc = check_handle(t)) return rc;
    if (!V || !Vq || !v_scale || !dims_ok(N, C, H, W, 1) || !dtype_ok(dtype) || !int8_mode_ok(mode)) return NOVA_EINVAL;
    const Geometry g = make_geometry(N, C, H, W, 1, t->m, t->r);
    if (g.T > 0x7fffffffLL) return NOVA_EINVAL;
    const long long elements = (long long)g.n * g.n * g.c_blocks * g.T * kChanBlock;
    const bool pos = mode == NOVA_INT8_PER_POSITION;
    return hip_result(launch_quantize_int8(V, Vq, v_scale, elements, g.n * g.n, (int)g.T, pos ? g.n * g.n : 1, pos ? 2 : 0,
                                           dtype, stream));
}

extern "C" int nova_contract_int8(const nova_transforms *t, const void *Uq, const void *Vq, const float *u_scales,
                                  const float *v_scale, int mode, void *M, size_t M_bytes, int N, int C, int H, int W,
                                  int K, int dequantise, void *stream)
{
    if (int rc = check_handle(t)) return rc;
    if (!Uq || !Vq || !M || !dims_ok(N, C, H, W, K) || !int8_mode_ok(mode)) return NOVA_EINVAL;
    if (dequantise && (!u_scales || !v_scale)) return NOVA_EINVAL;
    const Geometry g = make_geometry(N, C, H, W, K, t->m, t->r);
    if (M_bytes < m_bytes(g, NOVA_F32, 0)) return NOVA_ENOSPC;
    return hip_result(launch_contract_int8(Uq, Vq, M, u_scales, v_scale, mode, dequantise ? 1 : 0, g, stream));
}

// workspace of nova_winograd_conv2d_int8: V (storage format) | Vq | its scale | M (binary32), each 256-byte aligned
static size_t int8_parts(const Geometry &g, int dtype, size_t off[4])
{
    off[0] = 0;
    off[1] = off[0] + align256(v_bytes(g, dtype));
    off[2] = off[1] + align256(v_bytes(g, NOVA_F16) / 2);
    off[3] = off[2] + align256((size_t)g.n * g.n * sizeof(float));
    return off[3] + align256(m_bytes(g, NOVA_F32, 0));
}

extern "C" size_t nova_conv2d_int8_workspace_bytes(int N, int C, int H, int W, int K, int m, int r, int dtype)
{
    if (!dims_ok(N, C, H, W, K) || !device_tile_ok(m, r) || !dtype_ok(dtype)) return 0;
    size_t off[4];
    return int8_parts(make_geometry(N, C, H, W, K, m, r), dtype, off);
}

extern "C" int nova_winograd_conv2d_int8(const nova_transforms *t, const void *x, const void *Uq, const float *u_scales,
                                         int mode, void *y, int N, int C, int H, int W, int K, int dtype, int flags,
                                         void *workspace, size_t workspace_bytes, void *stream)
{
    if (int rc = check_handle(t)) return rc;
    if (!x || !Uq || !u_scales || !y || !workspace || !dims_ok(N, C, H, W, K) || !dtype_ok(dtype) || !int8_mode_ok(mode))
        return NOVA_EINVAL;
    if (((uintptr_t)workspace & 255) != 0 || (flags & NOVA_FLAG_M_F16)) return NOVA_EINVAL;
    if ((flags & NOVA_FLAG_POOL2) && (H % 2 != 0 || W % 2 != 0)) return NOVA_EINVAL;
    const Geometry g = make_geometry(N, C, H, W, K, t->m, t->r);
    if (g.T > 0x7fffffffLL) return NOVA_EINVAL;
    size_t off[4];
    if (int8_parts(g, dtype, off) > workspace_bytes) return NOVA_ENOSPC;
    char *ws = (char *)workspace;
    void *V = ws + off[0], *Vq = ws + off[1], *Mf = ws + off[3];
    float *v_scale = (float *)(ws + off[2]);
    if (int err = launch_input_transform(t, x, V, g, dtype, stream)) return hip_result(err);
    const long long elements = (long long)g.n * g.n * g.c_blocks * g.T * kChanBlock;
    const bool pos = mode == NOVA_INT8_PER_POSITION;
    if (int err = launch_quantize_int8(V, Vq, v_scale, elements, g.n * g.n, (int)g.T, pos ? g.n * g.n : 1, pos ? 2 : 0, dtype,
                                       stream))
        return hip_result(err);
    if (int err = launch_contract_int8(Uq, Vq, Mf, u_scales, v_scale, mode, 1, g, stream)) return hip_result(err);
    // the de-quantised products are binary32 whatever the storage format: the output transform's binary32-M path
    if (int err = launch_output_transform(t, Mf, y, g, dtype, flags, stream)) return hip_result(err);
    return NOVA_OK;
}

extern "C" int nova_relu_maxpool2x2(const void *in, void *out, int N, int C, int H, int W, int dtype,
                                    void *stream)
{
    if (!in || !out || !dims_ok(N, C, H, W, 1) || !dtype_ok(dtype)) return NOVA_EINVAL;
    return hip_result(launch_relu_maxpool2x2(in, out, N, C, H, W, dtype, stream));
}

extern "C" const char *nova_strerror(int code)
{
    switch (code) {
    case NOVA_OK: return "ok";
    case NOVA_EINVAL: return "invalid argument";
    case NOVA_EDUP: return "duplicate interpolation point";
    case NOVA_EOVERFLOW: return "exact arithmetic overflowed 64-bit numerator/denominator";
    case NOVA_EVERIFY: return "generated transforms fail the exact tensor identity";
    case NOVA_ENOSPC: return "workspace too small";
    case NOVA_EUNSUPPORTED: return "unsupported tile size or kernel size for the device path";
    case NOVA_EHIP: return "HIP call failed (see nova_last_hip_error)";
    case NOVA_ENOMEM: return "out of host memory";
    default: return "unknown error";
    }
}

extern "C" int nova_last_hip_error(void) { return g_last_hip_error; }
extern "C" const char *nova_version(void) { return "libnova 0.5 (gfx950)"; }
