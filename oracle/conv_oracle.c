/*
 * CPU oracle for r x r (r odd; 3 x 3 in the paper's experiments), stride-1, pad-(r-1)/2 convolution
 * and its Winograd F(m x m, r x r)
 * evaluation.  TEST INFRASTRUCTURE ONLY: plain, slow, written to be checked by eye.
 * It shares no code with the HIP library.
 *
 *   direct     the definition  y_i = sum_k g_k x_{i+k}  of Sec. 2.1 applied along both
 *              image axes and summed over input channels (no kernel flip, no bias).
 *   winograd   Y = A^T [ (G g G^T) * (B^T d B) ] A per n x n tile, n = m + r - 1
 *              (Sec. 2.1 steps 1-4 nested in 2D, App. "2D Extension via Kronecker
 *              Products"), channel sum taken in the transformed domain.
 *   emulated   the same with the intermediate tensors rounded to a storage format
 *              (binary16 or binary32) and the input transform carried out in binary32,
 *              which is the "fp16 storage, fp32 intermediates" set-up of
 *              Sec. "Float16 Precision Analysis" / Sec. 4.1.
 *
 * All tensors cross this interface as fp64 arrays (values that are already exactly
 * representable in the storage format when a storage format is emulated).
 * Layouts: x [N][C][H][W], g [K][C][r][r], y [N][K][H][W], matrices row-major with one
 * row per interpolation point (last row = the point at infinity).
 * Winograd-domain tensors: U [n*n][K][C], V [n*n][T][C], M [n*n][T][K] with
 * xi = i*n + j and t = (image*tiles_h + tile_row)*tiles_w + tile_col.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define MAXN 16 /* largest n = m + r - 1 handled */

int nova_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---------------------------------------------------------------- rounding helpers */

/* Nearest binary16 (ties to even, gradual underflow, overflow to infinity) of a double,
 * returned as a double.  Rounds once, directly from the fp64 value. */
static double round_to_f16(double v)
{
    if (isnan(v) || isinf(v) || v == 0.0) return v;
    double a = fabs(v);
    double q;                        /* spacing of binary16 numbers around a */
    if (a < ldexp(1.0, -14)) {
        q = ldexp(1.0, -24);         /* sub-normal range: fixed spacing */
    } else {
        int e;
        (void)frexp(a, &e);          /* a = f * 2^e, f in [0.5, 1)  =>  2^(e-1) <= a < 2^e */
        q = ldexp(1.0, (e - 1) - 10);
    }
    double r = nearbyint(a / q) * q; /* a/q is exact (power of two); nearbyint: ties to even */
    if (r > 65504.0) r = INFINITY;   /* 65520 and above round up to 2^16: not representable */
    return copysign(r, v);
}

static double round_to_f32(double v) { return (double)(float)v; }

static double round_storage(double v, int storage)
{
    return storage == 16 ? round_to_f16(v) : round_to_f32(v);
}

void nova_oracle_round_f16(const double *in, double *out, long count)
{
    for (long i = 0; i < count; ++i) out[i] = round_to_f16(in[i]);
}

/* ---------------------------------------------------------------- direct convolution */

int nova_oracle_direct_conv2d(const double *x, const double *g, double *y,
                              int N, int C, int H, int W, int K, int r)
{
    if (!x || !g || !y || N < 0 || C < 1 || H < 1 || W < 1 || K < 1 || r < 1 || r % 2 == 0) return -1;
    const int pad = (r - 1) / 2;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k) {
            double *yp = y + ((size_t)n * K + k) * H * W;
            for (size_t i = 0; i < (size_t)H * W; ++i) yp[i] = 0.0;
            for (int c = 0; c < C; ++c) {
                const double *xp = x + ((size_t)n * C + c) * H * W;
                const double *gp = g + ((size_t)k * C + c) * r * r;
                for (int a = 0; a < r; ++a)
                    for (int b = 0; b < r; ++b) {
                        double gv = gp[a * r + b];
                        for (int h = 0; h < H; ++h) {
                            int hh = h + a - pad;
                            if (hh < 0 || hh >= H) continue;
                            for (int w = 0; w < W; ++w) {
                                int ww = w + b - pad;
                                if (ww < 0 || ww >= W) continue;          /* zero border */
                                yp[(size_t)h * W + w] += gv * xp[(size_t)hh * W + ww];
                            }
                        }
                    }
            }
        }
    return 0;
}

/* ---------------------------------------------------------------- fp64 Winograd */

/* out (rows_l x cols_r) = L (rows_l x inner) * Mid (inner x inner2) * R^T, R (cols_r x inner2) */
static void sandwich_f64(const double *L, int rows_l, int inner,
                         const double *Mid, int inner2,
                         const double *R, int cols_r, double *out)
{
    double tmp[MAXN * MAXN];
    for (int i = 0; i < rows_l; ++i)
        for (int b = 0; b < inner2; ++b) {
            double s = 0.0;
            for (int a = 0; a < inner; ++a) s += L[i * inner + a] * Mid[a * inner2 + b];
            tmp[i * inner2 + b] = s;
        }
    for (int i = 0; i < rows_l; ++i)
        for (int j = 0; j < cols_r; ++j) {
            double s = 0.0;
            for (int b = 0; b < inner2; ++b) s += tmp[i * inner2 + b] * R[j * inner2 + b];
            out[i * cols_r + j] = s;
        }
}

static void load_tile(const double *plane, int H, int W, int h0, int w0, int n, int pad, double *d)
{
    for (int a = 0; a < n; ++a)
        for (int b = 0; b < n; ++b) {
            int hh = h0 - pad + a, ww = w0 - pad + b;   /* beyond the image reads as zero */
            d[a * n + b] = (hh >= 0 && hh < H && ww >= 0 && ww < W) ? plane[(size_t)hh * W + ww] : 0.0;
        }
}

int nova_oracle_winograd_conv2d_f64(const double *x, const double *g, double *y,
                                    int N, int C, int H, int W, int K, int m, int r,
                                    const double *A, const double *BT, const double *G)
{
    int n = m + r - 1, pad = (r - 1) / 2;
    if (!x || !g || !y || !A || !BT || !G || n > MAXN || m < 1 || r < 1 || r % 2 == 0) return -1;
    int th = (H + m - 1) / m, tw = (W + m - 1) / m;
    size_t nn = (size_t)n * n;
    double *U = malloc(sizeof(double) * nn * K * C);
    double *AT = malloc(sizeof(double) * m * n);
    if (!U || !AT) { free(U); free(AT); return -2; }
    for (int p = 0; p < n; ++p)
        for (int i = 0; i < m; ++i) AT[i * n + p] = A[p * m + i];
#pragma omp parallel for schedule(static)
    for (int kc = 0; kc < K * C; ++kc) {
        double u[MAXN * MAXN];
        sandwich_f64(G, n, r, g + (size_t)kc * r * r, r, G, n, u);    /* G g G^T */
        for (size_t xi = 0; xi < nn; ++xi) U[xi * K * C + kc] = u[xi];
    }
    int fail = 0;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int img = 0; img < N; ++img)
        for (int tr = 0; tr < th; ++tr) {
            double *V = malloc(sizeof(double) * nn * C);
            if (!V) { fail = 1; continue; }
            for (int tc = 0; tc < tw; ++tc) {
                double d[MAXN * MAXN], v[MAXN * MAXN], Mk[MAXN * MAXN], Y[MAXN * MAXN];
                for (int c = 0; c < C; ++c) {
                    load_tile(x + ((size_t)img * C + c) * H * W, H, W, tr * m, tc * m, n, pad, d);
                    sandwich_f64(BT, n, n, d, n, BT, n, v);           /* B^T d B */
                    for (size_t xi = 0; xi < nn; ++xi) V[xi * C + c] = v[xi];
                }
                for (int k = 0; k < K; ++k) {
                    for (size_t xi = 0; xi < nn; ++xi) {
                        const double *u = U + (xi * K + k) * C;
                        double s = 0.0;
                        for (int c = 0; c < C; ++c) s += u[c] * V[xi * C + c];
                        Mk[xi] = s;
                    }
                    sandwich_f64(AT, m, n, Mk, n, AT, m, Y);          /* A^T M A */
                    for (int p = 0; p < m; ++p)
                        for (int q = 0; q < m; ++q) {
                            int h = tr * m + p, w = tc * m + q;
                            if (h < H && w < W)
                                y[(((size_t)img * K + k) * H + h) * W + w] = Y[p * m + q];
                        }
                }
            }
            free(V);
        }
    free(U); free(AT);
    return fail ? -2 : 0;
}

/* ---------------------------------------------------------------- storage emulation */

/* One 1D input transform in binary32, the arithmetic contract of the fp16 / fp32 data
 * path:  out[p] = E_p + O_p,  where E_p (resp. O_p) is the fused-multiply-add chain
 * acc = fma(BT[p][a], v[a], acc), started from 0, over the even (resp. odd) indices a in
 * ascending order, skipping coefficients that are exactly zero, and the final sum is one
 * binary32 addition.  v has stride `vs`. */
static void input_transform_1d_f32(const float *BT, int n, const float *v, int vs, float *out, int os)
{
    for (int p = 0; p < n; ++p) {
        float even = 0.0f, odd = 0.0f;
        for (int a = 0; a < n; a += 2)
            if (BT[p * n + a] != 0.0f) even = fmaf(BT[p * n + a], v[a * vs], even);
        for (int a = 1; a < n; a += 2)
            if (BT[p * n + a] != 0.0f) odd = fmaf(BT[p * n + a], v[a * vs], odd);
        out[p * os] = even + odd;
    }
}

/*
 * storage   16 or 32: format of x, g (already exact in it), U, V and y.
 * m_storage 16 or 32: format M is rounded to after the fp64 channel sum.
 * v_exact   0: V = storage( B^T d B in binary32 with the chain order above, columns of d
 *              first, then rows )          -- the device contract
 *           1: V = storage( B^T d B in fp64 )  -- a single rounding, to measure the gap.
 * A32, BT32: matrices rounded once to binary32; G64: rounded once to binary64.
 * U_out, V_out, M_out: optional (may be NULL) copies of the Winograd-domain tensors.
 */
int nova_oracle_winograd_conv2d_emulated(const double *x, const double *g, double *y,
                                         int N, int C, int H, int W, int K, int m, int r,
                                         const float *A32, const float *BT32, const double *G64,
                                         int storage, int m_storage, int v_exact, int relu,
                                         double *U_out, double *V_out, double *M_out)
{
    int n = m + r - 1, pad = (r - 1) / 2;
    if (!x || !g || !y || !A32 || !BT32 || !G64 || n > MAXN || m < 1 || r < 1 || r % 2 == 0) return -1;
    if ((storage != 16 && storage != 32) || (m_storage != 16 && m_storage != 32)) return -1;
    int th = (H + m - 1) / m, tw = (W + m - 1) / m;
    size_t nn = (size_t)n * n, T = (size_t)N * th * tw;
    double *U = malloc(sizeof(double) * nn * K * C);
    double *AT = malloc(sizeof(double) * m * n);
    double *BT64 = malloc(sizeof(double) * nn);
    if (!U || !AT || !BT64) { free(U); free(AT); free(BT64); return -2; }
    for (int p = 0; p < n; ++p)
        for (int i = 0; i < m; ++i) AT[i * n + p] = (double)A32[p * m + i];
    for (size_t i = 0; i < nn; ++i) BT64[i] = (double)BT32[i];

    /* filter transform: fp64, one rounding to the storage format */
#pragma omp parallel for schedule(static)
    for (int kc = 0; kc < K * C; ++kc) {
        double u[MAXN * MAXN];
        sandwich_f64(G64, n, r, g + (size_t)kc * r * r, r, G64, n, u);
        for (size_t xi = 0; xi < nn; ++xi) U[xi * K * C + kc] = round_storage(u[xi], storage);
    }
    if (U_out) memcpy(U_out, U, sizeof(double) * nn * K * C);

    int fail = 0;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int img = 0; img < N; ++img)
        for (int tr = 0; tr < th; ++tr) {
            double *V = malloc(sizeof(double) * nn * C);
            if (!V) { fail = 1; continue; }
            for (int tc = 0; tc < tw; ++tc) {
                size_t t = ((size_t)img * th + tr) * tw + tc;
                double d[MAXN * MAXN], v[MAXN * MAXN], Mk[MAXN * MAXN], Y[MAXN * MAXN];
                for (int c = 0; c < C; ++c) {
                    load_tile(x + ((size_t)img * C + c) * H * W, H, W, tr * m, tc * m, n, pad, d);
                    if (v_exact) {
                        sandwich_f64(BT64, n, n, d, n, BT64, n, v);
                    } else {
                        float df[MAXN * MAXN], tf[MAXN * MAXN], vf[MAXN * MAXN];
                        for (size_t i = 0; i < nn; ++i) df[i] = (float)d[i];   /* exact */
                        for (int b = 0; b < n; ++b)     /* t[i][b] = sum_a BT[i][a] d[a][b] */
                            input_transform_1d_f32(BT32, n, df + b, n, tf + b, n);
                        for (int i = 0; i < n; ++i)     /* V[i][j] = sum_b t[i][b] BT[j][b] */
                            input_transform_1d_f32(BT32, n, tf + i * n, 1, vf + i * n, 1);
                        for (size_t i = 0; i < nn; ++i) v[i] = (double)vf[i];
                    }
                    for (size_t xi = 0; xi < nn; ++xi) {
                        V[xi * C + c] = round_storage(v[xi], storage);
                        if (V_out) V_out[(xi * T + t) * C + c] = V[xi * C + c];
                    }
                }
                for (int k = 0; k < K; ++k) {
                    for (size_t xi = 0; xi < nn; ++xi) {
                        const double *u = U + (xi * K + k) * C;
                        double s = 0.0;
                        for (int c = 0; c < C; ++c) s += u[c] * V[xi * C + c];
                        Mk[xi] = round_storage(s, m_storage);
                        if (M_out) M_out[(xi * T + t) * K + k] = Mk[xi];
                    }
                    sandwich_f64(AT, m, n, Mk, n, AT, m, Y);
                    for (int p = 0; p < m; ++p)
                        for (int q = 0; q < m; ++q) {
                            int h = tr * m + p, w = tc * m + q;
                            if (h < H && w < W) {
                                double out = Y[p * m + q];
                                if (relu && out < 0.0) out = 0.0;     /* NaN stays NaN */
                                y[(((size_t)img * K + k) * H + h) * W + w] = round_storage(out, storage);
                            }
                        }
                }
            }
            free(V);
        }
    free(U); free(AT); free(BT64);
    return fail ? -2 : 0;
}
