// Host side of libnova: exact Cook-Toom construction of A, B^T, G from interpolation points
// (Alg. "Symbolic Cook-Toom Construction"), exact verification of the bilinear identity
// (Sec. 2.4), rounded tables, and spectral condition numbers (Sec. 2.2).
#include <algorithm>
#include <cmath>
#include <new>

#include "internal.hpp"

using nova::Rat;
using nova::RatCtx;

namespace {

// prod_j (t - roots[j]) as ascending coefficients, skipping index `skip` (-1: none)
std::vector<Rat> expand_roots(RatCtx &cx, const std::vector<Rat> &roots, int skip)
{
    std::vector<Rat> poly(1);
    poly[0] = cx.make(1, 1);
    for (int j = 0; j < (int)roots.size(); ++j) {
        if (j == skip) continue;
        std::vector<Rat> next(poly.size() + 1);
        for (size_t d = 0; d < poly.size(); ++d) {
            next[d + 1] = cx.add(next[d + 1], poly[d]);
            next[d] = cx.sub(next[d], cx.mul(roots[j], poly[d]));
        }
        poly.swap(next);
    }
    return poly;
}

Rat power(RatCtx &cx, const Rat &base, int e)
{
    Rat r = cx.make(1, 1);
    for (int i = 0; i < e; ++i) r = cx.mul(r, base);
    return r;
}

// sum_p A[p][i] BT[p][j] G[p][k] == [j == i + k] for all i, j, k, exactly
bool identity_holds(RatCtx &cx, const nova_transforms &t)
{
    for (int i = 0; i < t.m; ++i)
        for (int j = 0; j < t.n; ++j)
            for (int k = 0; k < t.r; ++k) {
                Rat sum = cx.make(0, 1);
                for (int p = 0; p < t.n; ++p)
                    sum = cx.add(sum, cx.mul(cx.mul(t.A[p * t.m + i], t.BT[p * t.n + j]), t.G[p * t.r + k]));
                Rat want = cx.make(j == i + k ? 1 : 0, 1);
                if (!cx.ok || !RatCtx::eq(sum, want)) return false;
            }
    return true;
}

// Singular values by one-sided Jacobi rotations on the columns (rows >= cols), descending.
std::vector<double> singular_values(std::vector<double> a, int rows, int cols)
{
    for (int sweep = 0; sweep < 60; ++sweep) {
        double off = 0.0;
        for (int p = 0; p < cols - 1; ++p)
            for (int q = p + 1; q < cols; ++q) {
                double app = 0, aqq = 0, apq = 0;
                for (int i = 0; i < rows; ++i) {
                    app += a[i * cols + p] * a[i * cols + p];
                    aqq += a[i * cols + q] * a[i * cols + q];
                    apq += a[i * cols + p] * a[i * cols + q];
                }
                if (apq == 0.0) continue;
                off = std::max(off, std::fabs(apq) / std::sqrt(app * aqq));
                double zeta = (aqq - app) / (2.0 * apq);
                double tn = (zeta >= 0 ? 1.0 : -1.0) / (std::fabs(zeta) + std::sqrt(1.0 + zeta * zeta));
                double cs = 1.0 / std::sqrt(1.0 + tn * tn), sn = cs * tn;
                for (int i = 0; i < rows; ++i) {
                    double vp = a[i * cols + p], vq = a[i * cols + q];
                    a[i * cols + p] = cs * vp - sn * vq;
                    a[i * cols + q] = sn * vp + cs * vq;
                }
            }
        if (off < 1e-15) break;
    }
    std::vector<double> sv(cols);
    for (int j = 0; j < cols; ++j) {
        double s = 0;
        for (int i = 0; i < rows; ++i) s += a[i * cols + j] * a[i * cols + j];
        sv[j] = std::sqrt(s);
    }
    std::sort(sv.begin(), sv.end(), [](double x, double y) { return x > y; });
    return sv;
}

double kappa2(const std::vector<double> &mat, int rows, int cols)
{
    std::vector<double> a = mat;
    if (rows < cols) {   // transpose so that rows >= cols
        std::vector<double> tr((size_t)rows * cols);
        for (int i = 0; i < rows; ++i)
            for (int j = 0; j < cols; ++j) tr[(size_t)j * rows + i] = mat[(size_t)i * cols + j];
        a.swap(tr);
        std::swap(rows, cols);
    }
    std::vector<double> sv = singular_values(a, rows, cols);
    return sv.front() / sv.back();
}

const std::vector<Rat> *pick(const nova_transforms *t, int which, int *rows, int *cols)
{
    switch (which) {
    case NOVA_MATRIX_A: *rows = t->n; *cols = t->m; return &t->A;
    case NOVA_MATRIX_BT: *rows = t->n; *cols = t->n; return &t->BT;
    case NOVA_MATRIX_G: *rows = t->n; *cols = t->r; return &t->G;
    default: return nullptr;
    }
}

}  // namespace

namespace {

// the integer e with 1 <= 2^e * sum|row| < 2, by exact comparisons
int balancing_exponent(RatCtx &cx, const Rat *row, int len)
{
    Rat norm = cx.make(0, 1);
    for (int j = 0; j < len; ++j) {
        Rat mag = row[j];
        if (mag.num < 0) mag.num = -mag.num;
        norm = cx.add(norm, mag);
    }
    if (!cx.ok || norm.num == 0) { cx.ok = false; return 0; }
    // norm = num / den;  2^e * num >= den  and  2^e * num < 2 * den
    int e = 0;
    auto scaled_ge = [&](int ee, int factor) {           // 2^ee * num >= factor * den ?
        nova::i128 lhs = norm.num, rhs = norm.den * factor;
        if (ee >= 0) lhs = cx.mul(lhs, (nova::i128)1 << ee); else rhs = cx.mul(rhs, (nova::i128)1 << -ee);
        return lhs >= rhs;
    };
    while (cx.ok && e > -120 && scaled_ge(e, 2)) --e;
    while (cx.ok && e < 120 && !scaled_ge(e, 1)) ++e;
    return e;
}

Rat times_pow2(RatCtx &cx, const Rat &v, int e)
{
    return e >= 0 ? cx.mul(v, cx.make((nova::i128)1 << e, 1)) : cx.mul(v, cx.make(1, (nova::i128)1 << -e));
}

}  // namespace

namespace nova {
double spectral_condition(const std::vector<double> &mat, int rows, int cols) { return kappa2(mat, rows, cols); }
}

extern "C" int nova_make_transforms(const nova_rational *finite_points, int n_points, int m, int r,
                                    nova_transforms **out)
{
    return nova_make_transforms_ex(finite_points, n_points, m, r, NOVA_ROWS_PLAIN, nullptr, nullptr,
                                   NOVA_MATRIX_F32, out);
}

extern "C" int nova_make_transforms_ex(const nova_rational *finite_points, int n_points, int m, int r,
                                       int row_scaling, const int *log2_b, const int *log2_g,
                                       int matrix_dtype, nova_transforms **out)
{
    if (!out) return NOVA_EINVAL;
    *out = nullptr;
    if (!finite_points || m < 1 || r < 1) return NOVA_EINVAL;
    const int n = m + r - 1;
    if (n > nova::kMaxN || n_points != n - 1) return NOVA_EINVAL;
    if (row_scaling != NOVA_ROWS_PLAIN && row_scaling != NOVA_ROWS_BALANCED && row_scaling != NOVA_ROWS_GIVEN)
        return NOVA_EINVAL;
    if (matrix_dtype != NOVA_MATRIX_F32 && matrix_dtype != NOVA_MATRIX_F16 && matrix_dtype != NOVA_MATRIX_INT8)
        return NOVA_EINVAL;
    if (row_scaling == NOVA_ROWS_GIVEN) {
        if (!log2_b || !log2_g) return NOVA_EINVAL;
        for (int p = 0; p < n; ++p)
            if (log2_b[p] < -60 || log2_b[p] > 60 || log2_g[p] < -60 || log2_g[p] > 60) return NOVA_EINVAL;
    }

    RatCtx cx;
    nova_transforms *t = new (std::nothrow) nova_transforms;
    if (!t) return NOVA_ENOMEM;
    t->m = m; t->r = r; t->n = n;
    for (int p = 0; p < n - 1; ++p) {
        if (finite_points[p].den == 0 || finite_points[p].num == INT64_MIN || finite_points[p].den == INT64_MIN) {
            delete t;
            return NOVA_EINVAL;
        }
        t->points.push_back(cx.make(finite_points[p].num, finite_points[p].den));
    }
    for (int p = 0; p < n - 1; ++p)
        for (int q = p + 1; q < n - 1; ++q)
            if (RatCtx::eq(t->points[p], t->points[q])) { delete t; return NOVA_EDUP; }

    t->A.assign((size_t)n * m, cx.make(0, 1));
    t->G.assign((size_t)n * r, cx.make(0, 1));
    t->BT.assign((size_t)n * n, cx.make(0, 1));
    for (int p = 0; p < n - 1; ++p) {
        const Rat &alpha = t->points[p];
        Rat F = cx.make(1, 1);                       // Lagrange factor prod_{j != p} (alpha_p - alpha_j)
        for (int j = 0; j < n - 1; ++j)
            if (j != p) F = cx.mul(F, cx.sub(alpha, t->points[j]));
        Rat Finv = cx.inv(F);
        for (int i = 0; i < m; ++i) t->A[(size_t)p * m + i] = power(cx, alpha, i);
        for (int k = 0; k < r; ++k) t->G[(size_t)p * r + k] = cx.mul(power(cx, alpha, k), Finv);
        std::vector<Rat> Np = expand_roots(cx, t->points, p);   // degree n-2: n-1 coefficients
        for (int j = 0; j < n - 1; ++j) t->BT[(size_t)p * n + j] = Np[j];
    }
    t->A[(size_t)(n - 1) * m + (m - 1)] = cx.make(1, 1);
    t->G[(size_t)(n - 1) * r + (r - 1)] = cx.make(1, 1);
    std::vector<Rat> Mt = expand_roots(cx, t->points, -1);       // degree n-1: n coefficients
    for (int j = 0; j < n; ++j) t->BT[(size_t)(n - 1) * n + j] = Mt[j];

    if (!cx.ok) { delete t; return NOVA_EOVERFLOW; }
    for (const std::vector<Rat> *mat : {&t->A, &t->BT, &t->G})
        for (const Rat &e : *mat)
            if (!RatCtx::fits64(e)) { delete t; return NOVA_EOVERFLOW; }
    if (!identity_holds(cx, *t)) {
        int rc = cx.ok ? NOVA_EVERIFY : NOVA_EOVERFLOW;
        delete t;
        return rc;
    }

    // ---- optional power-of-two row scaling, exact, verified again
    t->log2_b.assign(n, 0);
    t->log2_g.assign(n, 0);
    if (row_scaling != NOVA_ROWS_PLAIN) {
        for (int p = 0; p < n; ++p) {
            t->log2_b[p] = row_scaling == NOVA_ROWS_GIVEN ? log2_b[p] : balancing_exponent(cx, &t->BT[(size_t)p * n], n);
            t->log2_g[p] = row_scaling == NOVA_ROWS_GIVEN ? log2_g[p] : balancing_exponent(cx, &t->G[(size_t)p * r], r);
        }
        if (!cx.ok) { delete t; return NOVA_EOVERFLOW; }
        for (int p = 0; p < n; ++p) {
            for (int j = 0; j < n; ++j) t->BT[(size_t)p * n + j] = times_pow2(cx, t->BT[(size_t)p * n + j], t->log2_b[p]);
            for (int k = 0; k < r; ++k) t->G[(size_t)p * r + k] = times_pow2(cx, t->G[(size_t)p * r + k], t->log2_g[p]);
            for (int i = 0; i < m; ++i) t->A[(size_t)p * m + i] = times_pow2(cx, t->A[(size_t)p * m + i], -(t->log2_b[p] + t->log2_g[p]));
        }
        if (!cx.ok) { delete t; return NOVA_EOVERFLOW; }
        for (const std::vector<Rat> *mat : {&t->A, &t->BT, &t->G})
            for (const Rat &e : *mat)
                if (!RatCtx::fits64(e)) { delete t; return NOVA_EOVERFLOW; }
        if (!identity_holds(cx, *t)) {
            int rc = cx.ok ? NOVA_EVERIFY : NOVA_EOVERFLOW;
            delete t;
            return rc;
        }
    }

    // canonical symmetric order: 0, +a1, -a1, +a2, -a2, ...
    bool sym = (n - 1) % 2 == 1 && RatCtx::is_zero(t->points[0]);
    for (int j = 1; sym && j + 1 < n - 1; j += 2)
        sym = RatCtx::eq(t->points[j], cx.neg(t->points[j + 1]));
    // the device kernels rely on what symmetry implies for the matrices; confirm it exactly
    for (int j = 1; sym && j + 1 < n - 1; j += 2)
        for (int a = 0; a < n; ++a) {
            const Rat &plus = t->BT[(size_t)j * n + a], &minus = t->BT[(size_t)(j + 1) * n + a];
            sym = sym && RatCtx::eq(minus, (a % 2 == 0) ? plus : cx.neg(plus));
            if (a == 0 || a == n - 1) sym = sym && RatCtx::is_zero(plus);
            if (a < m) {
                const Rat &ap = t->A[(size_t)j * m + a], &am = t->A[(size_t)(j + 1) * m + a];
                sym = sym && RatCtx::eq(am, (a % 2 == 0) ? ap : cx.neg(ap));
            }
        }
    for (int a = 0; sym && a < n; ++a) {
        if (a % 2 == 1) sym = RatCtx::is_zero(t->BT[a]);                           // row of 0: even polynomial
        else sym = RatCtx::is_zero(t->BT[(size_t)(n - 1) * n + a]);                 // row of infinity: odd
        if (a >= 1 && a < m) sym = sym && RatCtx::is_zero(t->A[a]);                // A row of 0 = e_0
    }
    t->symmetric = sym;

    t->matrix_dtype = matrix_dtype;
    auto fill = [&](const std::vector<Rat> &exact, std::vector<double> &t64, std::vector<float> &t32) {
        for (const Rat &e : exact) {
            if (matrix_dtype == NOVA_MATRIX_F16) {
                const double v = nova::rat_to_f16_value(e);      // exact in binary32 and binary64
                t64.push_back(v);
                t32.push_back((float)v);
            } else {
                t64.push_back(nova::rat_to_f64(e));
                t32.push_back(nova::rat_to_f32(e));
            }
        }
    };
    if (matrix_dtype == NOVA_MATRIX_INT8) {
        // per tensor: s = max|entry| / 127, code = round-half-even(entry / s), value = code * s, all exact
        auto quantise = [&](const std::vector<Rat> &exact, std::vector<int8_t> &codes, double &scale,
                            std::vector<double> &t64, std::vector<float> &t32) {
            Rat top = cx.make(0, 1);
            for (const Rat &e : exact) {
                Rat mag = e;
                if (mag.num < 0) mag.num = -mag.num;
                if (mag.num * top.den > top.num * mag.den) top = mag;       // entries fit 64 bits: no overflow
            }
            const Rat s = cx.mul(top, cx.make(1, 127));
            scale = nova::rat_to_f64(s);
            for (const Rat &e : exact) {
                const Rat scaled = cx.mul(e, cx.inv(s));                    // in [-127, 127]
                nova::i128 lo = scaled.num / scaled.den;                    // truncates toward zero
                if (scaled.num < 0 && lo * scaled.den != scaled.num) --lo;  // floor
                const nova::i128 rem2 = 2 * (scaled.num - lo * scaled.den); // 2 * fractional part * den
                if (rem2 > scaled.den || (rem2 == scaled.den && (lo % 2 != 0))) ++lo;
                if (lo > 127) lo = 127;
                if (lo < -128) lo = -128;
                codes.push_back((int8_t)lo);
                const Rat value = cx.mul(cx.make(lo, 1), s);
                if (!cx.ok || !RatCtx::fits64(value)) { cx.ok = false; return; }
                t64.push_back(nova::rat_to_f64(value));
                t32.push_back(nova::rat_to_f32(value));
            }
        };
        quantise(t->A, t->Aq, t->scale_q[0], t->A64, t->A32);
        quantise(t->BT, t->BTq, t->scale_q[1], t->BT64, t->BT32);
        quantise(t->G, t->Gq, t->scale_q[2], t->G64, t->G32);
        if (!cx.ok) { delete t; return NOVA_EOVERFLOW; }
    } else {
        fill(t->A, t->A64, t->A32);
        fill(t->BT, t->BT64, t->BT32);
        fill(t->G, t->G64, t->G32);
    }
    if (matrix_dtype == NOVA_MATRIX_F16) {
        // rounding may break what the paired kernels assume of the zero entries only if a non-zero
        // entry rounds to zero or infinity; +a / -a rows round alike, so the pairing itself survives
        for (const std::vector<double> *tab : {&t->A64, &t->BT64, &t->G64})
            for (double v : *tab)
                if (std::isinf(v)) { delete t; return NOVA_EOVERFLOW; }
    }
    *out = t;
    return NOVA_OK;
}

extern "C" int nova_get_row_scaling(const nova_transforms *t, int *log2_b, int *log2_g)
{
    if (!t) return NOVA_EINVAL;
    for (int p = 0; p < t->n; ++p) {
        if (log2_b) log2_b[p] = t->log2_b[p];
        if (log2_g) log2_g[p] = t->log2_g[p];
    }
    return NOVA_OK;
}

extern "C" int nova_get_matrix_int8(const nova_transforms *t, int which, int8_t *codes, double *scale)
{
    if (!t || t->matrix_dtype != NOVA_MATRIX_INT8 || !codes || !scale) return NOVA_EINVAL;
    const std::vector<int8_t> *src = which == NOVA_MATRIX_A ? &t->Aq : which == NOVA_MATRIX_BT ? &t->BTq
                                   : which == NOVA_MATRIX_G ? &t->Gq : nullptr;
    if (!src) return NOVA_EINVAL;
    std::copy(src->begin(), src->end(), codes);
    *scale = t->scale_q[which];
    return NOVA_OK;
}

extern "C" void nova_free_transforms(nova_transforms *t) { delete t; }

extern "C" int nova_transforms_shape(const nova_transforms *t, int *m, int *r, int *n, int *symmetric)
{
    if (!t) return NOVA_EINVAL;
    if (m) *m = t->m;
    if (r) *r = t->r;
    if (n) *n = t->n;
    if (symmetric) *symmetric = t->symmetric ? 1 : 0;
    return NOVA_OK;
}

extern "C" int nova_get_matrix(const nova_transforms *t, int which, nova_rational *out)
{
    int rows, cols;
    if (!t || !out) return NOVA_EINVAL;
    const std::vector<Rat> *mat = pick(t, which, &rows, &cols);
    if (!mat) return NOVA_EINVAL;
    for (size_t i = 0; i < mat->size(); ++i) {
        out[i].num = (int64_t)(*mat)[i].num;   // fits: checked at construction
        out[i].den = (int64_t)(*mat)[i].den;
    }
    return NOVA_OK;
}

extern "C" int nova_get_matrix_f64(const nova_transforms *t, int which, double *out)
{
    if (!t || !out) return NOVA_EINVAL;
    const std::vector<double> *src = which == NOVA_MATRIX_A ? &t->A64 : which == NOVA_MATRIX_BT ? &t->BT64
                                   : which == NOVA_MATRIX_G ? &t->G64 : nullptr;
    if (!src) return NOVA_EINVAL;
    std::copy(src->begin(), src->end(), out);
    return NOVA_OK;
}

extern "C" int nova_get_matrix_f32(const nova_transforms *t, int which, float *out)
{
    if (!t || !out) return NOVA_EINVAL;
    const std::vector<float> *src = which == NOVA_MATRIX_A ? &t->A32 : which == NOVA_MATRIX_BT ? &t->BT32
                                  : which == NOVA_MATRIX_G ? &t->G32 : nullptr;
    if (!src) return NOVA_EINVAL;
    std::copy(src->begin(), src->end(), out);
    return NOVA_OK;
}

extern "C" int nova_kappa(const nova_transforms *t, double out[4])
{
    if (!t || !out) return NOVA_EINVAL;
    const int nf = t->n - 1;
    std::vector<double> V((size_t)nf * nf);
    for (int p = 0; p < nf; ++p) {
        double alpha = nova::rat_to_f64(t->points[p]), pw = 1.0;
        // powers from the exact point: alpha^j rounded once would need the rational power; the
        // product of correctly rounded factors is accurate to a few ulp, ample for kappa
        for (int j = 0; j < nf; ++j) { V[(size_t)p * nf + j] = pw; pw *= alpha; }
    }
    out[0] = nf > 0 ? kappa2(V, nf, nf) : 1.0;
    out[1] = kappa2(t->A64, t->n, t->m);
    out[2] = kappa2(t->BT64, t->n, t->n);
    out[3] = kappa2(t->G64, t->n, t->r);
    return NOVA_OK;
}
