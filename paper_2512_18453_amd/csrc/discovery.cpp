// Host side of libnova: point discovery -- exhaustive search over symmetric configurations
// {0, +-p1, +-p2, ..} (Sec. "Symmetric Search", Alg. "Symmetric Search"), the evolution strategy over
// R^(n-1) (Sec. "Evolution Strategy", Alg. "Evolution Strategy for Winograd Point Discovery"), snapping
// a real number to a simple fraction (Sec. "Snap-to-Rational", Alg. "Snap-to-Rational") and the search
// among neighbouring fractions when snapping makes two points coincide (Sec. "Neighborhood Search").
#include <algorithm>
#include <cmath>
#include <thread>
#include <vector>

#include "internal.hpp"

namespace {

struct Frac { long long a, b; };                         // a / b, reduced, b > 0

long long gcd_ll(long long x, long long y)
{
    while (y) { long long t = x % y; x = y; y = t; }
    return x < 0 ? -x : x;
}

// all distinct a/b with 1 <= b <= d_max, 1 <= a <= bound * b, ascending
std::vector<Frac> positive_rationals(int d_max, int bound)
{
    std::vector<Frac> v;
    for (int b = 1; b <= d_max; ++b)
        for (int a = 1; a <= bound * b; ++a)
            if (gcd_ll(a, b) == 1) v.push_back({a, b});
    std::sort(v.begin(), v.end(), [](const Frac &x, const Frac &y) { return x.a * y.b < y.a * x.b; });
    return v;
}

// kappa_2 of the Vandermonde matrix of the finite points 0 (optional), +p, -p for every chosen p
double kappa_of(const std::vector<double> &values, const int *combo, int n_pairs, bool with_zero,
                std::vector<double> &scratch)
{
    const int finite = 2 * n_pairs + (with_zero ? 1 : 0);
    scratch.assign((size_t)finite * finite, 0.0);
    int row = 0;
    auto fill = [&](double alpha) {
        double pw = 1.0;
        for (int j = 0; j < finite; ++j) { scratch[(size_t)row * finite + j] = pw; pw *= alpha; }
        ++row;
    };
    if (with_zero) fill(0.0);
    for (int q = 0; q < n_pairs; ++q) { fill(values[combo[q]]); fill(-values[combo[q]]); }
    return nova::spectral_condition(scratch, finite, finite);
}

struct Best {
    double kappa = INFINITY;
    std::vector<int> combo;
    // lower kappa wins; equal kappa: the combination that comes first in lexicographic order
    bool beaten_by(double k, const int *c, int len) const
    {
        if (k < kappa) return true;
        if (k > kappa || combo.empty()) return k < kappa;
        return std::lexicographical_compare(c, c + len, combo.begin(), combo.end());
    }
};

// next combination of `len` indices out of [0, count) in lexicographic order; false at the end
bool next_combo(int *c, int len, int count)
{
    int i = len - 1;
    while (i >= 0 && c[i] == count - len + i) --i;
    if (i < 0) return false;
    ++c[i];
    for (int j = i + 1; j < len; ++j) c[j] = c[j - 1] + 1;
    return true;
}

}  // namespace

extern "C" int nova_symmetric_search(int m, int r, int d_max, nova_rational *points_out, double *kappa_out)
{
    if (m < 1 || r < 1 || !points_out || !kappa_out) return NOVA_EINVAL;
    const int n = m + r - 1, finite = n - 1;
    if (n > nova::kMaxN || finite < 2 || d_max < 1 || d_max > 64) return NOVA_EINVAL;
    const bool with_zero = finite % 2 == 1;
    const int n_pairs = with_zero ? (finite - 1) / 2 : finite / 2;
    const int bound = 5;
    const std::vector<Frac> cands = positive_rationals(d_max, bound);
    const int count = (int)cands.size();
    if (count < n_pairs) return NOVA_EINVAL;
    // refuse enumerations that would not end in reasonable time (C(count, n_pairs) > 2e8)
    double combos = 1.0;
    for (int i = 0; i < n_pairs; ++i) combos = combos * (count - i) / (i + 1);
    if (combos > 2e8) return NOVA_EUNSUPPORTED;
    std::vector<double> values(count);
    for (int i = 0; i < count; ++i) values[i] = (double)cands[i].a / (double)cands[i].b;   // correctly rounded

    // the combinations are dealt out by their first index; every worker keeps its own best and the
    // total order (kappa, lexicographic rank) makes the result independent of the number of workers
    unsigned workers = std::thread::hardware_concurrency();
    if (workers < 1) workers = 1;
    if (workers > 16) workers = 16;
    std::vector<Best> bests(workers);
    auto work = [&](unsigned w) {
        std::vector<int> c(n_pairs);
        std::vector<double> scratch;
        Best &best = bests[w];
        for (int first = (int)w; first + n_pairs <= count; first += (int)workers) {
            for (int j = 0; j < n_pairs; ++j) c[j] = first + j;
            do {
                const double k = kappa_of(values, c.data(), n_pairs, with_zero, scratch);
                if (best.beaten_by(k, c.data(), n_pairs)) { best.kappa = k; best.combo = c; }
            // the tail starts at first + 1, first + 2, .. and only ever grows, so it stays above c[0]
            } while (n_pairs > 1 && next_combo(c.data() + 1, n_pairs - 1, count));
        }
    };
    std::vector<std::thread> pool;
    for (unsigned w = 1; w < workers; ++w) pool.emplace_back(work, w);
    work(0);
    for (std::thread &th : pool) th.join();
    Best best;
    for (const Best &b : bests)
        if (!b.combo.empty() && best.beaten_by(b.kappa, b.combo.data(), n_pairs)) best = b;
    if (best.combo.empty()) return NOVA_EINVAL;

    int idx = 0;
    if (with_zero) points_out[idx++] = {0, 1};
    for (int q = 0; q < n_pairs; ++q) {
        const Frac &f = cands[best.combo[q]];
        points_out[idx++] = {f.a, f.b};
        points_out[idx++] = {-f.a, f.b};
    }
    // symbolic verification of the winner: exact construction and identity check
    nova_transforms *t = nullptr;
    const int rc = nova_make_transforms(points_out, finite, m, r, &t);
    if (rc != NOVA_OK) return rc;
    nova_free_transforms(t);
    *kappa_out = best.kappa;
    return NOVA_OK;
}

extern "C" int nova_snap_to_rational(double x, int d_max, nova_rational *out)
{
    if (!out || d_max < 1 || d_max > 1000 || !std::isfinite(x)) return NOVA_EINVAL;
    const int bound = 5;
    const double mag = std::fabs(x);
    if (mag >= (double)bound + 1.0) { *out = {x < 0 ? -bound : bound, 1}; return NOVA_OK; }   // d = 1 already gives +-5
    if (mag < std::ldexp(1.0, -40)) { *out = {0, 1}; return NOVA_OK; }           // nearer to 0 than to any 1/d
    // x = M * 2^-s exactly, M a 53-bit integer, 0 <= s <= 93
    int e = 0;
    const double fr = std::frexp(x, &e);                         // x = fr * 2^e, 0.5 <= |fr| < 1
    const long long M = (long long)std::ldexp(fr, 53);           // exact
    const int s = 53 - e;                                        // x = M * 2^-s; e <= 3 and e >= -39, so 50 <= s <= 92
    typedef __int128 i128;
    bool have = false;
    i128 best_num = 0;                                           // |x - a/d| = best_num / (best_d * 2^s)
    long long best_a = 0, best_d = 1;
    for (long long d = 1; d <= d_max; ++d)
        for (long long a = -bound * d; a <= bound * d; ++a) {
            i128 num = (i128)M * d - (i128)a * ((i128)1 << s);      // (a product: shifting a negative value left is undefined before C++20)
            if (num < 0) num = -num;
            // num / d < best_num / best_d  <=>  num * best_d < best_num * d
            if (!have || num * best_d < best_num * d) { have = true; best_num = num; best_a = a; best_d = d; }
        }
    const long long g = gcd_ll(best_a, best_d);
    *out = {best_a / (g ? g : 1), best_d / (g ? g : 1)};
    return NOVA_OK;
}

// ---------------------------------------------------------------------------------------------
// Evolution strategy.  The random numbers are an input (independent standard normal draws, consumed
// in the order the algorithm needs them), so that a run is a function of its arguments.
namespace {

constexpr double kLambdaMagnitude = 1e-3, kLambdaCondition = 1e-4;      // Table "Fitness function weights"

// coefficients (ascending) of prod (t - p_j) over all j except `skip` (-1: none); also the product of
// (p_skip - p_j)
void monic_product(const double *p, int count, int skip, std::vector<double> &coef, double *lagrange_factor)
{
    coef.assign(1, 1.0);
    double f = 1.0;
    for (int j = 0; j < count; ++j) {
        if (j == skip) continue;
        std::vector<double> next(coef.size() + 1);
        for (size_t k = 0; k < next.size(); ++k)
            next[k] = (k > 0 ? coef[k - 1] : 0.0) - p[j] * (k < coef.size() ? coef[k] : 0.0);
        coef.swap(next);
        if (skip >= 0) f *= p[skip] - p[j];
    }
    if (lagrange_factor) *lagrange_factor = f;
}

// f(p) = || T - T_rec(p) ||_F + lambda_1 |p|^2 / (n - 1) + lambda_2 log10(kappa(V) + 1); parts: tensor error,
// magnitude term |p|^2 / (n - 1), kappa.  +inf if anything is not finite (coinciding points)
double es_fitness(const double *p, int m, int r, double parts[3])
{
    const int n = m + r - 1, dim = n - 1;
    std::vector<double> A((size_t)n * m, 0.0), BT((size_t)n * n, 0.0), G((size_t)n * r, 0.0), coef;
    for (int q = 0; q < dim; ++q) {
        double f = 1.0;
        monic_product(p, dim, q, coef, &f);
        for (int j = 0; j < dim; ++j) BT[(size_t)q * n + j] = coef[j];
        double pw = 1.0;
        for (int i = 0; i < (m > r ? m : r); ++i) {
            if (i < m) A[(size_t)q * m + i] = pw;
            if (i < r) G[(size_t)q * r + i] = f != 0.0 ? pw / f : INFINITY;
            pw *= p[q];
        }
    }
    A[(size_t)(n - 1) * m + m - 1] = 1.0;
    G[(size_t)(n - 1) * r + r - 1] = 1.0;
    monic_product(p, dim, -1, coef, nullptr);
    for (int j = 0; j < n; ++j) BT[(size_t)(n - 1) * n + j] = coef[j];
    double sq = 0.0;
    for (int i = 0; i < m; ++i)
        for (int j = 0; j < n; ++j)
            for (int k = 0; k < r; ++k) {
                double rec = 0.0;
                for (int q = 0; q < n; ++q) rec += A[(size_t)q * m + i] * BT[(size_t)q * n + j] * G[(size_t)q * r + k];
                const double d = rec - (j == i + k ? 1.0 : 0.0);
                sq += d * d;
            }
    const double err = std::sqrt(sq);
    double mag = 0.0;
    for (int q = 0; q < dim; ++q) mag += p[q] * p[q];
    mag /= dim;
    std::vector<double> vander((size_t)dim * dim);
    for (int q = 0; q < dim; ++q) {
        double pw = 1.0;
        for (int j = 0; j < dim; ++j) { vander[(size_t)q * dim + j] = pw; pw *= p[q]; }
    }
    const double kappa = nova::spectral_condition(vander, dim, dim);
    double f = err + kLambdaMagnitude * mag + kLambdaCondition * std::log10(kappa + 1.0);
    if (!std::isfinite(f)) f = INFINITY;
    if (parts) { parts[0] = err; parts[1] = mag; parts[2] = kappa; }
    return f;
}

}  // namespace

extern "C" int nova_es_fitness(int m, int r, const double *points, double *fitness_out, double parts_out[3])
{
    if (m < 1 || r < 1 || !points || !fitness_out) return NOVA_EINVAL;
    const int n = m + r - 1;
    if (n > nova::kMaxN || n < 3) return NOVA_EINVAL;
    *fitness_out = es_fitness(points, m, r, parts_out);
    return NOVA_OK;
}

extern "C" size_t nova_es_normals_needed(int m, int r, int generations, int population, int restarts)
{
    if (m < 1 || r < 1 || generations < 1 || population < 1 || restarts < 1) return 0;
    return (size_t)restarts * (size_t)(m + r - 2) * (1 + (size_t)generations * population);
}

extern "C" int nova_evolution_strategy(int m, int r, int generations, int population, int restarts,
                                       const double *normals, size_t n_normals, double *points_out, double *fitness_out)
{
    if (!normals || !points_out || !fitness_out) return NOVA_EINVAL;
    const size_t need = nova_es_normals_needed(m, r, generations, population, restarts);
    const int n = m + r - 1, dim = n - 1;
    if (need == 0 || n_normals < need || n > nova::kMaxN || n < 3) return NOVA_EINVAL;
    const int elite_count = population / 4 > 1 ? population / 4 : 1;          // top 25 %
    const double *z = normals;
    std::vector<double> mu(dim), cands((size_t)population * dim), fits(population), next_mu(dim);
    std::vector<int> order(population);
    double best_f = INFINITY;
    bool have = false;
    for (int restart = 0; restart < restarts; ++restart) {
        for (int d = 0; d < dim; ++d) mu[d] = std::sqrt(0.5) * *z++;          // mu ~ N(0, 0.5 I)
        double sigma = 0.5;
        for (int gen = 0; gen < generations; ++gen) {
            const double f_parent = es_fitness(mu.data(), m, r, nullptr);
            for (int i = 0; i < population; ++i)
                for (int d = 0; d < dim; ++d) cands[(size_t)i * dim + d] = mu[d] + sigma * *z++;
            for (int i = 0; i < population; ++i) fits[i] = es_fitness(&cands[(size_t)i * dim], m, r, nullptr);
            for (int i = 0; i < population; ++i) order[i] = i;
            std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return fits[a] < fits[b]; });
            for (int d = 0; d < dim; ++d) {
                double acc = 0.0;
                for (int e = 0; e < elite_count; ++e) acc += cands[(size_t)order[e] * dim + d];
                next_mu[d] = acc / elite_count;
            }
            mu = next_mu;
            int better = 0;
            for (int i = 0; i < population; ++i) better += fits[i] < f_parent ? 1 : 0;
            const double success = (double)better / population;
            sigma = success > 0.2 ? sigma * 1.1 : sigma * 0.9;                  // the 1/5 rule
            sigma = sigma > 2.0 ? 2.0 : (sigma < 0.01 ? 0.01 : sigma);
            if (fits[order[0]] < best_f) {
                best_f = fits[order[0]];
                for (int d = 0; d < dim; ++d) points_out[d] = cands[(size_t)order[0] * dim + d];
                have = true;
            }
        }
    }
    if (!have) return NOVA_EVERIFY;           // every candidate of every generation was degenerate
    *fitness_out = best_f;
    return NOVA_OK;
}

extern "C" int nova_snap_points(int m, int r, const double *x, int d_max, nova_rational *points_out, double *kappa_out)
{
    if (m < 1 || r < 1 || !x || !points_out || !kappa_out || d_max < 1 || d_max > 64) return NOVA_EINVAL;
    const int n = m + r - 1, dim = n - 1, bound = 5;
    if (n > nova::kMaxN || n < 3) return NOVA_EINVAL;
    for (int d = 0; d < dim; ++d) {
        if (!std::isfinite(x[d])) return NOVA_EINVAL;
        if (int rc = nova_snap_to_rational(x[d], d_max, &points_out[d])) return rc;
    }
    auto same = [](const nova_rational &a, const nova_rational &b) { return a.num == b.num && a.den == b.den; };   // both reduced
    bool distinct = true;
    for (int i = 0; i < dim && distinct; ++i)
        for (int j = 0; j < i; ++j)
            if (same(points_out[i], points_out[j])) { distinct = false; break; }
    auto kappa_of_points = [&](const nova_rational *pts) {
        std::vector<double> vander((size_t)dim * dim);
        for (int q = 0; q < dim; ++q) {
            const double v = (double)pts[q].num / (double)pts[q].den;
            double pw = 1.0;
            for (int j = 0; j < dim; ++j) { vander[(size_t)q * dim + j] = pw; pw *= v; }
        }
        return nova::spectral_condition(vander, dim, dim);
    };
    if (!distinct) {
        // neighbourhood search: per point the candidates within 6/5 of its snapped value, nearest to its
        // continuous value first, as many as keep the number of combinations within 1e5
        int per_point = (int)std::floor(std::pow(1e5, 1.0 / dim) + 1e-9);
        if (per_point < 1) per_point = 1;
        struct Cand { long long a, b; };
        std::vector<Cand> every;                                 // all distinct fractions, ascending
        for (long long b = 1; b <= d_max; ++b)
            for (long long a = -bound * b; a <= bound * b; ++a)
                if (gcd_ll(a < 0 ? -a : a, b) == 1) every.push_back({a, b});       // (zero only as 0/1)
        std::sort(every.begin(), every.end(), [](const Cand &u, const Cand &v) { return u.a * v.b < v.a * u.b; });
        typedef __int128 i128;
        std::vector<std::vector<Cand>> choices(dim);
        for (int d = 0; d < dim; ++d) {
            const nova_rational s = points_out[d];
            std::vector<Cand> near;
            for (const Cand &c : every) {
                // |c - s| <= 6/5  <=>  5 |c.a s.den - s.num c.b| <= 6 c.b s.den
                i128 diff = (i128)c.a * s.den - (i128)s.num * c.b;
                if (diff < 0) diff = -diff;
                if (5 * diff <= (i128)6 * c.b * s.den) near.push_back(c);
            }
            // distance to the continuous value, compared exactly: x = M 2^-sh
            int e = 0;
            const double fr = std::frexp(x[d], &e);
            long long M = (long long)std::ldexp(fr, 53);
            int sh = 53 - e;
            if (x[d] == 0.0) { M = 0; sh = 0; }
            if (sh < 0 || sh > 100) return NOVA_EUNSUPPORTED;    // |x| beyond 2^53 or below 2^-47: not a point anyone means
            auto dist_less = [&](const Cand &u, const Cand &v) {
                // |M 2^-sh - u.a/u.b| < |.. v ..|  <=>  |M u.b - u.a 2^sh| v.b < |M v.b - v.a 2^sh| u.b
                const i128 unit = (i128)1 << sh;
                i128 du = (i128)M * u.b - (i128)u.a * unit, dv = (i128)M * v.b - (i128)v.a * unit;
                if (du < 0) du = -du;
                if (dv < 0) dv = -dv;
                const i128 l = du * v.b, rr = dv * u.b;
                if (l != rr) return l < rr;
                return u.a * v.b < v.a * u.b;                    // equally near: the smaller fraction first
            };
            std::sort(near.begin(), near.end(), dist_less);
            if ((int)near.size() > per_point) near.resize(per_point);
            if (near.empty()) return NOVA_EVERIFY;
            choices[d] = near;
        }
        std::vector<int> idx(dim, 0);
        std::vector<nova_rational> trial(dim), best(dim);
        double best_kappa = INFINITY;
        bool found = false;
        for (;;) {
            for (int d = 0; d < dim; ++d) trial[d] = {choices[d][idx[d]].a, choices[d][idx[d]].b};
            bool ok = true;
            for (int i = 0; i < dim && ok; ++i)
                for (int j = 0; j < i; ++j)
                    if (same(trial[i], trial[j])) { ok = false; break; }
            if (ok) {
                const double k = kappa_of_points(trial.data());
                // (permutations of one set differ in the last bits only: the first one enumerated stays)
                if (k < best_kappa * (1.0 - 1e-9)) { best_kappa = k; best = trial; found = true; }
            }
            int d = dim - 1;                                     // the last point varies fastest
            while (d >= 0 && ++idx[d] == (int)choices[d].size()) { idx[d] = 0; --d; }
            if (d < 0) break;
        }
        if (!found) return NOVA_EVERIFY;
        for (int d = 0; d < dim; ++d) points_out[d] = best[d];
    }
    nova_transforms *t = nullptr;                                // exact construction and identity check
    const int rc = nova_make_transforms(points_out, dim, m, r, &t);
    if (rc != NOVA_OK) return rc;
    nova_free_transforms(t);
    *kappa_out = kappa_of_points(points_out);
    return NOVA_OK;
}
