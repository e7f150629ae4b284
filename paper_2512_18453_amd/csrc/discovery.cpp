// Host side of libnova: the deterministic steps of point discovery -- exhaustive search over
// symmetric configurations {0, +-p1, +-p2, ..} (Sec. "Symmetric Search", Alg. "Symmetric Search")
// and snapping a real number to a simple fraction (Sec. "Snap-to-Rational", Alg. "Snap-to-Rational").
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
            i128 num = (i128)M * d - ((i128)a << s);
            if (num < 0) num = -num;
            // num / d < best_num / best_d  <=>  num * best_d < best_num * d
            if (!have || num * best_d < best_num * d) { have = true; best_num = num; best_a = a; best_d = d; }
        }
    const long long g = gcd_ll(best_a, best_d);
    *out = {best_a / (g ? g : 1), best_d / (g ? g : 1)};
    return NOVA_OK;
}
