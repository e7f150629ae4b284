// A walk through the host-only part of the C ABI (construction, matrices, discovery), for a build of the
// host sources with -fsanitize=address,undefined: the sanitizers report, this program only checks return
// codes.  It links transforms.cpp and discovery.cpp and nothing that needs a GPU.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../include/nova.h"

static int failures = 0;
#define EXPECT(cond)                                                          \
    do {                                                                      \
        if (!(cond)) { std::printf("host_selftest: line %d: %s\n", __LINE__, #cond); ++failures; } \
    } while (0)

static std::vector<nova_rational> paired(const std::vector<nova_rational> &magnitudes, bool with_zero)
{
    std::vector<nova_rational> p;
    if (with_zero) p.push_back({0, 1});
    for (const nova_rational &a : magnitudes) {
        p.push_back(a);
        p.push_back({-a.num, a.den});
    }
    return p;
}

static void walk_handle(const std::vector<nova_rational> &pts, int m, int r, int rows, int mdt)
{
    nova_transforms *t = nullptr;
    const int rc = nova_make_transforms_ex(pts.data(), (int)pts.size(), m, r, rows, nullptr, nullptr, mdt, &t);
    EXPECT(rc == NOVA_OK && t != nullptr);
    if (rc != NOVA_OK) return;
    int mm = 0, rr = 0, n = 0, sym = -1;
    EXPECT(nova_transforms_shape(t, &mm, &rr, &n, &sym) == NOVA_OK && mm == m && rr == r && n == m + r - 1);
    const int cols[3] = {m, n, r};
    for (int which = 0; which < 3; ++which) {
        std::vector<nova_rational> q((size_t)n * cols[which]);
        std::vector<double> d((size_t)n * cols[which]);
        std::vector<float> f((size_t)n * cols[which]);
        EXPECT(nova_get_matrix(t, which, q.data()) == NOVA_OK);
        EXPECT(nova_get_matrix_f64(t, which, d.data()) == NOVA_OK);
        EXPECT(nova_get_matrix_f32(t, which, f.data()) == NOVA_OK);
        std::vector<int8_t> codes((size_t)n * cols[which]);
        double scale = 0.0;
        const int rc8 = nova_get_matrix_int8(t, which, codes.data(), &scale);
        EXPECT(mdt == NOVA_MATRIX_INT8 ? (rc8 == NOVA_OK && scale > 0.0) : rc8 == NOVA_EINVAL);
    }
    EXPECT(nova_get_matrix(t, 3, nullptr) == NOVA_EINVAL);
    std::vector<int> lb(n), lg(n);
    EXPECT(nova_get_row_scaling(t, lb.data(), lg.data()) == NOVA_OK);
    double kappa[4];
    EXPECT(nova_kappa(t, kappa) == NOVA_OK && kappa[0] >= 1.0);
    nova_free_transforms(t);
}

int main()
{
    const std::vector<nova_rational> nova4 = {{5, 6}, {7, 6}}, nova6 = {{3, 5}, {1, 1}, {7, 6}},
                                     nova8 = {{2, 5}, {5, 6}, {1, 1}, {7, 6}}, std8 = {{1, 1}, {2, 1}, {3, 1}, {4, 1}};
    for (int mdt : {NOVA_MATRIX_F32, NOVA_MATRIX_F16, NOVA_MATRIX_INT8})
        for (int rows : {NOVA_ROWS_PLAIN, NOVA_ROWS_BALANCED}) {
            walk_handle(paired({{1, 1}}, true), 2, 3, rows, mdt);
            walk_handle(paired(nova4, true), 4, 3, rows, mdt);
            walk_handle(paired(nova6, true), 6, 3, rows, mdt);
            walk_handle(paired(nova8, true), 8, 3, rows, mdt);
            walk_handle(paired(std8, true), 8, 3, rows, mdt);
            walk_handle(paired(nova6, false), 5, 3, rows, mdt);       // an even number of finite points: no zero
        }
    // F(2,5), F(4,5), F(6,5): n - 1 = 5, 7, 9 finite points
    walk_handle(paired(nova4, true), 2, 5, NOVA_ROWS_PLAIN, NOVA_MATRIX_F32);
    walk_handle(paired(nova6, true), 4, 5, NOVA_ROWS_PLAIN, NOVA_MATRIX_F32);
    walk_handle(paired(nova8, true), 6, 5, NOVA_ROWS_PLAIN, NOVA_MATRIX_F32);
    // another order, an asymmetric set, explicit exponents
    {
        const std::vector<nova_rational> odd = {{1, 2}, {0, 1}, {-1, 3}, {2, 1}, {-3, 2}};
        walk_handle(odd, 4, 3, NOVA_ROWS_PLAIN, NOVA_MATRIX_F32);
        nova_transforms *t = nullptr;
        const int lb[6] = {1, -2, 0, 3, -1, 0}, lg[6] = {0, 1, -1, 2, 0, -3};
        EXPECT(nova_make_transforms_ex(odd.data(), 5, 4, 3, NOVA_ROWS_GIVEN, lb, lg, NOVA_MATRIX_F32, &t) == NOVA_OK);
        nova_free_transforms(t);
    }
    // refusals
    {
        nova_transforms *t = nullptr;
        const std::vector<nova_rational> dup = {{0, 1}, {1, 2}, {2, 4}, {1, 1}, {-1, 1}};
        EXPECT(nova_make_transforms(dup.data(), 5, 4, 3, &t) == NOVA_EDUP && t == nullptr);
        const std::vector<nova_rational> zero_den = {{0, 1}, {1, 0}, {2, 1}, {1, 1}, {-1, 1}};
        EXPECT(nova_make_transforms(zero_den.data(), 5, 4, 3, &t) == NOVA_EINVAL);
        EXPECT(nova_make_transforms(dup.data(), 4, 4, 3, &t) == NOVA_EINVAL);
        EXPECT(nova_make_transforms(nullptr, 5, 4, 3, &t) == NOVA_EINVAL);
        const std::vector<nova_rational> huge = paired({{1000003, 1}, {999983, 7}, {99991, 3}, {7919, 9973}, {104729, 11}, {15485863, 13}, {32452843, 17}}, true);
        const int rc = nova_make_transforms(huge.data(), (int)huge.size(), 14, 3, &t);
        EXPECT(rc == NOVA_EOVERFLOW || rc == NOVA_OK);
        if (rc == NOVA_OK) nova_free_transforms(t);
        nova_free_transforms(nullptr);
    }
    // discovery
    for (int m : {2, 4, 6}) {
        std::vector<nova_rational> pts(m + 1);
        double kappa = 0.0;
        EXPECT(nova_symmetric_search(m, 3, m == 6 ? 4 : 6, pts.data(), &kappa) == NOVA_OK && kappa >= 1.0);
    }
    {
        nova_rational q;
        for (double x : {0.0, 0.8333, -1.1666, 4.99, -5.5, 1e-9, 0.05}) EXPECT(nova_snap_to_rational(x, 10, &q) == NOVA_OK && q.den >= 1);
        EXPECT(nova_snap_to_rational(NAN, 10, &q) == NOVA_EINVAL);
        EXPECT(nova_snap_to_rational(0.5, 0, &q) == NOVA_EINVAL);
    }
    for (int m : {4, 8}) {
        const int dim = m + 1, generations = 6, population = 12, restarts = 2;
        const size_t need = nova_es_normals_needed(m, 3, generations, population, restarts);
        EXPECT(need == (size_t)restarts * ((size_t)dim + (size_t)generations * population * dim));
        std::vector<double> normals(need);
        uint64_t state = 0x9E3779B97F4A7C15ull + (uint64_t)m;
        for (size_t i = 0; i < need; i += 2) {              // Box-Muller on a 64-bit LCG: any reals would do
            state = state * 6364136223846793005ull + 1442695040888963407ull;
            const double u1 = ((state >> 11) + 1.0) / 9007199254740993.0;
            state = state * 6364136223846793005ull + 1442695040888963407ull;
            const double u2 = (state >> 11) / 9007199254740992.0;
            const double rad = std::sqrt(-2.0 * std::log(u1));
            normals[i] = rad * std::cos(6.283185307179586 * u2);
            if (i + 1 < need) normals[i + 1] = rad * std::sin(6.283185307179586 * u2);
        }
        std::vector<double> best(dim);
        double fitness = 0.0, parts[3];
        EXPECT(nova_evolution_strategy(m, 3, generations, population, restarts, normals.data(), need, best.data(), &fitness) == NOVA_OK);
        EXPECT(nova_evolution_strategy(m, 3, generations, population, restarts, normals.data(), need - 1, best.data(), &fitness) == NOVA_EINVAL);
        EXPECT(nova_es_fitness(m, 3, best.data(), &fitness, parts) == NOVA_OK && std::isfinite(fitness));
        std::vector<nova_rational> snapped(dim);
        double kappa = 0.0;
        EXPECT(nova_snap_points(m, 3, best.data(), 10, snapped.data(), &kappa) == NOVA_OK);
        // two coordinates that snap to the same fraction: the neighbourhood search has to separate them
        std::vector<double> close(dim, 0.0);
        for (int i = 0; i < dim; ++i) close[i] = 0.1 * i - 0.2;
        close[1] = close[0] + 1e-4;
        EXPECT(nova_snap_points(m, 3, close.data(), 10, snapped.data(), &kappa) == NOVA_OK && kappa >= 1.0);
        std::vector<double> same(dim, 0.25);
        double f2 = 0.0;
        EXPECT(nova_es_fitness(m, 3, same.data(), &f2, nullptr) == NOVA_OK && std::isinf(f2));
    }
    if (failures == 0) std::printf("host_selftest: ok\n");
    return failures == 0 ? 0 : 1;
}
