/* A walk through conv_oracle.c for a build with -fsanitize=address,undefined (test infrastructure, like the
 * file it includes): ragged shapes, both storage formats, every option, with the textbook F(2,3) matrices
 * and a plain F(4,3) set computed here.  The sanitizers report; this program checks return codes and that
 * the fp64 Winograd result equals the direct convolution to rounding. */
#include "conv_oracle.c"

#include <stdio.h>

static double frand(unsigned *state)
{
    *state = *state * 1664525u + 1013904223u;
    return ((double)(*state >> 8) / 16777216.0) * 2.0 - 1.0;
}

static int run(int N, int C, int H, int W, int K, int m, const double *A, const double *BT, const double *G)
{
    const int r = 3, n = m + r - 1;
    const int th = (H + m - 1) / m, tw = (W + m - 1) / m;
    const size_t nn = (size_t)n * n, T = (size_t)N * th * tw;
    unsigned state = 12345u + (unsigned)(H * 31 + W);
    double *x = malloc(sizeof(double) * N * C * H * W), *g = malloc(sizeof(double) * K * C * r * r);
    double *y0 = malloc(sizeof(double) * N * K * H * W), *y1 = malloc(sizeof(double) * N * K * H * W);
    double *U = malloc(sizeof(double) * nn * K * C), *V = malloc(sizeof(double) * nn * T * C), *M = malloc(sizeof(double) * nn * T * K);
    float *A32 = malloc(sizeof(float) * n * m), *BT32 = malloc(sizeof(float) * nn);
    int bad = 0;
    for (int i = 0; i < N * C * H * W; ++i) x[i] = frand(&state);
    for (int i = 0; i < K * C * r * r; ++i) g[i] = 0.3 * frand(&state);
    nova_oracle_round_f16(x, x, (long)N * C * H * W);
    nova_oracle_round_f16(g, g, (long)K * C * r * r);
    for (int i = 0; i < n * m; ++i) A32[i] = (float)A[i];
    for (size_t i = 0; i < nn; ++i) BT32[i] = (float)BT[i];
    bad |= nova_oracle_direct_conv2d(x, g, y0, N, C, H, W, K, r) != 0;
    bad |= nova_oracle_winograd_conv2d_f64(x, g, y1, N, C, H, W, K, m, r, A, BT, G) != 0;
    for (int i = 0; i < N * K * H * W; ++i) bad |= fabs(y0[i] - y1[i]) > 1e-9;
    for (int storage = 16; storage <= 32; storage += 16)
        for (int m_storage = 16; m_storage <= 32; m_storage += 16)
            for (int v_exact = 0; v_exact < 2; ++v_exact)
                for (int relu = 0; relu < 2; ++relu) {
                    bad |= nova_oracle_winograd_conv2d_emulated(x, g, y1, N, C, H, W, K, m, r, A32, BT32, G, storage, m_storage,
                                                                v_exact, relu, U, V, M) != 0;
                    bad |= nova_oracle_winograd_conv2d_emulated(x, g, y1, N, C, H, W, K, m, r, A32, BT32, G, storage, m_storage,
                                                                v_exact, relu, NULL, NULL, NULL) != 0;
                }
    bad |= nova_oracle_winograd_conv2d_emulated(x, g, y1, N, C, H, W, K, m, r, A32, BT32, G, 8, 32, 0, 0, NULL, NULL, NULL) != -1;
    free(x); free(g); free(y0); free(y1); free(U); free(V); free(M); free(A32); free(BT32);
    return bad;
}

int main(void)
{
    /* F(2,3), points 0, 1, -1 (and infinity) */
    const double A2[4 * 2] = {1, 0, 1, 1, 1, -1, 0, 1};
    const double BT2[4 * 4] = {-1, 0, 1, 0, 0, 1, 1, 0, 0, -1, 1, 0, 0, -1, 0, 1};       /* rows: prod_{j != p}(t - a_j), .. */
    const double G2[4 * 3] = {-1, 0, 0, 0.5, 0.5, 0.5, 0.5, -0.5, 0.5, 0, 0, 1};
    int bad = 0;
    /* the matrices above must satisfy the tensor identity, or the comparison in run() says so */
    bad |= run(2, 3, 5, 7, 2, 2, A2, BT2, G2);
    bad |= run(1, 1, 1, 1, 1, 2, A2, BT2, G2);
    bad |= run(3, 2, 8, 2, 3, 2, A2, BT2, G2);
    printf(bad ? "conv_oracle_selftest: FAILED\n" : "conv_oracle_selftest: ok (%d threads)\n", nova_oracle_threads());
    return bad;
}
