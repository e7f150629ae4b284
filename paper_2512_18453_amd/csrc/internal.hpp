// Shared between the host-side pieces of libnova: the transform handle, the coefficient
// packs handed to kernels by value, tensor geometry, and the launcher prototypes.
#pragma once
#include <cstddef>
#include <cstdint>
#include <vector>

#include "../../include/nova.h"
#include "rational.hpp"

namespace nova {

constexpr int kChanBlock = 32;   // channel blocking of U, V, M
constexpr int kMaxN = 16;        // largest n = m + r - 1 nova_make_transforms accepts

// Coefficients of one 1D input transform, n = N.
//   generic: the whole B^T, row-major.
//   symmetric (points 0, +a1, -a1, ...; H = (N-2)/2 pairs):
//     zero[H+1]  row of the point 0: coefficients at the even positions 0, 2, .., 2H
//     ev[j][H]   row of +a_j: coefficients at the even positions 2, 4, .., 2H
//     od[j][H]   row of +a_j: coefficients at the odd positions 1, 3, .., 2H-1
//     inf[H+1]   row of infinity: coefficients at the odd positions 1, 3, .., 2H+1
//   (all other entries of those rows are exactly zero, the row of -a_j has the same even and
//   the negated odd coefficients)
template <int N>
struct InCoef {
    static constexpr int H = (N - 2) / 2;
    float bt[N * N];
    float zero[H + 1];
    float ev[H > 0 ? H * H : 1];
    float od[H > 0 ? H * H : 1];
    float inf[H + 1];
};

// Coefficients of one 1D output transform for kernel size R: A (N x M) row-major, M = N - R + 1,
// and for the symmetric case pw[j][i] = A[row of +a_j][i] (a_j^i times the row's scale),
// zero = A[row of 0][0], inf = A[row of infinity][M-1] (both 1 unless the rows are rescaled).
template <int N, int R>
struct OutCoef {
    static constexpr int M = N - R + 1;
    static constexpr int H = (N - 2) / 2;
    float a[N * M];
    float pw[H > 0 ? H * M : 1];
    float zero, inf;
};

template <int N, int R>
struct FilterCoef {
    double g[N * R];
};

struct Geometry {
    int N, C, H, W, K, m, r, n;
    int tiles_h, tiles_w;
    long long T;          // tiles in the batch
    long long Tp;         // T rounded up to a multiple of 128: row count of M (rows >= T are scratch)
    int c_blocks, k_blocks;
    int Kp;               // K rounded up to the channel block
};

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

inline Geometry make_geometry(int N, int C, int H, int W, int K, int m, int r)
{
    Geometry g;
    g.N = N; g.C = C; g.H = H; g.W = W; g.K = K; g.m = m; g.r = r; g.n = m + r - 1;
    g.tiles_h = ceil_div(H, m);
    g.tiles_w = ceil_div(W, m);
    g.T = (long long)N * g.tiles_h * g.tiles_w;
    g.Tp = (g.T + 127) / 128 * 128;
    g.c_blocks = ceil_div(C, kChanBlock);
    g.k_blocks = ceil_div(K, kChanBlock);
    g.Kp = g.k_blocks * kChanBlock;
    return g;
}

inline size_t dtype_size(int dtype) { return dtype == NOVA_F16 ? 2 : 4; }

}  // namespace nova

struct nova_transforms {
    int m = 0, r = 0, n = 0;
    bool symmetric = false;
    int matrix_dtype = 0;                      // NOVA_MATRIX_F32 / NOVA_MATRIX_F16
    std::vector<int> log2_b, log2_g;           // row scaling in effect, n entries each
    std::vector<int8_t> Aq, BTq, Gq;           // NOVA_MATRIX_INT8: codes
    double scale_q[3] = {0, 0, 0};             //                   and scales of A, B^T, G
    std::vector<nova::Rat> points, A, BT, G;   // exact, row-major
    std::vector<double> A64, BT64, G64;        // rounded once
    std::vector<float> A32, BT32, G32;
};

// ---- kernel launchers (defined in the .hip files); all return a hipError_t as int ----
namespace nova {
void set_last_hip_error(int err);
// sigma_max / sigma_min of a row-major matrix (one-sided Jacobi)
double spectral_condition(const std::vector<double> &mat, int rows, int cols);
int device_cu_count();          // compute units of the current device (256 if the query fails)
// nova_winograd_conv2d's argument checks and slab loop; returns a NOVA_* code
int conv2d_with_workspace(const nova_transforms *t, const void *x, const void *U, void *y, int N, int C, int H,
                          int W, int K, int dtype, int flags, void *workspace, size_t workspace_bytes, void *stream);

int launch_filter_transform(const nova_transforms *t, const void *w, int K, int C, int dtype,
                            void *U, void *stream);
int launch_input_transform(const nova_transforms *t, const void *x, void *V, const Geometry &g,
                           int dtype, void *stream);
int launch_contract(const nova_transforms *t, const void *U, const void *V, void *M,
                    const Geometry &g, int dtype, int flags, void *stream);
int launch_output_transform(const nova_transforms *t, const void *M, void *y, const Geometry &g,
                            int dtype, int flags, void *stream);
// Contraction and output transform in one kernel (no M), for the shapes fused_contract_output_applies names;
// nova_winograd_conv2d takes it for those fused_contract_output_preferred names
bool fused_contract_output_applies(const nova_transforms *t, const Geometry &g, int dtype, int flags);
bool fused_contract_output_preferred(const nova_transforms *t, const Geometry &g, int dtype, int flags);
int launch_fused_contract_output(const nova_transforms *t, const void *U, const void *V, void *y, const Geometry &g,
                                 int dtype, int flags, void *stream);
// Few input channels (C <= few_channels_limit()): the output transform forms the products itself
// from V and a packed copy Uc of the filters' first channels (few_channels_filter_bytes), which
// launch_pack_few_channels writes from U.
int few_channels_limit();
size_t few_channels_filter_bytes(const Geometry &g, int dtype);
// ... and reads V in the compact layout [n*n][T][4] that launch_input_transform_few writes
size_t few_channels_input_bytes(const Geometry &g, int dtype);
int launch_input_transform_few(const nova_transforms *t, const void *x, void *Vc, const Geometry &g,
                               int dtype, void *stream);
int launch_pack_few_channels(const void *U, void *Uc, const Geometry &g, int dtype, void *stream);
int launch_output_transform_few(const nova_transforms *t, const void *V, const void *Uc, void *y,
                                const Geometry &g, int dtype, int flags, void *stream);
// INT8 operands in the Winograd domain: symmetric quantisation of a blocked tensor [positions][channel
// blocks][rows][32] with one scale (kind 0), one per row index (1) or one per position (2); integer
// contraction, raw (int32) or de-quantised (binary32) with the scales of the same kind
int launch_quantize_int8(const void *src, void *dst, void *scales, long long elements, int positions, int rows,
                         int n_scales, int kind, int dtype, void *stream);
int launch_contract_int8(const void *Uq, const void *Vq, void *Mo, const void *u_scales, const void *v_scale,
                         int scale_kind, int dequantise, const Geometry &g, void *stream);
int launch_relu_maxpool2x2(const void *in, void *out, int N, int C, int H, int W, int dtype,
                           void *stream);
}  // namespace nova
