/*
 * nova.h -- C ABI of libnova: 2D Winograd minimal-filtering convolution F(m x m, 3 x 3)
 * on AMD CDNA4 (gfx950), with Cook-Toom transform matrices A, B^T, G generated exactly
 * (rational arithmetic, host) from an arbitrary set of interpolation points.
 *
 * The algorithm (arxiv 2512.18453, Sec. 2.1 "Winograd Convolution via Cook-Toom", nested
 * in 2D as in App. "2D Extension via Kronecker Products"):
 *
 *     Y = A^T [ (G g G^T) * (B^T d B) ] A,   summed over input channels before A^T . A,
 *
 * for each n x n input tile d (n = m + r - 1, tiles at stride m over the image zero-padded by
 * (r-1)/2 pixels) and each r x r filter g (r = 3 in the paper's experiments, r = 5 its stated
 * extension); stride 1, correlation (no kernel flip), no bias.
 *
 * Conventions for every call
 *   - "host" pointers are ordinary process memory, "device" pointers are HIP device memory
 *     of the current device; nothing is copied between the two behind the caller's back.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Device work is
 *     enqueued on it and the call returns without waiting.
 *   - No call allocates or frees device memory, none keeps global state besides the last
 *     HIP error code (thread-local).
 *   - Return value: NOVA_OK (0) or a negative NOVA_E* code; nothing throws or aborts.
 *   - dtype selects the storage format of x, w, U, V, y: NOVA_F16 (IEEE binary16) or
 *     NOVA_F32.  Arithmetic: transforms in binary32 (filter transform in binary64),
 *     channel contraction on the matrix cores with binary32 accumulation.
 */
#ifndef NOVA_H
#define NOVA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct { int64_t num, den; } nova_rational;   /* den > 0 on output; den != 0 on input */
typedef struct nova_transforms nova_transforms;       /* opaque, host memory, immutable */

enum {
    NOVA_OK = 0,
    NOVA_EINVAL = -1,       /* null pointer, bad size, bad enum, zero denominator, wrong point count */
    NOVA_EDUP = -2,         /* two equal interpolation points (singular Vandermonde system) */
    NOVA_EOVERFLOW = -3,    /* an exact intermediate or matrix entry does not fit 64-bit num/den */
    NOVA_EVERIFY = -4,      /* the generated matrices fail the exact tensor identity (internal bug trap) */
    NOVA_ENOSPC = -5,       /* workspace too small */
    NOVA_EUNSUPPORTED = -6, /* valid request the device path does not implement (tile sizes other than
                               r = 3 with m in {2,4,6,8} and r = 5 with m in {2,4,6}) */
    NOVA_EHIP = -7,         /* a HIP call failed; see nova_last_hip_error() */
    NOVA_ENOMEM = -8        /* host allocation failed */
};

enum { NOVA_F32 = 0, NOVA_F16 = 1 };
enum { NOVA_MATRIX_A = 0, NOVA_MATRIX_BT = 1, NOVA_MATRIX_G = 2 };

/* flags of nova_winograd_conv2d / nova_output_transform / nova_contract */
enum {
    NOVA_FLAG_RELU = 1,     /* y = max(y, 0) fused into the output transform (NaN stays NaN) */
    NOVA_FLAG_M_F16 = 2,    /* NOVA_F16 only: keep the products M in binary16 instead of binary32 */
    NOVA_FLAG_POOL2 = 4     /* 2 x 2, stride-2 max-pool fused into the output transform (after the optional
                               ReLU): y is [N][K][H/2][W/2]; H and W must be even (NOVA_EINVAL otherwise);
                               a NaN in a window makes that output NaN.  The step between the blocks of a
                               VGG-style stack, without writing and re-reading the unpooled layer */
};

/* ------------------------------------------------------------------ transforms (host) */

/*
 * Exact Cook-Toom construction (Alg. "Symbolic Cook-Toom Construction"; Sec. 2.4).
 * finite_points: host array of n_points = m + r - 2 distinct rationals alpha_0 .. alpha_{n-2},
 * n = m + r - 1; the point at infinity is implicit and always last.  Row p of every matrix
 * belongs to alpha_p in the order given.
 *   A   (n x m)  A[p][i]  = alpha_p^i;                       infinity row = e_{m-1}
 *   G   (n x r)  G[p][k]  = alpha_p^k / F_p,  F_p = prod_{j != p} (alpha_p - alpha_j);   infinity row = e_{r-1}
 *   B^T (n x n)  row p = coefficients (ascending powers) of prod_{j != p} (t - alpha_j), then 0;
 *                infinity row = coefficients of prod_j (t - alpha_j)
 * The result is verified against the exact identity sum_p A[p][i] B^T[p][j] G[p][k] = [j == i + k]
 * before it is returned.  Any m >= 1, r >= 1 with n <= 16 is accepted here; the device calls
 * below need r == 3 with m in {2, 4, 6, 8}, or r == 5 with m in {2, 4, 6} (the 5 x 5 extension of
 * Sec. "Extension to 5 x 5 Kernels": same n as F(4,3) .. F(8,3)).
 * *out is owned by the caller: release with nova_free_transforms.
 */
int nova_make_transforms(const nova_rational *finite_points, int n_points, int m, int r,
                         nova_transforms **out);

/*
 * The same construction with two options.
 *
 * row_scaling -- the diagonal-scale form Y = D_A A^T [ (D_G G g) . (D_B B^T d) ] (related-work
 * discussion of learned diagonal scales; Table "Network-level ablation: points x scaling"),
 * restricted to powers of two with D_A D_G D_B = I, so the algorithm stays exact and only the range
 * of U and V moves:  row p of B^T is multiplied by 2^log2_b[p], row p of G by 2^log2_g[p], row p
 * of A by 2^-(log2_b[p] + log2_g[p]).
 *   NOVA_ROWS_PLAIN     no scaling (log2_b, log2_g ignored, may be NULL)
 *   NOVA_ROWS_BALANCED  the exponents that bring the absolute row sums of B^T and of G into
 *                       [1, 2): then |V| <= 4 max|x| and |U| <= 4 max|w| whatever the points
 *   NOVA_ROWS_GIVEN     log2_b, log2_g: host arrays of n = m + r - 1 exponents, each in [-60, 60]
 * The scaled matrices are verified against the exact identity again.  The device transforms share
 * work between the rows of +a and -a only if both rows carry the same exponents (always so for
 * NOVA_ROWS_BALANCED); otherwise the general kernels run.
 *
 * matrix_dtype -- what the device constants are rounded to (each entry once, from the exact value):
 *   NOVA_MATRIX_F32  A, B^T binary32, G binary64 (the default of nova_make_transforms)
 *   NOVA_MATRIX_F16  every entry to the nearest binary16 first (the variant with the matrices kept in
 *                    binary16: Sec. "Float16 Precision Analysis", Table "FP16 storage"); the rounded tables then hold those values
 *   NOVA_MATRIX_INT8 each of A, B^T, G quantised symmetrically per tensor (Sec. "INT8 Convolution
 *                    Error Validation"): scale s = max|entry| / 127, code = entry / s rounded to
 *                    nearest (ties to even) and saturated to [-128, 127], both computed exactly;
 *                    the rounded tables hold code * s (A, B^T to binary32, G to binary64).  This is
 *                    the configuration that reproduces the paper's printed INT8 error table.
 * The exact matrices (nova_get_matrix) are the unrounded ones in every case.
 * Errors as nova_make_transforms, plus NOVA_EINVAL for an unknown option or exponent out of range.
 */
#define NOVA_ROWS_PLAIN 0
#define NOVA_ROWS_BALANCED 1
#define NOVA_ROWS_GIVEN 2
#define NOVA_MATRIX_F32 0
#define NOVA_MATRIX_F16 1
#define NOVA_MATRIX_INT8 2
int nova_make_transforms_ex(const nova_rational *finite_points, int n_points, int m, int r,
                            int row_scaling, const int *log2_b, const int *log2_g, int matrix_dtype,
                            nova_transforms **out);
/* The exponents in effect (all zero for NOVA_ROWS_PLAIN): n entries each, either may be NULL. */
int nova_get_row_scaling(const nova_transforms *t, int *log2_b, int *log2_g);
/* INT8 codes (row-major, caller-allocated) and scale of one matrix of a handle made with
 * NOVA_MATRIX_INT8; NOVA_EINVAL for other handles.  *scale is s rounded to binary64. */
int nova_get_matrix_int8(const nova_transforms *t, int which, int8_t *codes, double *scale);
void nova_free_transforms(nova_transforms *t);

/*
 * Point discovery, the deterministic steps (host only).
 *
 * nova_symmetric_search: exhaustive search over symmetric configurations {0, +-p1, +-p2, ..}
 * (Sec. "Symmetric Search", Alg. "Symmetric Search"): n - 1 = m + r - 2 finite points, zero plus
 * (n - 2) / 2 pairs when n - 1 is odd, (n - 1) / 2 pairs when it is even; the magnitudes are all
 * a/b with 1 <= b <= d_max and 1 <= a <= 5b; the configuration with the lowest spectral condition
 * number of its Vandermonde matrix wins (first in lexicographic order of ascending magnitudes
 * among equals) and is verified exactly before it is returned.  With d_max = 6 this yields the
 * discovered point sets the paper prints for F(4,3), F(6,3) and F(8,3).
 * points_out: n - 1 entries, in the order 0, +p1, -p1, +p2, -p2, .. (ready for
 * nova_make_transforms); *kappa_out: its condition number.  1 <= d_max <= 64; NOVA_EUNSUPPORTED
 * if more than 2e8 combinations would have to be tried.  Uses up to 16 host threads.
 *
 * nova_snap_to_rational: the fraction a/b nearest to x with 1 <= b <= d_max, |a| <= 5b
 * (Sec. "Snap-to-Rational"); among equally near ones the first in the order b ascending, then a
 * ascending.  Exact comparison; *out is reduced.  1 <= d_max <= 1000, x finite.
 */
int nova_symmetric_search(int m, int r, int d_max, nova_rational *points_out, double *kappa_out);
int nova_snap_to_rational(double x, int d_max, nova_rational *out);

/*
 * The evolution strategy over R^(n-1) (Sec. "Evolution Strategy"; Alg. "Evolution Strategy for Winograd
 * Point Discovery"; Tables "Evolution Strategy hyperparameters" and "Fitness function weights"), host only.
 *
 * nova_es_fitness: f(p) = || T - T_rec(p) ||_F + 0.001 |p|^2 / (n - 1) + 0.0001 log10(kappa(V) + 1) for n - 1
 *   finite points given as doubles, T_rec the tensor rebuilt from the Cook-Toom matrices of p evaluated
 *   in binary64; parts_out (may be NULL): tensor error, |p|^2 / (n - 1), kappa(V).  +infinity when a part
 *   is not finite (coinciding points).
 * nova_evolution_strategy: `restarts` independent runs of `generations` generations with `population`
 *   candidates each: mean mu ~ N(0, 0.5 I), step sigma = 0.5; every generation samples mu + sigma eps,
 *   moves mu to the mean of the best quarter, multiplies sigma by 1.1 if more than 20 % of the
 *   candidates are fitter than the mean they were sampled around, else by 0.9 (kept within
 *   [0.01, 2]); the fittest candidate ever seen is returned (points_out: n - 1 doubles).
 *   The random numbers are an argument: `normals` holds at least nova_es_normals_needed(..)
 *   independent standard normal draws, consumed in order (per restart n - 1 for mu, then per generation
 *   population * (n - 1), candidate by candidate), so a run is a function of its arguments.
 *   The paper's values: generations 100, population 50, restarts 3.
 * nova_snap_points: the step after it (Sec. "Snap-to-Rational", "Neighborhood Search"): every coordinate
 *   to its nearest simple fraction (nova_snap_to_rational); if two coincide, each point gets the
 *   fractions within 6/5 of its snapped value, nearest to its continuous value first -- as many per
 *   point as keep the combinations within 1e5 -- and the combination of distinct points with the
 *   lowest kappa(V) wins (the first one enumerated, last point varying fastest, among those within a
 *   relative 1e-9 of each other); the result is verified exactly.  points_out: n - 1 entries in the order of x.
 * Errors: NOVA_EINVAL; NOVA_EVERIFY if no candidate was ever valid.
 */
int nova_es_fitness(int m, int r, const double *points, double *fitness_out, double parts_out[3]);
size_t nova_es_normals_needed(int m, int r, int generations, int population, int restarts);
int nova_evolution_strategy(int m, int r, int generations, int population, int restarts,
                            const double *normals, size_t n_normals, double *points_out, double *fitness_out);
int nova_snap_points(int m, int r, const double *x, int d_max, nova_rational *points_out, double *kappa_out);

/* m, r, n of a handle; `symmetric` = 1 when the points come as 0, +a1, -a1, +a2, -a2, ...
 * (the order for which the device transforms share work between +a and -a). Any pointer may be NULL. */
int nova_transforms_shape(const nova_transforms *t, int *m, int *r, int *n, int *symmetric);

/* Row-major copy of one matrix into caller-allocated host memory (n*m, n*n or n*r entries):
 * exact (NOVA_EOVERFLOW if an entry needs more than 64 bits), or rounded once to the nearest
 * binary64 / binary32 -- the tables the device code uses (B^T, A: binary32; G: binary64). */
int nova_get_matrix(const nova_transforms *t, int which, nova_rational *out);
int nova_get_matrix_f64(const nova_transforms *t, int which, double *out);
int nova_get_matrix_f32(const nova_transforms *t, int which, float *out);

/* Spectral condition numbers (Sec. 2.2 "Condition Number Definition"): out[0] = kappa_2 of the
 * square Vandermonde matrix of the finite points, out[1..3] = kappa_2 of A, B^T, G. */
int nova_kappa(const nova_transforms *t, double out[4]);

/* ------------------------------------------------------------------ device tensors */

/*
 * Winograd-domain layouts (device, opaque to most callers; documented for tests).
 * xi = i*n + j indexes the n*n transform-domain positions, t = (image*tiles_h + tile_row)*tiles_w
 * + tile_col the tiles, tiles_h = ceil(H/m), tiles_w = ceil(W/m).  Channels are blocked by 32:
 *   U [n*n][ceil(C/32)][Kp][32]   Kp = K rounded up to a multiple of 32; element (xi, k, c) at
 *                                 ((xi*ceil(C/32) + c/32)*Kp + k)*32 + c%32; padding is zero
 *   V [n*n][ceil(C/32)][T][32]    same with t in place of k and T in place of Kp
 *   M [n*n][ceil(K/32)][Tp][32]   Tp = T rounded up to a multiple of 128; element (xi, t, k) at
 *                                 ((xi*ceil(K/32) + k/32)*Tp + t)*32 + k%32; rows t >= T are scratch
 * U and V have the storage dtype; M is binary32 (binary16 with NOVA_FLAG_M_F16).
 */
size_t nova_filter_bytes(int K, int C, int m, int r, int dtype);                 /* size of U */
size_t nova_input_bytes(int N, int C, int H, int W, int m, int r, int dtype);    /* size of V, whole batch */
size_t nova_product_bytes(int N, int K, int H, int W, int m, int r, int dtype, int flags); /* size of M */

/*
 * Filter transform U = G g G^T (Sec. 2.1 step 2 in 2D), evaluated in binary64 and rounded once
 * to dtype.  w: device [K][C][r][r] of dtype; U: device, nova_filter_bytes(K, C, m, r, dtype) bytes,
 * fully overwritten (padding included).  Done once per weight set, off the per-call path.
 */
int nova_filter_transform(const nova_transforms *t, const void *w, int K, int C, int dtype,
                          void *U, void *stream);

/*
 * Workspace for nova_winograd_conv2d.  The call processes the batch in slabs of whole images so
 * that V and M of a slab stay cache resident; the slab size follows from the workspace it is
 * given (as many slabs as the largest size that fits would need, evened out: 16 + 16 images, not 20 + 12).  images_per_slab = 0 asks for the library's default (as many images as fit 256 MiB of
 * V and M, at least one), N for the whole batch in one pass.  Returns 0 for invalid arguments.
 * With C <= 4 (the first layer of an image network) the call keeps no M: the output transform forms
 * the products itself, and the workspace holds V in a compact 4-channel layout and a packed copy of the
 * filters' first four channels.
 */
size_t nova_conv2d_workspace_bytes(int N, int C, int H, int W, int K, int m, int r, int dtype, int flags,
                                   int images_per_slab);

/*
 * y = conv r x r (x, w), stride 1, zero border (r-1)/2 (3 x 3 with border 1 is the paper's case; the
 * 5 x 5 extension takes border 2, "same" output size), through F(m x m, r x r) with the handle's matrices:
 * input transform -> n*n channel contractions -> output transform, enqueued on `stream`.
 * With C <= 4 the contraction is done inside the output transform, as a binary32 multiply-add chain
 * over the channels (products of two stored values are exact in binary32), instead of on the matrix
 * unit; the result agrees with nova_contract + nova_output_transform to rounding, not bit for bit.
 * x: device [N][C][H][W]; U: from nova_filter_transform with the same handle, K, C, dtype;
 * y: device [N][K][H][W]; all of dtype.  H, W >= 1 arbitrary: the image is zero-extended to
 * whole tiles and the result cropped.  workspace: device, at least
 * nova_conv2d_workspace_bytes(..., images_per_slab = 1) bytes, 256-byte aligned; must not
 * overlap x, U, y.  Errors: NOVA_EINVAL, NOVA_EUNSUPPORTED, NOVA_ENOSPC, NOVA_EHIP.
 * Arithmetic contract of the input transform (what makes V reproducible bit for bit): each 1D
 * transform row is E + O in binary32, E / O = fused multiply-add chains over the even / odd
 * input indices in ascending order; columns of the tile first, then rows.
 */
int nova_winograd_conv2d(const nova_transforms *t, const void *x, const void *U, void *y,
                         int N, int C, int H, int W, int K, int dtype, int flags,
                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * nova_winograd_conv2d for callers that cannot allocate device memory or carry a workspace around:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, result and errors, but V and M of a slab live in a fixed array of
 * nova_static_workspace_bytes() = 64 MiB inside the library's device image (one copy per GPU, held
 * until the process ends) instead of a caller buffer; the batch is cut into as many slabs of whole
 * images as that size requires.  NOVA_ENOSPC if V and M of a single image exceed it (the shape then
 * needs nova_winograd_conv2d with a workspace of its own).  The call allocates and frees nothing;
 * the array's device address is looked up once per device (NOVA_EHIP if that fails).
 * All calls on one GPU share that GPU's array and nothing in it is expected to be zero or to
 * survive between calls: calls that overlap in time on one GPU (different streams, or threads)
 * race on it and must be serialised by the caller.
 */
size_t nova_static_workspace_bytes(void);
int nova_winograd_conv2d_static(const nova_transforms *t, const void *x, const void *U, void *y,
                                int N, int C, int H, int W, int K, int dtype, int flags, void *stream);

/* The three stages on their own (same arguments; V, M: device buffers for the N images passed).
 * V_bytes / M_bytes give the size of the buffer the call writes; the call returns NOVA_ENOSPC
 * before launching anything if that is less than nova_input_bytes / nova_product_bytes for the
 * shape (the kernels write whole padded blocks).  For tests and per-stage profiling. */
int nova_input_transform(const nova_transforms *t, const void *x, void *V, size_t V_bytes,
                         int N, int C, int H, int W, int dtype, void *stream);        /* Sec. 2.1 step 1 */
int nova_contract(const nova_transforms *t, const void *U, const void *V, void *M, size_t M_bytes,
                  int N, int C, int H, int W, int K, int dtype, int flags, void *stream); /* step 3 + channel sum */
int nova_output_transform(const nova_transforms *t, const void *M, size_t M_bytes, void *y,
                          int N, int K, int H, int W, int dtype, int flags, void *stream); /* step 4 */

/*
 * INT8 operands in the Winograd domain (Sec. 4.1 "INT8 Setup"; paragraph "CNN Quantization Setup":
 * the transform matrices stay in floating point, what is quantised are the weights and the
 * Winograd-domain tensors).  Symmetric quantisation without zero point: scale s = max|.| / 127,
 * code = value / s rounded to nearest (ties to even) and saturated to [-128, 127]; every
 * floating-point step that decides a code is binary32 and correctly rounded; a tensor (or channel)
 * that is all zero gets s = 1.  mode:
 *   NOVA_INT8_PER_TENSOR   one scale for U, one for V
 *   NOVA_INT8_PER_CHANNEL  one scale of U per output channel k (over all positions and input
 *                          channels), one for V (a scale that varied with the input channel could
 *                          not be pulled out of the channel sum)
 *   NOVA_INT8_PER_POSITION one scale per Winograd-domain position xi, for U and for V (n*n scales
 *                          each): the tap-wise scaling of the paper's related-work discussion
 * The channel contraction then runs on the codes, exactly, on the integer matrix cores:
 *   Mi[xi][t][k] = sum_c Vq[xi][t][c] Uq[xi][k][c]  (32-bit),  M = fl(fl(Mi) * fl(s_U[k] * s_V)).
 * Layouts as for U, V, M above with one byte per element (Uq, Vq) and 4 bytes per element (Mi, M).
 *
 * nova_quantize_filter_int8: U from nova_filter_transform (dtype) -> Uq (nova_filter_int8_bytes) and
 *   u_scales (device: 1 float, K floats, or n*n floats, by mode).  Once per weight set.
 * nova_quantize_input_int8: V from nova_input_transform (dtype, the N images passed) -> Vq
 *   (nova_input_int8_bytes) and v_scale (device: 1 float, or n*n floats per position; taken over
 *   these N images).
 * nova_contract_int8: M (device, nova_product_bytes(.., NOVA_F32, 0) bytes) receives the exact 32-bit
 *   sums (dequantise = 0; the scale pointers may then be NULL) or the de-quantised binary32 products
 *   (dequantise = 1), which nova_output_transform takes as they are.
 * nova_winograd_conv2d_int8: input transform, quantisation of V (one scale for the whole batch of
 *   the call), integer contraction, output transform, in one call; x, y of dtype as in
 *   nova_winograd_conv2d; workspace at least nova_conv2d_int8_workspace_bytes, 256-byte aligned; the
 *   batch is not cut into slabs (the scale of V belongs to the whole call).  NOVA_FLAG_M_F16 is
 *   refused (NOVA_EINVAL).
 * All are asynchronous on `stream` and allocate nothing.  Errors as for the calls above.
 */
enum { NOVA_INT8_PER_TENSOR = 0, NOVA_INT8_PER_CHANNEL = 1, NOVA_INT8_PER_POSITION = 2 };
size_t nova_filter_int8_bytes(int K, int C, int m, int r);
size_t nova_input_int8_bytes(int N, int C, int H, int W, int m, int r);
int nova_quantize_filter_int8(const nova_transforms *t, const void *U, int K, int C, int dtype, int mode,
                              void *Uq, float *u_scales, void *stream);
int nova_quantize_input_int8(const nova_transforms *t, const void *V, int N, int C, int H, int W, int dtype,
                             int mode, void *Vq, float *v_scale, void *stream);
int nova_contract_int8(const nova_transforms *t, const void *Uq, const void *Vq, const float *u_scales,
                       const float *v_scale, int mode, void *M, size_t M_bytes, int N, int C, int H, int W, int K,
                       int dequantise, void *stream);
size_t nova_conv2d_int8_workspace_bytes(int N, int C, int H, int W, int K, int m, int r, int dtype);
int nova_winograd_conv2d_int8(const nova_transforms *t, const void *x, const void *Uq, const float *u_scales,
                              int mode, void *y, int N, int C, int H, int W, int K, int dtype, int flags,
                              void *workspace, size_t workspace_bytes, void *stream);

/*
 * Steps 3 and 4 (Sec. 2.1) in one kernel: y = A^T [ sum_c U * V ] A per tile and output channel, the
 * products kept in registers and never written as M.  For layers with 64 input channels, where M is
 * most of the memory traffic: NOVA_F16 storage, points in the order 0, +a, -a, .., F(6,3) or F(8,3),
 * C = 64, K a multiple of 32, without NOVA_FLAG_M_F16; other requests: NOVA_EUNSUPPORTED.
 * U, V as for nova_contract; y, flags (ReLU, max-pool) as for nova_output_transform.  The result differs
 * from nova_contract + nova_output_transform by the order of the binary32 sums only.
 *
 * nova_conv2d_path says which kernels nova_winograd_conv2d runs for a layer shape (whatever the batch):
 * NOVA_PATH_STAGES (input transform, contraction, output transform), NOVA_PATH_FEW_CHANNELS (at most 4
 * input channels: compact V, the products formed inside the output transform) or NOVA_PATH_FUSED_OUTPUT
 * (input transform, then the kernel above: taken wherever it is supported).  Negative: an error code.
 * Host only.
 */
enum { NOVA_PATH_STAGES = 0, NOVA_PATH_FEW_CHANNELS = 1, NOVA_PATH_FUSED_OUTPUT = 2 };
int nova_conv2d_path(const nova_transforms *t, int C, int H, int W, int K, int dtype, int flags);
int nova_contract_output_fused(const nova_transforms *t, const void *U, const void *V, void *y,
                               int N, int C, int H, int W, int K, int dtype, int flags, void *stream);

/* out = maxpool2x2(max(in, 0)), stride 2, floor; in [N][C][H][W] -> out [N][C][H/2][W/2] (device).
 * The step between the blocks of a VGG-style stack. */
int nova_relu_maxpool2x2(const void *in, void *out, int N, int C, int H, int W, int dtype, void *stream);

/* ------------------------------------------------------------------ misc */
const char *nova_strerror(int code);
int nova_last_hip_error(void);     /* hipError_t of the last failed HIP call on this thread, 0 if none */
const char *nova_version(void);

#ifdef __cplusplus
}
#endif
#endif /* NOVA_H */
