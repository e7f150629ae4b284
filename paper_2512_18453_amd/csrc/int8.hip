// INT8 operands in the Winograd domain (Sec. 4.1 "INT8 Setup"; "CNN Quantization Setup"): the
// transformed weights U and the transformed input tiles V are quantised symmetrically -- scale
// s = max|.| / 127 per tensor, per output channel for U, or per Winograd-domain position; code = value / s rounded to nearest even,
// saturated to [-128, 127] -- and the channel contraction runs on the integer codes,
//     Mi[xi][t][k] = sum_c Vq[xi][t][c] * Uq[xi][k][c]        (exact, 32-bit accumulators),
// on the matrix cores (v_mfma_i32_32x32x32_i8).  The transforms themselves stay in floating point.
//
// Layouts as in the floating-point path, one byte per element: Uq [n*n][C/32][Kp][32],
// Vq [n*n][C/32][T][32]; Mi [n*n][K/32][Tp][32] of int32, or M of the same shape in binary32 with
// M = fl(fl(Mi) * fl(s_U[k] * s_V)).
// Every floating-point step that decides a code is binary32 and correctly rounded: s = max / 127,
// code = rint(value / s); a tensor or channel that is all zero has s = 1.
#include "device_common.hpp"

namespace nova {

typedef int int4v __attribute__((ext_vector_type(4)));
typedef int int16v __attribute__((ext_vector_type(16)));

__global__ void __launch_bounds__(256)
fill_u32_kernel(unsigned *dst, unsigned value, int count)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) dst[i] = value;
}

// largest magnitudes, as bit patterns (for non-negative binary32 numbers the order of the values is the
// order of their bit patterns, so an integer maximum does): top[row_group] over all elements whose
// row index (the second-to-last dimension: k of U, t of V) maps to that group; groups = 1 or rows
// which scale an 8-element piece p belongs to.  kind 0: the only one; 1: its row index inside a
// (position, channel block) plane; 2: its position xi (plane_pieces = pieces per position)
__device__ __forceinline__ int scale_index(long long p, int kind, int rows, long long plane_pieces)
{
    return kind == 0 ? 0 : kind == 1 ? (int)((p >> 2) % rows) : (int)(p / plane_pieces);
}

__device__ __forceinline__ float scale_of(unsigned top_bits)
{
    const float top = __uint_as_float(top_bits);
    return top > 0.0f ? __fdiv_rn(top, 127.0f) : 1.0f;
}

template <typename T>
__global__ void __launch_bounds__(256)
absmax_kernel(const T *__restrict__ src, unsigned *__restrict__ top, long long pieces, int rows, int valid,
              int kind, long long plane_pieces)
{
    // one 8-element piece per thread and step; a row of 32 channels is 4 pieces
    unsigned best = 0;
    int best_at = -1;
    for (long long p = (long long)blockIdx.x * blockDim.x + threadIdx.x; p < pieces; p += (long long)gridDim.x * blockDim.x) {
        const T *at = src + p * 8;
        float m = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) m = fmaxf(m, fabsf(load_f32(at + e)));
        const unsigned bits = __float_as_uint(m);
        if (kind != 0) {
            const int idx = scale_index(p, kind, rows, plane_pieces);
            if (idx != best_at) {
                if (best_at >= 0 && best_at < valid && best > 0) atomicMax(top + best_at, best);
                best_at = idx; best = 0;
            }
        }
        best = bits > best ? bits : best;
    }
    if (kind != 0) {
        if (best_at >= 0 && best_at < valid && best > 0) atomicMax(top + best_at, best);
        return;
    }
    // one atomic per wave
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const unsigned other = (unsigned)__shfl_xor((int)best, off);
        best = other > best ? other : best;
    }
    if ((threadIdx.x & 63) == 0 && best > 0) atomicMax(top, best);
}

template <typename T>
__global__ void __launch_bounds__(256)
quantize_kernel(const T *__restrict__ src, signed char *__restrict__ dst, const unsigned *__restrict__ top,
                long long pieces, int rows, int valid, int kind, long long plane_pieces)
{
    for (long long p = (long long)blockIdx.x * blockDim.x + threadIdx.x; p < pieces; p += (long long)gridDim.x * blockDim.x) {
        // (rows beyond `valid` are padding: all zero, and without a scale of their own)
        const int idx = scale_index(p, kind, rows, plane_pieces);
        const float s = scale_of(idx < valid ? top[idx] : 0u);
        const T *at = src + p * 8;
        unsigned lo = 0, hi = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float q = __builtin_rintf(__fdiv_rn(load_f32(at + e), s));         // ties to even
            q = q < -128.0f ? -128.0f : (q > 127.0f ? 127.0f : q);
            const unsigned byte = (unsigned)((int)q & 0xff);
            if (e < 4) lo |= byte << (8 * e); else hi |= byte << (8 * (e - 4));
        }
        typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
        *reinterpret_cast<u32x2 *>(dst + p * 8) = u32x2{lo, hi};
    }
}

// top (bit patterns of the largest magnitudes) -> scales, in place
__global__ void __launch_bounds__(256)
finish_scales_kernel(unsigned *top_then_scale, int count)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) top_then_scale[i] = __float_as_uint(scale_of(top_then_scale[i]));
}

// src: [positions][channel blocks][rows][32]; kind 0: one scale; 1: one per row index below n_scales (the
// other rows are zero padding); 2: one per position (n_scales = positions)
template <typename T>
static int quantize_rows(const void *src, void *dst, void *scales, long long elements, int rows, int n_scales,
                         int kind, long long plane_pieces, hipStream_t stream)
{
    const long long pieces = elements / 8;                  // rows are 32 elements: always whole pieces
    long long want = (pieces + 255) / 256;
    const unsigned blocks = (unsigned)(want < 1 ? 1 : want > 4096 ? 4096 : want);
    hipLaunchKernelGGL(fill_u32_kernel, dim3((n_scales + 255) / 256), dim3(256), 0, stream, (unsigned *)scales, 0u, n_scales);
    hipLaunchKernelGGL(absmax_kernel<T>, dim3(blocks), dim3(256), 0, stream, (const T *)src, (unsigned *)scales, pieces, rows,
                       n_scales, kind, plane_pieces);
    hipLaunchKernelGGL(quantize_kernel<T>, dim3(blocks), dim3(256), 0, stream, (const T *)src, (signed char *)dst,
                       (const unsigned *)scales, pieces, rows, n_scales, kind, plane_pieces);
    hipLaunchKernelGGL(finish_scales_kernel, dim3((n_scales + 255) / 256), dim3(256), 0, stream, (unsigned *)scales, n_scales);
    return (int)hipGetLastError();
}

int launch_quantize_int8(const void *src, void *dst, void *scales, long long elements, int positions, int rows,
                         int n_scales, int kind, int dtype, void *stream)
{
    if (positions < 1 || rows < 1 || elements % ((long long)positions * rows * kChanBlock) != 0) return (int)hipErrorInvalidValue;
    if ((kind == 0 && n_scales != 1) || (kind == 1 && (n_scales < 1 || n_scales > rows)) || (kind == 2 && n_scales != positions) ||
        kind < 0 || kind > 2)
        return (int)hipErrorInvalidValue;
    const long long plane_pieces = elements / positions / 8;
    return dtype == NOVA_F16 ? quantize_rows<f16>(src, dst, scales, elements, rows, n_scales, kind, plane_pieces, (hipStream_t)stream)
                             : quantize_rows<float>(src, dst, scales, elements, rows, n_scales, kind, plane_pieces, (hipStream_t)stream);
}

// ---- contraction.  A workgroup of 4 waves owns a BM x BN tile of one Mi[xi]; a step moves 32 channels
// (one 32x32x32 matrix instruction per pair of 32-row blocks) through double-buffered LDS, rows padded
// from 32 to 48 bytes so that the 16 lanes of a 128-bit read phase fall into different bank groups.
// The two halves of a wave supply the two 16-channel halves of a row; the sum over the 32 channels of
// a step does not depend on how the instruction orders them, as long as both operands use the same
// order -- they do: both are read with the same row and half-row indexing.
constexpr int kRowBytes8 = 48;

template <int BM, int BN, int WM, int WN, bool DEQUANT>
__global__ void __launch_bounds__(256)
contract_i8_kernel(const signed char *__restrict__ Uq, const signed char *__restrict__ Vq, void *__restrict__ Mo,
                   const float *__restrict__ u_scales, const float *__restrict__ v_scale, int scale_kind,
                   int T, int Tp, int Kp, int K, int c_blocks, int k_blocks, int row_blocks, int col_blocks)
{
    constexpr int MB = BM / WM / 32, NB = BN / WN / 32;
    static_assert(WM * WN == 4 && BM % (WM * 32) == 0 && BN % (WN * 32) == 0, "tile shape");
    static_assert(BM * 2 <= 256 && BN * 2 <= 256, "one 16-byte segment per thread and operand");
    __shared__ __align__(16) signed char lds_a[2][BM * kRowBytes8];
    __shared__ __align__(16) signed char lds_b[2][BN * kRowBytes8];

    unsigned bid = xcd_local_block_id(blockIdx.x, gridDim.x);
    const int cbk = bid % col_blocks; bid /= col_blocks;
    const int rbk = bid % row_blocks; bid /= row_blocks;
    const int xi = bid;
    const int t0 = rbk * BM, k0 = cbk * BN;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wm = wave / WN, wn = wave % WN;

    // segment s of an operand tile: row s/2, 16-byte half s%2; rows beyond the tensor are clamped to the
    // last valid row (their products are never stored)
    const int row = tid >> 1, halfrow = tid & 1;
    const bool has_a = tid < BM * 2, has_b = tid < BN * 2;
    int ta = t0 + row; if (ta > T - 1) ta = T - 1;
    int kb_row = k0 + row; if (kb_row > Kp - 1) kb_row = Kp - 1;
    const signed char *a_src = Vq + ((size_t)xi * c_blocks * T + ta) * kChanBlock + halfrow * 16;
    const signed char *b_src = Uq + ((size_t)xi * c_blocks * Kp + kb_row) * kChanBlock + halfrow * 16;
    const size_t a_step = (size_t)T * kChanBlock, b_step = (size_t)Kp * kChanBlock;
    const int dst_off = row * kRowBytes8 + halfrow * 16;

    int16v acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;

    int4v a_reg = {0, 0, 0, 0}, b_reg = {0, 0, 0, 0};
    auto load_global = [&](int cb) {
        if (has_a) a_reg = *reinterpret_cast<const int4v *>(a_src + cb * a_step);
        if (has_b) b_reg = *reinterpret_cast<const int4v *>(b_src + cb * b_step);
    };
    auto store_lds = [&](int buf) {
        if (has_a) *reinterpret_cast<int4v *>(&lds_a[buf][dst_off]) = a_reg;
        if (has_b) *reinterpret_cast<int4v *>(&lds_b[buf][dst_off]) = b_reg;
    };
    load_global(0);
    store_lds(0);
    __syncthreads();

    const int frag_row = lane & 31, frag_half = (lane >> 5) * 16;
    for (int cb = 0; cb < c_blocks; ++cb) {
        const int buf = cb & 1;
        if (cb + 1 < c_blocks) load_global(cb + 1);
        int4v af[MB], bf[NB];
#pragma unroll
        for (int i = 0; i < MB; ++i)
            af[i] = *reinterpret_cast<const int4v *>(&lds_a[buf][((wm * MB + i) * 32 + frag_row) * kRowBytes8 + frag_half]);
#pragma unroll
        for (int j = 0; j < NB; ++j)
            bf[j] = *reinterpret_cast<const int4v *>(&lds_b[buf][((wn * NB + j) * 32 + frag_row) * kRowBytes8 + frag_half]);
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int j = 0; j < NB; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[i], bf[j], acc[i][j], 0, 0, 0);
        if (cb + 1 < c_blocks) store_lds(buf ^ 1);
        __syncthreads();
    }

    // D[row][col] with A = V rows (tiles t), B = U rows (channels k): lane holds col = k = lane%32 and
    // rows t = 8*(e/4) + 4*(lane/32) + e%4
    const int col = lane & 31, row_base = (lane >> 5) * 4;
    // scale_kind 0: one scale each; 1: U per output channel; 2: both per position
    const float sv = DEQUANT ? v_scale[scale_kind == 2 ? xi : 0] : 0.0f;
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        const int kb = (k0 >> 5) + wn * NB + j;
        if (kb >= k_blocks) continue;
        const int k = kb * kChanBlock + col;
        float both = 0.0f;
        if constexpr (DEQUANT) both = u_scales[scale_kind == 1 ? (k < K ? k : K - 1) : scale_kind == 2 ? xi : 0] * sv;
        const size_t plane = ((size_t)xi * k_blocks + kb) * (size_t)Tp * kChanBlock + col;
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int t = t0 + (wm * MB + i) * 32 + (e >> 2) * 8 + row_base + (e & 3);
                if (t < T) {
                    if constexpr (DEQUANT) reinterpret_cast<float *>(Mo)[plane + (size_t)t * kChanBlock] = (float)acc[i][j][e] * both;
                    else reinterpret_cast<int *>(Mo)[plane + (size_t)t * kChanBlock] = acc[i][j][e];
                }
            }
    }
}

template <bool DEQUANT>
static int launch_ci8(const void *Uq, const void *Vq, void *Mo, const float *u_scales, const float *v_scale,
                      int scale_kind, const Geometry &g, hipStream_t stream)
{
    constexpr int BM = 128, BN = 128;
    const int row_blocks = ceil_div((int)g.T, BM), col_blocks = ceil_div(g.Kp, BN);
    const long long blocks = (long long)g.n * g.n * row_blocks * col_blocks;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL((contract_i8_kernel<BM, BN, 2, 2, DEQUANT>), dim3((unsigned)blocks), dim3(256), 0, stream,
                       (const signed char *)Uq, (const signed char *)Vq, Mo, u_scales, v_scale, scale_kind,
                       (int)g.T, (int)g.Tp, g.Kp, g.K, g.c_blocks, g.k_blocks, row_blocks, col_blocks);
    return (int)hipGetLastError();
}

int launch_contract_int8(const void *Uq, const void *Vq, void *Mo, const void *u_scales, const void *v_scale,
                         int scale_kind, int dequantise, const Geometry &g, void *stream)
{
    if (g.T > 0x7fffffffLL) return (int)hipErrorInvalidValue;
    return dequantise ? launch_ci8<true>(Uq, Vq, Mo, (const float *)u_scales, (const float *)v_scale, scale_kind, g, (hipStream_t)stream)
                      : launch_ci8<false>(Uq, Vq, Mo, (const float *)u_scales, (const float *)v_scale, scale_kind, g, (hipStream_t)stream);
}

}  // namespace nova
