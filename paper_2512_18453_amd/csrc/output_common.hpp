// What the output-transform kernels share: the 1D transform with A, the geometry of a tile group's
// output block in LDS, and the code that moves such a block to y.
#pragma once
#include <type_traits>

#include "device_common.hpp"

namespace nova {

// The 1D transform with A for points in the paired order (0, +a1, -a1, ..., infinity), in two steps that
// can be issued apart: sums and differences of the pairs, then one output at a time.
template <int N, int R>
__device__ __forceinline__ void output_transform_1d_pairs(const float (&v)[N], float (&s)[(N - 2) / 2 > 0 ? (N - 2) / 2 : 1],
                                                          float (&d)[(N - 2) / 2 > 0 ? (N - 2) / 2 : 1])
{
    constexpr int H = (N - 2) / 2;
#pragma unroll
    for (int j = 0; j < H; ++j) {
        s[j] = v[2 * j + 1] + v[2 * j + 2];
        d[j] = v[2 * j + 1] - v[2 * j + 2];
    }
}

// output i from the values at 0 and at infinity and the pairs' sums and differences
// (with unscaled rows zero = inf = pw[j][0] = 1 and these are plain sums)
template <int N, int R>
__device__ __forceinline__ float output_transform_1d_out(int i, float v_zero, float v_inf,
                                                         const float (&s)[(N - 2) / 2 > 0 ? (N - 2) / 2 : 1],
                                                         const float (&d)[(N - 2) / 2 > 0 ? (N - 2) / 2 : 1], const OutCoef<N, R> &k)
{
    constexpr int M = N - R + 1;
    constexpr int H = (N - 2) / 2;
    float acc = i == 0 ? k.zero * v_zero : (i == M - 1) ? k.inf * v_inf : 0.0f;
#pragma unroll
    for (int j = 0; j < H; ++j) acc = fma32(k.pw[j * M + i], (i & 1) ? d[j] : s[j], acc);
    if (M == 1) acc = fma32(k.inf, v_inf, acc);
    return acc;
}

template <int N, int R, bool SYM>
__device__ __forceinline__ void output_transform_1d(const float (&v)[N], float (&out)[N - R + 1], const OutCoef<N, R> &k)
{
    constexpr int M = N - R + 1;
    constexpr int H = (N - 2) / 2;
    if constexpr (SYM) {
        float s[H > 0 ? H : 1], d[H > 0 ? H : 1];
        output_transform_1d_pairs<N, R>(v, s, d);
#pragma unroll
        for (int i = 0; i < M; ++i) out[i] = output_transform_1d_out<N, R>(i, v[0], v[N - 1], s, d, k);
    } else {
#pragma unroll
        for (int i = 0; i < M; ++i) {
            float acc = 0.0f;
#pragma unroll
            for (int p = 0; p < N; ++p) acc = fma32(k.a[p * M + i], v[p], acc);
            out[i] = acc;
        }
    }
}

struct OutShape {
    int twb;          // tiles per group (all tile rows of the group together)
    int twc;          // tile columns per group
    int trb;          // tile rows per group
    int rows;         // output rows per group = trb * m
    int groups;       // tile groups per tile row
    int cols_pitch;   // LDS elements per output row of the group
    int k_pitch;      // LDS elements per channel
    int pieces;       // flat stores: 16-byte pieces that can touch one channel's run of rows * W elements
    unsigned piece_magic, w_magic, rows_magic;     // ceil(2^32 / d) for d = pieces, W, rows
    int pool;         // 1: 2 x 2 max-pool while storing (H, W even)
    unsigned half_rows_magic;                      // ceil(2^32 / (rows / 2)), rows / 2 >= 2
};

// How the block leaves LDS.
//   kStoreScalar  any W, any group: element by element, lanes along W
//   kStoreVec     W (and the group width) a multiple of a 16-byte piece, y 16-byte aligned
//   kStoreFlat    the group spans the image width (narrow images) and y is 16-byte aligned: the rows
//                 of one channel are one contiguous run of y, written in aligned 16-byte pieces
//                 whatever W is (element stores at its two ragged ends)
enum { kStoreScalar = 0, kStoreVec = 1, kStoreFlat = 2 };

// The [32 channels][rows][columns] block of a group, staged in LDS (channel pitch sh.k_pitch, row pitch
// sh.cols_pitch), to y [N][K][H][W] (or its 2 x 2 max-pooled form): lanes along W.  Called by all
// threads of the workgroup after a barrier; img, kb (block of 32 channels), tr (first tile row of the
// group), tc0 (first tile column) say where the block sits.
template <typename T, int M, int STG>
__device__ __forceinline__ void store_output_block(const T *lds, T *__restrict__ y, int img, int kb, int tr, int tc0,
                                                   int K, int H, int W, int tiles_w, const OutShape &sh)
{
    constexpr int PE = 16 / (int)sizeof(T);
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
    const int w0 = tc0 * M;
    int cols = sh.twc * M;
    if (w0 + cols > W) cols = W - w0;
    if (sh.pool) {
        // 2 x 2 max-pool on the way out: rows, columns, H, W, tr*M and w0 are all even, so no window
        // straddles two groups.  One output element per thread and round, lanes along the pooled row.
        const int Hp = H / 2, Wp = W / 2, pcols = cols / 2, prows = sh.rows / 2;
        if constexpr (STG == kStoreVec && sizeof(T) == 2) {
            // W, w0 and cols are multiples of a 16-byte piece of y and y is 16-byte aligned.  If they are multiples
            // of two pieces, the pooled rows leave in 16-byte pieces too: a thread takes 2 rows x 16 columns.
            if (W % (2 * PE) == 0 && w0 % (2 * PE) == 0 && cols % (2 * PE) == 0) {
                const int pieces = pcols / PE;
                const unsigned magic = (unsigned)((((unsigned long long)1 << 32) + pieces - 1) / pieces);
                const int slots = kChanBlock * prows * pieces;
                for (int s = threadIdx.x; s < slots; s += (int)blockDim.x) {
                    const int line = pieces > 1 ? (int)__umulhi((unsigned)s, magic) : s;
                    const int q = s - line * pieces;
                    const int kk = prows > 1 ? (int)__umulhi((unsigned)line, sh.half_rows_magic) : line;
                    const int pp = line - kk * prows;
                    const int k = kb * kChanBlock + kk, hp = (tr * M) / 2 + pp;
                    if (k >= K || hp >= Hp) continue;
                    const T *top = lds + kk * sh.k_pitch + 2 * pp * sh.cols_pitch + 2 * q * PE;     // 8-byte aligned
                    const T *bottom = top + sh.cols_pitch;
                    T a[2 * PE], b[2 * PE], out[PE];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        reinterpret_cast<u32x2 *>(a)[e] = reinterpret_cast<const u32x2 *>(top)[e];
                        reinterpret_cast<u32x2 *>(b)[e] = reinterpret_cast<const u32x2 *>(bottom)[e];
                    }
#pragma unroll
                    for (int e = 0; e < PE; ++e) {
                        const float v0 = (float)a[2 * e], v1 = (float)a[2 * e + 1], v2 = (float)b[2 * e], v3 = (float)b[2 * e + 1];
                        float best = v0;                                  // a NaN in the window wins
                        best = (v1 > best || v1 != v1) ? v1 : best;
                        best = (v2 > best || v2 != v2) ? v2 : best;
                        best = (v3 > best || v3 != v3) ? v3 : best;
                        out[e] = (T)best;                                 // one of the four values: exact
                    }
                    u32x4 piece;
                    __builtin_memcpy(&piece, out, 16);
                    __builtin_nontemporal_store(piece, reinterpret_cast<u32x4 *>(y + (((size_t)img * K + k) * Hp + hp) * Wp + w0 / 2 + q * PE));
                }
                return;
            }
        }
        const unsigned pc_magic = (unsigned)((((unsigned long long)1 << 32) + pcols - 1) / pcols);
        const int slots = kChanBlock * prows * pcols;
        for (int s = threadIdx.x; s < slots; s += (int)blockDim.x) {
            const int line = pcols > 1 ? (int)__umulhi((unsigned)s, pc_magic) : s;
            const int qq = s - line * pcols;
            const int kk = prows > 1 ? (int)__umulhi((unsigned)line, sh.half_rows_magic) : line;
            const int pp = line - kk * prows;
            const int k = kb * kChanBlock + kk, hp = (tr * M) / 2 + pp;
            if (k >= K || hp >= Hp) continue;
            const T *win = lds + kk * sh.k_pitch + 2 * pp * sh.cols_pitch + 2 * qq;
            const float a = load_f32(win), b = load_f32(win + 1);
            const float c = load_f32(win + sh.cols_pitch), d = load_f32(win + sh.cols_pitch + 1);
            float best = a;                                   // a NaN in the window wins
            best = (b > best || b != b) ? b : best;
            best = (c > best || c != c) ? c : best;
            best = (d > best || d != d) ? d : best;
            store_from_f32(y + (((size_t)img * K + k) * Hp + hp) * Wp + w0 / 2 + qq, best);
        }
        return;
    }
    if constexpr (STG == kStoreVec) {
        // W, w0 and cols are multiples of PE and y is 16-byte aligned
        const int pieces = cols / PE;
        const unsigned magic = (unsigned)((((unsigned long long)1 << 32) + pieces - 1) / pieces);
        const int slots = kChanBlock * sh.rows * pieces;
        for (int s = threadIdx.x; s < slots; s += (int)blockDim.x) {
            const int line = pieces > 1 ? (int)__umulhi((unsigned)s, magic) : s;
            const int q = s - line * pieces;
            const int kk = (int)__umulhi((unsigned)line, sh.rows_magic), p = line - kk * sh.rows;
            const int k = kb * kChanBlock + kk, h = tr * M + p;
            if (k >= K || h >= H) continue;
            const u32x2 *in = reinterpret_cast<const u32x2 *>(lds + kk * sh.k_pitch + p * sh.cols_pitch + q * PE);
            const u32x2 lo = in[0], hi = in[1];
            u32x4 *dst = reinterpret_cast<u32x4 *>(y + (((size_t)img * K + k) * H + h) * W + w0 + q * PE);
            __builtin_nontemporal_store(u32x4{lo.x, lo.y, hi.x, hi.y}, dst);    // y is not read again by this call
        }
    } else if constexpr (STG == kStoreFlat) {
        // the group spans the width: rows h0 .. h1-1 of one channel are one run of y
        const int h0 = tr * M;
        int h1 = h0 + sh.rows; if (h1 > H) h1 = H;
        const int run = (h1 - h0) * W;
        const int slots = kChanBlock * sh.pieces;
        for (int s = threadIdx.x; s < slots; s += (int)blockDim.x) {
            const int kk = (int)__umulhi((unsigned)s, sh.piece_magic);
            const int kq = s - kk * sh.pieces;
            const int k = kb * kChanBlock + kk;
            if (k >= K) continue;
            const long long e0 = (((long long)img * K + k) * H + h0) * W;         // first element of the run
            const long long p0 = (e0 & ~(long long)(PE - 1)) + (long long)kq * PE;   // piece, aligned in y
            const int rel = (int)(p0 - e0);                                        // -(PE-1) .. run-1 if needed
            if (rel >= run) continue;
            // (row, column) of the piece's first element inside the run, then step along it
            const int q = rel < 0 ? 0 : rel;
            int hr = (int)__umulhi((unsigned)q, sh.w_magic);
            int w = q - hr * W;
            const T *src = lds + kk * sh.k_pitch;
            T val[PE];
#pragma unroll
            for (int e = 0; e < PE; ++e) {
                const int pos = rel + e;
                val[e] = (T)0.0f;
                if (pos >= 0 && pos < run) {
                    val[e] = src[hr * sh.cols_pitch + w];
                    if (++w == W) { w = 0; ++hr; }
                }
            }
            if (rel >= 0 && rel + PE <= run) {
                u32x4 piece;
                __builtin_memcpy(&piece, val, 16);
                __builtin_nontemporal_store(piece, reinterpret_cast<u32x4 *>(y + p0));
            } else {
#pragma unroll
                for (int e = 0; e < PE; ++e)
                    if (rel + e >= 0 && rel + e < run) y[p0 + e] = val[e];
            }
        }
    } else {
        const unsigned magic = (unsigned)((((unsigned long long)1 << 32) + cols - 1) / cols);
        const int slots = kChanBlock * sh.rows * cols;
        for (int s = threadIdx.x; s < slots; s += (int)blockDim.x) {
            const int line = cols > 1 ? (int)__umulhi((unsigned)s, magic) : s;
            const int q = s - line * cols;
            const int kk = (int)__umulhi((unsigned)line, sh.rows_magic), p = line - kk * sh.rows;
            const int k = kb * kChanBlock + kk, h = tr * M + p;
            if (k >= K || h >= H) continue;
            y[(((size_t)img * K + k) * H + h) * W + w0 + q] = lds[kk * sh.k_pitch + p * sh.cols_pitch + q];
        }
    }
}

template <int N, int R>
static void fill_out_coef(const nova_transforms *t, OutCoef<N, R> &k)
{
    constexpr int M = N - R + 1, H = OutCoef<N, R>::H;
    for (int i = 0; i < N * M; ++i) k.a[i] = t->A32[i];
    for (int j = 0; j < H; ++j)
        for (int i = 0; i < M; ++i) k.pw[j * M + i] = t->A32[(2 * j + 1) * M + i];
    k.zero = t->A32[0];
    k.inf = t->A32[(N - 1) * M + (M - 1)];
}

template <int N, int R, typename T>
static size_t out_shape(int twb, int trb, OutShape &sh)
{
    constexpr int M = N - R + 1;
    sh.twb = twb * trb;
    sh.twc = twb;
    sh.trb = trb;
    sh.rows = trb * M;
    sh.rows_magic = (unsigned)((((unsigned long long)1 << 32) + sh.rows - 1) / sh.rows);
    sh.cols_pitch = (twb * M + 3) / 4 * 4;              // rows stay 8-byte aligned
    int kp = sh.rows * sh.cols_pitch;                   // multiple of 4
    // channel pitch 4 * odd elements: 8-byte aligned rows, and the 32 channels of a half-wave
    // writing one (row, column) fall into different banks
    if ((kp / 4) % 2 == 0) kp += 4;
    sh.k_pitch = kp;
    sh.pieces = 1; sh.piece_magic = 0; sh.w_magic = 0;
    sh.pool = 0;
    sh.half_rows_magic = sh.rows / 2 > 1 ? (unsigned)((((unsigned long long)1 << 32) + sh.rows / 2 - 1) / (sh.rows / 2)) : 0;
    return (size_t)kChanBlock * kp * sizeof(T);
}


}  // namespace nova
