// Output transform Y = A^T M A (Sec. 2.1 step 4, nested in 2D), cropped to H x W and written as
// y [N][K][H][W];  M [n*n][K/32][Tp][32] holds the channel-summed products (Tp = T rounded up to
// a multiple of 128; the extra rows are never read).
//
// One workgroup takes one image, one tile row, a group of TWB neighbouring tiles (for narrow
// images, where a tile row has few tiles: TRB neighbouring tile rows of full width) and one block of
// 32 output channels; thread = one tile x one channel, so the n*n loads of a half-wave are 128
// (fp32 M) contiguous bytes each and a workgroup reads TWB*128 contiguous bytes per xi.  The
// m x m results go through LDS so that the global stores run along W.
// For points given as 0, +a, -a, ... the rows of +a and -a enter only through their sum (even
// output index) or difference (odd output index), which halves the multiplications.  Binary32
// arithmetic, one rounding to the storage format at the store; optional fused ReLU.
//
// Few input channels (C <= 4, the first layer of an image network): the products are not read
// from M but formed here, M[xi][t][k] = sum_c V[xi][t][c] U[xi][k][c] as a binary32 multiply-add
// chain over c (the factors are exact in binary32), from V in a compact layout Vc [n*n][T][4] and a packed copy
// Uc [n*n][Kp][4] of the first four channels of U.  M, n*n*T*K values that would be written and
// read once whatever C is, then never exists.
#include <type_traits>

#include "output_common.hpp"

namespace nova {

// channels the few-channel path covers (one 8-byte binary16 / 16-byte binary32 load per operand)
constexpr int kFewChannels = 4;

// CF = 0: products read from Mp (MT: their type).  CF = kFewChannels: products formed from Vp
// [n*n][Ttot][CF] and Uc [n*n][k_blocks*32][CF]; MT = f16 rounds each product to binary16 first,
// as storing M in binary16 would.
template <int N, int R, typename T, typename MT, bool SYM, int STG, bool RELU, int CF>
__global__ void __launch_bounds__(512)
output_transform_kernel(const MT *__restrict__ Mp, const T *__restrict__ Vp, const T *__restrict__ Uc,
                        T *__restrict__ y, int K, int H, int W,
                        int tiles_h, int tiles_w, int k_blocks, long long Ttot, OutShape sh,
                        OutCoef<N, R> coef)
{
    constexpr int M = N - R + 1;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    T *lds = reinterpret_cast<T *>(lds_raw);

    unsigned bid = xcd_local_block_id(blockIdx.x, gridDim.x);
    const int row_groups = (tiles_h + sh.trb - 1) / sh.trb;
    const int tg = bid % sh.groups; bid /= sh.groups;
    const int tr = (bid % row_groups) * sh.trb; bid /= row_groups;      // first tile row of the group
    const int kb = bid % k_blocks; bid /= k_blocks;
    const int img = bid;
    const int tc0 = sh.trb > 1 ? 0 : tg * sh.twb;

    if constexpr (CF > 0) {
        // few-channel path: what the workgroup needs of V ([tile of the group][xi][CF]) and of the
        // packed filters ([xi][32 channels][CF]) goes to LDS first, all loads in flight together;
        // the region is reused for the output block once every thread has its results
        typedef T few_t __attribute__((ext_vector_type(CF > 0 ? CF : 1)));
        few_t *Vs = reinterpret_cast<few_t *>(lds), *Us = Vs + N * N * sh.twb;
        const few_t *Vg = reinterpret_cast<const few_t *>(Vp), *Ug = reinterpret_cast<const few_t *>(Uc);
        for (int s = threadIdx.x; s < N * N * sh.twb; s += (int)blockDim.x) {
            const int xi = s / sh.twb, jj = s - xi * sh.twb;
            int sr = 0, sc = jj;
            if (sh.trb > 1) { sr = jj / tiles_w; sc = jj - sr * tiles_w; }
            few_t val;
#pragma unroll
            for (int c = 0; c < CF; ++c) val[c] = (T)0.0f;
            if (tc0 + sc < tiles_w && tr + sr < tiles_h) {
                const long long t = ((long long)img * tiles_h + tr + sr) * tiles_w + tc0 + sc;
                val = Vg[(size_t)xi * Ttot + t];
            }
            Vs[jj * (N * N) + xi] = val;
        }
        for (int s = threadIdx.x; s < N * N * kChanBlock; s += (int)blockDim.x) {
            const int xi = s / kChanBlock, kk = s - xi * kChanBlock;
            Us[s] = Ug[((size_t)xi * k_blocks + kb) * kChanBlock + kk];
        }
        __syncthreads();
    }

    const int j = threadIdx.x >> 5, k_in = threadIdx.x & 31;
    int jr = 0, jc = j;                       // tile row and column inside the group
    if (sh.trb > 1) { jr = j / tiles_w; jc = j - jr * tiles_w; }
    const bool active = j < sh.twb && tc0 + jc < tiles_w && tr + jr < tiles_h;
    // (few-channel path: the results wait in registers, binary16 ones two to a register, until every
    // thread has read its operands)
    typedef typename std::conditional<sizeof(T) == 2, unsigned int, float>::type held_t;
    constexpr int kHeldPer = sizeof(T) == 2 ? 2 : 1;
    held_t held[CF > 0 ? (M * M + kHeldPer - 1) / kHeldPer : 1];
    if (active) {
        const long long t = ((long long)img * tiles_h + tr + jr) * tiles_w + tc0 + jc;
        // plane base of each xi is uniform (scalar registers); the offset inside the plane is per
        // thread and fits 32 bits (checked by the launcher)
        const size_t xi_stride = (size_t)k_blocks * Ttot * kChanBlock;
        const unsigned in_plane = (unsigned)((((size_t)kb * Ttot + t) * kChanBlock + k_in) * sizeof(MT));   // bytes

        float z[M][N];                    // A^T M, column by column
#pragma unroll
        for (int b = 0; b < N; ++b) {
            float v[N], o[M];
            if constexpr (CF > 0) {
                typedef T few_t __attribute__((ext_vector_type(CF > 0 ? CF : 1)));
                const few_t *Vs = reinterpret_cast<const few_t *>(lds) + j * (N * N), *Us = reinterpret_cast<const few_t *>(lds) + N * N * sh.twb + k_in;
                few_t vv[N], uu[N];
#pragma unroll
                for (int a = 0; a < N; ++a) {
                    vv[a] = Vs[a * N + b];
                    uu[a] = Us[(a * N + b) * kChanBlock];
                }
#pragma unroll
                for (int a = 0; a < N; ++a) {
                    float acc = 0.0f;
#pragma unroll
                    for (int c = 0; c < CF; ++c) acc = fma32((float)vv[a][c], (float)uu[a][c], acc);
                    if constexpr (sizeof(MT) == 2) acc = (float)round_twice(acc, (f16 *)nullptr);
                    v[a] = acc;
                }
            } else {
#pragma unroll
                for (int a = 0; a < N; ++a) {
                    const NOVA_GLOBAL MT *src = plane_element(Mp + (size_t)(a * N + b) * xi_stride, in_plane);
                    // last use of M.  In binary32 it is the largest tensor of the call and is read with the
                    // streaming hint, so that it leaves the last-level cache behind it; in binary16 the
                    // hint measured slower (its lines are better left to be overwritten in the cache)
                    if constexpr (sizeof(MT) == 4) v[a] = (float)__builtin_nontemporal_load(src);
                    else v[a] = (float)*src;
                }
            }
            output_transform_1d<N, R, SYM>(v, o, coef);
#pragma unroll
            for (int p = 0; p < M; ++p) z[p][b] = o[p];
        }
        T *dst = lds + k_in * sh.k_pitch + jr * M * sh.cols_pitch + jc * M;
#pragma unroll
        for (int p = 0; p < M; ++p) {
            float o[M];
            output_transform_1d<N, R, SYM>(z[p], o, coef);
#pragma unroll
            for (int q = 0; q < M; ++q) {
                float val = o[q];
                if constexpr (RELU) val = val < 0.0f ? 0.0f : val;      // NaN stays NaN
                if constexpr (CF > 0) {
                    if constexpr (sizeof(T) == 2) {
                        const f16 hv = (f16)val;
                        unsigned short bits;
                        __builtin_memcpy(&bits, &hv, 2);
                        const int at = p * M + q;
                        if ((at & 1) == 0) held[at >> 1] = bits;
                        else held[at >> 1] |= (unsigned int)bits << 16;
                    } else {
                        held[p * M + q] = val;
                    }
                } else {
                    store_from_f32(dst + p * sh.cols_pitch + q, val);
                }
            }
        }
    }
    if constexpr (CF > 0) {
        __syncthreads();                      // the operands in LDS have been read
        if (active) {
            T *dst = lds + k_in * sh.k_pitch + jr * M * sh.cols_pitch + jc * M;
#pragma unroll
            for (int p = 0; p < M; ++p)
#pragma unroll
                for (int q = 0; q < M; ++q) {
                    const int at = p * M + q;
                    if constexpr (sizeof(T) == 2) {
                        const unsigned short bits = (unsigned short)(held[at >> 1] >> ((at & 1) * 16));
                        __builtin_memcpy(dst + p * sh.cols_pitch + q, &bits, 2);
                    } else {
                        __builtin_memcpy(dst + p * sh.cols_pitch + q, &held[at], 4);
                    }
                }
        }
    }
    __syncthreads();

    store_output_block<T, M, STG>(lds, y, img, kb, tr, tc0, K, H, W, tiles_w, sh);
}

// Uc[xi][k][c] = U[xi][0][k][c] for c < kFewChannels (U [n*n][1][Kp][32])
template <typename T>
__global__ void __launch_bounds__(256)
pack_few_channels_kernel(const T *__restrict__ U, T *__restrict__ Uc, long long rows)
{
    const long long row = (long long)blockIdx.x * blockDim.x + threadIdx.x;      // (xi, k)
    if (row >= rows) return;
#pragma unroll
    for (int c = 0; c < kFewChannels; ++c) Uc[row * kFewChannels + c] = U[row * kChanBlock + c];
}

// CF = 0: Mp holds the products.  CF = kFewChannels: Mp is V, and `few_u` the packed filters.
template <int N, int R, typename T, typename MT, int CF>
static int launch_ot(const nova_transforms *t, const void *Mp, const void *few_u, void *y, const Geometry &g, int flags,
                     hipStream_t stream)
{
    constexpr int M = N - R + 1;
    constexpr int PE = 16 / (int)sizeof(T);
    OutCoef<N, R> coef;
    fill_out_coef<N, R>(t, coef);
    OutShape sh;
    // LDS of a group: the output block, and on the few-channel path the staged operands in the same region
    auto lds_need = [&](int twb, int trb) {
        size_t need = out_shape<N, R, T>(twb, trb, sh);
        if (CF > 0) {
            const size_t staged = (size_t)N * N * (twb * trb + kChanBlock) * CF * sizeof(T);
            if (staged > need) need = staged;
        }
        return need;
    };
    // (few-channel path: smaller groups, so that more of them fit a compute unit: nothing is gained from
    // wide reads of M there)
    int twb_max = CF > 0 ? 8 : 16;
    while (twb_max > 1 && lds_need(twb_max, 1) > 64 * 1024) --twb_max;
    sh.groups = ceil_div(g.tiles_w, twb_max);
    const int twb = ceil_div(g.tiles_w, sh.groups);     // tiles of one tile row per group
    // narrow images: a group spans the width; give it as many tile rows as keep it within 8 tiles
    // (more per workgroup measured slower: 56 x 56 with 2 x 7 tiles 42 us against 39 us with 7)
    int trb = 1;
    if (sh.groups == 1) {
        trb = 8 / twb;
        if (trb < 1) trb = 1;
        if (trb > g.tiles_h) trb = g.tiles_h;
        while (trb > 1 && lds_need(twb, trb) > 64 * 1024) --trb;
    }
    trb = ceil_div(g.tiles_h, ceil_div(g.tiles_h, trb));    // same number of groups, evenly sized
    const size_t lds_bytes = lds_need(twb, trb);           // (leaves sh.groups alone)
    if (lds_bytes > 64 * 1024) return (int)hipErrorInvalidValue;
    if (CF == 0 && (size_t)g.k_blocks * g.Tp * kChanBlock * sizeof(MT) >= ((size_t)1 << 32)) return (int)hipErrorInvalidValue;
    if (CF > 0 && g.C > CF) return (int)hipErrorInvalidValue;
    const bool aligned = ((uintptr_t)y % 16) == 0;
    const bool vec = g.W % PE == 0 && aligned && (sh.groups == 1 || (twb * M) % PE == 0);
    // (W >= 2 and at least two pieces: the reciprocals used for the divisions do not exist for 1)
    const bool flat = !vec && aligned && sh.groups == 1 && g.W >= 2 && sh.rows * g.W + 2 * (PE - 1) >= 2 * PE &&
                      (long long)sh.rows * g.W < (1 << 15);
    if (flat) {
        sh.pieces = (sh.rows * g.W + 2 * (PE - 1)) / PE;
        sh.piece_magic = (unsigned)((((unsigned long long)1 << 32) + sh.pieces - 1) / sh.pieces);
        sh.w_magic = (unsigned)((((unsigned long long)1 << 32) + g.W - 1) / g.W);
    }
    sh.pool = (flags & NOVA_FLAG_POOL2) ? 1 : 0;
    const int threads = ((sh.twb * 32 + 63) / 64) * 64;
    const long long blocks = (long long)sh.groups * ceil_div(g.tiles_h, trb) * g.k_blocks * g.N;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return (int)hipErrorInvalidValue;
    void (*kern)(const MT *, const T *, const T *, T *, int, int, int, int, int, int, long long, OutShape, OutCoef<N, R>);
    const bool relu = (flags & NOVA_FLAG_RELU) != 0;
    const int stg = vec ? kStoreVec : flat ? kStoreFlat : kStoreScalar;
    auto pick = [&](auto sym) {
        constexpr bool S = decltype(sym)::value;
        switch (stg) {
        case kStoreVec:  return relu ? output_transform_kernel<N, R, T, MT, S, kStoreVec, true, CF> : output_transform_kernel<N, R, T, MT, S, kStoreVec, false, CF>;
        case kStoreFlat: return relu ? output_transform_kernel<N, R, T, MT, S, kStoreFlat, true, CF> : output_transform_kernel<N, R, T, MT, S, kStoreFlat, false, CF>;
        default:         return relu ? output_transform_kernel<N, R, T, MT, S, kStoreScalar, true, CF> : output_transform_kernel<N, R, T, MT, S, kStoreScalar, false, CF>;
        }
    };
    kern = t->symmetric ? pick(std::true_type{}) : pick(std::false_type{});
    if constexpr (CF > 0)
        hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(threads), lds_bytes, stream,
                           (const MT *)nullptr, (const T *)Mp, (const T *)few_u, (T *)y, g.K, g.H, g.W, g.tiles_h, g.tiles_w,
                           g.k_blocks, g.T, sh, coef);
    else
        hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(threads), lds_bytes, stream,
                           (const MT *)Mp, (const T *)nullptr, (const T *)nullptr, (T *)y, g.K, g.H, g.W, g.tiles_h,
                           g.tiles_w, g.k_blocks, g.Tp, sh, coef);
    return (int)hipGetLastError();
}

template <int N, int R, int CF>
static int launch_ot_n(const nova_transforms *t, const void *Mp, const void *few_u, void *y, const Geometry &g, int dtype,
                       int flags, hipStream_t s)
{
    if (dtype == NOVA_F32) return launch_ot<N, R, float, float, CF>(t, Mp, few_u, y, g, flags, s);
    if (flags & NOVA_FLAG_M_F16) return launch_ot<N, R, f16, f16, CF>(t, Mp, few_u, y, g, flags, s);
    return launch_ot<N, R, f16, float, CF>(t, Mp, few_u, y, g, flags, s);
}

template <int CF>
static int launch_ot_any(const nova_transforms *t, const void *Mp, const void *few_u, void *y, const Geometry &g,
                         int dtype, int flags, hipStream_t s)
{
    if (t->r == 3) {
        switch (t->n) {
        case 4: return launch_ot_n<4, 3, CF>(t, Mp, few_u, y, g, dtype, flags, s);
        case 6: return launch_ot_n<6, 3, CF>(t, Mp, few_u, y, g, dtype, flags, s);
        case 8: return launch_ot_n<8, 3, CF>(t, Mp, few_u, y, g, dtype, flags, s);
        case 10: return launch_ot_n<10, 3, CF>(t, Mp, few_u, y, g, dtype, flags, s);
        }
    } else if (t->r == 5) {
        switch (t->n) {
        case 6: return launch_ot_n<6, 5, CF>(t, Mp, few_u, y, g, dtype, flags, s);
        case 8: return launch_ot_n<8, 5, CF>(t, Mp, few_u, y, g, dtype, flags, s);
        case 10: return launch_ot_n<10, 5, CF>(t, Mp, few_u, y, g, dtype, flags, s);
        }
    }
    return (int)hipErrorInvalidValue;
}

int launch_output_transform(const nova_transforms *t, const void *Mp, void *y, const Geometry &g,
                            int dtype, int flags, void *stream)
{
    return launch_ot_any<0>(t, Mp, nullptr, y, g, dtype, flags, (hipStream_t)stream);
}

int few_channels_limit() { return kFewChannels; }

size_t few_channels_filter_bytes(const Geometry &g, int dtype)
{
    return (size_t)g.n * g.n * g.Kp * kFewChannels * dtype_size(dtype);
}

int launch_pack_few_channels(const void *U, void *Uc, const Geometry &g, int dtype, void *stream)
{
    const long long rows = (long long)g.n * g.n * g.Kp;
    const unsigned blocks = (unsigned)((rows + 255) / 256);
    if (dtype == NOVA_F16)
        hipLaunchKernelGGL(pack_few_channels_kernel<f16>, dim3(blocks), dim3(256), 0, (hipStream_t)stream,
                           (const f16 *)U, (f16 *)Uc, rows);
    else
        hipLaunchKernelGGL(pack_few_channels_kernel<float>, dim3(blocks), dim3(256), 0, (hipStream_t)stream,
                           (const float *)U, (float *)Uc, rows);
    return (int)hipGetLastError();
}

int launch_output_transform_few(const nova_transforms *t, const void *V, const void *Uc, void *y,
                                const Geometry &g, int dtype, int flags, void *stream)
{
    return launch_ot_any<kFewChannels>(t, V, Uc, y, g, dtype, flags, (hipStream_t)stream);
}

}  // namespace nova
