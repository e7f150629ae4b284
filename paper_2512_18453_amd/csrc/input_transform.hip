// Input transform V = B^T d B (Sec. 2.1 step 1, nested in 2D) for every n x n tile of the
// zero-padded image, x [N][C][H][W] -> V [n*n][C/32][T][32].
//
// One workgroup takes one image, one tile row, a group of TWB neighbouring tiles and one block
// of 32 channels.  The (n rows) x (TWB*m + 2 columns) x 32-channel input strip is staged in LDS
// with the channel index fastest, so that global reads run along W and the per-thread tile reads
// (thread = one tile x one channel, 32 consecutive lanes = 32 consecutive channels) hit 32
// different LDS words.  Each thread then transforms its tile in registers and writes n*n values,
// 64 (fp16) or 128 (fp32) contiguous bytes per half-wave and position xi; the TWB tiles of the
// group are adjacent in t, so a workgroup writes TWB*64 contiguous bytes per xi.
//
// Arithmetic contract (binary32): a 1D transform row is E + O, with E / O fused multiply-add
// chains over the even / odd input indices in ascending order, columns of the tile first, then
// rows.  For points given as 0, +a, -a, ... the rows of +a and -a share E and O (the even
// coefficients agree, the odd ones are negated), which gives bit-identical results at half the
// multiplications.  The result is rounded once to the storage format.
#include "device_common.hpp"

namespace nova {

template <int N, bool SYM>
__device__ __forceinline__ void input_transform_1d(const float (&v)[N], float (&out)[N], const InCoef<N> &k)
{
    constexpr int H = (N - 2) / 2;
    if constexpr (SYM) {
        float e0 = 0.0f;
#pragma unroll
        for (int q = 0; q <= H; ++q) e0 = fma32(k.zero[q], v[2 * q], e0);
        out[0] = e0;
#pragma unroll
        for (int j = 0; j < H; ++j) {
            float E = 0.0f, O = 0.0f;
#pragma unroll
            for (int q = 0; q < H; ++q) E = fma32(k.ev[j * H + q], v[2 * q + 2], E);
#pragma unroll
            for (int q = 0; q < H; ++q) O = fma32(k.od[j * H + q], v[2 * q + 1], O);
            out[2 * j + 1] = E + O;
            out[2 * j + 2] = E - O;
        }
        float oi = 0.0f;
#pragma unroll
        for (int q = 0; q <= H; ++q) oi = fma32(k.inf[q], v[2 * q + 1], oi);
        out[N - 1] = oi;
    } else {
#pragma unroll
        for (int p = 0; p < N; ++p) {
            float E = 0.0f, O = 0.0f;
#pragma unroll
            for (int a = 0; a < N; a += 2) E = fma32(k.bt[p * N + a], v[a], E);
#pragma unroll
            for (int a = 1; a < N; a += 2) O = fma32(k.bt[p * N + a], v[a], O);
            out[p] = E + O;
        }
    }
}

template <typename T> struct LdsPitch;
template <> struct LdsPitch<f16> { static constexpr int value = kChanBlock + 2; };   // 17 words: odd
template <> struct LdsPitch<float> { static constexpr int value = kChanBlock + 1; }; // 33 words: odd

template <int N, typename T, bool SYM>
__global__ void __launch_bounds__(512)
input_transform_kernel(const T *__restrict__ x, T *__restrict__ V, int C, int H, int W,
                       int tiles_h, int tiles_w, int twb, int groups, int c_blocks, long long Ttot,
                       InCoef<N> coef)
{
    constexpr int M = N - 2;
    constexpr int CP = LdsPitch<T>::value;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    T *lds = reinterpret_cast<T *>(lds_raw);

    // block -> (image, channel block, tile row, tile group); group fastest
    unsigned bid = xcd_local_block_id(blockIdx.x, gridDim.x);
    const int tg = bid % groups; bid /= groups;
    const int tr = bid % tiles_h; bid /= tiles_h;
    const int cb = bid % c_blocks; bid /= c_blocks;
    const int img = bid;

    const int tc0 = tg * twb;
    const int cols = twb * M + 2;
    const int h_lo = tr * M - 1;          // image row of strip row 0
    const int w_lo = tc0 * M - 1;         // image column of strip column 0

    // ---- stage the strip: one (channel, row) line per wave iteration, lanes along W
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int n_waves = (blockDim.x + 63) >> 6;
    for (int line = wave; line < kChanBlock * N; line += n_waves) {
        const int c_in = line / N, a = line - c_in * N;
        const int c = cb * kChanBlock + c_in;
        const int h = h_lo + a;
        const bool row_ok = c < C && h >= 0 && h < H;
        const T *src = x + (((size_t)img * C + (row_ok ? c : 0)) * H + (row_ok ? h : 0)) * W;
        for (int col = lane; col < cols; col += 64) {
            const int w = w_lo + col;
            T val = (T)0.0f;
            if (row_ok && w >= 0 && w < W) val = src[w];
            lds[(a * cols + col) * CP + c_in] = val;
        }
    }
    __syncthreads();

    // ---- transform: thread = (tile j of the group, channel c_in)
    const int j = threadIdx.x >> 5, c_in = threadIdx.x & 31;
    if (j >= twb || tc0 + j >= tiles_w) return;

    float tmp[N][N];
#pragma unroll
    for (int b = 0; b < N; ++b) {
        float d[N], o[N];
#pragma unroll
        for (int a = 0; a < N; ++a) d[a] = load_f32(&lds[(a * cols + j * M + b) * CP + c_in]);
        input_transform_1d<N, SYM>(d, o, coef);
#pragma unroll
        for (int i = 0; i < N; ++i) tmp[i][b] = o[i];
    }

    const long long t = ((long long)img * tiles_h + tr) * tiles_w + tc0 + j;
    const size_t xi_stride = (size_t)c_blocks * Ttot * kChanBlock;
    T *dst = V + ((size_t)cb * Ttot + t) * kChanBlock + c_in;
#pragma unroll
    for (int i = 0; i < N; ++i) {
        float o[N];
        input_transform_1d<N, SYM>(tmp[i], o, coef);
#pragma unroll
        for (int jj = 0; jj < N; ++jj) store_rounded_twice(dst + (size_t)(i * N + jj) * xi_stride, o[jj]);
    }
}

template <int N>
static void fill_in_coef(const nova_transforms *t, InCoef<N> &k)
{
    constexpr int H = InCoef<N>::H;
    for (int i = 0; i < N * N; ++i) k.bt[i] = t->BT32[i];
    for (int q = 0; q <= H; ++q) {
        k.zero[q] = t->BT32[0 * N + 2 * q];
        k.inf[q] = t->BT32[(N - 1) * N + 2 * q + 1];
    }
    for (int j = 0; j < H; ++j)
        for (int q = 0; q < H; ++q) {
            k.ev[j * H + q] = t->BT32[(2 * j + 1) * N + 2 * q + 2];
            k.od[j * H + q] = t->BT32[(2 * j + 1) * N + 2 * q + 1];
        }
}

template <int N, typename T>
static int launch_it(const nova_transforms *t, const void *x, void *V, const Geometry &g, hipStream_t stream)
{
    constexpr int M = N - 2;
    constexpr int CP = LdsPitch<T>::value;
    InCoef<N> coef;
    fill_in_coef<N>(t, coef);
    // tiles per group: at most 16 (512 threads) and an LDS strip of at most 64 KiB
    const int lds_budget = 64 * 1024;
    int twb_max = (lds_budget / (int)(N * CP * sizeof(T)) - 2) / M;
    twb_max = twb_max > 16 ? 16 : (twb_max < 1 ? 1 : twb_max);
    const int groups = ceil_div(g.tiles_w, twb_max);
    const int twb = ceil_div(g.tiles_w, groups);
    const size_t lds_bytes = (size_t)N * (twb * M + 2) * CP * sizeof(T);
    const int threads = ((twb * 32 + 63) / 64) * 64;
    const long long blocks = (long long)groups * g.tiles_h * g.c_blocks * g.N;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return (int)hipErrorInvalidValue;
    auto kern = t->symmetric ? input_transform_kernel<N, T, true> : input_transform_kernel<N, T, false>;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(threads), lds_bytes, stream,
                       (const T *)x, (T *)V, g.C, g.H, g.W, g.tiles_h, g.tiles_w, twb, groups,
                       g.c_blocks, g.T, coef);
    return (int)hipGetLastError();
}

int launch_input_transform(const nova_transforms *t, const void *x, void *V, const Geometry &g,
                           int dtype, void *stream)
{
    hipStream_t s = (hipStream_t)stream;
    const bool h = dtype == NOVA_F16;
    switch (t->n) {
    case 4: return h ? launch_it<4, f16>(t, x, V, g, s) : launch_it<4, float>(t, x, V, g, s);
    case 6: return h ? launch_it<6, f16>(t, x, V, g, s) : launch_it<6, float>(t, x, V, g, s);
    case 8: return h ? launch_it<8, f16>(t, x, V, g, s) : launch_it<8, float>(t, x, V, g, s);
    case 10: return h ? launch_it<10, f16>(t, x, V, g, s) : launch_it<10, float>(t, x, V, g, s);
    default: return (int)hipErrorInvalidValue;
    }
}

}  // namespace nova
