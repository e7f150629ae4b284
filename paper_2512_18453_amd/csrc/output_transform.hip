// Output transform Y = A^T M A (Sec. 2.1 step 4, nested in 2D), cropped to H x W and written as
// y [N][K][H][W];  M [n*n][K/32][T][32] holds the channel-summed products.
//
// One workgroup takes one image, one tile row, a group of TWB neighbouring tiles and one block of
// 32 output channels; thread = one tile x one channel, so the n*n loads of a half-wave are 128
// (fp32 M) contiguous bytes each and a workgroup reads TWB*128 contiguous bytes per xi.  The
// m x m results go through LDS so that the global stores run along W.
// For points given as 0, +a, -a, ... the rows of +a and -a enter only through their sum (even
// output index) or difference (odd output index), which halves the multiplications.  Binary32
// arithmetic, one rounding to the storage format at the store; optional fused ReLU.
#include "device_common.hpp"

namespace nova {

template <int N, bool SYM>
__device__ __forceinline__ void output_transform_1d(const float (&v)[N], float (&out)[N - 2], const OutCoef<N> &k)
{
    constexpr int M = N - 2;
    constexpr int H = (N - 2) / 2;
    if constexpr (SYM) {
        float s[H > 0 ? H : 1], d[H > 0 ? H : 1];
#pragma unroll
        for (int j = 0; j < H; ++j) {
            s[j] = v[2 * j + 1] + v[2 * j + 2];
            d[j] = v[2 * j + 1] - v[2 * j + 2];
        }
        float y0 = v[0];
#pragma unroll
        for (int j = 0; j < H; ++j) y0 += s[j];
        out[0] = y0;
#pragma unroll
        for (int i = 1; i < M; ++i) {
            float acc = (i == M - 1) ? v[N - 1] : 0.0f;
#pragma unroll
            for (int j = 0; j < H; ++j) acc = fma32(k.pw[j * M + i], (i & 1) ? d[j] : s[j], acc);
            out[i] = acc;
        }
        if constexpr (M == 1) out[0] += v[N - 1];
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

template <int N, typename T, typename MT, bool SYM>
__global__ void __launch_bounds__(512)
output_transform_kernel(const MT *__restrict__ Mp, T *__restrict__ y, int K, int H, int W,
                        int tiles_h, int tiles_w, int twb, int groups, int k_blocks, long long Ttot,
                        int cols_pitch, int k_pitch, int relu, OutCoef<N> coef)
{
    constexpr int M = N - 2;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    T *lds = reinterpret_cast<T *>(lds_raw);

    unsigned bid = xcd_local_block_id(blockIdx.x, gridDim.x);
    const int tg = bid % groups; bid /= groups;
    const int tr = bid % tiles_h; bid /= tiles_h;
    const int kb = bid % k_blocks; bid /= k_blocks;
    const int img = bid;
    const int tc0 = tg * twb;

    const int j = threadIdx.x >> 5, k_in = threadIdx.x & 31;
    if (j < twb && tc0 + j < tiles_w) {
        const long long t = ((long long)img * tiles_h + tr) * tiles_w + tc0 + j;
        const size_t xi_stride = (size_t)k_blocks * Ttot * kChanBlock;
        const MT *src = Mp + ((size_t)kb * Ttot + t) * kChanBlock + k_in;

        float z[M][N];                    // A^T M, column by column
#pragma unroll
        for (int b = 0; b < N; ++b) {
            float v[N], o[M];
#pragma unroll
            for (int a = 0; a < N; ++a) v[a] = load_f32(src + (size_t)(a * N + b) * xi_stride);
            output_transform_1d<N, SYM>(v, o, coef);
#pragma unroll
            for (int p = 0; p < M; ++p) z[p][b] = o[p];
        }
        T *dst = lds + k_in * k_pitch + j * M;
#pragma unroll
        for (int p = 0; p < M; ++p) {
            float o[M];
            output_transform_1d<N, SYM>(z[p], o, coef);
#pragma unroll
            for (int q = 0; q < M; ++q) {
                float val = o[q];
                if (relu) val = val < 0.0f ? 0.0f : val;      // NaN stays NaN
                store_from_f32(dst + p * cols_pitch + q, val);
            }
        }
    }
    __syncthreads();

    // ---- store: one (channel, row) line per wave iteration, lanes along W
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int n_waves = (blockDim.x + 63) >> 6;
    const int w0 = tc0 * M;
    int cols = twb * M;
    if (w0 + cols > W) cols = W - w0;
    for (int line = wave; line < kChanBlock * M; line += n_waves) {
        const int kk = line / M, p = line - kk * M;
        const int k = kb * kChanBlock + kk;
        const int h = tr * M + p;
        if (k >= K || h >= H) continue;
        T *out = y + (((size_t)img * K + k) * H + h) * W + w0;
        const T *in = lds + kk * k_pitch + p * cols_pitch;
        for (int col = lane; col < cols; col += 64) out[col] = in[col];
    }
}

template <int N>
static void fill_out_coef(const nova_transforms *t, OutCoef<N> &k)
{
    constexpr int M = N - 2, H = OutCoef<N>::H;
    for (int i = 0; i < N * M; ++i) k.a[i] = t->A32[i];
    for (int j = 0; j < H; ++j)
        for (int i = 0; i < M; ++i) k.pw[j * M + i] = t->A32[(2 * j + 1) * M + i];
}

template <int N, typename T, typename MT>
static int launch_ot(const nova_transforms *t, const void *Mp, void *y, const Geometry &g, int flags,
                     hipStream_t stream)
{
    constexpr int M = N - 2;
    OutCoef<N> coef;
    fill_out_coef<N>(t, coef);
    const int lds_budget = 64 * 1024;
    int twb_max = (lds_budget / (int)(kChanBlock * M * sizeof(T)) - 4) / M;
    twb_max = twb_max > 16 ? 16 : (twb_max < 1 ? 1 : twb_max);
    const int groups = ceil_div(g.tiles_w, twb_max);
    const int twb = ceil_div(g.tiles_w, groups);
    const int cols_pitch = twb * M;
    // per-channel pitch: an odd number of 32-bit words, so that the 32 channels of a half-wave
    // land in different banks when they write the same (row, column)
    int k_pitch = M * cols_pitch;
    if (sizeof(T) == 2) { while ((k_pitch % 2) != 0 || ((k_pitch / 2) % 2) == 0) ++k_pitch; }
    else                { while ((k_pitch % 2) == 0) ++k_pitch; }
    const size_t lds_bytes = (size_t)kChanBlock * k_pitch * sizeof(T);
    const int threads = ((twb * 32 + 63) / 64) * 64;
    const long long blocks = (long long)groups * g.tiles_h * g.k_blocks * g.N;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return (int)hipErrorInvalidValue;
    auto kern = t->symmetric ? output_transform_kernel<N, T, MT, true> : output_transform_kernel<N, T, MT, false>;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(threads), lds_bytes, stream,
                       (const MT *)Mp, (T *)y, g.K, g.H, g.W, g.tiles_h, g.tiles_w, twb, groups,
                       g.k_blocks, g.T, cols_pitch, k_pitch, (flags & NOVA_FLAG_RELU) ? 1 : 0, coef);
    return (int)hipGetLastError();
}

template <int N>
static int launch_ot_n(const nova_transforms *t, const void *Mp, void *y, const Geometry &g, int dtype,
                       int flags, hipStream_t s)
{
    if (dtype == NOVA_F32) return launch_ot<N, float, float>(t, Mp, y, g, flags, s);
    if (flags & NOVA_FLAG_M_F16) return launch_ot<N, f16, f16>(t, Mp, y, g, flags, s);
    return launch_ot<N, f16, float>(t, Mp, y, g, flags, s);
}

int launch_output_transform(const nova_transforms *t, const void *Mp, void *y, const Geometry &g,
                            int dtype, int flags, void *stream)
{
    hipStream_t s = (hipStream_t)stream;
    switch (t->n) {
    case 4: return launch_ot_n<4>(t, Mp, y, g, dtype, flags, s);
    case 6: return launch_ot_n<6>(t, Mp, y, g, dtype, flags, s);
    case 8: return launch_ot_n<8>(t, Mp, y, g, dtype, flags, s);
    case 10: return launch_ot_n<10>(t, Mp, y, g, dtype, flags, s);
    default: return (int)hipErrorInvalidValue;
    }
}

}  // namespace nova
