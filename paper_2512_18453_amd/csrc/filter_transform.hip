// Filter transform U = G g G^T (Sec. 2.1 step 2, nested in 2D) of R x R kernels, one thread per
// (k, c) pair.
// Evaluated in binary64 with G rounded once to binary64, result rounded once to the storage
// format, written in the channel-blocked layout U[xi][c/32][Kp][32] (zero in the padding).
// Runs once per weight set, so it is written for exactness, not speed.
#include "device_common.hpp"

namespace nova {

template <int N, int R, typename T>
__global__ void __launch_bounds__(256)
filter_transform_kernel(const T *__restrict__ w, T *__restrict__ U, int K, int C, int Kp, int c_blocks,
                        FilterCoef<N, R> coef)
{
    const long long total = (long long)c_blocks * Kp * kChanBlock;
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int c_in = (int)(idx % kChanBlock);
    const int k = (int)((idx / kChanBlock) % Kp);
    const int cb = (int)(idx / ((long long)kChanBlock * Kp));
    const int c = cb * kChanBlock + c_in;
    const size_t xi_stride = (size_t)c_blocks * Kp * kChanBlock;
    T *dst = U + idx;

    if (k >= K || c >= C) {
        for (int xi = 0; xi < N * N; ++xi) dst[xi * xi_stride] = (T)0.0f;
        return;
    }
    double g[R * R];
    const T *src = w + ((size_t)k * C + c) * (R * R);
#pragma unroll
    for (int i = 0; i < R * R; ++i) g[i] = (double)load_f32(src + i);

    double tmp[N][R];                     // G g
#pragma unroll
    for (int i = 0; i < N; ++i)
#pragma unroll
        for (int b = 0; b < R; ++b) {
            double s = 0.0;
#pragma unroll
            for (int a = 0; a < R; ++a) s += coef.g[i * R + a] * g[a * R + b];
            tmp[i][b] = s;
        }
#pragma unroll
    for (int i = 0; i < N; ++i)
#pragma unroll
        for (int j = 0; j < N; ++j) {     // (G g) G^T
            double s = 0.0;
#pragma unroll
            for (int b = 0; b < R; ++b) s += tmp[i][b] * coef.g[j * R + b];
            dst[(size_t)(i * N + j) * xi_stride] = round_f64_to(s, (T *)nullptr);
        }
}

template <int N, int R, typename T>
static int launch_ft(const nova_transforms *t, const void *w, int K, int C, void *U, hipStream_t stream)
{
    FilterCoef<N, R> coef;
    for (int i = 0; i < N * R; ++i) coef.g[i] = t->G64[i];
    const int c_blocks = ceil_div(C, kChanBlock);
    const int Kp = ceil_div(K, kChanBlock) * kChanBlock;
    const long long total = (long long)c_blocks * Kp * kChanBlock;
    const unsigned blocks = (unsigned)((total + 255) / 256);
    hipLaunchKernelGGL((filter_transform_kernel<N, R, T>), dim3(blocks), dim3(256), 0, stream,
                       (const T *)w, (T *)U, K, C, Kp, c_blocks, coef);
    return (int)hipGetLastError();
}

int launch_filter_transform(const nova_transforms *t, const void *w, int K, int C, int dtype, void *U,
                            void *stream)
{
    hipStream_t s = (hipStream_t)stream;
    const bool h = dtype == NOVA_F16;
    if (t->r == 3) {
        switch (t->n) {
        case 4: return h ? launch_ft<4, 3, f16>(t, w, K, C, U, s) : launch_ft<4, 3, float>(t, w, K, C, U, s);
        case 6: return h ? launch_ft<6, 3, f16>(t, w, K, C, U, s) : launch_ft<6, 3, float>(t, w, K, C, U, s);
        case 8: return h ? launch_ft<8, 3, f16>(t, w, K, C, U, s) : launch_ft<8, 3, float>(t, w, K, C, U, s);
        case 10: return h ? launch_ft<10, 3, f16>(t, w, K, C, U, s) : launch_ft<10, 3, float>(t, w, K, C, U, s);
        }
    } else if (t->r == 5) {
        switch (t->n) {
        case 6: return h ? launch_ft<6, 5, f16>(t, w, K, C, U, s) : launch_ft<6, 5, float>(t, w, K, C, U, s);
        case 8: return h ? launch_ft<8, 5, f16>(t, w, K, C, U, s) : launch_ft<8, 5, float>(t, w, K, C, U, s);
        case 10: return h ? launch_ft<10, 5, f16>(t, w, K, C, U, s) : launch_ft<10, 5, float>(t, w, K, C, U, s);
        }
    }
    return (int)hipErrorInvalidValue;
}

}  // namespace nova
