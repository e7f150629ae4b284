// ReLU followed by a 2x2, stride-2 max-pool: the step between the blocks of a VGG-style stack.
// in [N][C][H][W] -> out [N][C][H/2][W/2]; memory bound, one thread per output element with the
// lanes running along the output row.
#include "device_common.hpp"

namespace nova {

template <typename T>
__global__ void __launch_bounds__(256)
relu_maxpool2x2_kernel(const T *__restrict__ in, T *__restrict__ out, long long planes, int H, int W)
{
    const int Ho = H / 2, Wo = W / 2;
    const long long total = planes * Ho * Wo;
    for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
         idx += (long long)gridDim.x * blockDim.x) {
        const int wo = (int)(idx % Wo);
        const int ho = (int)((idx / Wo) % Ho);
        const long long plane = idx / ((long long)Wo * Ho);
        const T *src = in + (plane * H + 2 * ho) * W + 2 * wo;
        const float a = load_f32(src), b = load_f32(src + 1), c = load_f32(src + W), d = load_f32(src + W + 1);
        // a NaN input makes the output NaN, like the comparison-based CPU definition
        float m = a;
        m = (b > m || b != b) ? b : m;
        m = (c > m || c != c) ? c : m;
        m = (d > m || d != d) ? d : m;
        m = m < 0.0f ? 0.0f : m;
        store_from_f32(out + idx, m);
    }
}

int launch_relu_maxpool2x2(const void *in, void *out, int N, int C, int H, int W, int dtype, void *stream)
{
    const long long planes = (long long)N * C;
    const long long total = planes * (H / 2) * (W / 2);
    if (total == 0) return 0;
    long long blocks = (total + 255) / 256;
    if (blocks > 256 * 64) blocks = 256 * 64;
    hipStream_t s = (hipStream_t)stream;
    if (dtype == NOVA_F16)
        hipLaunchKernelGGL(relu_maxpool2x2_kernel<f16>, dim3((unsigned)blocks), dim3(256), 0, s,
                           (const f16 *)in, (f16 *)out, planes, H, W);
    else
        hipLaunchKernelGGL(relu_maxpool2x2_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, s,
                           (const float *)in, (float *)out, planes, H, W);
    return (int)hipGetLastError();
}

}  // namespace nova
