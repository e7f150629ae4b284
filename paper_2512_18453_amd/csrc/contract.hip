// Winograd-domain contraction over input channels (Sec. 2.1 step 3, summed over channels):
//     M[xi][t][k] = sum_c V[xi][t][c] * U[xi][k][c]      for each of the n*n positions xi,
// i.e. n*n independent (T x C) . (C x K) matrix products.  Both operands are stored with the
// contraction index blocked by 32 and fastest (V [xi][C/32][T][32], U [xi][C/32][Kp][32]), so a
// (rows x 32-channel) operand tile is one contiguous piece of memory and every lane's MFMA
// fragment is a 16-byte read.
//
// binary16 path: v_mfma_f32_32x32x16_f16, binary32 accumulation.  A workgroup of 4 waves owns a
// BM x BN tile of one M[xi]; the channel loop moves 32 channels per step through double-buffered
// LDS (rows padded from 64 to 80 bytes, which spreads the 16 lanes of a 128-bit read phase over
// all 64 banks), global loads for step s+1 are issued before the MFMAs of step s.
// binary32 path: same layouts, plain FMA tiles (validation path, not tuned).
#include "device_common.hpp"

namespace nova {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef unsigned int uint4v __attribute__((ext_vector_type(4)));

constexpr int kRowHalves = 40;   // LDS row pitch of a 32-channel operand row, in binary16 units (80 B)

template <int BM, int BN, int WM, int WN, typename MT>
__global__ void __launch_bounds__(256)
contract_f16_kernel(const f16 *__restrict__ U, const f16 *__restrict__ V, MT *__restrict__ Mo,
                    int T, int Kp, int c_blocks, int k_blocks, int row_blocks, int col_blocks)
{
    constexpr int MB = BM / WM / 32;          // 32x32 MFMA blocks per wave, rows
    constexpr int NB = BN / WN / 32;          // and columns
    constexpr int A_SEGS = BM * 4 / 256;      // 16-byte segments per thread and stage
    constexpr int B_SEGS = (BN * 4 + 255) / 256;
    static_assert(WM * WN == 4 && BM % (WM * 32) == 0 && BN % (WN * 32) == 0, "tile shape");

    __shared__ __align__(16) f16 lds_a[2][BM * kRowHalves];
    __shared__ __align__(16) f16 lds_b[2][BN * kRowHalves];

    unsigned bid = xcd_local_block_id(blockIdx.x, gridDim.x);
    const int cbk = bid % col_blocks; bid /= col_blocks;
    const int rbk = bid % row_blocks; bid /= row_blocks;
    const int xi = bid;
    const int t0 = rbk * BM, k0 = cbk * BN;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wm = wave / WN, wn = wave % WN;

    // per-thread global segments: segment s -> (row s/4, 16-byte piece s%4); rows beyond the
    // tensor are clamped to the last valid row (their products are never stored)
    const f16 *a_src[A_SEGS];
    const f16 *b_src[B_SEGS];
    int a_dst[A_SEGS], b_dst[B_SEGS];
#pragma unroll
    for (int i = 0; i < A_SEGS; ++i) {
        const int s = tid + i * 256, row = s >> 2, piece = s & 3;
        int t = t0 + row; if (t > T - 1) t = T - 1;
        a_src[i] = V + ((size_t)xi * c_blocks * T + t) * kChanBlock + piece * 8;
        a_dst[i] = row * kRowHalves + piece * 8;
    }
#pragma unroll
    for (int i = 0; i < B_SEGS; ++i) {
        const int s = tid + i * 256, row = s >> 2, piece = s & 3;
        int k = k0 + row; if (k > Kp - 1) k = Kp - 1;
        b_src[i] = U + ((size_t)xi * c_blocks * Kp + k) * kChanBlock + piece * 8;
        b_dst[i] = row * kRowHalves + piece * 8;
    }
    const size_t a_step = (size_t)T * kChanBlock, b_step = (size_t)Kp * kChanBlock;

    float16v acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    uint4v a_reg[A_SEGS], b_reg[B_SEGS];
    auto load_global = [&](int cb) {
#pragma unroll
        for (int i = 0; i < A_SEGS; ++i) a_reg[i] = *reinterpret_cast<const uint4v *>(a_src[i] + cb * a_step);
#pragma unroll
        for (int i = 0; i < B_SEGS; ++i)
            if (BN * 4 >= 256 || tid + i * 256 < BN * 4)
                b_reg[i] = *reinterpret_cast<const uint4v *>(b_src[i] + cb * b_step);
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_SEGS; ++i) *reinterpret_cast<uint4v *>(&lds_a[buf][a_dst[i]]) = a_reg[i];
#pragma unroll
        for (int i = 0; i < B_SEGS; ++i)
            if (BN * 4 >= 256 || tid + i * 256 < BN * 4)
                *reinterpret_cast<uint4v *>(&lds_b[buf][b_dst[i]]) = b_reg[i];
    };

    load_global(0);
    store_lds(0);
    __syncthreads();

    const int frag_row = lane & 31, frag_k = (lane >> 5) * 8;
    for (int cb = 0; cb < c_blocks; ++cb) {
        const int buf = cb & 1;
        if (cb + 1 < c_blocks) load_global(cb + 1);
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            half8 af[MB], bf[NB];
#pragma unroll
            for (int i = 0; i < MB; ++i)
                af[i] = *reinterpret_cast<const half8 *>(
                    &lds_a[buf][((wm * MB + i) * 32 + frag_row) * kRowHalves + kk * 16 + frag_k]);
#pragma unroll
            for (int j = 0; j < NB; ++j)
                bf[j] = *reinterpret_cast<const half8 *>(
                    &lds_b[buf][((wn * NB + j) * 32 + frag_row) * kRowHalves + kk * 16 + frag_k]);
#pragma unroll
            for (int i = 0; i < MB; ++i)
#pragma unroll
                for (int j = 0; j < NB; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
        if (cb + 1 < c_blocks) store_lds(buf ^ 1);
        __syncthreads();
    }

    // D[row][col]: lane holds col = lane%32 and rows 8*(e/4) + 4*(lane/32) + e%4
    const int col = lane & 31, row_base = (lane >> 5) * 4;
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        const int kb = (k0 >> 5) + wn * NB + j;
        if (kb >= k_blocks) continue;
        MT *dst = Mo + ((size_t)xi * k_blocks + kb) * (size_t)T * kChanBlock + col;
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int t = t0 + (wm * MB + i) * 32 + (e >> 2) * 8 + row_base + (e & 3);
                if (t < T) store_from_f32(dst + (size_t)t * kChanBlock, acc[i][j][e]);
            }
    }
}

// binary32: 64 x 64 tile, 256 threads, 4 x 4 outputs per thread
__global__ void __launch_bounds__(256)
contract_f32_kernel(const float *__restrict__ U, const float *__restrict__ V, float *__restrict__ Mo,
                    int T, int Kp, int c_blocks, int k_blocks, int row_blocks, int col_blocks)
{
    __shared__ float lds_a[64][kChanBlock + 1];
    __shared__ float lds_b[64][kChanBlock + 1];
    unsigned bid = blockIdx.x;
    const int cbk = bid % col_blocks; bid /= col_blocks;
    const int rbk = bid % row_blocks; bid /= row_blocks;
    const int xi = bid;
    const int t0 = rbk * 64, k0 = cbk * 64;
    const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;

    float acc[4][4] = {};
    for (int cb = 0; cb < c_blocks; ++cb) {
        for (int e = tid; e < 64 * kChanBlock; e += 256) {
            const int row = e >> 5, c = e & 31;
            int t = t0 + row; if (t > T - 1) t = T - 1;
            int k = k0 + row; if (k > Kp - 1) k = Kp - 1;
            lds_a[row][c] = V[(((size_t)xi * c_blocks + cb) * T + t) * kChanBlock + c];
            lds_b[row][c] = U[(((size_t)xi * c_blocks + cb) * Kp + k) * kChanBlock + c];
        }
        __syncthreads();
#pragma unroll 8
        for (int c = 0; c < kChanBlock; ++c) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = lds_a[ty + 16 * i][c]; b[i] = lds_b[tx + 16 * i][c]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fma32(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int t = t0 + ty + 16 * i, k = k0 + tx + 16 * j;
            if (t < T && (k >> 5) < k_blocks)
                Mo[(((size_t)xi * k_blocks + (k >> 5)) * T + t) * kChanBlock + (k & 31)] = acc[i][j];
        }
}

template <int BM, int BN, int WM, int WN, typename MT>
static int launch_c16(const void *U, const void *V, void *Mo, const Geometry &g, hipStream_t stream)
{
    const int row_blocks = ceil_div((int)g.T, BM), col_blocks = ceil_div(g.Kp, BN);
    const long long blocks = (long long)g.n * g.n * row_blocks * col_blocks;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL((contract_f16_kernel<BM, BN, WM, WN, MT>), dim3((unsigned)blocks), dim3(256), 0, stream,
                       (const f16 *)U, (const f16 *)V, (MT *)Mo, (int)g.T, g.Kp, g.c_blocks, g.k_blocks,
                       row_blocks, col_blocks);
    return (int)hipGetLastError();
}

template <typename MT>
static int launch_c16_shape(const void *U, const void *V, void *Mo, const Geometry &g, hipStream_t s)
{
    if (g.Kp >= 128) return launch_c16<128, 128, 2, 2, MT>(U, V, Mo, g, s);
    if (g.Kp >= 64) return launch_c16<128, 64, 2, 2, MT>(U, V, Mo, g, s);
    return launch_c16<128, 32, 4, 1, MT>(U, V, Mo, g, s);
}

int launch_contract(const nova_transforms *, const void *U, const void *V, void *Mo, const Geometry &g,
                    int dtype, int flags, void *stream)
{
    hipStream_t s = (hipStream_t)stream;
    if (g.T > 0x7fffffffLL) return (int)hipErrorInvalidValue;
    if (dtype == NOVA_F16)
        return (flags & NOVA_FLAG_M_F16) ? launch_c16_shape<f16>(U, V, Mo, g, s)
                                         : launch_c16_shape<float>(U, V, Mo, g, s);
    const int row_blocks = ceil_div((int)g.T, 64), col_blocks = ceil_div(g.Kp, 64);
    const long long blocks = (long long)g.n * g.n * row_blocks * col_blocks;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(contract_f32_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (const float *)U,
                       (const float *)V, (float *)Mo, (int)g.T, g.Kp, g.c_blocks, g.k_blocks, row_blocks,
                       col_blocks);
    return (int)hipGetLastError();
}

}  // namespace nova
