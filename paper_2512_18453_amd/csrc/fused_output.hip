// Contraction and output transform in one kernel, for layers with 64 input channels (the early
// layers of an image network, where the products M -- n*n values per tile and output channel, written
// once and read once whatever C is -- are most of the memory traffic and the matrix work is small).
// M never exists in memory: Y = A^T [ sum_c U * V ] A is formed per (tile, channel) pair from
// matrix-unit results that stay in registers (Sec. 2.1 steps 3 and 4).
//
// A workgroup of 8 waves takes 16 neighbouring tiles (one group of a tile row, or a few tile rows of
// a narrow image) and 64 output channels; a wave takes 8 of those channels.  Per Winograd-domain
// position xi a wave forms a 16 x 16 block (v_mfma_f32_16x16x32_f16, binary32 accumulation over the
// input channels) of which only 8 rows are used: the matrix unit leaves each lane 4 results (rows
// 4 * (lane / 16) + 0..3 of column lane % 16), and the transform state of a (tile, channel) pair is
// m*m + m values, so a lane can carry two pairs, not four -- rows 2 and 3 of every group of four repeat
// rows 0 and 1 and their results are dropped.  The matrix unit has the time: the kernel is bound by
// memory and by the vector ALU.
//   lane = (tile lane % 16, channels 2 * (lane / 16) + {0, 1} of the wave's eight)
// The positions are visited row by row, xi = i * n + j.  When the n products of a row i are there, the
// lane transforms them along j (w[q] = sum_j A[j][q] M[i][j]) and folds the row into its m x m
// outputs, Y[p][q] += A[i][p] w[q]; the rows of +a and -a enter together through their sum and
// difference, which halves the multiplications (as in the separate output transform).  The row loop
// is unrolled by two -- rows 2d and 2d + 1 -- so that buffers, ring places and the fold are the same
// code for every d: the fold after row 2d takes the pair (2d - 1, 2d) with the coefficient row fold[d]
// (for d = 0 the carried row is zero and fold[0] = (A[0][0], 0, ...): the point 0), row n - 1 (the
// point at infinity) is added after the loop.
//
// Operands.  V[xi] of the 16 tiles (64 channels: 2 KiB) is shared by the 8 waves: two LDS buffers of
// one row of positions each, filled by direct global->LDS loads a row ahead, one barrier per row.
// U[xi] of a wave's 8 channels (1 KiB) is private to the wave: a ring of one row of positions in LDS,
// refilled for the next row, half a row at a time, right after the half has been read, and waited for
// by the wave alone (vector-memory operations of a wave complete in the order issued, so "at most
// the loads issued after these are outstanding" is a count).  Every LDS address in the loop is a
// per-lane base plus an immediate.  U comes from L2 (the whole of U is under a MB at these channel
// counts), V from memory, once per group of 64 output channels.
// LDS rows of 64 bytes (32 channels) are XOR-swizzled by 16-byte piece, so that the 128-bit fragment
// reads of 16 lanes fall into 16 different bank groups; the loads fix each lane's place in LDS, so a
// lane fetches the piece that belongs there.
// At the end the m x m results of all pairs go through LDS as [32 channels][rows][columns] blocks (two
// passes of 32 channels) and leave as in the separate output transform, with its ReLU / max-pool options.
#include "output_common.hpp"

namespace nova {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));

constexpr int kFusedTiles = 16;        // tiles per workgroup: the columns of the matrix instruction
constexpr int kFusedWaves = 8;
constexpr int kFusedWaveChannels = 8;  // output channels per wave
constexpr int kFusedChannels = kFusedWaves * kFusedWaveChannels;
constexpr int kFusedCB = 2;            // blocks of 32 input channels

// fold[d][p]: d = 0: (A[0][0], 0, ..., 0); d >= 1: the coefficients of the pair of points d (A[2d - 1][p])
template <int N, int R>
struct FoldCoef {
    float c[(N / 2) * (N - R + 1)];
};

template <int N, int R, int STG>
__global__ void __launch_bounds__(64 * kFusedWaves, 2)
fused_contract_output_kernel(const f16 *__restrict__ U, const f16 *__restrict__ V, f16 *__restrict__ y,
                             int K, int H, int W, int tiles_h, int tiles_w, int Kp, long long Ttot, int k_groups,
                             int relu, OutShape sh, OutCoef<N, R> coef, FoldCoef<N, R> fold)
{
    constexpr int M = N - R + 1;
    constexpr int CB = kFusedCB;
    constexpr int G = N / 2;                          // positions whose U is waited for, read and refilled together
    constexpr int V_CHUNK = kFusedTiles * 64;         // bytes: 16 tiles x 32 channels
    constexpr int V_ROW = N * CB * V_CHUNK;           // one row of positions
    constexpr int U_STAGE = CB * kFusedWaveChannels * 64;     // bytes of one position: 2 blocks x 8 channels x 32 channels in
    constexpr int U_RING = N * U_STAGE;
    constexpr int V_LOADS = (N * CB + kFusedWaves - 1) / kFusedWaves;      // chunks of a row per wave, at most
    constexpr bool V_EVEN = (N * CB) % kFusedWaves == 0;
    static_assert(N % 2 == 0 && V_LOADS >= 2 && V_LOADS <= 5 && G <= 5 && N * CB - (V_LOADS - 1) * kFusedWaves > 0, "pipeline shape");
    extern __shared__ __align__(1024) unsigned char lds_raw[];
    const unsigned lds_base = (unsigned)(size_t)((__attribute__((address_space(3))) void *)lds_raw);

    const int lane = (int)(threadIdx.x & 63);
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));

    // block -> (image, tile rows, tile group, group of 64 output channels); the channel groups of one
    // tile group are neighbours and run on the same XCD, so that V is fetched into one L2 only
    unsigned bid = xcd_local_block_id(blockIdx.x, gridDim.x);
    const int kg = bid % k_groups; bid /= k_groups;
    const int row_groups = (tiles_h + sh.trb - 1) / sh.trb;
    const int tg = bid % sh.groups; bid /= sh.groups;
    const int tr = (bid % row_groups) * sh.trb; bid /= row_groups;
    const int img = bid;
    const int tc0 = sh.trb > 1 ? 0 : tg * sh.twb;
    // the group's tiles are neighbours in t (a group of several tile rows spans the image width)
    const long long t0 = ((long long)img * tiles_h + tr) * tiles_w + tc0;
    const int k0 = kg * kFusedChannels, kw0 = k0 + wave * kFusedWaveChannels;

    // ---- direct loads.  A 64-byte row r of a chunk holds its four 16-byte pieces in the places
    // piece ^ ((r / 4) % 4); lane l of a load writes 16 bytes at its base + 16 l.
    // V: one load = one chunk (16 tiles of one channel block): lane l -> row l / 4, place l % 4; the
    //    N * CB chunks of a row are dealt out to the waves, chunk = wave + 8 s.
    // U: one load = one position (8 channels each of the two channel blocks): lane l -> block l / 32,
    //    row (l / 4) % 8, place l % 4.
    const int v_row_l = lane >> 2, v_piece_l = (lane & 3) ^ ((lane >> 4) & 3);
    long long v_t = t0 + v_row_l;
    if (v_t > Ttot - 1) v_t = Ttot - 1;               // rows past the end: reread the last tile (never used)
    const unsigned v_lane_off = (unsigned)(((unsigned)v_t * kChanBlock + (unsigned)v_piece_l * 8u) * sizeof(f16));
    const size_t v_cb_stride = (size_t)Ttot * kChanBlock;          // elements per channel block of a position
    const size_t u_cb_stride = (size_t)Kp * kChanBlock;
    const int u_row_l = (lane >> 2) & 7, u_piece_l = (lane & 3) ^ ((u_row_l >> 2) & 3);
    const unsigned u_lane_off = (unsigned)((((unsigned)(lane >> 5) * (unsigned)u_cb_stride) + (unsigned)(kw0 + u_row_l) * kChanBlock +
                                            (unsigned)u_piece_l * 8u) * sizeof(f16));
    const bool v_all = V_EVEN || wave + (V_LOADS - 1) * kFusedWaves < N * CB;      // this wave has a chunk in the last round
    const f16 *v_fill = uniform_pointer(V + (size_t)wave * v_cb_stride);          // the wave's first chunk of the row issued next
    const f16 *u_fill = U;                                                        // the position of U issued next
    const unsigned v_lds = lds_base + (unsigned)(wave * V_CHUNK);
    const unsigned u_lds = lds_base + (unsigned)(2 * V_ROW + wave * U_RING);
    auto issue_v_row = [&](int buf) __attribute__((always_inline)) {
        const unsigned at = (unsigned)__builtin_amdgcn_readfirstlane((int)(v_lds + (unsigned)(buf * V_ROW)));
        if (v_all) {
            const void *planes[V_LOADS];
#pragma unroll
            for (int s = 0; s < V_LOADS; ++s) planes[s] = uniform_pointer(v_fill + (size_t)(s * kFusedWaves) * v_cb_stride);
            global_to_lds16_run<V_LOADS, kFusedWaves * V_CHUNK>(planes, v_lane_off, at);
        } else {
            const void *planes[V_LOADS - 1];
#pragma unroll
            for (int s = 0; s < V_LOADS - 1; ++s) planes[s] = uniform_pointer(v_fill + (size_t)(s * kFusedWaves) * v_cb_stride);
            global_to_lds16_run<V_LOADS - 1, kFusedWaves * V_CHUNK>(planes, v_lane_off, at);
        }
        v_fill += (size_t)(N * CB) * v_cb_stride;
    };
    auto issue_u_half = [&](int half) __attribute__((always_inline)) {
        const void *planes[G];
#pragma unroll
        for (int s = 0; s < G; ++s) planes[s] = uniform_pointer(u_fill + (size_t)(s * CB) * u_cb_stride);
        const unsigned at = (unsigned)__builtin_amdgcn_readfirstlane((int)(u_lds + (unsigned)(half * G * U_STAGE)));
        global_to_lds16_run<G, U_STAGE>(planes, u_lane_off, at);
        u_fill += (size_t)(G * CB) * u_cb_stride;
    };

    // ---- fragment reads.  A operand (U): lane supplies row lane % 16 of the 16 x 32 block, channels
    // 8 * (lane / 16) .. + 7 of the 32; rows 4g + {0, 1} and again 4g + {2, 3} are the wave's channels
    // 2g + {0, 1}.  B operand (V): column lane % 16 = tile, the same channels.
    const int f_row = lane & 15, f_piece = lane >> 4;
    const int a_chan = 2 * (f_row >> 2) + (f_row & 1);                       // 0..7
    const unsigned char *a_at = lds_raw + 2 * V_ROW + wave * U_RING + a_chan * 64 + ((f_piece ^ ((a_chan >> 2) & 3)) * 16);
    const unsigned char *b_at = lds_raw + f_row * 64 + ((f_piece ^ ((f_row >> 2) & 3)) * 16);

    // ---- the lane's two pairs: tile lane % 16, channels kw0 + 2 * (lane / 16) + {0, 1}
    float Y[2][M][M];
    float carried[2][M];              // the row before, transformed along j
#pragma unroll
    for (int e = 0; e < 2; ++e) {
#pragma unroll
        for (int q = 0; q < M; ++q) carried[e][q] = 0.0f;
#pragma unroll
        for (int p = 0; p < M; ++p)
#pragma unroll
            for (int q = 0; q < M; ++q) Y[e][p][q] = 0.0f;
    }

    // One row of positions: products of the row, transformed along j, into w.  BUF: the buffer of V that
    // holds the row.  Order of this wave's loads around it: ..., V(row), U(row, first half), U(row,
    // second half), [row starts] V(row + 1), U(row + 1, first half), U(row + 1, second half), ...
    auto row = [&](auto buf_tag, bool more, float (&w)[2][M]) __attribute__((always_inline)) {
        constexpr int BUF = decltype(buf_tag)::value;
        // this wave's chunks of V(row) have landed: the two halves of U(row) were issued after them
        asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
        __syncthreads();              // everyone's have; everyone is done with the row before, whose buffer is free
        float m_row[N][2];
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            // U of this half has landed.  Issued after it: first half -- the second half; second half --
            // V(row + 1) and U(row + 1, first half), if there is a next row
            if (half == 0) asm volatile("s_waitcnt vmcnt(%0)" : : "n"(G) : "memory");
            else if (!more) asm volatile("s_waitcnt vmcnt(0)" : : : "memory");
            else if (v_all) asm volatile("s_waitcnt vmcnt(%0)" : : "n"(G + V_LOADS) : "memory");
            else asm volatile("s_waitcnt vmcnt(%0)" : : "n"(G + V_LOADS - 1) : "memory");
            if (half == 0 && more) issue_v_row(BUF ^ 1);
            float4v acc[G];
#pragma unroll
            for (int jj = 0; jj < G; ++jj) {
                const int j = half * G + jj;
                acc[jj] = float4v{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) {
                    const half8 a = *reinterpret_cast<const half8 *>(a_at + j * U_STAGE + cb * (U_STAGE / CB));
                    const half8 b = *reinterpret_cast<const half8 *>(b_at + BUF * V_ROW + (j * CB + cb) * V_CHUNK);
                    acc[jj] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, acc[jj], 0, 0, 0);
                }
            }
#pragma unroll
            for (int jj = 0; jj < G; ++jj) {
                m_row[half * G + jj][0] = acc[jj][0];
                m_row[half * G + jj][1] = acc[jj][1];
            }
            if (more) {
                // the places of this half are free once its fragment reads have returned
                asm volatile("s_waitcnt lgkmcnt(0)" : : : "memory");
                issue_u_half(half);
            }
        }
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            float v[N];
#pragma unroll
            for (int j = 0; j < N; ++j) v[j] = m_row[j][e];
            output_transform_1d<N, R, true>(v, w[e], coef);
        }
    };

    issue_v_row(0);
    issue_u_half(0);
    issue_u_half(1);
#pragma unroll 1
    for (int d = 0; d < N / 2; ++d) {
        float w[2][M];
        row(std::integral_constant<int, 0>{}, true, w);
        // rows 2d - 1 (+a, carried) and 2d (-a) enter through their sum and difference
        const float *c = fold.c + d * M;
#pragma unroll
        for (int e = 0; e < 2; ++e)
#pragma unroll
            for (int p = 0; p < M; ++p) {
                const float cp = c[p];
#pragma unroll
                for (int q = 0; q < M; ++q) {
                    const float sd = (p & 1) ? carried[e][q] - w[e][q] : carried[e][q] + w[e][q];
                    Y[e][p][q] = fma32(cp, sd, Y[e][p][q]);
                }
            }
        row(std::integral_constant<int, 1>{}, d + 1 < N / 2, carried);
    }
    // row n - 1: the point at infinity
#pragma unroll
    for (int e = 0; e < 2; ++e)
#pragma unroll
        for (int q = 0; q < M; ++q) Y[e][M - 1][q] = fma32(coef.inf, carried[e][q], Y[e][M - 1][q]);

    // ---- the results leave through LDS, 32 channels at a time
    f16 *stage = reinterpret_cast<f16 *>(lds_raw);
    const int tile = lane & 15;
    int jr = 0, jc = tile;
    if (sh.trb > 1) { jr = tile / tiles_w; jc = tile - jr * tiles_w; }
    const bool active = tile < sh.twb && tc0 + jc < tiles_w && tr + jr < tiles_h;
#pragma unroll 1
    for (int pass = 0; pass < kFusedChannels / kChanBlock; ++pass) {
        __syncthreads();              // the operand buffers (first pass) or the block before have been read
        if (active && (wave >> 2) == pass) {
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int k_in = (wave & 3) * kFusedWaveChannels + 2 * (lane >> 4) + e;
                f16 *dst = stage + k_in * sh.k_pitch + jr * M * sh.cols_pitch + jc * M;
#pragma unroll
                for (int p = 0; p < M; ++p)
#pragma unroll
                    for (int q = 0; q < M; ++q) {
                        float val = Y[e][p][q];
                        if (relu) val = val < 0.0f ? 0.0f : val;      // NaN stays NaN
                        dst[p * sh.cols_pitch + q] = (f16)val;
                    }
            }
        }
        __syncthreads();
        store_output_block<f16, M, STG>(stage, y, img, k0 / kChanBlock + pass, tr, tc0, K, H, W, tiles_w, sh);
    }
}

template <int N, int R>
static int launch_fused_shape(const nova_transforms *t, const void *U, const void *V, void *y, const Geometry &g, int flags,
                              hipStream_t stream)
{
    constexpr int M = N - R + 1;
    constexpr int PE = 8;
    constexpr int CB = kFusedCB;
    OutCoef<N, R> coef;
    fill_out_coef<N, R>(t, coef);
    FoldCoef<N, R> fold;
    for (int p = 0; p < M; ++p) fold.c[p] = p == 0 ? coef.zero : 0.0f;
    for (int d = 1; d < N / 2; ++d)
        for (int p = 0; p < M; ++p) fold.c[d * M + p] = coef.pw[(d - 1) * M + p];
    OutShape sh;
    sh.groups = ceil_div(g.tiles_w, kFusedTiles);
    const int twb = ceil_div(g.tiles_w, sh.groups);
    int trb = 1;
    if (sh.groups == 1) {
        trb = kFusedTiles / twb;
        if (trb > g.tiles_h) trb = g.tiles_h;
        trb = ceil_div(g.tiles_h, ceil_div(g.tiles_h, trb));     // same number of groups, evenly sized
    }
    const size_t stage_bytes = out_shape<N, R, f16>(twb, trb, sh);
    const size_t loop_bytes = (size_t)2 * N * CB * kFusedTiles * 64 + (size_t)kFusedWaves * N * CB * kFusedWaveChannels * 64;
    const size_t lds_bytes = stage_bytes > loop_bytes ? stage_bytes : loop_bytes;
    if (lds_bytes > 160 * 1024 || sh.twb > kFusedTiles) return (int)hipErrorInvalidValue;
    // 32-bit byte offsets inside one position of V
    if ((size_t)CB * g.T * kChanBlock * sizeof(f16) >= ((size_t)1 << 32)) return (int)hipErrorInvalidValue;
    const bool aligned = ((uintptr_t)y % 16) == 0;
    const bool vec = g.W % PE == 0 && aligned && (sh.groups == 1 || (twb * M) % PE == 0);
    const bool flat = !vec && aligned && sh.groups == 1 && g.W >= 2 && sh.rows * g.W + 2 * (PE - 1) >= 2 * PE &&
                      (long long)sh.rows * g.W < (1 << 15);
    if (flat) {
        sh.pieces = (sh.rows * g.W + 2 * (PE - 1)) / PE;
        sh.piece_magic = (unsigned)((((unsigned long long)1 << 32) + sh.pieces - 1) / sh.pieces);
        sh.w_magic = (unsigned)((((unsigned long long)1 << 32) + g.W - 1) / g.W);
    }
    sh.pool = (flags & NOVA_FLAG_POOL2) ? 1 : 0;
    const int k_groups = g.Kp / kFusedChannels;
    const long long blocks = (long long)sh.groups * ceil_div(g.tiles_h, trb) * k_groups * g.N;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return (int)hipErrorInvalidValue;
    auto kern = vec ? fused_contract_output_kernel<N, R, kStoreVec>
              : flat ? fused_contract_output_kernel<N, R, kStoreFlat> : fused_contract_output_kernel<N, R, kStoreScalar>;
    static bool raised[3] = {false, false, false};          // more than 64 KiB of dynamic LDS: asked for once per kernel
    const int which = vec ? 0 : flat ? 1 : 2;
    if (!raised[which]) {
        NOVA_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                         160 * 1024));
        raised[which] = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(64 * kFusedWaves), lds_bytes, stream,
                       (const f16 *)U, (const f16 *)V, (f16 *)y, g.K, g.H, g.W, g.tiles_h, g.tiles_w, g.Kp, g.T, k_groups,
                       (flags & NOVA_FLAG_RELU) ? 1 : 0, sh, coef, fold);
    return (int)hipGetLastError();
}

// Shapes the fused kernel takes: binary16 storage, products not rounded to binary16, points in the paired
// order, F(6,3) or F(8,3), C = 64, K a multiple of 64.
bool fused_contract_output_applies(const nova_transforms *t, const Geometry &g, int dtype, int flags)
{
    return dtype == NOVA_F16 && !(flags & NOVA_FLAG_M_F16) && t->symmetric && t->r == 3 && (t->n == 8 || t->n == 10) &&
           g.C == kFusedCB * kChanBlock && g.K % kFusedChannels == 0 && g.T <= 0x7fffffffLL;
}

int launch_fused_contract_output(const nova_transforms *t, const void *U, const void *V, void *y, const Geometry &g,
                                 int dtype, int flags, void *stream)
{
    if (!fused_contract_output_applies(t, g, dtype, flags)) return (int)hipErrorInvalidValue;
    hipStream_t s = (hipStream_t)stream;
    if (t->n == 10) return launch_fused_shape<10, 3>(t, U, V, y, g, flags, s);
    return launch_fused_shape<8, 3>(t, U, V, y, g, flags, s);
}

}  // namespace nova
