// Contraction and output transform in one kernel, for layers with 64 input channels (the early
// layers of an image network, where the products M -- n*n values per tile and output channel, written
// once and read once whatever C is -- are most of the memory traffic and the matrix work is small).
// M never exists in memory: Y = A^T [ sum_c U * V ] A is formed per (tile, channel) pair from
// matrix-unit results that stay in registers (Sec. 2.1 steps 3 and 4).
//
// A workgroup of 4 waves takes a block of up to 16 tiles (trb tile rows x twc tile columns, the shape
// that wastes the fewest of the 16 slots over the image) and 32 output channels; a wave takes 8 of those
// channels.  Two workgroups share a compute unit (80 KB of LDS and at most 256 registers each), so that the
// head and the tail of one -- waiting for the first operands, converting, staging and storing the results,
// 40 % of its life -- overlap the other's main loop (8 waves as one workgroup per unit: 3-19 % slower).
// Per Winograd-domain position xi a wave forms a 16 x 16 block (v_mfma_f32_16x16x32_f16, binary32
// accumulation over the input channels) of which only 8 rows are used: the matrix unit leaves each lane 4 results (rows
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
// code for every d: the pair of rows (2d - 1, 2d) is folded with the coefficient row fold[d] (for d = 0
// the carried row is zero and fold[0] = (A[0][0], 0, ...): the point 0), row n - 1 (the point at
// infinity) is added after the loop.  The vector work on a row runs a row late, cut into slices that
// sit between the matrix instructions of the next row, whose fragments are read two positions ahead.
//
// Operands.  V[xi] of the 16 tiles (64 channels: 2 KiB) is shared by the 4 waves: two LDS buffers of
// one row of positions each, filled by direct global->LDS loads a row ahead, one barrier per row.
// U[xi] of a wave's 8 channels (1 KiB) is private to the wave: a ring of one row of positions in LDS,
// refilled for the next row, half a row at a time, right after the half has been read, and waited for
// by the wave alone (vector-memory operations of a wave complete in the order issued, so "at most
// the loads issued after these are outstanding" is a count).  Every LDS address in the loop is a
// per-lane base plus an immediate.  U comes from L2 (the whole of U is under a MB at these channel
// counts), V from memory or L2, once per group of 32 output channels (neighbouring workgroups).
// LDS rows of 64 bytes (32 channels) are XOR-swizzled by 16-byte piece -- piece ^ ((row / 2) % 4), the
// pattern that a 128-bit fragment read of rows lane % 16 takes fastest (timed: 2.9 clocks per wave-wide
// read against 4.5 without it or with (row / 4) % 4, which is the right one for rows lane % 32); the
// loads fix each lane's place in LDS, so a lane fetches the piece that belongs there.
// At the end the m x m results of all pairs go through LDS as a [32 channels][rows][columns] block and
// leave as in the separate output transform, with its ReLU / max-pool options.
#include "output_common.hpp"

namespace nova {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));

constexpr int kFusedTiles = 16;        // tiles per workgroup: the columns of the matrix instruction
constexpr int kFusedWaves = 4;         // 32 output channels per workgroup; two workgroups share a compute unit
constexpr int kFusedWaveChannels = 8;  // output channels per wave
constexpr int kFusedChannels = kFusedWaves * kFusedWaveChannels;
constexpr int kFusedCB = 2;            // blocks of 32 input channels

// The value is formed before this point of the program and used after it: arithmetic without side effects
// is otherwise free to drift to its first use, past the matrix instructions it is meant to sit between.
__device__ __forceinline__ void stays_here(float &x) { asm volatile("" : "+v"(x)); }

template <int I, int COUNT, typename F>
__device__ __forceinline__ void static_for_from(F &&f)
{
    if constexpr (I < COUNT) {
        f(std::integral_constant<int, I>{});
        static_for_from<I + 1, COUNT>(f);
    }
}
template <int COUNT, typename F>
__device__ __forceinline__ void static_for(F &&f) { static_for_from<0, COUNT>(f); }

// fold[d][p]: d = 0: (A[0][0], 0, ..., 0); d >= 1: the coefficients of the pair of points d (A[2d - 1][p])
template <int N, int R>
struct FoldCoef {
    float c[(N / 2) * (N - R + 1)];
};

template <int N, int R, int STG>
__global__ void __launch_bounds__(64 * kFusedWaves, 2)
fused_contract_output_kernel(const f16 *__restrict__ U, const f16 *__restrict__ V, f16 *__restrict__ y,
                             int K, int H, int W, int tiles_h, int tiles_w, int Kp, long long Ttot, int k_groups,
                             int relu, int one_pass, OutShape sh, OutCoef<N, R> coef, FoldCoef<N, R> fold)
{
    constexpr int M = N - R + 1;
    constexpr int CB = kFusedCB;
    constexpr int HP = (N - 2) / 2;                   // pairs of points +a, -a
    constexpr int G = N / 2;                          // positions whose U is waited for, read and refilled together
    constexpr int kFusedAhead = 2;                    // positions whose fragments are read ahead of the matrix instructions
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
    const int tc0 = tg * sh.twc;
    // tile j of the group: row j / twc, column j % twc of a block of trb x twc tiles
    const long long t0 = ((long long)img * tiles_h + tr) * tiles_w + tc0;
    const int k0 = kg * kFusedChannels, kw0 = k0 + wave * kFusedWaveChannels;

    // ---- direct loads.  A 64-byte row r of a chunk holds its four 16-byte pieces in the places
    // piece ^ ((r / 2) % 4); lane l of a load writes 16 bytes at its base + 16 l.
    // V: one load = one chunk (16 tiles of one channel block): lane l -> row l / 4, place l % 4; the
    //    N * CB chunks of a row are dealt out to the waves, chunk = wave + 8 s.
    // U: one load = one position (8 channels each of the two channel blocks): lane l -> block l / 32,
    //    row (l / 4) % 8, place l % 4.
    const int v_row_l = lane >> 2, v_piece_l = (lane & 3) ^ ((v_row_l >> 1) & 3);
    long long v_t = t0 + (long long)(v_row_l / sh.twc) * tiles_w + v_row_l % sh.twc;
    if (v_t > Ttot - 1) v_t = Ttot - 1;               // rows past the end: reread the last tile (never used)
    const unsigned v_lane_off = (unsigned)(((unsigned)v_t * kChanBlock + (unsigned)v_piece_l * 8u) * sizeof(f16));
    const size_t v_cb_stride = (size_t)Ttot * kChanBlock;          // elements per channel block of a position
    const size_t u_cb_stride = (size_t)Kp * kChanBlock;
    const int u_row_l = (lane >> 2) & 7, u_piece_l = (lane & 3) ^ ((u_row_l >> 1) & 3);
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
    const unsigned char *a_at = lds_raw + 2 * V_ROW + wave * U_RING + a_chan * 64 + ((f_piece ^ ((a_chan >> 1) & 3)) * 16);
    const unsigned char *b_at = lds_raw + f_row * 64 + ((f_piece ^ ((f_row >> 1) & 3)) * 16);

    // ---- the lane's two pairs: tile lane % 16, channels kw0 + 2 * (lane / 16) + {0, 1}
    float Y[2][M][M];
#pragma unroll
    for (int e = 0; e < 2; ++e)
#pragma unroll
        for (int p = 0; p < M; ++p)
#pragma unroll
            for (int q = 0; q < M; ++q) Y[e][p][q] = 0.0f;

    // One row of positions: the products of the row into m_out.  A half row at a time: wait for its U,
    // then position by position -- fragment reads kFusedAhead positions ahead of the matrix instructions
    // that take them, and between the matrix instructions a slice of the vector work on the rows before
    // (valu0 / valu1: slice jj of the first / second half), in exactly this order (the scheduler is
    // fenced off after every position: left alone it reads each fragment just before its use and waits).
    // BUF: the buffer of V that holds the row.  Order of this wave's loads around it: ..., V(row),
    // U(row, first half), U(row, second half), [row starts] V(row + 1), U(row + 1, first half), ...
    auto row = [&](auto buf_tag, bool more, float (&m_out)[N][2], auto &&valu0, auto &&valu1) __attribute__((always_inline)) {
        constexpr int BUF = decltype(buf_tag)::value;
        // this wave's chunks of V(row) have landed: the two halves of U(row) were issued after them
        asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
        __syncthreads();              // everyone's have; everyone is done with the row before, whose buffer is free
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            // U of this half has landed.  Issued after it: first half -- the second half; second half --
            // V(row + 1) and U(row + 1, first half), if there is a next row
            if (half == 0) asm volatile("s_waitcnt vmcnt(%0)" : : "n"(G) : "memory");
            else if (!more) asm volatile("s_waitcnt vmcnt(0)" : : : "memory");
            else if (v_all) asm volatile("s_waitcnt vmcnt(%0)" : : "n"(G + V_LOADS) : "memory");
            else asm volatile("s_waitcnt vmcnt(%0)" : : "n"(G + V_LOADS - 1) : "memory");
            if (half == 0 && more) issue_v_row(BUF ^ 1);
            half8 fa[G][CB], fb[G][CB];
            float4v acc[G];
            auto read_fragments = [&](int jj) __attribute__((always_inline)) {
                const int j = half * G + jj;
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) {
                    fa[jj][cb] = *reinterpret_cast<const half8 *>(a_at + j * U_STAGE + cb * (U_STAGE / CB));
                    fb[jj][cb] = *reinterpret_cast<const half8 *>(b_at + BUF * V_ROW + (j * CB + cb) * V_CHUNK);
                }
            };
#pragma unroll
            for (int jj = 0; jj < kFusedAhead && jj < G; ++jj) read_fragments(jj);
            __builtin_amdgcn_sched_barrier(0);
            static_for<G>([&](auto jj_tag) __attribute__((always_inline)) {
                constexpr int jj = decltype(jj_tag)::value;
                if (jj + kFusedAhead < G) read_fragments(jj + kFusedAhead);
                acc[jj] = float4v{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) acc[jj] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fa[jj][cb], fb[jj][cb], acc[jj], 0, 0, 0);
                if (half == 0) valu0(jj_tag); else valu1(jj_tag);
                __builtin_amdgcn_sched_barrier(0);
            });
#pragma unroll
            for (int jj = 0; jj < G; ++jj) {
                m_out[half * G + jj][0] = acc[jj][0];
                m_out[half * G + jj][1] = acc[jj][1];
            }
            if (more) {
                // the places of this half are free once its fragment reads have returned
                asm volatile("s_waitcnt lgkmcnt(0)" : : : "memory");
                issue_u_half(half);
            }
        }
    };

    // Slices of the vector work.  The transform of a finished row along j, for one of the lane's two pairs:
    // slice 0 forms the pairs' sums and differences, slice k >= 1 the outputs 2k - 2 and 2k - 1.
    static_assert(M == 2 * (G - 1), "slices of the row transform");
    float pair_s[HP], pair_d[HP];
    auto transform_slice = [&](auto jj_tag, auto e_tag, const float (&m_in)[N][2], float (&out)[M]) __attribute__((always_inline)) {
        constexpr int jj = decltype(jj_tag)::value, e = decltype(e_tag)::value;
        if constexpr (jj == 0) {
            float v[N];
#pragma unroll
            for (int j = 0; j < N; ++j) v[j] = m_in[j][e];
            output_transform_1d_pairs<N, R>(v, pair_s, pair_d);
#pragma unroll
            for (int j = 0; j < HP; ++j) { stays_here(pair_s[j]); stays_here(pair_d[j]); }
        } else {
#pragma unroll
            for (int i = 2 * jj - 2; i < 2 * jj; ++i) {
                out[i] = output_transform_1d_out<N, R>(i, m_in[0][e], m_in[N - 1][e], pair_s, pair_d, coef);
                stays_here(out[i]);
            }
        }
    };
    // The fold of the rows +a (odd, `carried`) and -a (even, `w`) of a pair of points into Y, through their
    // sum and difference: slice k < m / 2 takes the output rows 2k and 2k + 1.
    float carried[2][M], w[2][M];
    auto fold_slice = [&](auto jj_tag, auto e_tag, const float *c) __attribute__((always_inline)) {
        constexpr int jj = decltype(jj_tag)::value, e = decltype(e_tag)::value;
        if constexpr (2 * jj < M) {
#pragma unroll
            for (int p = 2 * jj; p < 2 * jj + 2; ++p) {
                const float cp = c[p];
#pragma unroll
                for (int q = 0; q < M; ++q) {
                    const float sd = (p & 1) ? carried[e][q] - w[e][q] : carried[e][q] + w[e][q];
                    Y[e][p][q] = fma32(cp, sd, Y[e][p][q]);
                    stays_here(Y[e][p][q]);
                }
            }
        }
    };
    constexpr std::integral_constant<int, 0> kFirst{};
    constexpr std::integral_constant<int, 1> kSecond{};

    issue_v_row(0);
    issue_u_half(0);
    issue_u_half(1);
    float m_even[N][2], m_odd[N][2];
#pragma unroll
    for (int j = 0; j < N; ++j) m_odd[j][0] = m_odd[j][1] = 0.0f;      // "row -1"
#pragma unroll
    for (int q = 0; q < M; ++q) carried[1][q] = w[1][q] = 0.0f;          // "pair -1" of the second pair
    // In turn d: row 2d while row 2d - 1 is transformed (-> carried) and the lane's second pair takes the
    // pair of points d - 1 (for d = 0: zeros); row 2d + 1 while row 2d is transformed (-> w) and the lane's
    // first pair takes the pair of points d (for d = 0: "row -1", zeros, and row 0, the point 0).
#pragma unroll 1
    for (int d = 0; d < N / 2; ++d) {
        const float *c_before = fold.c + (d > 0 ? d - 1 : 0) * M;
        const float *c_this = fold.c + d * M;
        row(kFirst, true, m_even,
            [&](auto jj) __attribute__((always_inline)) { transform_slice(jj, kFirst, m_odd, carried[0]); fold_slice(jj, kSecond, c_before); },
            [&](auto jj) __attribute__((always_inline)) { transform_slice(jj, kSecond, m_odd, carried[1]); });
        row(kSecond, d + 1 < N / 2, m_odd,
            [&](auto jj) __attribute__((always_inline)) { transform_slice(jj, kFirst, m_even, w[0]); },
            [&](auto jj) __attribute__((always_inline)) { transform_slice(jj, kSecond, m_even, w[1]); fold_slice(jj, kFirst, c_this); });
    }
    static_for<G>([&](auto jj) __attribute__((always_inline)) { fold_slice(jj, kSecond, fold.c + (N / 2 - 1) * M); });
    // row n - 1: the point at infinity
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        float v[N], last[M];
#pragma unroll
        for (int j = 0; j < N; ++j) v[j] = m_odd[j][e];
        output_transform_1d<N, R, true>(v, last, coef);
#pragma unroll
        for (int q = 0; q < M; ++q) Y[e][M - 1][q] = fma32(coef.inf, last[q], Y[e][M - 1][q]);
    }

    // ---- the results leave through LDS: all 64 channels at once if the block fits, else 32 at a time
    f16 *stage = reinterpret_cast<f16 *>(lds_raw);
    const int tile = lane & 15;
    const int jr = tile / sh.twc, jc = tile - jr * sh.twc;
    const bool active = tile < sh.twb && tc0 + jc < tiles_w && tr + jr < tiles_h;
    const float floor_at = relu ? 0.0f : -__builtin_inff();          // val < floor ? floor : val keeps a NaN
    constexpr int KB = kFusedChannels / kChanBlock;
    const int per_pass = one_pass ? KB : 1;
#pragma unroll 1
    for (int pass = 0; pass < KB; pass += per_pass) {
        __syncthreads();              // the operand buffers (first pass) or the block before have been read
        if (active && (one_pass || (wave >> 2) == pass)) {
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int k_in = (one_pass ? wave : (wave & 3)) * kFusedWaveChannels + 2 * (lane >> 4) + e;
                f16 *dst = stage + k_in * sh.k_pitch + jr * M * sh.cols_pitch + jc * M;
#pragma unroll
                for (int p = 0; p < M; ++p)
#pragma unroll
                    for (int q = 0; q < M; ++q) {
                        const float val = Y[e][p][q];
                        dst[p * sh.cols_pitch + q] = (f16)(val < floor_at ? floor_at : val);
                    }
            }
        }
        __syncthreads();
        for (int blk = 0; blk < per_pass; ++blk)
            store_output_block<f16, M, STG>(stage + blk * kChanBlock * sh.k_pitch, y, img, k0 / kChanBlock + pass + blk, tr, tc0,
                                            K, H, W, tiles_w, sh);
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
    // The 16 tile slots of a workgroup are a block of trb x twc tiles.  Chosen: the block shape with the lowest
    // estimated cost per tile of the image -- slots launched (ragged last blocks and twc * trb < 16 waste some)
    // times a factor 1 + 1.2 / twc for narrow blocks (short runs of V and of y; fitted to timings: 4 x 4 blocks
    // cost 1.14-1.22 times what full rows of 10-14 tiles cost per slot) -- among those whose output block leaves
    // in 16-byte stores (its width a whole number of pieces, or one block spanning the image width).
    const bool aligned = ((uintptr_t)y % 16) == 0;
    int twb = 1, trb = 1;
    double best = -1.0;
    for (int tc = 1; tc <= kFusedTiles && tc <= g.tiles_w; ++tc)
        for (int tr = 1; tr * tc <= kFusedTiles && tr <= g.tiles_h; ++tr) {
            const int across = ceil_div(g.tiles_w, tc), down = ceil_div(g.tiles_h, tr);
            const bool fast = aligned && (across == 1 || (g.W % PE == 0 && (tc * M) % PE == 0));
            const double used = (double)g.tiles_w * g.tiles_h / ((double)across * down * kFusedTiles);
            const double merit = used / (1.0 + 1.2 / tc) * (fast ? 1.0 : 0.5);
            if (merit > best * (1.0 + 1e-9)) { best = merit; twb = tc; trb = tr; }
        }
    OutShape sh;
    sh.groups = ceil_div(g.tiles_w, twb);
    const size_t stage_bytes = out_shape<N, R, f16>(twb, trb, sh);
    const size_t loop_bytes = (size_t)2 * N * CB * kFusedTiles * 64 + (size_t)kFusedWaves * N * CB * kFusedWaveChannels * 64;
    constexpr int KB = kFusedChannels / kChanBlock;
    const int one_pass = KB * stage_bytes <= 160 * 1024 ? 1 : 0;      // all blocks of 32 channels staged together
    const size_t out_bytes = one_pass ? KB * stage_bytes : stage_bytes;
    const size_t lds_bytes = out_bytes > loop_bytes ? out_bytes : loop_bytes;
    if (lds_bytes > 160 * 1024 || sh.twb > kFusedTiles) return (int)hipErrorInvalidValue;
    // 32-bit byte offsets inside one position of V
    if ((size_t)CB * g.T * kChanBlock * sizeof(f16) >= ((size_t)1 << 32)) return (int)hipErrorInvalidValue;
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
                       (flags & NOVA_FLAG_RELU) ? 1 : 0, one_pass, sh, coef, fold);
    return (int)hipGetLastError();
}

// Shapes the fused kernel takes: binary16 storage, products not rounded to binary16, points in the paired
// order, F(6,3) or F(8,3), C = 64, K a multiple of 32.
bool fused_contract_output_applies(const nova_transforms *t, const Geometry &g, int dtype, int flags)
{
    return dtype == NOVA_F16 && !(flags & NOVA_FLAG_M_F16) && t->symmetric && t->r == 3 && (t->n == 8 || t->n == 10) &&
           g.C == kFusedCB * kChanBlock && g.K % kFusedChannels == 0 && g.T <= 0x7fffffffLL;
}

// ... and those for which nova_winograd_conv2d takes it: all of them (measured against contraction + output
// transform on one MI355X, F(8,3) and F(6,3), 224 x 224 down to 13 x 13: faster on every shape it takes).
bool fused_contract_output_preferred(const nova_transforms *t, const Geometry &g, int dtype, int flags)
{
    return fused_contract_output_applies(t, g, dtype, flags);
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
