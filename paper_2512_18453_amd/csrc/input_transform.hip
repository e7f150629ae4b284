// Input transform V = B^T d B (Sec. 2.1 step 1, nested in 2D) for every n x n tile of the
// zero-padded image, x [N][C][H][W] -> V [n*n][C/32][T][32].
//
// One workgroup takes one image, one tile row, a group of TWB neighbouring tiles and one block
// of 32 channels (for narrow images, where a tile row has few tiles: TRB neighbouring tile rows
// of full width).  The 32-channel x (TRB*m + r - 1 rows) x (TWB*m + r - 1 columns) input strip is
// staged in LDS in the order it has in memory (16-byte pieces, all loads of a round in flight
// together), with a channel pitch that keeps the per-thread window reads free of bank conflicts.
// Thread = one tile x one channel (32 consecutive lanes = 32 consecutive channels); a pair of waves
// shares two tiles and splits the rows of the transform between them.  The n*n results of a tile
// go back through LDS as [tile][xi][32 channels], so that they leave in 16-byte stores: the tiles
// of a group are adjacent in t, so a workgroup writes TWB*64 (fp16) contiguous bytes per xi.
//
// Arithmetic contract (binary32): a 1D transform row is E + O, with E / O fused multiply-add
// chains over the even / odd input indices in ascending order, columns of the tile first, then
// rows.  For points given as 0, +a, -a, ... the rows of +a and -a share E and O (the even
// coefficients agree, the odd ones are negated), which gives bit-identical results at half the
// multiplications.  The result is rounded once to the storage format.
#include "device_common.hpp"

namespace nova {

// Rows [LO, HI) of one 1D transform: out[p - LO] = sum_a B^T[p][a] v[a] in the contracted order.
// With SYM the range must not cut a (+a, -a) pair of rows (rows 2q+1, 2q+2).
template <int N, bool SYM, int LO, int HI>
__device__ __forceinline__ void input_transform_rows(const float (&v)[N], float (&out)[HI - LO], const InCoef<N> &k)
{
    constexpr int H = (N - 2) / 2;
    if constexpr (SYM) {
        if constexpr (LO == 0) {
            float e0 = 0.0f;
#pragma unroll
            for (int q = 0; q <= H; ++q) e0 = fma32(k.zero[q], v[2 * q], e0);
            out[0] = e0;
        }
#pragma unroll
        for (int j = 0; j < H; ++j) {
            if (2 * j + 1 >= LO && 2 * j + 2 < HI) {
                float E = 0.0f, O = 0.0f;
#pragma unroll
                for (int q = 0; q < H; ++q) E = fma32(k.ev[j * H + q], v[2 * q + 2], E);
#pragma unroll
                for (int q = 0; q < H; ++q) O = fma32(k.od[j * H + q], v[2 * q + 1], O);
                out[2 * j + 1 - LO] = E + O;
                out[2 * j + 2 - LO] = E - O;
            }
        }
        if constexpr (HI == N) {
            float oi = 0.0f;
#pragma unroll
            for (int q = 0; q <= H; ++q) oi = fma32(k.inf[q], v[2 * q + 1], oi);
            out[N - 1 - LO] = oi;
        }
    } else {
#pragma unroll
        for (int p = LO; p < HI; ++p) {
            float E = 0.0f, O = 0.0f;
#pragma unroll
            for (int a = 0; a < N; a += 2) E = fma32(k.bt[p * N + a], v[a], E);
#pragma unroll
            for (int a = 1; a < N; a += 2) O = fma32(k.bt[p * N + a], v[a], O);
            out[p - LO] = E + O;
        }
    }
}

// Where the rows are split between the two waves that share a tile pair: half 0 takes rows
// [0, SP), half 1 rows [SP, N); SP is odd so that no (+a, -a) pair of rows is cut.
template <int N> struct RowSplit { static constexpr int value = ((N / 2) % 2 == 1) ? N / 2 : N / 2 + 1; };

// LDS strip: [32 channels][N rows][row_pitch columns], columns fastest (the order of x in
// memory, so staging moves 16-byte pieces); strip column lc holds image column w_al + lc, where
// w_al is the first needed column w_lo rounded down to a whole piece.  The channel pitch is
// 4 * odd elements: rows stay 8-byte aligned for the staging writes, and the 32 channels that a
// half-wave reads at one (row, column) fall into 32 different banks.
struct StripShape {
    int twb;         // tiles per group (all tile rows of the group together)
    int trb;         // tile rows per group; > 1 only if a group spans the image width
    int rows;        // strip rows = trb * m + r - 1
    unsigned rows_magic;    // ceil(2^32 / rows)
    int groups;      // tile groups per tile row
    int pieces;      // 16-byte pieces per strip row (vector path) / columns per row (scalar path)
    int row_pitch;   // elements
    int ch_pitch;    // elements
    unsigned piece_magic;   // ceil(2^32 / pieces): s / pieces == mulhi(s, magic) while s * pieces < 2^32
    unsigned w_magic;       // the same for W (flat staging)
    int cs, passes, iters;  // vector staging: channels per chunk of a wave, passes of 64 lanes per chunk, chunks per wave
    unsigned slot_magic;    // ceil(2^32 / (rows * pieces))
};

// How the strip gets into LDS.
//   kStageScalar  any W, any group: element by element, lanes along W
//   kStageVec     W a multiple of a 16-byte piece and x 16-byte aligned: pieces never straddle rows
//   kStageFlat    the group spans the whole image width (narrow images) and x is 16-byte aligned:
//                 the rows a strip needs are one contiguous run of each channel plane, fetched in
//                 aligned 16-byte pieces whatever W is and scattered to their (row, column) in LDS
enum { kStageScalar = 0, kStageVec = 1, kStageFlat = 2 };

template <int N, typename T, bool SYM, bool ALIGNED, int LO, int HI>
__device__ __forceinline__ void transform_rows_of_tile(const T *tile, int row_pitch, T *mine, int xi_pitch,
                                                       const InCoef<N> &coef)
{
    // columns of the tile first: tmp[i - LO][b] = sum_a B^T[i][a] d[a][b] for this wave's rows i
    float tmp[HI - LO][N];
    T win[N][N];                                  // the tile window d[a][b] in storage format
    if constexpr (ALIGNED) {
        // m = 8 and a strip whose column 0 is a multiple of 8: columns 1..8 of every window row are
        // one aligned 16-byte (fp16) or two aligned 16-byte (fp32) reads; an unaligned wide LDS read
        // costs several passes
        constexpr int PE = 16 / (int)sizeof(T);
        typedef T vecT __attribute__((ext_vector_type(PE)));
#pragma unroll
        for (int a = 0; a < N; ++a) {
            const T *row = tile + a * row_pitch;
            win[a][0] = row[0];
#pragma unroll
            for (int v = 0; v < 8 / PE; ++v) {
                const vecT piece = *reinterpret_cast<const vecT *>(__builtin_assume_aligned(row + 1 + v * PE, 16));
#pragma unroll
                for (int e = 0; e < PE; ++e) win[a][1 + v * PE + e] = piece[e];
            }
            win[a][9] = row[9];
        }
    } else {
#pragma unroll
        for (int a = 0; a < N; ++a)
#pragma unroll
            for (int b = 0; b < N; ++b) win[a][b] = tile[a * row_pitch + b];
    }
#pragma unroll
    for (int b = 0; b < N; ++b) {
        float d[N], o[HI - LO];
#pragma unroll
        for (int a = 0; a < N; ++a) d[a] = (float)win[a][b];
        input_transform_rows<N, SYM, LO, HI>(d, o, coef);
#pragma unroll
        for (int i = 0; i < HI - LO; ++i) tmp[i][b] = o[i];
    }
    // then along each of those rows: V[i][j] = sum_b tmp[i][b] B^T[j][b], rounded to storage
#pragma unroll
    for (int i = LO; i < HI; ++i) {
        float o[N];
        input_transform_rows<N, SYM, 0, N>(tmp[i - LO], o, coef);
#pragma unroll
        for (int jj = 0; jj < N; ++jj) mine[((i - LO) * N + jj) * xi_pitch] = round_twice(o[jj], (T *)nullptr);
    }
}

template <int N, int R, typename T, bool SYM, int STG>
__global__ void __launch_bounds__(N <= 8 ? 640 : 512)     // (n <= 8: groups of up to 10 tiles)
input_transform_kernel(const T *__restrict__ x, T *__restrict__ V, int C, int H, int W,
                       int tiles_h, int tiles_w, int c_blocks, long long Ttot, long long x_elems,
                       StripShape sh, InCoef<N> coef)
{
    constexpr bool VEC = STG == kStageVec;
    constexpr int M = N - R + 1;                 // outputs per tile side = tile stride
    constexpr int PAD = (R - 1) / 2;             // zero border of the convolution
    constexpr int PE = 16 / (int)sizeof(T);      // elements per 16-byte piece
    constexpr int SP = RowSplit<N>::value;
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
    extern __shared__ __align__(16) unsigned char lds_raw[];
    T *lds = reinterpret_cast<T *>(lds_raw);

    // block -> (image, channel block, tile row, tile group); group fastest
    unsigned bid = xcd_local_block_id(blockIdx.x, gridDim.x);
    const int row_groups = (tiles_h + sh.trb - 1) / sh.trb;
    const int tg = bid % sh.groups; bid /= sh.groups;
    const int tr = (bid % row_groups) * sh.trb; bid /= row_groups;      // first tile row of the group
    const int cb = bid % c_blocks; bid /= c_blocks;
    const int img = bid;

    const int tc0 = sh.trb > 1 ? 0 : tg * sh.twb;
    const int h_lo = tr * M - PAD;        // image row of strip row 0
    const int w_lo = tc0 * M - PAD;       // first image column the group needs
    int w_al = w_lo;                      // image column of strip column 0

    // ---- stage the strip [32 channels][N rows][columns] in the order it has in memory
    if constexpr (VEC) {
        // W is a multiple of PE and x is 16-byte aligned: every piece is wholly inside or outside
        // the image.  All loads of a round are issued before the first LDS write waits on them.
        w_al = (w_lo + PE) / PE * PE - PE;        // floor to a multiple of PE (w_lo >= -PAD >= -PE)
        // A wave takes sh.cs whole channels at a time (1 unless the strip of one channel has fewer
        // than 64 pieces) and its lanes run over their (channel, row, piece) slots in sh.passes passes
        // of 64.  What a lane does in one pass -- its offset in the channel plane, its place in LDS,
        // whether the piece lies inside the image -- is decoded once and holds for every chunk of
        // channels the wave visits; a chunk only moves the (scalar) plane base and the LDS base.
        const int a_lo = h_lo < 0 ? -h_lo : 0, a_hi = H - h_lo < sh.rows ? H - h_lo : sh.rows;
        const int q_lo = w_al < 0 ? (-w_al) / PE : 0, q_hi = (W - w_al) / PE < sh.pieces ? (W - w_al) / PE : sh.pieces;
        const int c_lim = C - cb * kChanBlock < kChanBlock ? C - cb * kChanBlock : kChanBlock;
        const unsigned a_span = (unsigned)(a_hi - a_lo), q_span = (unsigned)(q_hi - q_lo);
        const T *blk = x + ((size_t)img * C + (size_t)cb * kChanBlock) * H * W;
        const int HW = H * W;
        const int slots = sh.rows * sh.pieces;                       // per channel
        const int lane = (int)(threadIdx.x & 63);
        const int wave_u = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
        const int n_waves = (int)(blockDim.x >> 6);
        constexpr int PU = 2, IU = 4;              // passes x chunks whose loads are in flight together
        for (int p0 = 0; p0 < sh.passes; p0 += PU) {
            int dst[PU], room[PU];
            unsigned src[PU];
            bool slot[PU], inside[PU];
#pragma unroll
            for (int pp = 0; pp < PU; ++pp) {
                const int s = lane + 64 * (p0 + pp);
                const int c_sub = (int)__umulhi((unsigned)s, sh.slot_magic);
                const int rem = s - c_sub * slots;
                const int a = (int)__umulhi((unsigned)rem, sh.piece_magic), q = rem - a * sh.pieces;
                slot[pp] = p0 + pp < sh.passes && c_sub < sh.cs;
                room[pp] = c_lim - c_sub;                     // the chunk's first channel must stay below this
                inside[pp] = slot[pp] && (unsigned)(a - a_lo) < a_span && (unsigned)(q - q_lo) < q_span;
                dst[pp] = c_sub * sh.ch_pitch + a * sh.row_pitch + q * PE;
                src[pp] = (unsigned)(c_sub * HW + (h_lo + a) * W + w_al + q * PE) * (unsigned)sizeof(T);
            }
            // a lane outside the image never loads: its registers keep the zeros it writes to LDS
            u32x4 val[IU][PU];
#pragma unroll
            for (int u = 0; u < IU; ++u)
#pragma unroll
                for (int pp = 0; pp < PU; ++pp) val[u][pp] = u32x4{0u, 0u, 0u, 0u};
            for (int it0 = 0; it0 < sh.iters; it0 += IU) {
                if (c_lim < kChanBlock) {
                    // ragged channel block: a lane may load for one chunk and not for the next
#pragma unroll
                    for (int u = 0; u < IU; ++u)
#pragma unroll
                        for (int pp = 0; pp < PU; ++pp) val[u][pp] = u32x4{0u, 0u, 0u, 0u};
                }
#pragma unroll
                for (int u = 0; u < IU; ++u) {
                    const int c0 = ((it0 + u) * n_waves + wave_u) * sh.cs;       // wave-uniform
                    if (c0 < kChanBlock) {
                        const T *plane = blk + (size_t)c0 * HW;
#pragma unroll
                        for (int pp = 0; pp < PU; ++pp)
                            if (inside[pp] && c0 < room[pp])
                                // x is not read again by this call: streaming hint, so that it does not
                                // push V and M out of the last-level cache
                                val[u][pp] = __builtin_nontemporal_load(
                                    reinterpret_cast<const NOVA_GLOBAL u32x4 *>(plane_element(plane, src[pp])));
                    }
                }
#pragma unroll
                for (int u = 0; u < IU; ++u) {
                    const int c0 = ((it0 + u) * n_waves + wave_u) * sh.cs;
                    if (c0 < kChanBlock) {
#pragma unroll
                        for (int pp = 0; pp < PU; ++pp)
                            if (slot[pp]) {
                                u32x2 *p = reinterpret_cast<u32x2 *>(lds + c0 * sh.ch_pitch + dst[pp]);
                                p[0] = u32x2{val[u][pp].x, val[u][pp].y};
                                p[1] = u32x2{val[u][pp].z, val[u][pp].w};
                            }
                    }
                }
            }
        }
    } else if constexpr (STG == kStageFlat) {
        // The group spans the image width (tc0 = 0, w_lo = -PAD).  Rows h0..h1 of one channel are one
        // run of (h1 - h0 + 1) * W elements; it is covered with 16-byte pieces aligned in x (their
        // ends may belong to neighbouring rows or channels: those elements are dropped), and every
        // element goes to its own (row, column) of the strip.  What the image does not cover
        // (halo column and rows, tile padding) is zeroed first.
        {
            const int words = kChanBlock * sh.ch_pitch * (int)sizeof(T) / 8;     // ch_pitch: a multiple of 4 elements
            u32x2 *z = reinterpret_cast<u32x2 *>(lds);
            for (int s = threadIdx.x; s < words; s += (int)blockDim.x) z[s] = u32x2{0u, 0u};
        }
        __syncthreads();
        const int h0 = h_lo < 0 ? 0 : h_lo;
        const int h1 = h_lo + sh.rows - 1 > H - 1 ? H - 1 : h_lo + sh.rows - 1;
        const int run = (h1 - h0 + 1) * W;
        const int slots = kChanBlock * sh.pieces;
        constexpr int RT = 4;
        for (int base = threadIdx.x; base < slots; base += RT * (int)blockDim.x) {
            T val[RT][PE];
            int rel[RT], c_of[RT];
#pragma unroll
            for (int r = 0; r < RT; ++r) {
                const int s = base + r * (int)blockDim.x;
                const int c_in = (int)__umulhi((unsigned)s, sh.piece_magic);
                const int k = s - c_in * sh.pieces;
                const int c = cb * kChanBlock + c_in;
                const long long e0 = (((long long)img * C + c) * H + h0) * W;     // first element of the run
                const long long p0 = (e0 & ~(long long)(PE - 1)) + (long long)k * PE;
                rel[r] = (int)(p0 - e0);                                           // -(PE-1) .. run-1 if needed
                c_of[r] = c_in;
                const bool ok = s < slots && c < C && rel[r] < run;
                if (!ok) rel[r] = run;                                             // nothing of it is used
#pragma unroll
                for (int e = 0; e < PE; ++e) val[r][e] = (T)0.0f;
                if (ok) {
                    if (p0 + PE <= x_elems) {
                        const u32x4 piece = *reinterpret_cast<const u32x4 *>(x + p0);
                        __builtin_memcpy(val[r], &piece, 16);
                    } else {
                        // the last piece of x when its size is not a multiple of a piece
#pragma unroll
                        for (int e = 0; e < PE; ++e)
                            if (p0 + e < x_elems) val[r][e] = x[p0 + e];
                    }
                }
            }
#pragma unroll
            for (int r = 0; r < RT; ++r) {
                // (row, column) of the first element that belongs to the run, then step along it
                int q = rel[r] < 0 ? 0 : rel[r];
                int hr = (int)__umulhi((unsigned)q, sh.w_magic);
                int w = q - hr * W;
                T *row0 = lds + c_of[r] * sh.ch_pitch + (h0 - h_lo) * sh.row_pitch + PAD;  // column of w = 0
#pragma unroll
                for (int e = 0; e < PE; ++e) {
                    const int pos = rel[r] + e;
                    if (pos >= 0 && pos < run) {
                        row0[hr * sh.row_pitch + w] = val[r][e];
                        if (++w == W) { w = 0; ++hr; }
                    }
                }
            }
        }
    } else {
        // any W: element-wise, lanes along W
        const int cols = sh.pieces;
        const int slots = kChanBlock * sh.rows * cols;
        constexpr int RT = 8;
        for (int base = threadIdx.x; base < slots; base += RT * (int)blockDim.x) {
            T val[RT];
            int dst[RT];
#pragma unroll
            for (int r = 0; r < RT; ++r) {
                const int s = base + r * (int)blockDim.x;
                const int line = (int)__umulhi((unsigned)s, sh.piece_magic);
                const int q = s - line * cols;
                const int c_in = (int)__umulhi((unsigned)line, sh.rows_magic), a = line - c_in * sh.rows;
                const int c = cb * kChanBlock + c_in, h = h_lo + a, w = w_al + q;
                const bool ok = s < slots && c < C && h >= 0 && h < H && w >= 0 && w < W;
                dst[r] = s < slots ? c_in * sh.ch_pitch + a * sh.row_pitch + q : -1;
                val[r] = (T)0.0f;
                if (ok) val[r] = x[(((size_t)img * C + c) * H + h) * W + w];
            }
#pragma unroll
            for (int r = 0; r < RT; ++r)
                if (dst[r] >= 0) lds[dst[r]] = val[r];
        }
    }
    __syncthreads();

    // ---- transform.  Waves come in pairs that share two tiles: lane = (tile of the pair, channel),
    // and the two waves of a pair take the transform rows [0, SP) and [SP, N) -- half the registers
    // per thread, twice the waves, and no work done twice (the rows of a 1D transform are
    // independent once no +a/-a pair is cut).  The results are collected in registers first ...
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int j = (wave >> 1) * 2 + (lane >> 5), c_in = lane & 31, half = wave & 1;
    int jr = 0, jc = j;                       // tile row and column inside the group
    if (sh.trb > 1) { jr = j / tiles_w; jc = j - jr * tiles_w; }
    const bool active = j < sh.twb && tc0 + jc < tiles_w && tr + jr < tiles_h;
    const T *tile = lds + c_in * sh.ch_pitch + jr * M * sh.row_pitch + (w_lo - w_al) + jc * M;
    constexpr int ROWS_MAX = SP > N - SP ? SP : N - SP;
    T res[ROWS_MAX * N];
    if (active) {
        constexpr bool AL = VEC && N == 10 && R == 3;   // window column 1 = image column 8*(tc0+j): 16-byte aligned
        if (half == 0) transform_rows_of_tile<N, T, SYM, AL, 0, SP>(tile, sh.row_pitch, res, 1, coef);
        else           transform_rows_of_tile<N, T, SYM, AL, SP, N>(tile, sh.row_pitch, res, 1, coef);
    }
    __syncthreads();                          // the strip has been read; its LDS is reused below

    // ... and go back through LDS as [tile of the group][xi][32 channels], so that they leave in
    // 16-byte stores (2-byte stores, one per lane and position, are what limits this kernel
    // otherwise): for one xi the tiles of the group are adjacent in V, twb*64 contiguous bytes.
    // A tile takes (N*N + 1) rows of 32 channels: the spare row shifts neighbouring tiles by a
    // quarter (binary16) or half (binary32) of the banks, so that the 16-byte reads below, which
    // run over tiles within one xi, do not collide.
    constexpr int TS = (N * N + 1) * kChanBlock;              // elements per tile
    if (active) {
        const int count = half == 0 ? SP * N : (N - SP) * N;
        T *mine = lds + j * TS + (half == 0 ? 0 : SP * N * kChanBlock) + c_in;
#pragma unroll
        for (int e = 0; e < ROWS_MAX * N; ++e)
            if (e < count) mine[e * kChanBlock] = res[e];
    }
    __syncthreads();
    {
        constexpr int PPR = kChanBlock / PE;               // 16-byte pieces per (xi, tile) row
        // tiles of the group that exist; consecutive tile rows of full width are adjacent in t
        int valid = tiles_w - tc0; if (valid > sh.twb) valid = sh.twb; if (valid < 0) valid = 0;
        if (sh.trb > 1) {
            int tile_rows = tiles_h - tr; if (tile_rows > sh.trb) tile_rows = sh.trb;
            valid = tile_rows * tiles_w;
        }
        const long long t0 = ((long long)img * tiles_h + tr) * tiles_w + tc0;
        const size_t in_plane = ((size_t)cb * Ttot + t0) * kChanBlock;
        const size_t xi_stride = (size_t)c_blocks * Ttot * kChanBlock;
        const int n_waves = (int)blockDim.x >> 6;
        const int wave_u = __builtin_amdgcn_readfirstlane(wave);
        // a lane moves the same piece of every xi: piece lane of the valid * PPR <= 64 that one xi has
        const bool on = lane < valid * PPR;
        const T *src = lds + (lane / PPR) * TS + (lane % PPR) * PE;
        constexpr int UN = 4;                               // LDS reads in flight before the stores
        for (int xi0 = wave_u; xi0 < N * N; xi0 += UN * n_waves) {
            u32x4 piece[UN];
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int xi = xi0 + u * n_waves;
                if (xi < N * N && on) piece[u] = *reinterpret_cast<const u32x4 *>(src + xi * kChanBlock);
            }
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int xi = xi0 + u * n_waves;
                if (xi < N * N && on) {
                    T *plane = V + (size_t)xi * xi_stride + in_plane;
                    *reinterpret_cast<NOVA_GLOBAL u32x4 *>(plane_element(plane, (unsigned)lane * 16u)) = piece[u];
                }
            }
        }
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

// Strip geometry for groups of `trb` tile rows x `twb` tiles; returns the LDS bytes it needs.
template <int N, int R, typename T>
static size_t strip_shape(int twb, int trb, bool vec, StripShape &sh)
{
    sh.w_magic = 0;
    constexpr int M = N - R + 1;
    constexpr int PE = 16 / (int)sizeof(T);
    const int need = twb * M + R - 1;                   // columns w_lo .. w_lo + need - 1
    sh.trb = trb;
    sh.rows = trb * M + R - 1;
    sh.rows_magic = (unsigned)((((unsigned long long)1 << 32) + sh.rows - 1) / sh.rows);
    if (vec) {
        // worst-case offset of w_lo inside its piece is PE - 1
        sh.pieces = (need + PE - 1 + PE - 1) / PE;
        sh.row_pitch = sh.pieces * PE;
    } else {
        sh.pieces = need;
        sh.row_pitch = (need + 3) / 4 * 4;
    }
    // channel pitch: an odd multiple of 16 bytes on the vector path (aligned 128-bit reads, and the
    // 16 lanes of one read phase cover all 64 banks), else 4 * odd elements
    const int unit = vec ? 16 / (int)sizeof(T) : 4;
    int chp = (sh.rows * sh.row_pitch + unit - 1) / unit * unit;
    if ((chp / unit) % 2 == 0) chp += unit;
    sh.ch_pitch = chp;
    sh.twb = twb * trb;
    sh.piece_magic = (unsigned)((((unsigned long long)1 << 32) + sh.pieces - 1) / sh.pieces);
    return (size_t)kChanBlock * chp * sizeof(T);
}

template <int N, int R, typename T>
static int launch_it(const nova_transforms *t, const void *x, void *V, const Geometry &g, hipStream_t stream)
{
    constexpr int PE = 16 / (int)sizeof(T);
    InCoef<N> coef;
    fill_in_coef<N>(t, coef);
    // (vector path: byte offsets inside one block of 32 channel planes are 32-bit)
    const bool vec = g.W % PE == 0 && ((uintptr_t)x % 16) == 0 &&
                     (long long)kChanBlock * g.H * g.W * (long long)sizeof(T) < (1LL << 31);
    // tiles per group: at most 8 (two waves per tile pair, 512 threads); a row of 9 or 10 tiles (56 x 56 at
    // m = 6) is taken whole for n <= 8 instead of split 5 + 5 (wider rows measured slower in groups of 10:
    // 224 x 224 at m = 6, 234 against 174 us); the LDS block holds first
    // the strip, then the results [xi][tile][32], and may take at most 64 KiB
    StripShape sh;
    auto lds_need = [&](int twb, int trb) {
        const size_t strip = strip_shape<N, R, T>(twb, trb, vec, sh);
        const size_t out_stage = (size_t)(N * N + 1) * twb * trb * kChanBlock * sizeof(T);
        return strip > out_stage ? strip : out_stage;
    };
    // (binary16 only: the store loop moves one position's valid * 32 / PE <= 64 pieces in one step)
    int twb_max = (N <= 8 && sizeof(T) == 2 && g.tiles_w > 8 && g.tiles_w <= 10) ? 10 : 8;
    while (twb_max > 1 && lds_need(twb_max, 1) > 64 * 1024) --twb_max;
    sh.groups = ceil_div(g.tiles_w, twb_max);
    const int twb = ceil_div(g.tiles_w, sh.groups);      // tiles of one tile row per group
    // narrow images: a group spans the width; give it as many tile rows as keep it within 8 tiles
    int trb = 1;
    if (sh.groups == 1) {
        trb = 8 / twb;
        if (trb < 1) trb = 1;
        if (trb > g.tiles_h) trb = g.tiles_h;
        while (trb > 1 && lds_need(twb, trb) > 64 * 1024) --trb;
    }
    trb = ceil_div(g.tiles_h, ceil_div(g.tiles_h, trb));    // same number of groups, evenly sized
    const size_t lds_bytes = lds_need(twb, trb);         // (leaves sh.groups alone)
    if (lds_bytes > 64 * 1024 || sh.pieces < 2) return (int)hipErrorInvalidValue;
    // narrow images whose width is not a whole number of pieces: flat staging
    // (W >= 2: the reciprocal used for divisions by W does not exist for 1; such images take the scalar path)
    const bool flat = !vec && sh.groups == 1 && ((uintptr_t)x % 16) == 0 && g.W >= 2 &&
                      (long long)sh.rows * g.W < (1 << 15);
    if (flat) {
        sh.pieces = (sh.rows * g.W + 2 * (PE - 1)) / PE;    // pieces that can touch a run of rows*W elements
        sh.piece_magic = (unsigned)((((unsigned long long)1 << 32) + sh.pieces - 1) / sh.pieces);
        sh.w_magic = (unsigned)((((unsigned long long)1 << 32) + g.W - 1) / g.W);
    }
    const int threads = ((sh.twb + 1) / 2) * 128;        // a pair of waves per pair of tiles
    {
        const int slots = sh.rows * sh.pieces;           // pieces of one channel's strip
        sh.cs = 1;
        while (sh.cs < kChanBlock && sh.cs * 2 * slots <= 64) sh.cs *= 2;
        sh.passes = ceil_div(sh.cs * slots, 64);
        sh.iters = ceil_div(kChanBlock, (threads / 64) * sh.cs);
        sh.slot_magic = (unsigned)((((unsigned long long)1 << 32) + slots - 1) / slots);
    }
    const long long blocks = (long long)sh.groups * ceil_div(g.tiles_h, trb) * g.c_blocks * g.N;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return (int)hipErrorInvalidValue;
    void (*kern)(const T *, T *, int, int, int, int, int, int, long long, long long, StripShape, InCoef<N>);
    if (t->symmetric)
        kern = vec ? input_transform_kernel<N, R, T, true, kStageVec>
             : flat ? input_transform_kernel<N, R, T, true, kStageFlat> : input_transform_kernel<N, R, T, true, kStageScalar>;
    else
        kern = vec ? input_transform_kernel<N, R, T, false, kStageVec>
             : flat ? input_transform_kernel<N, R, T, false, kStageFlat> : input_transform_kernel<N, R, T, false, kStageScalar>;
    const long long x_elems = (long long)g.N * g.C * g.H * g.W;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(threads), lds_bytes, stream,
                       (const T *)x, (T *)V, g.C, g.H, g.W, g.tiles_h, g.tiles_w, g.c_blocks, g.T, x_elems, sh, coef);
    return (int)hipGetLastError();
}

int launch_input_transform(const nova_transforms *t, const void *x, void *V, const Geometry &g,
                           int dtype, void *stream)
{
    hipStream_t s = (hipStream_t)stream;
    const bool h = dtype == NOVA_F16;
    if (t->r == 3) {
        switch (t->n) {
        case 4: return h ? launch_it<4, 3, f16>(t, x, V, g, s) : launch_it<4, 3, float>(t, x, V, g, s);
        case 6: return h ? launch_it<6, 3, f16>(t, x, V, g, s) : launch_it<6, 3, float>(t, x, V, g, s);
        case 8: return h ? launch_it<8, 3, f16>(t, x, V, g, s) : launch_it<8, 3, float>(t, x, V, g, s);
        case 10: return h ? launch_it<10, 3, f16>(t, x, V, g, s) : launch_it<10, 3, float>(t, x, V, g, s);
        }
    } else if (t->r == 5) {
        switch (t->n) {
        case 6: return h ? launch_it<6, 5, f16>(t, x, V, g, s) : launch_it<6, 5, float>(t, x, V, g, s);
        case 8: return h ? launch_it<8, 5, f16>(t, x, V, g, s) : launch_it<8, 5, float>(t, x, V, g, s);
        case 10: return h ? launch_it<10, 5, f16>(t, x, V, g, s) : launch_it<10, 5, float>(t, x, V, g, s);
        }
    }
    return (int)hipErrorInvalidValue;
}

// ---- Few input channels (C <= 4): V in the compact layout Vc [n*n][T][4] that the few-channel
// output transform reads (no 32-channel blocks: 3 of 32 channels would carry data).  One pair of
// waves takes 16 neighbouring tiles of a tile row and the 4 channels, lane = (tile, channel); the
// two waves split the transform rows as above.  Same arithmetic contract; channels >= C are zero.
constexpr int kFewIn = 4;                  // channels
constexpr int kFewTiles = 64 / kFewIn;     // tiles per group

template <int N, int R, typename T, bool SYM>
__global__ void __launch_bounds__(128)
input_transform_few_kernel(const T *__restrict__ x, T *__restrict__ Vc, int C, int H, int W,
                           int tiles_h, int tiles_w, int groups, long long Ttot, int row_pitch, InCoef<N> coef)
{
    constexpr int M = N - R + 1;
    constexpr int PAD = (R - 1) / 2;
    constexpr int SP = RowSplit<N>::value;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    T *lds = reinterpret_cast<T *>(lds_raw);

    unsigned bid = blockIdx.x;
    const int tg = bid % groups; bid /= groups;
    const int tr = bid % tiles_h; bid /= tiles_h;
    const int img = bid;
    const int tc0 = tg * kFewTiles;
    const int h_lo = tr * M - PAD, w_lo = tc0 * M - PAD;
    const int cols = kFewTiles * M + R - 1;
    const int ch_pitch = N * row_pitch;

    // strip [4 channels][N rows][cols], lanes along W; outside the image and for channels >= C: zero
    const unsigned cols_magic = (unsigned)((((unsigned long long)1 << 32) + cols - 1) / cols);
    const int slots = kFewIn * N * cols;
    constexpr int RT = 8;
    for (int base = threadIdx.x; base < slots; base += RT * (int)blockDim.x) {
        T val[RT];
        int dst[RT];
#pragma unroll
        for (int r = 0; r < RT; ++r) {
            const int s = base + r * (int)blockDim.x;
            const int line = (int)__umulhi((unsigned)s, cols_magic);       // (channel, row)
            const int q = s - line * cols;
            const int c = line / N, a = line - c * N;
            const int h = h_lo + a, w = w_lo + q;
            const bool ok = s < slots && c < C && h >= 0 && h < H && w >= 0 && w < W;
            dst[r] = s < slots ? c * ch_pitch + a * row_pitch + q : -1;
            val[r] = (T)0.0f;
            if (ok) val[r] = x[(((size_t)img * C + c) * H + h) * W + w];
        }
#pragma unroll
        for (int r = 0; r < RT; ++r)
            if (dst[r] >= 0) lds[dst[r]] = val[r];
    }
    __syncthreads();

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int j = lane / kFewIn, c_in = lane % kFewIn;
    if (tc0 + j >= tiles_w) return;
    const T *tile = lds + c_in * ch_pitch + j * M;
    constexpr int ROWS_MAX = SP > N - SP ? SP : N - SP;
    T res[ROWS_MAX * N];
    if (wave == 0) transform_rows_of_tile<N, T, SYM, false, 0, SP>(tile, row_pitch, res, 1, coef);
    else           transform_rows_of_tile<N, T, SYM, false, SP, N>(tile, row_pitch, res, 1, coef);

    // a wave writes 64 consecutive values (16 tiles x 4 channels) per xi
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const int first = wave_u == 0 ? 0 : SP * N, count = wave_u == 0 ? SP * N : (N - SP) * N;
    const long long t0 = ((long long)img * tiles_h + tr) * tiles_w + tc0;
    const unsigned off = (unsigned)lane * (unsigned)sizeof(T);
#pragma unroll
    for (int e = 0; e < ROWS_MAX * N; ++e)
        if (e < count) {
            T *plane = Vc + ((size_t)(first + e) * Ttot + t0) * kFewIn;
            *reinterpret_cast<NOVA_GLOBAL T *>(plane_element(plane, off)) = res[e];
        }
}

template <int N, int R, typename T>
static int launch_it_few(const nova_transforms *t, const void *x, void *Vc, const Geometry &g, hipStream_t stream)
{
    constexpr int M = N - R + 1;
    if (g.C > kFewIn) return (int)hipErrorInvalidValue;
    InCoef<N> coef;
    fill_in_coef<N>(t, coef);
    const int groups = ceil_div(g.tiles_w, kFewTiles);
    const int row_pitch = (kFewTiles * M + R - 1 + 3) / 4 * 4;
    const size_t lds_bytes = (size_t)kFewIn * N * row_pitch * sizeof(T);
    const long long blocks = (long long)groups * g.tiles_h * g.N;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return (int)hipErrorInvalidValue;
    auto kern = t->symmetric ? input_transform_few_kernel<N, R, T, true> : input_transform_few_kernel<N, R, T, false>;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(128), lds_bytes, stream,
                       (const T *)x, (T *)Vc, g.C, g.H, g.W, g.tiles_h, g.tiles_w, groups, g.T, row_pitch, coef);
    return (int)hipGetLastError();
}

size_t few_channels_input_bytes(const Geometry &g, int dtype)
{
    return (size_t)g.n * g.n * (size_t)g.T * kFewIn * dtype_size(dtype);
}

int launch_input_transform_few(const nova_transforms *t, const void *x, void *Vc, const Geometry &g,
                               int dtype, void *stream)
{
    hipStream_t s = (hipStream_t)stream;
    const bool h = dtype == NOVA_F16;
    if (t->r == 3) {
        switch (t->n) {
        case 4: return h ? launch_it_few<4, 3, f16>(t, x, Vc, g, s) : launch_it_few<4, 3, float>(t, x, Vc, g, s);
        case 6: return h ? launch_it_few<6, 3, f16>(t, x, Vc, g, s) : launch_it_few<6, 3, float>(t, x, Vc, g, s);
        case 8: return h ? launch_it_few<8, 3, f16>(t, x, Vc, g, s) : launch_it_few<8, 3, float>(t, x, Vc, g, s);
        case 10: return h ? launch_it_few<10, 3, f16>(t, x, Vc, g, s) : launch_it_few<10, 3, float>(t, x, Vc, g, s);
        }
    } else if (t->r == 5) {
        switch (t->n) {
        case 6: return h ? launch_it_few<6, 5, f16>(t, x, Vc, g, s) : launch_it_few<6, 5, float>(t, x, Vc, g, s);
        case 8: return h ? launch_it_few<8, 5, f16>(t, x, Vc, g, s) : launch_it_few<8, 5, float>(t, x, Vc, g, s);
        case 10: return h ? launch_it_few<10, 5, f16>(t, x, Vc, g, s) : launch_it_few<10, 5, float>(t, x, Vc, g, s);
        }
    }
    return (int)hipErrorInvalidValue;
}

}  // namespace nova
