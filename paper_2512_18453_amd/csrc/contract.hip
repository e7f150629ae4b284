// Winograd-domain contraction over input channels (Sec. 2.1 step 3, summed over channels):
//     M[xi][t][k] = sum_c V[xi][t][c] * U[xi][k][c]      for each of the n*n positions xi,
// i.e. n*n independent (T x C) . (C x K) matrix products.  Both operands are stored with the
// contraction index blocked by 32 and fastest (V [xi][C/32][T][32], U [xi][C/32][Kp][32]), so a
// (rows x 32-channel) operand tile is one contiguous piece of memory and every lane's MFMA
// fragment is a 16-byte read.
//
// binary16 path: v_mfma_f32_32x32x16_f16, binary32 accumulation, two kernels.
//   streaming kernel (C = 64, 128 or 256 and K a multiple of 64; further down): U stays in
//     registers, V streams once through an LDS ring filled by direct global->LDS loads;
//   tiled kernel (everything else): a workgroup of 4 waves owns a BM x BN tile of one M[xi]; the
//     channel loop moves 32 channels per step through double-buffered LDS (rows padded from 64 to
//     80 bytes, which spreads the 16 lanes of a 128-bit read phase over all 64 banks), global loads
//     for step s+1 are issued before the MFMAs of step s.
// binary32 path: same layouts, plain FMA tiles (validation path, not tuned).
#include <type_traits>

#include "device_common.hpp"

namespace nova {

int device_cu_count()
{
    static int cached[64] = {};
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cached[dev] == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cached[dev] = n;
    }
    return cached[dev];
}

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef unsigned int uint4v __attribute__((ext_vector_type(4)));

constexpr int kRowHalves = 40;   // LDS row pitch of a 32-channel operand row, in binary16 units (80 B)

template <int BM, int BN, int WM, int WN, typename MT>
__global__ void __launch_bounds__(256)
contract_f16_kernel(const f16 *__restrict__ U, const f16 *__restrict__ V, MT *__restrict__ Mo,
                    int T, int Tp, int Kp, int c_blocks, int k_blocks, int row_blocks, int col_blocks)
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
        MT *dst = Mo + ((size_t)xi * k_blocks + kb) * (size_t)Tp * kChanBlock + col;
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int t = t0 + (wm * MB + i) * 32 + (e >> 2) * 8 + row_base + (e & 3);
                if (t < T) store_from_f32(dst + (size_t)t * kChanBlock, acc[i][j][e]);
            }
    }
}

// ---------------------------------------------------------------------------------------------
// Weight-stationary streaming variant.
//
// The contraction is bound by HBM traffic (V in, M out), not by the matrix cores, and a tiled
// GEMM that reloads U and V per output tile is held back by load latency: it never has enough
// bytes in flight.  Here a workgroup keeps its slice of U[xi] -- NB*32 output channels x all C
// input channels per wave -- in VGPRs as ready-made MFMA fragments, and streams its share of
// V[xi] exactly once through a ring of S stages in LDS, filled by direct global->LDS loads (no
// destination registers), S-1 stages in flight.  A stage is SR = 32*WM consecutive tiles t with
// all C channels, so each stage yields finished outputs (no accumulation across stages) which go
// straight from the accumulators to M.  A segment = all stages of one (k-group, xi): the unit
// that shares one set of U fragments.  The grid is sized to what is resident at once (OCC
// workgroups per CU); if that is at least the number of segments, each segment is split among
// several workgroups and nobody reloads U, otherwise each workgroup takes a contiguous, equal
// share of all stages and walks through it segment by segment.
//   WN x WM waves; WN split the output channels, WM the rows of a stage.
//   CB = C/32 (fixes the registers for the U fragments).
// Two workgroups per CU where registers and LDS allow: the stores throttle the wave that issues
// them when HBM writes back up, and a second workgroup's MFMAs and loads fill those gaps.
//
// Waiting.  The hardware retires the vector-memory operations of a wave in issue order, and
// `s_waitcnt vmcnt(X)` waits until at most X are outstanding; so an operation with at least X
// younger ones is complete after the wait.  The compiler's own bookkeeping cannot express "all
// but the newest S-2 stages" across the loop, so the streaming loads and the stores are issued
// through inline assembly (which it does not count) and waited for with explicit counts.  Every
// stage issues exactly NP loads and NS stores per thread, nothing conditional; the compiler's own
// loads of U are complete before the loop over stages starts.
// The direct loads write LDS, not registers, so nothing the compiler allocates is written behind
// its back; their "memory" clobber keeps LDS reads from moving across them.
// Addresses are `uniform 64-bit base (scalar registers) + 32-bit per-lane byte offset`: one VGPR
// per access instead of two, which this kernel's register budget needs.
__device__ __forceinline__ void stream_to_lds16(const void *uniform_base, unsigned byte_offset, unsigned lds_wave_base)
{
    global_to_lds16<false>(uniform_base, byte_offset, lds_wave_base);
}
template <int IMM>
__device__ __forceinline__ void stream_store(float *uniform_base, unsigned byte_offset, float a, float b, float c, float d)
{
    typedef float float4v __attribute__((ext_vector_type(4)));
    const float4v v = {a, b, c, d};
    asm volatile("global_store_dwordx4 %0, %1, %2 offset:%3" : : "v"(byte_offset), "v"(v), "s"(uniform_base), "n"(IMM) : "memory");
}
template <int IMM>
__device__ __forceinline__ void stream_store(f16 *uniform_base, unsigned byte_offset, float a, float b, float c, float d)
{
    typedef _Float16 half4 __attribute__((ext_vector_type(4)));
    const half4 v = {(f16)a, (f16)b, (f16)c, (f16)d};
    asm volatile("global_store_dwordx2 %0, %1, %2 offset:%3" : : "v"(byte_offset), "v"(v), "s"(uniform_base), "n"(IMM) : "memory");
}
template <int X>
__device__ __forceinline__ void stream_wait()
{
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(X < 63 ? X : 63) : "memory");
}
// wait for the loads of the i-th stage of this workgroup (i counted from its first stage):
// younger operations = (S-2) stages of loads plus the stores of the min(i, S-1) stages completed
// since that stage was issued
template <int I, int S, int NP, int NS>
__device__ __forceinline__ void stream_wait_stage(int i)
{
    if constexpr (I == S - 1) {
        stream_wait<(S - 2) * NP + NS * (S - 1)>();
    } else {
        if (i == I) stream_wait<(S - 2) * NP + NS * I>();
        else stream_wait_stage<I + 1, S, NP, NS>(i);
    }
}

// WN x WM waves: WN split the output channels (NB blocks of 32 each, so WN*NB*32 per workgroup),
// WM split the rows of a stage (SR = 32*WM tiles).  OCC = workgroups per CU the registers and the
// LDS ring are budgeted for: with two, one workgroup's MFMAs overlap the other's stores, which
// throttle the issuing wave when HBM writes back up.
template <int WN, int WM, int NB, int CB, int S, int OCC, typename MT>
// (the second launch bound is waves per SIMD: a workgroup puts WN*WM/4 on each)
__global__ void __launch_bounds__(64 * WN * WM, (OCC * WN * WM + 3) / 4)
contract_stream_kernel(const f16 *__restrict__ U, const f16 *__restrict__ V, MT *__restrict__ Mo,
                       int T, int Tp, int Kp, int k_blocks, int stages_per_xi, int xi_count, int items_total, int wgs_per_seg)
{
    constexpr int THREADS = 64 * WN * WM;
    constexpr int SR = 32 * WM;                      // rows (tiles t) per stage
    constexpr int NP = CB * SR * 4 / THREADS;        // 16-byte loads per thread and stage
    constexpr int NS = 4 * NB;                       // stores per thread and stage
    constexpr int STAGE_BYTES = CB * SR * 64;        // [CB][SR] rows of 32 binary16 channels
    static_assert(NP >= 1 && NP * THREADS == CB * SR * 4 && S >= 3 && S * STAGE_BYTES * OCC <= 144 * 1024,
                  "pipeline shape");
    static_assert(THREADS / 4 % 16 == 0, "the swizzle term (r/4)%4 must not depend on the piece index i");

    __shared__ __align__(1024) unsigned char ring[S * STAGE_BYTES];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int frag_row = lane & 31;
    const unsigned ring_base = (unsigned)(size_t)((__attribute__((address_space(3))) void *)ring);

    // Work items: item = ((kg * xi_count) + xi) * stages_per_xi + tb; a run of stages_per_xi items
    // with the same (kg, xi) is a segment and needs one load of U fragments.  If there are at least
    // as many workgroups as segments, wgs_per_seg of them share each segment and nobody reloads U in
    // mid-stream; otherwise every workgroup takes a contiguous, equal share of all items.
    // (Workgroups that are neighbours in this order run on the same XCD, so a U[xi] slice shared by
    // several of them is fetched into one L2 only.)
    const unsigned wg = xcd_local_block_id(blockIdx.x, gridDim.x);
    int g0, g1;
    if (wgs_per_seg > 0) {
        const int seg0 = wg / wgs_per_seg, part = wg - seg0 * wgs_per_seg;
        g0 = seg0 * stages_per_xi + (int)((long long)stages_per_xi * part / wgs_per_seg);
        g1 = seg0 * stages_per_xi + (int)((long long)stages_per_xi * (part + 1) / wgs_per_seg);
    } else {
        g0 = (int)((long long)items_total * wg / gridDim.x);
        g1 = (int)((long long)items_total * (wg + 1) / gridDim.x);
    }
    if (g0 >= g1) return;

    // Piece p = tid + THREADS*i of a stage sits at LDS offset 16*p: row r = p/4 of the stage
    // ([channel block][tile] order), physical 16-byte slot p%4.  The logical slot (which 8 channels
    // of the row) is XOR-ed with (r/4)%4, so that the 16 rows a 128-bit fragment read touches in one
    // phase fall into 16 different bank groups.  Each lane picks the global address that belongs in
    // its fixed LDS slot.
    const int p_q = (tid & 3) ^ ((tid >> 4) & 3);        // (r/4)%4 with r = tid/4 + (THREADS/4)*i
    // fragment reads: row cb*SR + wm*32 + frag_row, logical slot 2*kk + lane/32
    const int swz = (frag_row >> 2) & 3;                 // (r/4)%4 of those rows (SR is a multiple of 32)
    int frag_off[2];
    for (int kk = 0; kk < 2; ++kk) frag_off[kk] = (wm * 32 + frag_row) * 64 + (((kk * 2 + (lane >> 5)) ^ swz) * 16);
    const unsigned u_lane_off = (unsigned)((frag_row * kChanBlock + (lane >> 5) * 8) * (int)sizeof(f16));

    // One pass of the outer loop = the part of this workgroup's range that lies in one segment.
    for (int g = g0; g < g1;) {
        const int seg = g / stages_per_xi;                 // = kg * xi_count + xi
        const int kg = seg / xi_count, xi = seg - kg * xi_count;
        const int tb0 = g - seg * stages_per_xi;
        int count = stages_per_xi - tb0;                   // stages of this pass
        if (count > g1 - g) count = g1 - g;
        g += count;
        const f16 *v_plane = uniform_pointer(V + (size_t)xi * CB * T * kChanBlock);

        // stage j of the pass -> ring slot; past the end of the pass the loads are still issued
        // (the wait counts assume a fixed number per stage) but every lane rereads the first 16
        // bytes of the plane: one cached request
        auto issue_stage = [&](int j, int slot) __attribute__((always_inline)) {
            const bool surplus = j > count - 1;
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                const int r = (tid >> 2) + i * (THREADS / 4);    // row of the stage: [channel block][tile]
                const int cb = r / SR, row = r % SR;             // SR is a power of two
                int t = (tb0 + j) * SR + row; if (t > T - 1) t = T - 1;      // rows past the end: reread the last
                const unsigned off = surplus ? 0u : ((unsigned)(cb * T + t) * kChanBlock + (unsigned)p_q * 8u) * (unsigned)sizeof(f16);
                stream_to_lds16(v_plane, off, ring_base + slot * STAGE_BYTES + (i * THREADS + wave * 64) * 16);
            }
        };
        for (int j = 0; j < S - 1; ++j) issue_stage(j, j);       // S-1 stages in flight

        // this wave's NB*32 output channels x all C channels of U[xi], as ready-made MFMA fragments:
        // uniform base per (block of 32 channels out, block of 32 channels in) + one per-lane offset
        half8 ufrag[NB][CB][2];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const int k0 = ((kg * WN + wn) * NB + nb) * 32;               // k0 + 31 < Kp: Kp is a multiple of WN*NB*32
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                const f16 *blk = U + (((size_t)xi * CB + cb) * Kp + k0) * kChanBlock;
#pragma unroll
                for (int kk = 0; kk < 2; ++kk)
                    ufrag[nb][cb][kk] = *reinterpret_cast<const NOVA_GLOBAL half8 *>(plane_element(blk + kk * 16, u_lane_off));
            }
        }
        // Pin the fragments here: each empty statement below consumes and redefines one of them, so
        // the compiler must have the load issued and waited for at this point and cannot sink either
        // into the loop.  Its wait for the youngest of them is vmcnt(0), which also covers the S-1
        // stages above (they are older); from here on only operations issued through inline
        // assembly are outstanding, as the counts in the loop assume.
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                for (int kk = 0; kk < 2; ++kk) asm volatile("" : "+v"(ufrag[nb][cb][kk]));
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

        MT *m_plane = uniform_pointer(Mo + ((size_t)xi * k_blocks + (size_t)(kg * WN + wn) * NB) * Tp * kChanBlock);
        // lane holds t = lane%32 and output channels 8*(e/4) + 4*(lane/32) + e%4 of each block:
        // four consecutive channels per store; rows up to Tp exist, so no store is conditional
        unsigned m_off = ((unsigned)(tb0 * SR + wm * 32 + frag_row) * kChanBlock + (unsigned)(lane >> 5) * 4u) * (unsigned)sizeof(MT);
        int slot = 0;
        for (int j = 0; j < count; ++j) {
            stream_wait_stage<0, S, NP, NS>(j);                // this wave's pieces of stage j have landed
            __syncthreads();                                   // everyone's have; slot-1 is free again
            issue_stage(j + S - 1, slot == 0 ? S - 1 : slot - 1);

            // acc[nb] = U-block (32 output channels) x V-stage rows (32 tiles): D[row = k][col = t]
            float16v acc[NB];
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[nb][e] = 0.0f;
            const unsigned char *stage = ring + slot * STAGE_BYTES;
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                for (int kk = 0; kk < 2; ++kk) {
                    const half8 vf = *reinterpret_cast<const half8 *>(stage + cb * SR * 64 + frag_off[kk]);
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
                        acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ufrag[nb][cb][kk], vf, acc[nb], 0, 0, 0);
                    // keep the fragment reads of later channel blocks from being hoisted all the way
                    // up: sixteen 128-bit fragments in flight at once do not fit the register budget
                    if (kk == 1) __builtin_amdgcn_sched_barrier(0);
                }

            // The stores are inline assembly and read the accumulators directly; the compiler inserts
            // the wait states an MFMA result needs before a vector-memory instruction may read it
            // only for instructions it schedules itself, so they are spelled out here (the longest
            // requirement, for a 16-pass MFMA, is 18).
            asm volatile("s_nop 15\n\ts_nop 7" ::: "memory");
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                MT *plane = m_plane + (size_t)nb * Tp * kChanBlock;
                stream_store<0 * 8 * (int)sizeof(MT)>(plane, m_off, acc[nb][0], acc[nb][1], acc[nb][2], acc[nb][3]);
                stream_store<1 * 8 * (int)sizeof(MT)>(plane, m_off, acc[nb][4], acc[nb][5], acc[nb][6], acc[nb][7]);
                stream_store<2 * 8 * (int)sizeof(MT)>(plane, m_off, acc[nb][8], acc[nb][9], acc[nb][10], acc[nb][11]);
                stream_store<3 * 8 * (int)sizeof(MT)>(plane, m_off, acc[nb][12], acc[nb][13], acc[nb][14], acc[nb][15]);
            }
            m_off += (unsigned)(SR * kChanBlock) * (unsigned)sizeof(MT);
            slot = slot == S - 1 ? 0 : slot + 1;
        }
        // the surplus prefetches of the tail must land before the ring is refilled or released,
        // and every wave must be done reading before the next pass overwrites it
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
    }
}

// binary32: 64 x 64 tile, 256 threads, 4 x 4 outputs per thread
__global__ void __launch_bounds__(256)
contract_f32_kernel(const float *__restrict__ U, const float *__restrict__ V, float *__restrict__ Mo,
                    int T, int Tp, int Kp, int c_blocks, int k_blocks, int row_blocks, int col_blocks)
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
                Mo[(((size_t)xi * k_blocks + (k >> 5)) * Tp + t) * kChanBlock + (k & 31)] = acc[i][j];
        }
}

template <int BM, int BN, int WM, int WN, typename MT>
static int launch_c16(const void *U, const void *V, void *Mo, const Geometry &g, hipStream_t stream)
{
    const int row_blocks = ceil_div((int)g.T, BM), col_blocks = ceil_div(g.Kp, BN);
    const long long blocks = (long long)g.n * g.n * row_blocks * col_blocks;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL((contract_f16_kernel<BM, BN, WM, WN, MT>), dim3((unsigned)blocks), dim3(256), 0, stream,
                       (const f16 *)U, (const f16 *)V, (MT *)Mo, (int)g.T, (int)g.Tp, g.Kp, g.c_blocks, g.k_blocks,
                       row_blocks, col_blocks);
    return (int)hipGetLastError();
}

template <int WN, int WM, int NB, int CB, int S, int OCC, typename MT>
static int launch_stream(const void *U, const void *V, void *Mo, const Geometry &g, hipStream_t stream)
{
    constexpr int SR = 32 * WM;
    const int slots = device_cu_count() * OCC;           // workgroups resident at once
    const int stages_per_xi = ceil_div((int)g.T, SR);
    const int kgroups = g.Kp / (WN * NB * 32);
    const long long segs = (long long)kgroups * g.n * g.n;
    const long long items = segs * stages_per_xi;
    if (items <= 0 || items > 0x7fffffffLL) return (int)hipErrorInvalidValue;
    // 32-bit byte offsets inside one xi plane of V and one (xi, channel block) plane of M
    if ((size_t)g.c_blocks * g.T * kChanBlock * sizeof(f16) >= ((size_t)1 << 32) ||
        (size_t)g.Tp * kChanBlock * sizeof(MT) >= ((size_t)1 << 32)) return (int)hipErrorInvalidValue;
    int wgs_per_seg = (int)(slots / segs);
    if (wgs_per_seg > stages_per_xi) wgs_per_seg = stages_per_xi;
    const int blocks = wgs_per_seg > 0 ? (int)(segs * wgs_per_seg) : (int)(items < slots ? items : slots);
    hipLaunchKernelGGL((contract_stream_kernel<WN, WM, NB, CB, S, OCC, MT>), dim3(blocks), dim3(64 * WN * WM), 0, stream,
                       (const f16 *)U, (const f16 *)V, (MT *)Mo, (int)g.T, (int)g.Tp, g.Kp, g.k_blocks,
                       stages_per_xi, g.n * g.n, (int)items, wgs_per_seg);
    return (int)hipGetLastError();
}

template <typename MT>
static int launch_c16_tiled(const void *U, const void *V, void *Mo, const Geometry &g, hipStream_t s)
{
    if (g.Kp >= 128) return launch_c16<128, 128, 2, 2, MT>(U, V, Mo, g, s);
    if (g.Kp >= 64) return launch_c16<128, 64, 2, 2, MT>(U, V, Mo, g, s);
    return launch_c16<128, 32, 4, 1, MT>(U, V, Mo, g, s);
}

template <typename MT>
static int launch_c16_shape(const void *U, const void *V, void *Mo, const Geometry &g, hipStream_t s)
{
    // streaming kernel: C in {64, 128, 256} and K a multiple of the workgroup's channel span
    // (C = 512 variants, 16 channel blocks in 128 fragment registers at one workgroup per CU, measured
    // no faster than the tiled kernel at T = 512 and slower at T = 128);
    // ring depth S: as many stages as fit about 128 KiB of LDS, at most 8
    const int cb = g.c_blocks;
    const int wn = g.Kp % 256 == 0 ? 4 : g.Kp % 128 == 0 ? 2 : g.Kp % 64 == 0 ? 1 : 0;
    {
        //                                            WN WM NB CB  S OCC
        if (wn == 4 && cb == 8) return launch_stream<8, 1, 1, 8, 4, 2, MT>(U, V, Mo, g, s);   // 8 waves x 32 channels
        if (wn == 4 && cb == 4) return launch_stream<4, 1, 2, 4, 8, 2, MT>(U, V, Mo, g, s);
        if (wn == 4 && cb == 2) return launch_stream<4, 1, 2, 2, 8, 2, MT>(U, V, Mo, g, s);
        if (wn == 2 && cb == 8) return launch_stream<2, 2, 2, 8, 4, 1, MT>(U, V, Mo, g, s);
        if (wn == 2 && cb == 4) return launch_stream<2, 2, 2, 4, 4, 2, MT>(U, V, Mo, g, s);
        if (wn == 2 && cb == 2) return launch_stream<2, 2, 2, 2, 8, 2, MT>(U, V, Mo, g, s);
        if (wn == 1 && cb == 4) return launch_stream<1, 4, 2, 4, 4, 1, MT>(U, V, Mo, g, s);
        if (wn == 1 && cb == 2) return launch_stream<1, 4, 2, 2, 4, 2, MT>(U, V, Mo, g, s);
    }
    return launch_c16_tiled<MT>(U, V, Mo, g, s);       // other shapes: tiled kernel
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
                       (const float *)V, (float *)Mo, (int)g.T, (int)g.Tp, g.Kp, g.c_blocks, g.k_blocks, row_blocks,
                       col_blocks);
    return (int)hipGetLastError();
}

}  // namespace nova
