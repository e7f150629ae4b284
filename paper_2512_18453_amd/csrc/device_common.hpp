// Device-side helpers shared by the libnova kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include "internal.hpp"

namespace nova {

typedef _Float16 f16;

// storage <-> binary32; the binary16 conversion rounds to nearest even, keeps sub-normals and
// overflows to infinity (v_cvt_f16_f32).
__device__ __forceinline__ float load_f32(const float *p) { return *p; }
__device__ __forceinline__ float load_f32(const f16 *p) { return (float)*p; }
__device__ __forceinline__ void store_from_f32(float *p, float v) { *p = v; }
__device__ __forceinline__ void store_from_f32(f16 *p, float v) { *p = (f16)v; }

// binary32 -> storage as its own rounding step.  Without the barrier the compiler merges a
// fused multiply-add and the conversion into one v_fma_mixlo_f16, which rounds the exact
// a*b+c once to binary16 and therefore disagrees, in the last place, with "round to binary32,
// then to binary16" -- the order the input-transform contract prescribes.
template <typename P> __device__ __forceinline__ void store_rounded_twice(P *p, float v);
template <> __device__ __forceinline__ void store_rounded_twice(float *p, float v) { *p = v; }
template <> __device__ __forceinline__ void store_rounded_twice(f16 *p, float v)
{
    asm volatile("" : "+v"(v));
    *p = (f16)v;
}
__device__ __forceinline__ float round_twice(float v, float *) { return v; }
__device__ __forceinline__ f16 round_twice(float v, f16 *)
{
    asm volatile("" : "+v"(v));
    return (f16)v;
}

__device__ __forceinline__ float fma32(float a, float b, float c) { return __builtin_fmaf(a, b, c); }

// binary64 -> storage with a single rounding.  For binary16 the value first goes to binary32
// with round-to-odd (the inexact bit survives in the last place), after which the
// round-to-nearest-even conversion to binary16 cannot double round (24 >= 11 + 2 bits).
__device__ __forceinline__ float round_f64_to(double v, float *) { return (float)v; }
__device__ __forceinline__ f16 round_f64_to(double v, f16 *)
{
    float f = (float)v;                           // nearest even
    if (!(__builtin_fabs(v) <= 3.0e38) || (double)f == v) return (f16)f;   // exact, huge, inf or NaN
    unsigned bits = __float_as_uint(f);
    bool away = __builtin_fabs((double)f) > __builtin_fabs(v);   // rounded away from zero?
    if (away) bits -= 1;                          // step back to the truncated magnitude
    bits |= 1u;                                   // inexact: force the last place odd
    return (f16)__uint_as_float(bits);
}

// A pointer into global memory formed as `wave-uniform base + 32-bit per-thread byte offset`.
// The base is pinned to scalar registers and made opaque to the optimizer, so the access is
// selected with a scalar base operand instead of per-thread 64-bit address arithmetic on the
// vector ALU; the result is typed as a global-memory pointer so that it stays a global access.
#define NOVA_GLOBAL __attribute__((address_space(1)))
template <typename P>
__device__ __forceinline__ NOVA_GLOBAL P *plane_element(P *uniform_base, unsigned byte_offset)
{
    unsigned long long bits = reinterpret_cast<unsigned long long>(uniform_base);
    asm volatile("" : "+s"(bits));
    NOVA_GLOBAL char *base = reinterpret_cast<NOVA_GLOBAL char *>(bits);
    return reinterpret_cast<NOVA_GLOBAL P *>(base + byte_offset);
}

// The same pointer, read from the first active lane into scalar registers: for values every lane
// computes alike but which the compiler keeps in vector registers (inline-assembly operands with
// an "s" constraint need them in scalar ones).
template <typename P>
__device__ __forceinline__ P *uniform_pointer(P *p)
{
    const unsigned long long bits = reinterpret_cast<unsigned long long>(p);
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)bits);
    const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(bits >> 32));
    return reinterpret_cast<P *>(((unsigned long long)hi << 32) | lo);
}

// One 16-byte piece per lane from global memory straight into LDS (no destination registers):
// lane i of the wave reads uniform_base + byte_offset (its own) and writes LDS address
// lds_wave_base + 16 * i; lanes switched off by the execution mask do neither.  The hardware takes
// the LDS base from M0, a register the compiler reserves for uses of its own and cannot be told
// about as clobbered, so the statement hands it back as it found it.  The load counts in vmcnt like
// any vector-memory load; the compiler does not know that it writes LDS, so whoever reads that
// memory waits (s_waitcnt vmcnt) and synchronises explicitly.  NT: streaming cache hint.
template <bool NT>
__device__ __forceinline__ void global_to_lds16(const void *uniform_base, unsigned byte_offset, unsigned lds_wave_base)
{
    unsigned saved_m0;
    if constexpr (NT)
        asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3 nt\n\ts_mov_b32 m0, %0"
                     : "=&s"(saved_m0) : "s"(lds_wave_base), "v"(byte_offset), "s"(uniform_base) : "memory");
    else
        asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3\n\ts_mov_b32 m0, %0"
                     : "=&s"(saved_m0) : "s"(lds_wave_base), "v"(byte_offset), "s"(uniform_base) : "memory");
}

// COUNT such loads in one statement (M0 saved and handed back once): load k takes the 64 pieces at
// planes[k] + byte_offset to LDS at lds_wave_base + k * LDS_STEP.
#define NOVA_DMA_FIRST "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %4\n\t"
#define NOVA_DMA_NEXT(P) "s_add_u32 m0, m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, " P "\n\t"
#define NOVA_DMA_LAST "s_mov_b32 m0, %0"
template <int COUNT, int LDS_STEP>
__device__ __forceinline__ void global_to_lds16_run(const void *const (&planes)[COUNT], unsigned byte_offset, unsigned lds_wave_base)
{
    static_assert(COUNT >= 1 && COUNT <= 5, "loads per statement");
    unsigned saved_m0;
    if constexpr (COUNT == 1)
        asm volatile(NOVA_DMA_FIRST NOVA_DMA_LAST
                     : "=&s"(saved_m0) : "s"(lds_wave_base), "v"(byte_offset), "n"(LDS_STEP), "s"(planes[0]) : "memory", "scc");
    else if constexpr (COUNT == 2)
        asm volatile(NOVA_DMA_FIRST NOVA_DMA_NEXT("%5") NOVA_DMA_LAST
                     : "=&s"(saved_m0) : "s"(lds_wave_base), "v"(byte_offset), "n"(LDS_STEP), "s"(planes[0]), "s"(planes[1])
                     : "memory", "scc");
    else if constexpr (COUNT == 3)
        asm volatile(NOVA_DMA_FIRST NOVA_DMA_NEXT("%5") NOVA_DMA_NEXT("%6") NOVA_DMA_LAST
                     : "=&s"(saved_m0)
                     : "s"(lds_wave_base), "v"(byte_offset), "n"(LDS_STEP), "s"(planes[0]), "s"(planes[1]), "s"(planes[2])
                     : "memory", "scc");
    else if constexpr (COUNT == 4)
        asm volatile(NOVA_DMA_FIRST NOVA_DMA_NEXT("%5") NOVA_DMA_NEXT("%6") NOVA_DMA_NEXT("%7") NOVA_DMA_LAST
                     : "=&s"(saved_m0)
                     : "s"(lds_wave_base), "v"(byte_offset), "n"(LDS_STEP), "s"(planes[0]), "s"(planes[1]), "s"(planes[2]),
                       "s"(planes[3])
                     : "memory", "scc");
    else
        asm volatile(NOVA_DMA_FIRST NOVA_DMA_NEXT("%5") NOVA_DMA_NEXT("%6") NOVA_DMA_NEXT("%7") NOVA_DMA_NEXT("%8") NOVA_DMA_LAST
                     : "=&s"(saved_m0)
                     : "s"(lds_wave_base), "v"(byte_offset), "n"(LDS_STEP), "s"(planes[0]), "s"(planes[1]), "s"(planes[2]),
                       "s"(planes[3]), "s"(planes[4])
                     : "memory", "scc");
}
#undef NOVA_DMA_FIRST
#undef NOVA_DMA_NEXT
#undef NOVA_DMA_LAST

// s_waitcnt vmcnt(n) for a wave-uniform run-time n: waits until at most min(n, 31) of the wave's
// vector-memory operations are outstanding (the count is an immediate of the instruction, hence the
// decision tree: five comparisons; waiting for fewer than n is always safe).
template <int LO = 0, int HI = 31>
__device__ __forceinline__ void wait_vmcnt_at_most(int n)
{
    if constexpr (LO == HI) {
        asm volatile("s_waitcnt vmcnt(%0)" : : "n"(LO) : "memory");
    } else {
        constexpr int MID = (LO + HI + 1) / 2;
        if (n >= MID) wait_vmcnt_at_most<MID, HI>(n);
        else wait_vmcnt_at_most<LO, MID - 1>(n);
    }
}

// blockIdx.x -> logical block id such that consecutive logical ids run on the same XCD
// (hardware deals consecutive workgroup ids round-robin over the 8 XCDs, each with its own L2).
__device__ __forceinline__ unsigned xcd_local_block_id(unsigned id, unsigned total)
{
    constexpr unsigned kXcd = 8;
    unsigned full = total / kXcd * kXcd;
    if (id >= full) return id;                    // ragged tail: leave as is
    return (id % kXcd) * (total / kXcd) + id / kXcd;
}

}  // namespace nova

#define NOVA_HIP_TRY(expr)                                   \
    do {                                                     \
        hipError_t nova_err_ = (expr);                       \
        if (nova_err_ != hipSuccess) return (int)nova_err_;  \
    } while (0)
