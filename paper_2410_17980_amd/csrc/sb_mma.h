// Device-side building blocks shared by the bf16 kernels: vector types, the
// base-2 softplus, LDS swizzles and the transposing-load helper.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sb {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

#define SB_LDS(T, p) ((__attribute__((address_space(3))) T*)(p))

constexpr float SB_LOG2E = 1.4426950408889634f;
constexpr float SB_LN2 = 0.6931471805599453f;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// sp2(x) = log2(1 + 2^x), the base-2 softplus: -sp2 is log2(1 - sigma(z)) and
// x - sp2 is log2(sigma(z)) for x = z*log2(e).  For x > 128 the power overflows
// to +inf and so does the log; the true value is then x itself to fp32
// precision, and the median of (log, x, 128) picks it.  Below that the log
// lies between x and 128 and is the median.  x = -inf gives 0.
__device__ __forceinline__ float sp2(float x)
{
    return __builtin_amdgcn_fmed3f(fast_log2(1.0f + fast_exp2(x)), x, 128.0f);
}

// MFMA 32x32 accumulator register r of lane (n, hh) is output row
// 8*(r/4) + 4*hh + r%4.  Feeding MFMA row rho from tile row perm_row(rho)
// makes lane (n, hh) own the 16 CONSECUTIVE tile rows 16*hh + r, r = 0..15.
__device__ __forceinline__ int perm_row(int rho)
{
    return 16 * ((rho >> 2) & 1) + 4 * (rho >> 3) + (rho & 3);
}

// LDS tiles are [row][D] bf16, unpadded, with the 16-byte chunk index of a row
// xor-ed by a function of the row so that both access patterns are conflict free:
//   (a) A/B-operand reads: 16 lanes read the same chunk of 16 different rows;
//   (b) transposing reads: 16 lanes read 32 B of each of 4 consecutive rows,
//       and the two quarter-waves of a half-wave the other 32 B of the same 64 B.
// swz_perm is for tiles whose operand reads go through perm_row (the 16 rows are
// {0..7, 16..23} + 8k), swz_nat for tiles read in natural row order (rows 0..15 + 16k).
// A row holds D/8 chunks (16 at D = 128, 8 at D = 64, 4 at D = 32), so 1, 2 or 4 rows
// share the 64 banks and the xor needs 4, 3 or 2 bits.
template <int D> __device__ __forceinline__ int swz_perm(int row)
{
    static_assert(D == 32 || D == 64 || D == 128, "head dimension");
    if (D == 128) return ((row & 3) << 2) | ((row >> 2) & 1) | (((row >> 4) & 1) << 1);
    if (D == 64) return (((row >> 1) & 1) << 2) | ((row >> 2) & 1) | (((row >> 4) & 1) << 1);
    return ((row >> 2) & 1) | (((row >> 4) & 1) << 1);
}
template <int D> __device__ __forceinline__ int swz_nat(int row)
{
    static_assert(D == 32 || D == 64 || D == 128, "head dimension");
    if (D == 128) return ((row & 3) << 2) | ((row >> 2) & 3);
    if (D == 64) return (((row >> 1) & 1) << 2) | ((row >> 2) & 3);
    return (row >> 2) & 3;
}

// byte offset of 16-byte chunk c of tile row `row`
template <int D> __device__ __forceinline__ int tile_off_perm(int row, int c)
{
    return row * (D * 2) + ((c ^ swz_perm<D>(row)) << 4);
}
template <int D> __device__ __forceinline__ int tile_off_nat(int row, int c)
{
    return row * (D * 2) + ((c ^ swz_nat<D>(row)) << 4);
}

// Two transposing loads (ds_read_b64_tr_b16) glued into one MFMA operand: the
// K-dimension elements 0..3 come from p_lo, 4..7 from p_hi.  Within each group of
// 16 lanes, lane i supplies the address of row i/4, columns 4*(i%4)..+3 and
// receives column i of the four rows.
__device__ __forceinline__ bf16x8 tr_pair(const char* p_lo, const char* p_hi)
{
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(SB_LDS(s16x4, p_lo));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(SB_LDS(s16x4, p_hi));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

// both half-waves' copies of a per-lane float: returns (value of lane n, value of lane n+32)
__device__ __forceinline__ void both_halves(float v, float& lo, float& hi)
{
    auto sw = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(int, v), __builtin_bit_cast(int, v), false, false);
    lo = __builtin_bit_cast(float, (int)sw[0]);
    hi = __builtin_bit_cast(float, (int)sw[1]);
}

// LDS byte address of a pointer into a __shared__ array.  A generic pointer to LDS is the LDS
// address in its low half and the aperture in its high half, so this is a truncation; the
// address-space cast would add a null check (compare + select) per use.
__device__ __forceinline__ uint32_t lds_offset(const char* p)
{
    return (uint32_t)(uintptr_t)p;
}

// LDS accesses by 32-bit LDS byte address (integer arithmetic on addresses, xor included,
// stays in the LDS address space this way)
typedef __attribute__((address_space(3))) const u32x4* lds_cu32x4_ptr;
typedef __attribute__((address_space(3))) u32x4* lds_u32x4_ptr;
typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;
__device__ __forceinline__ u32x4 lds_load16(uint32_t addr) { return *(lds_cu32x4_ptr)(uintptr_t)(addr); }
__device__ __forceinline__ void lds_store16(uint32_t addr, bf16x8 v)
{
    *(lds_u32x4_ptr)(uintptr_t)(addr) = __builtin_bit_cast(u32x4, v);
}
// tr_pair by LDS address
__device__ __forceinline__ bf16x8 tr_pair_at(uint32_t a_lo, uint32_t a_hi)
{
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(uintptr_t)(a_lo));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(uintptr_t)(a_hi));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

// Direct global -> LDS copy of 16 bytes per lane (global_load_lds_dwordx4): lane l
// of the wave writes LDS bytes [lds_base + 16 l, +16) with the 16 bytes at its own
// global address; lds_base must be wave-uniform.  Issued through inline assembly so
// that the compiler's wait-count pass does not see an LDS write it would guard
// every later LDS read against; the caller orders it with dma_wait<N>() + barrier.
// Completion is counted in vmcnt, in issue order.  The LDS base travels in M0, which
// is handed over as a register operand: the compiler writes it and knows it is in use
// (the s_nop covers the wait state between a scalar write of M0 and this instruction,
// which the compiler cannot see into).
__device__ __forceinline__ void dma16_to_lds(const void* gptr, const char* lds_base)
{
    const uint32_t lds = __builtin_amdgcn_readfirstlane(lds_offset(lds_base));
    asm volatile("s_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :: "{m0}"(lds), "v"(gptr) : "memory");
}

// same, with the global address given as a wave-uniform base plus a per-lane byte offset
__device__ __forceinline__ void dma16_to_lds_saddr(const void* gbase, int lane_off, const char* lds_base)
{
    const uint32_t lds = __builtin_amdgcn_readfirstlane(lds_offset(lds_base));
    const uint64_t b = (uint64_t)(uintptr_t)gbase;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)b);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
    const uint64_t sb = ((uint64_t)hi << 32) | lo;
    asm volatile("s_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "{m0}"(lds), "v"(lane_off), "s"(sb) : "memory");
}

// wait until at most N of this wave's vector-memory operations are outstanding
template <int N> __device__ __forceinline__ void dma_wait()
{
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// workgroup barrier without the compiler's "wait for everything" fence: the caller
// has already waited for exactly what must be visible
__device__ __forceinline__ void barrier_nofence()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// workgroup barrier that first waits for this wave's LDS operations (its writes are then
// visible to the others, its reads have returned)
__device__ __forceinline__ void barrier_lds()
{
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

}  // namespace sb
