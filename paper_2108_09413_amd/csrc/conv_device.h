// Device helpers shared by the convolution kernels: LDS swizzle, requantisation,
// clamp and byte packing.
#ifndef ISR_CONV_DEVICE_H
#define ISR_CONV_DEVICE_H

#include <type_traits>

#include "isr_internal.h"

namespace isr {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// 16-byte chunk swizzle inside an LDS row of CPR chunks (64 or 128 bytes): spreads equal chunk indices of
// neighbouring rows over different banks for the 128-bit fragment reads.  The LDS serves such a read 16
// consecutive lanes at a time from 64 banks of 4 bytes, so 16 consecutive rows reading one logical chunk must
// cover 256 bytes exactly once: the rows that share a 256-byte line (4 rows of 64 bytes, 2 of 128) keep the
// chunk, each next group of rows moves it on by one (measured: as fast as contiguous reads; XOR with the
// low row bits instead costs 13-14 % of the read rate).
template <int CPR>
__device__ __forceinline__ int swz(int row) { return CPR == 4 ? ((row >> 2) & 3) : ((row >> 1) & 7); }

// RHA(acc * M0, 31 + shift) on magnitude and sign, 32x32->64 multiply-add:
//   |acc| * (M0 << 1) + 2^(31+shift) = 2 * (|acc| * M0 + 2^(30+shift)),
// so the rounded quotient is the high word shifted right by `shift`.
__device__ __forceinline__ int requant(int acc, uint32_t m0x2, uint32_t rnd_lo, uint32_t rnd_hi, uint32_t sh) {
    uint32_t mag = (uint32_t)(acc < 0 ? -acc : acc);
    uint64_t prod = (uint64_t)mag * (uint64_t)m0x2 + (((uint64_t)rnd_hi << 32) | rnd_lo);
    int r = (int)((uint32_t)(prod >> 32) >> sh);
    return acc < 0 ? -r : r;
}

// Same result from one signed 32x32+64 multiply-add when 2 <= shift <= 22:
//   z_out + RHA(v, s) = floor((v + 2^(s-1) - [v<0] + z_out 2^s) / 2^s),  v = acc M0, s = 31 + shift.
// 2^(s-1) + z_out 2^s is a multiple of 2^32 (chi holds its high word), and
// subtracting [v<0] turns the 64-bit addend into (chi + m : m) with m = acc >> 31.
__device__ __forceinline__ int requant_fast(int acc, int m0, int chi, int shm1) {
    int m = acc >> 31;
    long addend = (long)(((unsigned long)(uint32_t)(chi + m) << 32) | (uint32_t)m);
    long w = (long)acc * (long)m0 + addend;
    return (int)(w >> 32) >> shm1;
}

// The same again for a layer whose products acc * M0 can never be an exact half
// (ConvParams::tie_free): with the low word of the rounding term gone only the high
// word of the product is needed.
__device__ __forceinline__ int requant_tie_free(int acc, int m0, int chi, int shm1) {
    return (__mulhi(acc, m0) + chi) >> shm1;
}

template <bool TIE_FREE>
__device__ __forceinline__ int requant_q(int acc, int m0, int chi, int shm1) {
    if constexpr (TIE_FREE) return requant_tie_free(acc, m0, chi, shm1);
    else return requant_fast(acc, m0, chi, shm1);
}

// clamp(v, lo, hi) for lo <= hi in one instruction
__device__ __forceinline__ int clamp3(int v, int lo, int hi) {
    int r;
    asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(v), "v"(lo), "v"(hi));
    return r;
}

// Residual add on the int8 result q of the convolution and the int8 residual r8 (second
// requantisation): v = q Ms + r8 Mr + c0, out = clamp((v + k + (v >> 31)) >> sh, lo, 127)
// with k = 2^(sh-1) + z_out 2^sh; 24-bit multiplies: |q|, |r8| <= 2^7, |multipliers| < 2^23.
template <bool TIE_FREE>
__device__ __forceinline__ int fused_add(int q, int r8, const ConvParams &p) {
    if constexpr (TIE_FREE) {
        const int v = __mul24(q, p.add_mul_self) + (p.add_c0 + p.add_k) + __mul24(r8, p.add_mul_res);
        return clamp3(v >> p.add_sh, p.add_lo, 127);
    }
    const int v = __mul24(q, p.add_mul_self) + p.add_c0 + __mul24(r8, p.add_mul_res);
    return clamp3((v + p.add_k + (v >> 31)) >> p.add_sh, p.add_lo, 127);
}

// low bytes of four registers -> one dword (3 byte-permutes)
__device__ __forceinline__ uint32_t pack4(int a, int b, int c, int d) {
    uint32_t lo = __builtin_amdgcn_perm((uint32_t)b, (uint32_t)a, 0x0c0c0400u);
    uint32_t hi = __builtin_amdgcn_perm((uint32_t)d, (uint32_t)c, 0x0c0c0400u);
    return __builtin_amdgcn_perm(hi, lo, 0x05040100u);
}

// 16 bytes per lane from global memory into LDS: lane l of the wave writes bytes
// [16 l, 16 l + 16) after the wave-uniform LDS address `lptr`.
#define ISR_GLOBAL_TO_LDS16(gptr, lptr)                                                             \
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(gptr),        \
                                     (__attribute__((address_space(3))) void *)(lptr), 16, 0, 0)

// Wave-uniform LDS byte address of `p` as a plain integer, and a direct-to-LDS load that takes its destination
// from one: the compiler then cannot tie the load to the array and puts no vmcnt(0) in front of every later
// read of that array (which would serialise refill and compute); the kernel's own waits and barriers order them.
__device__ __forceinline__ uint32_t lds_address(const void *p) {
    return (uint32_t)__builtin_amdgcn_readfirstlane((int)(uintptr_t)(const __attribute__((address_space(3))) void *)p);
}
#define ISR_GLOBAL_TO_LDS16_AT(gptr, lds_u32)                                                       \
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(gptr),        \
                                     (__attribute__((address_space(3))) void *)(uintptr_t)(lds_u32), 16, 0, 0)

// The compiler does not order LDS reads after loads that write LDS; this wait does.
template <int N>
__device__ __forceinline__ void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

}  // namespace isr

#endif
