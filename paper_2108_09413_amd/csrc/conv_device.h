// Device helpers shared by the convolution kernels: LDS swizzle, requantisation,
// clamp and byte packing.
#ifndef ISR_CONV_DEVICE_H
#define ISR_CONV_DEVICE_H

#include "isr_internal.h"

namespace isr {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// 16-byte chunk swizzle inside an LDS row of CPR chunks: spreads equal chunk
// indices of neighbouring rows over different banks for the 128-bit fragment reads
// (8 consecutive rows must cover all 32 banks).
template <int CPR>
__device__ __forceinline__ int swz(int row) { return CPR == 4 ? (((row >> 1) ^ (row >> 3)) & 3) : (row & 7); }

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

// clamp(v, lo, hi) for lo <= hi in one instruction
__device__ __forceinline__ int clamp3(int v, int lo, int hi) {
    int r;
    asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(v), "v"(lo), "v"(hi));
    return r;
}

// low bytes of four registers -> one dword (3 byte-permutes)
__device__ __forceinline__ uint32_t pack4(int a, int b, int c, int d) {
    uint32_t lo = __builtin_amdgcn_perm((uint32_t)b, (uint32_t)a, 0x0c0c0400u);
    uint32_t hi = __builtin_amdgcn_perm((uint32_t)d, (uint32_t)c, 0x0c0c0400u);
    return __builtin_amdgcn_perm(hi, lo, 0x05040100u);
}

}  // namespace isr

#endif
