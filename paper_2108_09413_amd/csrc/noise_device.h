// The device sampler of the noise stage, shared by the kernels that draw noisy pixels:
//   x + delta, delta ~ discrete Gaussian (Def. 3.3), saturated to [0,255], recentred to int8.
// Randomness: Philox4x32-10 keyed by the seed; counter (p >> 2, sample, image, 2*phase + half)
// with p the logical [C][H][W] pixel index; word p & 3; half 0 supplies the high 32 bits of the
// uniform 64-bit u, half 1 the low 32 bits.  The low half is generated only when the high word
// ties with a threshold.
#ifndef ISR_NOISE_DEVICE_H
#define ISR_NOISE_DEVICE_H

#include "isr_internal.h"

namespace isr {

__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t out[4]) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;   // one 32x32->64 multiply gives both halves
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        c0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        c1 = (uint32_t)p1;
        c2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c3 = (uint32_t)p0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

struct NoiseLds {
    uint32_t hi[NOISE_TABLE_MAX + 2];   // entries >= n hold 0xFFFFFFFF
    uint32_t lo[NOISE_TABLE_MAX];
    uint16_t guide[NOISE_GUIDE_SIZE + 2];
};

// #{j < n : T[j] <= u} when the guide bucket holds more than one candidate or the
// high word ties with a threshold: binary search inside the bucket, then the
// 64-bit comparison for the (rare) equal high words.
__device__ __noinline__ int threshold_count_slow(const NoiseLds &t, int n, uint32_t uhi, uint32_t grp,
                                                 uint32_t sample, uint32_t image, uint32_t phase, uint32_t key0,
                                                 uint32_t key1, int word) {
    const uint32_t b = uhi >> (32 - NOISE_GUIDE_BITS);
    int lo = t.guide[b], hi = t.guide[b + 1];    // every threshold with high word < uhi lies below guide[b+1]
    while (lo < hi) {                             // first index whose high word is >= uhi
        int mid = (lo + hi) >> 1;
        if (t.hi[mid] < uhi) lo = mid + 1; else hi = mid;
    }
    int c = lo;
    if (c < n && t.hi[c] == uhi) {
        uint32_t lo4[4];
        philox4x32_10(grp, sample, image, phase * 2u + 1u, key0, key1, lo4);
        const uint32_t ulo = lo4[word & 3];
        while (c < n && t.hi[c] == uhi && t.lo[c] <= ulo) ++c;
    }
    return c;
}

// Stages a table into LDS (all threads of the workgroup; followed by a barrier at the caller).
__device__ __forceinline__ void stage_noise_table(NoiseLds &t, const DeviceNoiseTable *tab, int tid, int nthreads) {
    for (int i = tid; i < (int)NOISE_TABLE_MAX; i += nthreads) {
        t.hi[i] = tab->hi[i];
        t.lo[i] = tab->lo[i];
    }
    if (tid < 2) t.hi[NOISE_TABLE_MAX + tid] = 0xFFFFFFFFu;
    for (int i = tid; i < (int)(NOISE_GUIDE_SIZE + 2) / 2; i += nthreads)   // two 16-bit entries per word
        ((uint32_t *)t.guide)[i] = ((const uint32_t *)tab->guide)[i];
}

// Four horizontally adjacent noisy pixels (x4 * 4 .. x4 * 4 + 3 of row y) of one copy as NHWC4 words:
// byte c of word j = clamp(x[c][y][4 x4 + j] + delta, 0, 255) - 128, byte 3 = 0.
__device__ __forceinline__ void noisy_quad(const NoiseLds &t, int n, int dmin, const uint8_t *xim, int C, int H, int W, int y,
                                           int x4, uint32_t sample, uint32_t image_id, uint32_t phase, uint32_t key0,
                                           uint32_t key1, uint32_t packed[4]) {
    packed[0] = packed[1] = packed[2] = packed[3] = 0;
#pragma unroll
    for (int c = 0; c < 3; ++c) {
        if (c < C) {
            const uint32_t pix = (uint32_t)((c * H + y) * W + x4 * 4);   // multiple of 4
            const uint32_t grp = pix >> 2;
            uint32_t hi[4];
            philox4x32_10(grp, sample, image_id, phase * 2u, key0, key1, hi);
            const uint32_t px4 = *(const uint32_t *)(xim + pix);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t u = hi[j];
                int cnt = t.guide[u >> (32 - NOISE_GUIDE_BITS)];
                const uint32_t t0 = t.hi[cnt], t1 = t.hi[cnt + 1];
                cnt += t0 < u;
                // common case: at most one threshold below u in the bucket and no tie
                if ((t0 < u ? t1 : t0) <= u)
                    cnt = threshold_count_slow(t, n, u, grp, sample, image_id, phase, key0, key1, j);
                int v = (int)((px4 >> (8 * j)) & 0xFF) + dmin + cnt;
                v = (v < 0 ? 0 : (v > 255 ? 255 : v)) - 128;
                packed[j] |= (uint32_t)(v & 0xFF) << (8 * c);
            }
        }
    }
}

__device__ __forceinline__ void resolve_noise_source(const NoiseSource &s, long copy, const uint8_t *&xim,
                                                     const DeviceNoiseTable *&tab, uint32_t &image_id, uint32_t &sample) {
    xim = s.x; tab = s.table; image_id = s.image; sample = s.sample_begin + (uint32_t)copy;
    if (s.items) {
        const uint64_t slot = s.slot_begin + (uint64_t)copy, item = slot / s.n_per_item;
        const NoiseItem it = s.items[item];
        xim = s.x + (size_t)it.image * s.C * s.H * s.W;
        tab = s.table + it.table_slot;
        image_id = it.image_id;
        sample = (uint32_t)(slot - item * s.n_per_item);
    }
}

}  // namespace isr

#endif
