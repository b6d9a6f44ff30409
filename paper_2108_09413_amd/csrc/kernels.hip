// Memory-bound stages of the Monte-Carlo loop: noise injection, residual add,
// pooling, the FC + argmax + vote tally.
#include "noise_device.h"

namespace isr {

typedef int v4i __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------
// Noise: x + delta, delta ~ discrete Gaussian (Def. 3.3), saturated to [0,255],
// recentred to int8, written as NHWC4 (4th channel 0).
//
// Randomness: Philox4x32-10 keyed by the seed; counter (p >> 2, sample, image,
// 2*phase + half) with p the logical [C][H][W] pixel index; word p & 3; half 0
// supplies the high 32 bits of the uniform 64-bit u, half 1 the low 32 bits.
// The low half is generated only when the high word ties with a threshold.

__global__ __launch_bounds__(256) void noise_kernel(const NoiseParams p) {
    __shared__ NoiseLds t;
    // what this workgroup draws: one image, one table, a range of sample indices, a range of output copies
    const uint8_t *xim = p.x;
    const DeviceNoiseTable *tab = p.table;
    uint32_t image_id = p.image, sample_begin = p.sample_begin, count = p.count;
    long out_copy0 = 0;
    if (p.items) {   // batch mode: grid row = item; its slots that fall into this chunk
        const uint64_t item = (uint64_t)p.item_first + blockIdx.y;
        const uint64_t first = item * p.n_per_item, last = first + p.n_per_item, chunk_end = p.slot_begin + p.count;
        const uint64_t lo = first > p.slot_begin ? first : p.slot_begin, hi = last < chunk_end ? last : chunk_end;
        if (hi <= lo) return;   // uniform over the workgroup
        const NoiseItem it = p.items[item];
        xim = p.x + (size_t)it.image * p.C * p.H * p.W;
        tab = p.table + it.table_slot;
        image_id = it.image_id;
        sample_begin = (uint32_t)(lo - first);
        count = (uint32_t)(hi - lo);
        out_copy0 = (long)(lo - p.slot_begin);
    }
    stage_noise_table(t, tab, threadIdx.x, 256);
    const int n = (int)tab->n;
    const int dmin = tab->dmin;
    __syncthreads();

    const int W4 = p.W >> 2;
    const long groups_per_sample = (long)p.H * W4;
    const long total = groups_per_sample * count;
    for (long g = (long)blockIdx.x * 256 + threadIdx.x; g < total; g += (long)gridDim.x * 256) {
        const uint32_t s_local = (uint32_t)(g / groups_per_sample);
        const int rem = (int)(g - (long)s_local * groups_per_sample);
        const int y = rem / W4, x4 = rem - y * W4;
        const uint32_t sample = sample_begin + s_local;
        uint32_t packed[4];
        noisy_quad(t, n, dmin, xim, p.C, p.H, p.W, y, x4, sample, image_id, p.phase, p.key0, p.key1, packed);
        v4i o = {(int)packed[0], (int)packed[1], (int)packed[2], (int)packed[3]};
        *(v4i *)(p.out + ((out_copy0 + s_local) * groups_per_sample + rem) * 16) = o;
    }
}

hipError_t launch_noise(const NoiseParams &p, hipStream_t st) {
    if (p.count == 0) return hipSuccess;
    if (p.C < 1 || p.C > 3 || (p.W & 3) != 0) return hipErrorInvalidValue;
    unsigned rows = 1;
    uint32_t per_row = p.count;
    if (p.items) {
        if (p.n_per_item == 0 || p.item_count == 0 || p.item_count > 65535) return hipErrorInvalidValue;
        rows = p.item_count;
        if (p.n_per_item < per_row) per_row = p.n_per_item;
    }
    long total = (long)p.H * (p.W >> 2) * per_row;
    long blocks = (total + 255) / 256;
    const long cap = rows >= 4 ? 256 : 256 * 4;   // the table is staged into LDS once per workgroup
    if (blocks > cap) blocks = cap;
    set_kernel_name("noise_kernel");
    hipLaunchKernelGGL(noise_kernel, dim3((unsigned)blocks, rows), dim3(256), 0, st, p);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Noise bank: the discrete-Gaussian draws themselves (no image, no saturation), int16, for
// noise that is sampled ahead of training and stored.  Same generator and counter layout as
// above with the tensor index in the sample word, the bank id in the image word and phase 2;
// the whole threshold table (2R entries) is searched, bucketed by a guide table on the top
// 12 bits; the guide and the high words are staged into LDS (dynamic, 4 bytes per threshold),
// the low words stay in global memory (read on a tie of the high words only).

// #{j < n : T[j] <= u} when the guide bucket of u holds more than one candidate or the high
// word ties with a threshold (rare): binary search inside the bucket, then the low words.
__device__ __noinline__ int bank_count_slow(const uint32_t *thi_s, const uint16_t *guide, const NoiseBankParams &p,
                                            uint32_t u, uint32_t grp, uint32_t tensor, int word) {
    const uint32_t b = u >> (32 - NOISE_GUIDE_BITS);
    int a = guide[b], e = guide[b + 1];              // thresholds with a high word below u end before guide[b + 1]
    while (a < e) {                                  // first index whose high word is >= u
        const int mid = (a + e) >> 1;
        if (thi_s[mid] < u) a = mid + 1; else e = mid;
    }
    int c = a;
    if (c < p.n && thi_s[c] == u) {                  // equal high words: the low words decide
        uint32_t lo[4];
        philox4x32_10(grp, tensor, p.bank, 5u, p.key0, p.key1, lo);
        while (c < p.n && thi_s[c] == u && p.tlo[c] <= lo[word & 3]) ++c;
    }
    return c;
}

__global__ __launch_bounds__(256) void noise_bank_kernel(const NoiseBankParams p) {
    __shared__ uint16_t guide[NOISE_GUIDE_SIZE + 2];
    extern __shared__ uint32_t thi_s[];              // n high words, then two entries of 0xFFFFFFFF
    for (int i = threadIdx.x; i < (int)(NOISE_GUIDE_SIZE + 2) / 2; i += 256)
        ((uint32_t *)guide)[i] = ((const uint32_t *)p.guide)[i];
    for (int i = threadIdx.x; i < p.n + 2; i += 256) thi_s[i] = i < p.n ? p.thi[i] : 0xFFFFFFFFu;
    __syncthreads();
    const uint64_t groups_per_tensor = p.d >> 2, total = groups_per_tensor * p.count;
    for (uint64_t g = (uint64_t)blockIdx.x * 256 + threadIdx.x; g < total; g += (uint64_t)gridDim.x * 256) {
        const uint32_t t = (uint32_t)(g / groups_per_tensor), grp = (uint32_t)(g - (uint64_t)t * groups_per_tensor);
        const uint32_t tensor = p.first + t;
        uint32_t hi[4];
        philox4x32_10(grp, tensor, p.bank, 4u, p.key0, p.key1, hi);
        int d4[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t u = hi[j];
            int c = guide[u >> (32 - NOISE_GUIDE_BITS)];
            const uint32_t t0 = thi_s[c], t1 = thi_s[c + 1];
            c += t0 < u;
            // common case: at most one threshold below u in the bucket and no tie
            if ((t0 < u ? t1 : t0) <= u) c = bank_count_slow(thi_s, guide, p, u, grp, tensor, j);
            d4[j] = c - p.R;
        }
        const uint32_t w0 = (uint32_t)(d4[0] & 0xFFFF) | ((uint32_t)d4[1] << 16), w1 = (uint32_t)(d4[2] & 0xFFFF) | ((uint32_t)d4[3] << 16);
        *(uint2 *)(p.out + ((uint64_t)t * p.d + 4ull * grp)) = make_uint2(w0, w1);
    }
}

hipError_t launch_noise_bank(const NoiseBankParams &p, hipStream_t st) {
    if (p.count == 0) return hipSuccess;
    if (p.d == 0 || (p.d & 3) != 0 || p.n < 2 || p.n > 32768 || !p.thi || !p.tlo || !p.guide || !p.out) return hipErrorInvalidValue;
    const uint64_t total = (uint64_t)(p.d >> 2) * p.count;
    uint64_t blocks = (total + 255) / 256;
    if (blocks > 256 * 8) blocks = 256 * 8;
    const size_t lds = ((size_t)p.n + 2) * 4;   // at most 128 KiB plus the 8 KiB guide: within the 160 KiB of a CU (sigma 1024 needs 72 KiB)
    hipError_t e = hipFuncSetAttribute((const void *)noise_bank_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    set_kernel_name("noise_bank_kernel");
    hipLaunchKernelGGL(noise_bank_kernel, dim3((unsigned)blocks), dim3(256), lds, st, p);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Residual add of two int8 tensors with requantisation:
//   out = clamp(z_o + RHA((qa - za) Ma + (qb - zb) Mb, shift), relu ? z_o : -128, 127)

__device__ __forceinline__ int rha64(long v, int s) {
    if (s == 0) return (int)v;
    long half = 1L << (s - 1);
    return (int)(v >= 0 ? (v + half) >> s : -((-v + half) >> s));
}

__global__ __launch_bounds__(256) void add_kernel(const AddParams p) {
    const int lo = p.relu ? p.zo : -128;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < p.n16; i += (long)gridDim.x * 256) {
        v4i va = *(const v4i *)(p.a + i * 16), vb = *(const v4i *)(p.b + i * 16), vo;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            uint32_t packed = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                int qa = (int)(int8_t)((uint32_t)va[d] >> (8 * e));
                int qb = (int)(int8_t)((uint32_t)vb[d] >> (8 * e));
                long v = (long)(qa - p.za) * p.Ma + (long)(qb - p.zb) * p.Mb;
                int r = p.zo + rha64(v, p.sh);
                r = r < lo ? lo : (r > 127 ? 127 : r);
                packed |= (uint32_t)(r & 0xFF) << (8 * e);
            }
            vo[d] = (int)packed;
        }
        *(v4i *)(p.out + i * 16) = vo;
    }
}

hipError_t launch_add(const AddParams &p, hipStream_t st) {
    if (p.n16 <= 0) return hipSuccess;
    long blocks = (p.n16 + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    set_kernel_name("add_kernel");
    hipLaunchKernelGGL(add_kernel, dim3((unsigned)blocks), dim3(256), 0, st, p);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Max pooling over in-bounds taps, NHWC, 16 channels per thread.

__global__ __launch_bounds__(256) void maxpool_kernel(const PoolParams p) {
    const int c16 = p.Cp >> 4;
    const long total = (long)p.B * p.Ho * p.Wo * c16;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        int cg = (int)(i % c16);
        long pix = i / c16;
        int ox = (int)(pix % p.Wo);
        long t = pix / p.Wo;
        int oy = (int)(t % p.Ho);
        long b = t / p.Ho;
        int best[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) best[e] = -128;
        for (int ky = 0; ky < p.k; ++ky) {
            int iy = oy * p.stride - p.pad + ky;
            if ((unsigned)iy >= (unsigned)p.H) continue;
            for (int kx = 0; kx < p.k; ++kx) {
                int ix = ox * p.stride - p.pad + kx;
                if ((unsigned)ix >= (unsigned)p.W) continue;
                v4i v = *(const v4i *)(p.in + ((b * p.H + iy) * p.W + ix) * p.Cp + cg * 16);
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    int q = (int)(int8_t)((uint32_t)v[e >> 2] >> (8 * (e & 3)));
                    best[e] = q > best[e] ? q : best[e];
                }
            }
        }
        v4i o;
#pragma unroll
        for (int d = 0; d < 4; ++d)
            o[d] = (int)((uint32_t)(best[4 * d] & 0xFF) | ((uint32_t)(best[4 * d + 1] & 0xFF) << 8) |
                         ((uint32_t)(best[4 * d + 2] & 0xFF) << 16) | ((uint32_t)best[4 * d + 3] << 24));
        *(v4i *)(p.out + pix * p.Cp + cg * 16) = o;
    }
}

hipError_t launch_maxpool(const PoolParams &p, hipStream_t st) {
    long total = (long)p.B * p.Ho * p.Wo * (p.Cp >> 4);
    if (total <= 0) return hipSuccess;
    long blocks = (total + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    set_kernel_name("maxpool_kernel");
    hipLaunchKernelGGL(maxpool_kernel, dim3((unsigned)blocks), dim3(256), 0, st, p);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Global average pooling: S = sum over H*W of (q - z_in), requantised like a
// convolution output with a scalar (M0, shift); 4 channels per thread.

__global__ __launch_bounds__(256) void gap_kernel(const GapParams p) {
    const int c4 = p.Cp >> 2;
    const long total = (long)p.B * c4;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        int cg = (int)(i % c4);
        long b = i / c4;
        const int8_t *src = p.in + b * p.HW * p.Cp + cg * 4;
        int s[4] = {0, 0, 0, 0};
        for (int t = 0; t < p.HW; ++t) {
            uint32_t v = *(const uint32_t *)(src + (long)t * p.Cp);
#pragma unroll
            for (int e = 0; e < 4; ++e) s[e] += (int)(int8_t)(v >> (8 * e));
        }
        uint32_t packed = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            long v = (long)(s[e] - p.HW * p.zp_in) * p.M0;
            int r = p.zp_out + rha64(v, 31 + p.sh);
            r = r < -128 ? -128 : (r > 127 ? 127 : r);
            packed |= (uint32_t)(r & 0xFF) << (8 * e);
        }
        *(uint32_t *)(p.out + b * p.Cp + cg * 4) = packed;
    }
}

hipError_t launch_gap(const GapParams &p, hipStream_t st) {
    long total = (long)p.B * (p.Cp >> 2);
    if (total <= 0) return hipSuccess;
    long blocks = (total + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    set_kernel_name("gap_kernel");
    hipLaunchKernelGGL(gap_kernel, dim3((unsigned)blocks), dim3(256), 0, st, p);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// FC logits (int32, no requantisation), wavefront argmax (lowest index among
// maxima) and vote histogram: one wave per sample, LDS histogram per block,
// one global atomic per class per block.

constexpr int FC_MAX_CLASSES = 1024;

__global__ __launch_bounds__(256) void fc_vote_kernel(const FcParams p) {
    __shared__ uint32_t hist[FC_MAX_CLASSES];
    for (int i = threadIdx.x; i < p.classes; i += 256) hist[i] = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (long s = (long)blockIdx.x * 4 + wave; s < p.B; s += (long)gridDim.x * 4) {
        const int8_t *a = p.in + s * p.Kp;
        int best = INT32_MIN, best_idx = 0x7FFFFFFF;
        for (int c = lane; c < p.classes; c += 64) {
            // weights are stored [K / 16][classes_p][16]: the 64 classes of a pass read 1 KiB contiguous
            const int8_t *w = p.w + (long)c * 16;
            int acc = p.bias[c];
#pragma unroll 4
            for (int k = 0; k < p.Kp; k += 16) {
                v4i va = *(const v4i *)(a + k), vw = *(const v4i *)(w + (long)(k >> 4) * p.classes_p * 16);
#pragma unroll
                for (int d = 0; d < 4; ++d) acc = __builtin_amdgcn_sdot4(va[d], vw[d], acc, false);
            }
            if (p.logits) p.logits[s * p.classes + c] = acc;
            if (acc > best) { best = acc; best_idx = c; }   // ascending c keeps the lowest index
        }
        // wave reduction: larger logit wins, then the lower class index
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            int ob = __shfl_xor(best, off, 64), oi = __shfl_xor(best_idx, off, 64);
            if (ob > best || (ob == best && oi < best_idx)) { best = ob; best_idx = oi; }
        }
        if (lane == 0) {
            if (p.argmax) p.argmax[s] = best_idx;
            if (p.counts) {
                if (p.n_per_item) atomicAdd(&p.counts[(p.slot_begin + (uint64_t)s) / p.n_per_item * p.classes + best_idx], 1u);
                else atomicAdd(&hist[best_idx], 1u);
            }
        }
    }
    __syncthreads();
    if (p.counts && !p.n_per_item)
        for (int i = threadIdx.x; i < p.classes; i += 256)
            if (hist[i]) atomicAdd(&p.counts[i], hist[i]);
}

// The same for long feature vectors, with the four waves of a workgroup on ONE sample: each wave
// sums a quarter of K for all classes (lane = class) with 16 independent weight loads in
// flight, the partial sums meet in LDS.  The one-wave form above waits for memory 128 times in
// a row at K = 2048.  Integer sums, so the order of the additions is free.
__global__ __launch_bounds__(256) void fc_vote_ksplit_kernel(const FcParams p) {
    __shared__ int part[4][FC_MAX_CLASSES];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int kq = p.Kp >> 2;                        // K bytes per wave, a multiple of 256
    for (long s = blockIdx.x; s < p.B; s += gridDim.x) {
        const int8_t *a = p.in + s * p.Kp + wave * kq;
        for (int c = lane; c < p.classes; c += 64) {
            const int8_t *w = p.w + ((long)(wave * kq >> 4) * p.classes_p + c) * 16;
            int acc = 0;
            for (int k0 = 0; k0 < kq; k0 += 256) {
                v4i vw[16];
#pragma unroll
                for (int j = 0; j < 16; ++j) vw[j] = *(const v4i *)(w + (long)((k0 >> 4) + j) * p.classes_p * 16);
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const v4i va = *(const v4i *)(a + k0 + 16 * j);
#pragma unroll
                    for (int d = 0; d < 4; ++d) acc = __builtin_amdgcn_sdot4(va[d], vw[j][d], acc, false);
                }
            }
            part[wave][c] = acc;
        }
        __syncthreads();
        if (wave == 0) {
            int best = INT32_MIN, best_idx = 0x7FFFFFFF;
            for (int c = lane; c < p.classes; c += 64) {
                const int acc = p.bias[c] + part[0][c] + part[1][c] + part[2][c] + part[3][c];
                if (p.logits) p.logits[s * p.classes + c] = acc;
                if (acc > best) { best = acc; best_idx = c; }   // ascending c keeps the lowest index
            }
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                int ob = __shfl_xor(best, off, 64), oi = __shfl_xor(best_idx, off, 64);
                if (ob > best || (ob == best && oi < best_idx)) { best = ob; best_idx = oi; }
            }
            if (lane == 0) {
                if (p.argmax) p.argmax[s] = best_idx;
                if (p.counts) {
                    const uint64_t row = p.n_per_item ? (p.slot_begin + (uint64_t)s) / p.n_per_item : 0;
                    atomicAdd(&p.counts[row * p.classes + best_idx], 1u);
                }
            }
        }
        __syncthreads();   // part is free for the next sample
    }
}

hipError_t launch_fc(const FcParams &p, hipStream_t st) {
    if (p.B <= 0) return hipSuccess;
    if (p.classes < 1 || p.classes > FC_MAX_CLASSES || p.Kp % 16 != 0 || p.classes_p < p.classes) return hipErrorInvalidValue;
    if (p.Kp % 1024 == 0) {
        long blocks = p.B;
        if (blocks > 256 * 16) blocks = 256 * 16;
        set_kernel_name("fc_vote_ksplit_kernel");
        hipLaunchKernelGGL(fc_vote_ksplit_kernel, dim3((unsigned)blocks), dim3(256), 0, st, p);
        return hipGetLastError();
    }
    long blocks = ((long)p.B + 3) / 4;
    if (blocks > 256 * 8) blocks = 256 * 8;
    set_kernel_name("fc_vote_kernel");
    hipLaunchKernelGGL(fc_vote_kernel, dim3((unsigned)blocks), dim3(256), 0, st, p);
    return hipGetLastError();
}

__global__ void fill_u32_kernel(uint32_t *p, uint32_t v, size_t n) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = v;
}

hipError_t launch_fill_u32(uint32_t *p, uint32_t value, size_t n, hipStream_t st) {
    if (n == 0) return hipSuccess;
    size_t blocks = (n + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)blocks), dim3(256), 0, st, p, value, n);
    return hipGetLastError();
}

}  // namespace isr
