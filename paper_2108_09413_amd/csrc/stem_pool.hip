// First layer fused with the max pooling that follows it: 7x7 stride-2 convolution
// (pad 3) of the noisy NHWC4 image into 64 channels, requantisation + clamp, then
// 3x3 stride-2 max pooling (pad 1, in-bounds taps only) -- the convolution output
// never goes to HBM.
//
// One workgroup (4 waves) makes P pooled rows of one sample.  It stages in LDS
//   * the 64 x 256-byte weight matrix (K = (ky, kx padded to 8, channel padded to 4)),
//   * the 4P + 7 input rows the band needs, shifted right by 3 pixels and padded with the
//     input zero-point, so that the 16 K-bytes of an MFMA fragment lane -- 4 horizontally
//     adjacent taps x 4 channels -- are 16 contiguous, 8-byte aligned LDS bytes,
//   * the 2P + 1 convolution rows as int8 [pixel][64 channels],
// computes the convolution with v_mfma_i32_32x32x32_i8 (one K step per kernel row ky,
// both operands read from LDS, no global gather), and pools out of LDS.
#include "conv_device.h"

namespace isr {

namespace {

constexpr int SP_WMAX = 224;            // widest input row held in LDS
constexpr int SP_K = 7, SP_KP = 256;    // kernel size; padded K bytes per output channel

// 16 channels of pixel `n` sit at chunk (c ^ spswz(n)) of its 64-byte row: the 128-bit
// stores of 16 consecutive pixels then hit 16 different bank groups
__device__ __forceinline__ int spswz(int n) { return (n >> 2) & 3; }

template <int P>
__global__ __launch_bounds__(256, 2) void stem_pool_kernel(const StemPoolParams p) {
    constexpr int CR = 2 * P + 1;             // convolution rows of the band
    constexpr int IR = 2 * CR + 5;            // input rows of the band
    constexpr int PWMAX = SP_WMAX + 8;        // patch row stride in pixels (3 left, >= 4 right padding + alignment)
    constexpr int WOMAX = SP_WMAX / 2;
    __shared__ __attribute__((aligned(16))) int8_t Wl[64 * SP_KP];
    __shared__ __attribute__((aligned(16))) int8_t In[IR * PWMAX * 4];
    __shared__ __attribute__((aligned(16))) int8_t Cv[CR * WOMAX * 64];
    __shared__ int prm[4][64];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nbands = (p.Hp + P - 1) / P;
    const int b = blockIdx.x / nbands, p0 = (blockIdx.x % nbands) * P;
    const int cy0 = 2 * p0 - 1;               // first convolution row of the band (may be -1)
    const int iy0 = 2 * cy0 - 3;              // first input row of the band
    const int PW = p.W + 8;                   // patch row stride in pixels
    const uint32_t zb = (uint32_t)(p.zp_in & 0xFF) * 0x01010101u;

    // weights: row r, 16-byte chunk c at chunk position c ^ (r & 15)
    for (int i = tid; i < 64 * (SP_KP / 16); i += 256) {
        const int r = i >> 4, c = i & 15;
        *(v4i *)(&Wl[r * SP_KP + ((c ^ (r & 15)) << 4)]) = *(const v4i *)(p.w + (long)r * SP_KP + c * 16);
    }
    if (tid < 64) { prm[0][tid] = p.bias[tid]; prm[1][tid] = p.m0s[tid]; prm[2][tid] = p.chi[tid]; prm[3][tid] = p.shm1[tid]; }
    // input patch: pixel (row r, input column x) at patch column x + 3
    const int wchunks = p.W >> 2;             // 16-byte chunks (4 pixels) per input row
    for (int i = tid; i < IR * wchunks; i += 256) {
        const int r = i / wchunks, c = i - r * wchunks, iy = iy0 + r;
        v4i v = {(int)zb, (int)zb, (int)zb, (int)zb};
        if ((unsigned)iy < (unsigned)p.H) v = *(const v4i *)(p.in + (((long)b * p.H + iy) * p.W + 4 * c) * 4);
        int *dst = (int *)(&In[(r * PW + 3 + 4 * c) * 4]);
        dst[0] = v[0]; dst[1] = v[1]; dst[2] = v[2]; dst[3] = v[3];
    }
    for (int i = tid; i < IR * 8; i += 256) {   // 3 columns left, 5 right of the image
        const int r = i >> 3, c = i & 7;
        *(int *)(&In[(r * PW + (c < 3 ? c : p.W + c)) * 4]) = (int)zb;
    }
    __syncthreads();

    // ---- convolution of the band: CR x Wo pixels in fragments of 32, 64 channels ----
    const int npix = CR * p.Wo, nfrag = (npix + 31) >> 5;
    const int half = lane >> 5;
    const int lo = p.relu ? p.zp_out : -128;
    for (int f = wave; f < nfrag; f += 4) {
        int n = f * 32 + (lane & 31);
        const bool live = n < npix;
        if (!live) n = 0;
        const int cyl = n / p.Wo, ox = n - cyl * p.Wo;
        const int8_t *bsrc = &In[((2 * cyl) * PW + 2 * ox + 4 * half) * 4];
        v16i acc[2];
#pragma unroll
        for (int fm = 0; fm < 2; ++fm)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[fm][i] = prm[0][fm * 32 + 16 * half + i];
#pragma unroll
        for (int ky = 0; ky < SP_K; ++ky) {
            const long long b0 = *(const long long *)(bsrc + ky * PW * 4), b1 = *(const long long *)(bsrc + ky * PW * 4 + 8);
            const v4i fb = {(int)b0, (int)(b0 >> 32), (int)b1, (int)(b1 >> 32)};
#pragma unroll
            for (int fm = 0; fm < 2; ++fm) {
                const int r = fm * 32 + (lane & 31), c = ky * 2 + half;
                const v4i fa = *(const v4i *)(&Wl[r * SP_KP + ((c ^ (r & 15)) << 4)]);
                acc[fm] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa, fb, acc[fm], 0, 0, 0);
            }
        }
        const int cy = cy0 + cyl;
        const bool inside = (unsigned)cy < (unsigned)p.Ho;   // rows outside the image never win the max
#pragma unroll
        for (int fm = 0; fm < 2; ++fm) {
            const int oc = fm * 32 + 16 * half;
            int q[16];
#pragma unroll
            for (int i = 0; i < 16; ++i)
                q[i] = inside ? clamp3(requant_fast(acc[fm][i], prm[1][oc + i], prm[2][oc + i], prm[3][oc + i]), lo, 127) : -128;
            const v4i v = {(int)pack4(q[0], q[1], q[2], q[3]), (int)pack4(q[4], q[5], q[6], q[7]),
                           (int)pack4(q[8], q[9], q[10], q[11]), (int)pack4(q[12], q[13], q[14], q[15])};
            if (live) *(v4i *)(&Cv[n * 64 + (((oc >> 4) ^ spswz(n)) << 4)]) = v;
        }
    }
    __syncthreads();

    // ---- 3x3 stride-2 max pooling out of LDS: 16 channels per thread and item ----
    const int items = P * p.Wp * 4;
    for (int i = tid; i < items; i += 256) {
        const int cg = i & 3, px = (i >> 2) % p.Wp, pyl = (i >> 2) / p.Wp;
        const int py = p0 + pyl;
        if (py >= p.Hp) continue;
        int best[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) best[e] = -128;
#pragma unroll
        for (int ky = 0; ky < 3; ++ky)
#pragma unroll
            for (int kx = 0; kx < 3; ++kx) {
                const int cx = 2 * px - 1 + kx;
                if ((unsigned)cx >= (unsigned)p.Wo) continue;
                const int n = (2 * pyl + ky) * p.Wo + cx;
                const v4i v = *(const v4i *)(&Cv[n * 64 + ((cg ^ spswz(n)) << 4)]);
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int q = (int)(int8_t)((uint32_t)v[e >> 2] >> (8 * (e & 3)));
                    best[e] = q > best[e] ? q : best[e];
                }
            }
        const v4i o = {(int)pack4(best[0], best[1], best[2], best[3]), (int)pack4(best[4], best[5], best[6], best[7]),
                       (int)pack4(best[8], best[9], best[10], best[11]), (int)pack4(best[12], best[13], best[14], best[15])};
        *(v4i *)(p.out + ((((long)b * p.Hp + py) * p.Wp + px) << 6) + cg * 16) = o;
    }
}

}  // namespace

bool stem_pool_supported(int k, int stride, int pad, int cout_p, int H, int W, int fast_requant, int pool_k,
                         int pool_stride, int pool_pad) {
    return k == SP_K && stride == 2 && pad == 3 && cout_p == 64 && fast_requant && pool_k == 3 && pool_stride == 2 &&
           pool_pad == 1 && W % 4 == 0 && W >= 8 && W <= SP_WMAX && H >= 1;
}

hipError_t launch_stem_pool(const StemPoolParams &p, hipStream_t st) {
    if (p.B <= 0) return hipSuccess;
    // geometry the kernel assumes: 7x7/2 pad 3 then 3x3/2 pad 1
    if (p.W % 4 != 0 || p.W < 8 || p.W > SP_WMAX || p.Ho != (p.H - 1) / 2 + 1 || p.Wo != (p.W - 1) / 2 + 1 ||
        p.Hp != (p.Ho - 1) / 2 + 1 || p.Wp != (p.Wo - 1) / 2 + 1 || !p.in || !p.out || !p.w)
        return hipErrorInvalidValue;
    constexpr int P = 2;
    const long blocks = (long)p.B * ((p.Hp + P - 1) / P);
    if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((stem_pool_kernel<P>), dim3((unsigned)blocks), dim3(256), 0, st, p);
    return hipGetLastError();
}

}  // namespace isr
