// First layer fused with the max pooling that follows it: 7x7 stride-2 convolution
// (pad 3) of the noisy NHWC4 image into 64 channels, then 3x3 stride-2 max pooling
// (pad 1, in-bounds taps only), then requantisation + clamp -- in that order: for a
// positive multiplier the requantisation z + RHA(acc M0, s) and the clamp are
// non-decreasing in acc, so the maximum over a window of requantised values equals
// the requantised maximum of the int32 accumulators.  Pooling the accumulators first
// requantises a quarter of the values and nothing but the pooled tensor leaves the CU.
//
// A wave makes 2 pooled rows x 31 pooled columns; 4 waves (2 row pairs x 2 column
// strips, or 4 row pairs for images of at most 31 pooled columns) share in LDS
//   * the 64 x 256-byte weight matrix (K = (ky, kx padded to 8, channel padded to 4)),
//   * the input rows of their band, shifted right by 3 pixels and padded with the input
//     zero-point, so that the 16 K-bytes of an MFMA fragment lane -- 4 horizontally
//     adjacent taps x 4 channels -- are 16 contiguous, 8-byte aligned LDS bytes.
// Per convolution row the wave computes one MFMA fragment of the 32 even columns
// 2 px and one of the odd columns 2 px - 1 (v_mfma_i32_32x32x32_i8, one K step per
// kernel row, both operands from LDS, no global gather); the horizontal maximum of a
// pooled pixel is then lane-local but for the right neighbour, fetched with a DPP
// wave shift, and the vertical maximum runs in registers over the 5 rows.
#include <climits>

#include "conv_device.h"
#include "noise_device.h"

namespace isr {

namespace {

constexpr int SP_WMAX = 224;            // widest input row held in LDS
constexpr int SP_K = 7, SP_KP = 256;    // kernel size; padded K bytes per output channel
constexpr int SP_STRIP = 31;            // pooled columns per wave
// input band: 23 rows of up to 232 pixels (two strips) or 39 rows of up to 132 (one strip)
constexpr int SP_IN_BYTES = 23 * (SP_WMAX + 8) * 4;
static_assert(39 * (4 * SP_STRIP + 8) * 4 <= SP_IN_BYTES, "one-strip band fits");

__global__ __launch_bounds__(256, 3) void stem_pool_kernel(const StemPoolParams p) {
    __shared__ __attribute__((aligned(16))) int8_t Wl[64 * SP_KP];
    __shared__ __attribute__((aligned(16))) int8_t In[SP_IN_BYTES];
    __shared__ int prm[4][64];
    __shared__ NoiseLds ntab;                 // the sampler's table when the kernel draws its own input

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nstrips = (p.Wp + SP_STRIP - 1) / SP_STRIP;       // 1 or 2 (checked by the launcher)
    const int P = 2 * (4 / nstrips);                            // pooled rows per workgroup
    const int nbands = (p.Hp + P - 1) / P;
    const int b = blockIdx.x / nbands, p0 = (blockIdx.x % nbands) * P;
    const int cy0 = 2 * p0 - 1;               // first convolution row of the band (may be -1)
    const int iy0 = 2 * cy0 - 3;              // first input row of the band
    const int IR = 4 * P + 7;                 // input rows of the band
    const int PW = p.W + 8;                   // patch row stride in pixels
    const uint32_t zb = (uint32_t)(p.zp_in & 0xFF) * 0x01010101u;

    // weights: row r, 16-byte chunk c at chunk position c ^ (r & 15)
    for (int i = tid; i < 64 * (SP_KP / 16); i += 256) {
        const int r = i >> 4, c = i & 15;
        *(v4i *)(&Wl[r * SP_KP + ((c ^ (r & 15)) << 4)]) = *(const v4i *)(p.w + (long)r * SP_KP + c * 16);
    }
    if (tid < 64) { prm[0][tid] = p.bias[tid]; prm[1][tid] = p.m0s[tid]; prm[2][tid] = p.chi[tid]; prm[3][tid] = p.shm1[tid]; }
    // input band: pixel (row r, input column x) at patch column x + 3
    const int wchunks = p.W >> 2;             // 16-byte chunks (4 pixels) per input row
    if (p.fused_noise) {
        // the noisy rows are drawn here instead of being read back from memory: the stream is counter-based,
        // so the rows that neighbouring bands share are simply drawn again, bit for bit the same
        const uint8_t *xim;
        const DeviceNoiseTable *tab;
        uint32_t image_id, sample;
        resolve_noise_source(p.noise, b, xim, tab, image_id, sample);
        stage_noise_table(ntab, tab, tid, 256);
        const int n = (int)tab->n, dmin = tab->dmin;
        __syncthreads();
        for (int i = tid; i < IR * wchunks; i += 256) {
            const int r = i / wchunks, c = i - r * wchunks, iy = iy0 + r;
            uint32_t v[4] = {zb, zb, zb, zb};
            if ((unsigned)iy < (unsigned)p.H)
                noisy_quad(ntab, n, dmin, xim, p.noise.C, p.H, p.W, iy, c, sample, image_id, p.noise.phase, p.noise.key0, p.noise.key1, v);
            int *dst = (int *)(&In[(r * PW + 3 + 4 * c) * 4]);
            dst[0] = (int)v[0]; dst[1] = (int)v[1]; dst[2] = (int)v[2]; dst[3] = (int)v[3];
        }
    } else {
        for (int i = tid; i < IR * wchunks; i += 256) {
            const int r = i / wchunks, c = i - r * wchunks, iy = iy0 + r;
            v4i v = {(int)zb, (int)zb, (int)zb, (int)zb};
            if ((unsigned)iy < (unsigned)p.H) v = *(const v4i *)(p.in + (((long)b * p.H + iy) * p.W + 4 * c) * 4);
            int *dst = (int *)(&In[(r * PW + 3 + 4 * c) * 4]);
            dst[0] = v[0]; dst[1] = v[1]; dst[2] = v[2]; dst[3] = v[3];
        }
    }
    for (int i = tid; i < IR * 8; i += 256) {   // 3 columns left, 5 right of the image
        const int r = i >> 3, c = i & 7;
        *(int *)(&In[(r * PW + (c < 3 ? c : p.W + c)) * 4]) = (int)zb;
    }
    __syncthreads();

    // ---- this wave: pooled rows py0, py0 + 1, pooled columns px0 .. px0 + 30 ----
    const int strip = wave % nstrips, rg = wave / nstrips;
    const int py0 = p0 + 2 * rg, px0 = strip * SP_STRIP;
    if (py0 >= p.Hp) return;                  // wave-uniform; no barrier follows
    const int l = lane & 31, half = lane >> 5;
    const int px = px0 + l;
    const bool pxok = l < SP_STRIP && px < p.Wp;
    const int oxe = pxok ? 2 * px : 0;                         // even fragment: column 2 px
    const int oxo_raw = 2 * (px0 + l) - 1;                     // odd fragment: column 2 px - 1 (left neighbour)
    const bool ook = oxo_raw >= 0 && oxo_raw < p.Wo;           // also the right neighbour of lane l - 1
    const int oxo = ook ? oxo_raw : 0;
    const int8_t *srce = &In[(2 * oxe + 4 * half) * 4], *srco = &In[(2 * oxo + 4 * half) * 4];
    const int rowbytes = PW * 4;
    const int lo = p.relu ? p.zp_out : -128;

#pragma unroll 1
    for (int fm = 0; fm < 2; ++fm) {
        const int oc = fm * 32 + 16 * half;   // first of the 16 channels this lane holds
        v4i fa[SP_K];
#pragma unroll
        for (int ky = 0; ky < SP_K; ++ky) {
            const int r = fm * 32 + l, c = ky * 2 + half;
            fa[ky] = *(const v4i *)(&Wl[r * SP_KP + ((c ^ (r & 15)) << 4)]);
        }
        v16i binit;
#pragma unroll
        for (int i = 0; i < 16; ++i) binit[i] = prm[0][oc + i];
        int va[16], vb[16];                   // running maxima of the two pooled rows
#pragma unroll
        for (int i = 0; i < 16; ++i) va[i] = vb[i] = INT_MIN;

        auto emit_as = [&](const int *v, int py, auto tie_free) {
            int q[16];
#pragma unroll
            for (int i = 0; i < 16; ++i)
                q[i] = clamp3(requant_q<decltype(tie_free)::value>(v[i], prm[1][oc + i], prm[2][oc + i], prm[3][oc + i]), lo, 127);
            const v4i o = {(int)pack4(q[0], q[1], q[2], q[3]), (int)pack4(q[4], q[5], q[6], q[7]),
                           (int)pack4(q[8], q[9], q[10], q[11]), (int)pack4(q[12], q[13], q[14], q[15])};
            *(v4i *)(p.out + ((((long)b * p.Hp + py) * p.Wp + px) << 6) + oc) = o;
        };
        auto emit = [&](const int *v, int py) {
            if (py >= p.Hp || !pxok) return;
            if (p.tie_free) emit_as(v, py, std::true_type{});
            else emit_as(v, py, std::false_type{});
        };

#pragma unroll
        for (int r = 0; r < 5; ++r) {
            const int cyl = 4 * rg + r, cy = cy0 + cyl;       // convolution row: local, global
            if ((unsigned)cy < (unsigned)p.Ho) {              // rows outside the image never win the max
                v16i ae = binit, ao = binit;
#pragma unroll
                for (int ky = 0; ky < SP_K; ++ky) {
                    const int off = (2 * cyl + ky) * rowbytes;
                    const long long e0 = *(const long long *)(srce + off), e1 = *(const long long *)(srce + off + 8);
                    const long long o0 = *(const long long *)(srco + off), o1 = *(const long long *)(srco + off + 8);
                    const v4i fe = {(int)e0, (int)(e0 >> 32), (int)e1, (int)(e1 >> 32)};
                    const v4i fo = {(int)o0, (int)(o0 >> 32), (int)o1, (int)(o1 >> 32)};
                    ae = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[ky], fe, ae, 0, 0, 0);
                    ao = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[ky], fo, ao, 0, 0, 0);
                }
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int left = ook ? ao[i] : INT_MIN;
                    // lane + 1 holds column 2 px + 1 (wave_shl:1 reads the next lane)
                    const int right = __builtin_amdgcn_update_dpp(INT_MIN, left, 0x130, 0xf, 0xf, false);
                    int h = ae[i] > left ? ae[i] : left;
                    h = h > right ? h : right;
                    if (r <= 2) va[i] = va[i] > h ? va[i] : h;
                    if (r >= 2) vb[i] = vb[i] > h ? vb[i] : h;
                }
            }
            if (r == 2) emit(va, py0);
            if (r == 4) emit(vb, py0 + 1);
        }
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
    // geometry the kernel assumes: 7x7/2 pad 3 then 3x3/2 pad 1, at most two strips of pooled columns
    if (p.W % 4 != 0 || p.W < 8 || p.W > SP_WMAX || p.Ho != (p.H - 1) / 2 + 1 || p.Wo != (p.W - 1) / 2 + 1 ||
        p.Hp != (p.Ho - 1) / 2 + 1 || p.Wp != (p.Wo - 1) / 2 + 1 || p.Wp > 2 * SP_STRIP || !p.out || !p.w)
        return hipErrorInvalidValue;
    if (p.fused_noise) {
        const NoiseSource &ns = p.noise;
        if (!ns.x || !ns.table || ns.C < 1 || ns.C > 3 || ns.H != p.H || ns.W != p.W || (ns.items && ns.n_per_item == 0)) return hipErrorInvalidValue;
    } else if (!p.in) {
        return hipErrorInvalidValue;
    }
    const int nstrips = (p.Wp + SP_STRIP - 1) / SP_STRIP, P = 2 * (4 / nstrips);
    if ((4 * P + 7) * (p.W + 8) * 4 > SP_IN_BYTES) return hipErrorInvalidValue;
    const long blocks = (long)p.B * ((p.Hp + P - 1) / P);
    if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
    set_kernel_name(p.fused_noise ? "stem_pool_kernel (+noise)" : "stem_pool_kernel");
    hipLaunchKernelGGL(stem_pool_kernel, dim3((unsigned)blocks), dim3(256), 0, st, p);
    return hipGetLastError();
}

}  // namespace isr
