// Kernels of the two floating-point comparison systems of the paper's evaluation (section
// "Experiments": FloatRS-quant, FloatRS-fp): continuous Gaussian noise on the image, then either
// rounding back onto the pixel grid (the int8 network follows) or the fp32 network, whose
// convolutions run here as implicit GEMMs on the fp32 MFMA.
#include <hip/hip_runtime.h>

#include "isr_internal.h"
#include "noise_device.h"

namespace isr {

namespace {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef int v4i __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------
// The binary32 standard-normal sampler.  Every step is one IEEE operation (+, -, *, /, sqrt,
// rounded once, never contracted into a fused multiply-add), so a draw is the same bit pattern
// on any conforming machine:
//   Box-Muller on two 32-bit words (wa, wb): u = ((wa >> 8) + 1) / 2^24 in (0, 1],
//   v = (wb >> 8) / 2^24 in [0, 1);  z_a = sqrt(-2 ln u) cos(2 pi v), z_b = sqrt(-2 ln u) sin(2 pi v);
//   ln by range reduction to [sqrt(1/2), sqrt(2)] and the atanh series, cos / sin by octant and the
//   Taylor polynomials on [0, pi/4).

// -ln(n / 2^24), n in [1, 2^24].
__device__ __forceinline__ float neg_log_u24(uint32_t n) {
#pragma clang fp contract(off)
    const float f = (float)n;                                  // exact
    const uint32_t bits = __float_as_uint(f);
    int E = (int)(bits >> 23) - 127;                           // n = m 2^E, m in [1, 2)
    float m = __uint_as_float((bits & 0x7FFFFFu) | 0x3F800000u);
    if (m > 1.41421354f) { m = m * 0.5f; E += 1; }
    const float k = (float)(24 - E);
    const float s = __fdiv_rn(m - 1.0f, m + 1.0f);             // ln m = 2 atanh(s)
    const float s2 = s * s;
    float p = 0.222222224f;
    p = p * s2; p = p + 0.285714298f;
    p = p * s2; p = p + 0.400000006f;
    p = p * s2; p = p + 0.666666687f;
    p = p * s2; p = p + 2.0f;
    const float lnm = s * p;
    const float a = k * 0.693145752f;                          // ln 2 = hi + lo; k * hi is exact
    const float b = k * 1.42860677e-06f;
    const float d = a - lnm;
    return d + b;
}

// cos and sin of 2 pi t / 2^24, t in [0, 2^24).
__device__ __forceinline__ void cos_sin_turn24(uint32_t t, float &co, float &si) {
#pragma clang fp contract(off)
    const uint32_t octant = t >> 21, q = t & 0x1FFFFFu;
    const float phi = (float)q * 3.74507039e-07f;              // (pi/4) / 2^21
    const float x2 = phi * phi;
    float c = -2.755732e-07f;
    c = c * x2; c = c + 2.48015876e-05f;
    c = c * x2; c = c - 0.00138888892f;
    c = c * x2; c = c + 0.0416666679f;
    c = c * x2; c = c - 0.5f;
    c = c * x2; c = c + 1.0f;
    float s = 2.75573188e-06f;
    s = s * x2; s = s - 0.000198412701f;
    s = s * x2; s = s + 0.00833333377f;
    s = s * x2; s = s - 0.166666672f;
    s = s * x2; s = s + 1.0f;
    s = s * phi;
    float d = c - s, e = c + s;
    d = d * 0.707106769f;
    e = e * 0.707106769f;
    switch (octant) {
    case 0: co = c; si = s; break;
    case 1: co = d; si = e; break;
    case 2: co = -s; si = c; break;
    case 3: co = -e; si = d; break;
    case 4: co = -c; si = -s; break;
    case 5: co = -d; si = -e; break;
    case 6: co = s; si = -c; break;
    default: co = e; si = -d; break;
    }
}

__device__ __forceinline__ void box_muller(uint32_t wa, uint32_t wb, float &za, float &zb) {
#pragma clang fp contract(off)
    const float l = neg_log_u24((wa >> 8) + 1u);
    // the correctly rounded binary32 root: the binary64 root rounded once more (53 >= 2 * 24 + 2 bits make the
    // second rounding harmless); the fast binary32 root instruction alone is off by one unit in a sixth of the draws
    const float r = (float)sqrt((double)(2.0f * l));
    float c, s;
    cos_sin_turn24(wb >> 8, c, s);
    za = r * c;
    zb = r * s;
}

// One thread per four horizontally adjacent pixels of one copy: per channel one Philox call gives
// the four draws of logical elements (c*H + y)*W + 4 x4 .. + 3.
__global__ __launch_bounds__(256) void float_noise_kernel(const FloatNoiseParams p) {
#pragma clang fp contract(off)
    const int W4 = p.W >> 2;
    const long groups_per_sample = (long)p.H * W4;
    const long total = groups_per_sample * p.count;
    for (long g = (long)blockIdx.x * 256 + threadIdx.x; g < total; g += (long)gridDim.x * 256) {
        const uint32_t s_local = (uint32_t)(g / groups_per_sample);
        const int rem = (int)(g - (long)s_local * groups_per_sample);
        const int y = rem / W4, x4 = rem - y * W4;
        float v[3][4];
#pragma unroll
        for (int c = 0; c < 3; ++c) {
#pragma unroll
            for (int j = 0; j < 4; ++j) v[c][j] = p.quant ? 128.0f : p.center;   // absent channels: code 0 / real value 0
            if (c < p.C) {
                const uint32_t pix = (uint32_t)((c * p.H + y) * p.W + x4 * 4);
                uint32_t w[4];
                philox4x32_10(pix >> 2, p.sample_begin + s_local, p.image, 8u + p.phase, p.key0, p.key1, w);
                float z[4];
                box_muller(w[0], w[1], z[0], z[1]);
                box_muller(w[2], w[3], z[2], z[3]);
                const uint32_t px4 = *(const uint32_t *)(p.x + pix);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float sz = p.sigma * z[j];
                    v[c][j] = (float)((px4 >> (8 * j)) & 0xFF) + sz;
                }
            }
        }
        const long o = (long)s_local * groups_per_sample + rem;
        if (p.quant) {
            int packed[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint32_t word = 0;
#pragma unroll
                for (int c = 0; c < 3; ++c) {
                    float r = rintf(v[c][j]);
                    r = r < 0.0f ? 0.0f : (r > 255.0f ? 255.0f : r);
                    word |= (uint32_t)(((int)r - 128) & 0xFF) << (8 * c);
                }
                packed[j] = (int)word;
            }
            *(v4i *)((int8_t *)p.out + o * 16) = v4i{packed[0], packed[1], packed[2], packed[3]};
        } else {
            float *dst = (float *)p.out + o * 16;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                *(v4f *)(dst + 4 * j) = v4f{v[0][j] - p.center, v[1][j] - p.center, v[2][j] - p.center, 0.0f};
        }
    }
}

// ---------------------------------------------------------------------------
// fp32 convolution: implicit GEMM on v_mfma_f32_32x32x2_f32.  A = weights (rows = output channels),
// B = im2col pixels (columns), K = (tap, channel) cut into quads of 4 consecutive channels; a step
// of the main loop covers 4 quads.  Both operands are staged in LDS as [quad][row][4 floats]; in a
// step's MFMA pair index the lanes 0-31 (k = 0) take their element from quad 2h and the lanes 32-63
// (k = 1) from quad 2h + 1, so each lane reads one 16-byte vector per fragment and uses all of it.
// Global loads of the next step are issued before the MFMAs of the current one (registers), stored
// to the other LDS stage after them; one barrier per step.
//
// Workgroup tile: 32 MT WM channels x 32 NT WN pixels, four waves as WM x WN.

template <int MT, int NT, int WM, int WN>
__global__ __launch_bounds__(256, 2) void fconv_kernel(const FConvParams p) {
    constexpr int BM = 32 * MT * WM, BN = 32 * NT * WN;
    constexpr int ASTR = BM * 4 + 8, BSTR = BN * 4 + 8;        // floats per quad row group; +8 words keeps the 4 quads on distinct banks
    constexpr int STAGE = 4 * ASTR + 4 * BSTR;
    constexpr int NA = (BM * 4 + 255) / 256, NB = BN * 4 / 256;
    static_assert(WM * WN == 4 && BN * 4 % 256 == 0, "four waves; whole float4 rounds for the pixel operand");
    __shared__ __attribute__((aligned(16))) float lds[2 * STAGE];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WM, wn = wave / WM;
    const int half = lane >> 5, l32 = lane & 31;
    const int mtiles = p.Cout_pp / BM;
    // Workgroup ids are dealt round-robin over the 8 XCDs (each with its own L2): renumber them so that an XCD
    // works on a contiguous run of tiles, in which the channel tiles of one pixel tile are neighbours and
    // share that pixel tile through the XCD's L2.
    const long nb = gridDim.x, per = nb >> 3, rem = nb & 7;
    const long xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const long bid = xcd * per + (xcd < rem ? xcd : rem) + slot;   // XCD x owns per (+1 for x < rem) consecutive ids
    const int ch0 = (int)(bid % mtiles) * BM;
    const long px0 = (bid / mtiles) * BN;

    const int bq = tid & 3;
    int b_iy0[NB], b_ix0[NB];
    long b_base[NB];
    bool b_ok[NB];
    const int hw_o = p.Ho * p.Wo;
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        const long P = px0 + (tid >> 2) + 64 * j;
        b_ok[j] = P < p.npix;
        const long Pc = b_ok[j] ? P : 0;
        const int b = (int)(Pc / hw_o), r = (int)(Pc - (long)b * hw_o);
        const int oy = r / p.Wo, ox = r - oy * p.Wo;
        b_iy0[j] = oy * p.stride - p.pad;
        b_ix0[j] = ox * p.stride - p.pad;
        b_base[j] = (long)b * p.H * p.W;
    }

    v16f acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    v4f ga[NA], gb[NB];
    auto gload = [&](int step) {
#pragma unroll
        for (int j = 0; j < NA; ++j) {
            const int idx = tid + 256 * j;
            if (idx < BM * 4) {
                const int q = idx / BM, row = idx % BM;
                ga[j] = *(const v4f *)(p.w + ((long)(step * 4 + q) * p.Cout_pp + ch0 + row) * 4);
            }
        }
        const int e = p.ktab[step * 4 + bq];
        const int dy = e >> 24, dx = (e >> 16) & 0xFF, coff = e & 0xFFFF;
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const int iy = b_iy0[j] + dy, ix = b_ix0[j] + dx;
            const bool inb = b_ok[j] && e >= 0 && (unsigned)iy < (unsigned)p.H && (unsigned)ix < (unsigned)p.W;
            gb[j] = inb ? *(const v4f *)(p.in + (b_base[j] + (long)iy * p.W + ix) * p.Cin_p + coff) : v4f{0.f, 0.f, 0.f, 0.f};
        }
    };
    auto lstore = [&](int stage) {
        float *A = lds + stage * STAGE, *B = A + 4 * ASTR;
#pragma unroll
        for (int j = 0; j < NA; ++j) {
            const int idx = tid + 256 * j;
            if (idx < BM * 4) *(v4f *)(A + (idx / BM) * ASTR + (idx % BM) * 4) = ga[j];
        }
#pragma unroll
        for (int j = 0; j < NB; ++j) *(v4f *)(B + bq * BSTR + ((tid >> 2) + 64 * j) * 4) = gb[j];
    };

    const int nsteps = p.Kq >> 2;
    gload(0);
    lstore(0);
    __syncthreads();
    for (int step = 0; step < nsteps; ++step) {
        if (step + 1 < nsteps) gload(step + 1);
        const float *A = lds + (step & 1) * STAGE, *B = A + 4 * ASTR;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int q = 2 * h + half;
            v4f af[MT], bf[NT];
#pragma unroll
            for (int i = 0; i < MT; ++i) af[i] = *(const v4f *)(A + q * ASTR + ((wm * MT + i) * 32 + l32) * 4);
#pragma unroll
            for (int j = 0; j < NT; ++j) bf[j] = *(const v4f *)(B + q * BSTR + ((wn * NT + j) * 32 + l32) * 4);
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int i = 0; i < MT; ++i)
#pragma unroll
                    for (int j = 0; j < NT; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i][e], bf[j][e], acc[i][j], 0, 0, 0);
        }
        if (step + 1 < nsteps) lstore((step + 1) & 1);
        __syncthreads();
    }

    // epilogue: with the weight rows in MFMA row order a lane holds 16 consecutive channels of one pixel
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const long P = px0 + (wn * NT + j) * 32 + l32;
        if (P >= p.npix) continue;
#pragma unroll
        for (int i = 0; i < MT; ++i) {
            const int chb = ch0 + (wm * MT + i) * 32 + 16 * half;
            if (chb >= p.Cout_p) continue;                     // Cout_p is a multiple of 16: the run is stored whole or not at all
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int ch = chb + 4 * g;
                const v4f bias = *(const v4f *)(p.bias + ch), scale = *(const v4f *)(p.scale + ch);
                v4f t;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    t[e] = (acc[i][j][4 * g + e] + bias[e]) * scale[e];
                    if (p.relu) t[e] = fmaxf(t[e], 0.0f);
                }
                if (p.res) {
                    const v4f r = *(const v4f *)(p.res + P * p.Cout_p + ch);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        t[e] = p.ma * t[e] + p.mb * r[e];
                        if (p.add_relu) t[e] = fmaxf(t[e], 0.0f);
                    }
                }
                *(v4f *)(p.out + P * p.Cout_p + ch) = t;
            }
        }
    }
}

__global__ __launch_bounds__(256) void fadd_kernel(const FAddParams p) {
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < p.n4; i += (long)gridDim.x * 256) {
        const v4f a = ((const v4f *)p.a)[i], b = ((const v4f *)p.b)[i];
        v4f o;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            o[e] = p.ma * a[e] + p.mb * b[e];
            if (p.relu) o[e] = fmaxf(o[e], 0.0f);
        }
        ((v4f *)p.out)[i] = o;
    }
}

// One thread per (copy, output pixel, 4 channels): max over the in-bounds taps.
__global__ __launch_bounds__(256) void fmaxpool_kernel(const FPoolParams p) {
    const int c4n = p.Cp >> 2;
    const long total = (long)p.B * p.Ho * p.Wo * c4n;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        const int c4 = (int)(i % c4n);
        long r = i / c4n;
        const int ox = (int)(r % p.Wo);
        r /= p.Wo;
        const int oy = (int)(r % p.Ho), b = (int)(r / p.Ho);
        v4f best = {0.f, 0.f, 0.f, 0.f};
        bool any = false;
        for (int ky = 0; ky < p.k; ++ky) {
            const int iy = oy * p.stride - p.pad + ky;
            if (iy < 0 || iy >= p.H) continue;
            for (int kx = 0; kx < p.k; ++kx) {
                const int ix = ox * p.stride - p.pad + kx;
                if (ix < 0 || ix >= p.W) continue;
                const v4f q = *(const v4f *)(p.in + (((long)b * p.H + iy) * p.W + ix) * p.Cp + 4 * c4);
                if (!any) best = q;
                else
#pragma unroll
                    for (int e = 0; e < 4; ++e) best[e] = fmaxf(best[e], q[e]);
                any = true;
            }
        }
        *(v4f *)(p.out + (((long)b * p.Ho + oy) * p.Wo + ox) * p.Cp + 4 * c4) = best;
    }
}

// One thread per (copy, 4 channels): scale * sum over the H x W positions.
__global__ __launch_bounds__(256) void fgap_kernel(const FGapParams p) {
    const int c4n = p.Cp >> 2;
    const long total = (long)p.B * c4n;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        const int c4 = (int)(i % c4n);
        const long b = i / c4n;
        v4f s = {0.f, 0.f, 0.f, 0.f};
        const float *src = p.in + b * p.HW * p.Cp + 4 * c4;
        for (int j = 0; j < p.HW; ++j) {
            const v4f q = *(const v4f *)(src + (long)j * p.Cp);
#pragma unroll
            for (int e = 0; e < 4; ++e) s[e] += q[e];
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) s[e] *= p.scale;
        *(v4f *)(p.out + b * p.Cp + 4 * c4) = s;
    }
}

// One wave per copy: the class with the largest logit (lowest index among equals) and its vote.
__global__ __launch_bounds__(64) void fvote_kernel(const FVoteParams p) {
    const int b = blockIdx.x, lane = threadIdx.x;
    const float *lg = p.logits + (long)b * p.stride;
    float best = 0.f;
    int arg = 0x7FFFFFFF;
    for (int c = lane; c < p.classes; c += 64) {
        const float v = lg[c];
        if (arg == 0x7FFFFFFF || v > best) { best = v; arg = c; }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float ob = __shfl_xor(best, off);
        const int oa = __shfl_xor(arg, off);
        if (oa != 0x7FFFFFFF && (arg == 0x7FFFFFFF || ob > best || (ob == best && oa < arg))) { best = ob; arg = oa; }
    }
    if (lane == 0) {
        if (p.argmax) p.argmax[b] = arg;
        if (p.counts) atomicAdd(p.counts + arg, 1u);
    }
}

long grid_for(long items, long cap = 256L * 32) {
    long blocks = (items + 255) / 256;
    return blocks < 1 ? 1 : (blocks > cap ? cap : blocks);
}

}  // namespace

hipError_t launch_float_noise(const FloatNoiseParams &p, hipStream_t st) {
    if (p.count == 0) return hipSuccess;
    if (p.C < 1 || p.C > 3 || (p.W & 3) != 0 || !(p.sigma >= 0.0f)) return hipErrorInvalidValue;
    const long total = (long)p.H * (p.W >> 2) * p.count;
    set_kernel_name(p.quant ? "float_noise_kernel (rounded)" : "float_noise_kernel");
    hipLaunchKernelGGL(float_noise_kernel, dim3((unsigned)grid_for(total)), dim3(256), 0, st, p);
    return hipGetLastError();
}

int fconv_tile_m(int cout_p) { return cout_p <= 32 ? 32 : (cout_p <= 64 ? 64 : 128); }

hipError_t launch_fconv(const FConvParams &p, hipStream_t st) {
    if (p.npix <= 0) return hipSuccess;
    const int bm = fconv_tile_m(p.Cout_p);
    if (p.Kq <= 0 || (p.Kq & 3) || p.Cout_pp % bm != 0 || p.Cout_p > p.Cout_pp || (p.Cout_p & 15) || (p.Cin_p & 3))
        return hipErrorInvalidValue;
    const long ptiles = ((long)p.npix + 127) / 128, blocks = ptiles * (p.Cout_pp / bm);
    if (blocks > 0x7FFFFFFFL) return hipErrorInvalidValue;
    if (bm == 128) {
        set_kernel_name("fconv_kernel<128 x 128>");
        hipLaunchKernelGGL((fconv_kernel<2, 2, 2, 2>), dim3((unsigned)blocks), dim3(256), 0, st, p);
    } else if (bm == 64) {
        set_kernel_name("fconv_kernel<64 x 128>");
        hipLaunchKernelGGL((fconv_kernel<2, 1, 1, 4>), dim3((unsigned)blocks), dim3(256), 0, st, p);
    } else {
        set_kernel_name("fconv_kernel<32 x 128>");
        hipLaunchKernelGGL((fconv_kernel<1, 1, 1, 4>), dim3((unsigned)blocks), dim3(256), 0, st, p);
    }
    return hipGetLastError();
}

hipError_t launch_fadd(const FAddParams &p, hipStream_t st) {
    if (p.n4 <= 0) return hipSuccess;
    set_kernel_name("fadd_kernel");
    hipLaunchKernelGGL(fadd_kernel, dim3((unsigned)grid_for(p.n4)), dim3(256), 0, st, p);
    return hipGetLastError();
}

hipError_t launch_fmaxpool(const FPoolParams &p, hipStream_t st) {
    if (p.B <= 0) return hipSuccess;
    if (p.Cp & 3) return hipErrorInvalidValue;
    set_kernel_name("fmaxpool_kernel");
    hipLaunchKernelGGL(fmaxpool_kernel, dim3((unsigned)grid_for((long)p.B * p.Ho * p.Wo * (p.Cp >> 2))), dim3(256), 0, st, p);
    return hipGetLastError();
}

hipError_t launch_fgap(const FGapParams &p, hipStream_t st) {
    if (p.B <= 0) return hipSuccess;
    if (p.Cp & 3) return hipErrorInvalidValue;
    set_kernel_name("fgap_kernel");
    hipLaunchKernelGGL(fgap_kernel, dim3((unsigned)grid_for((long)p.B * (p.Cp >> 2))), dim3(256), 0, st, p);
    return hipGetLastError();
}

hipError_t launch_fvote(const FVoteParams &p, hipStream_t st) {
    if (p.B <= 0) return hipSuccess;
    if (p.classes < 1) return hipErrorInvalidValue;
    set_kernel_name("fvote_kernel");
    hipLaunchKernelGGL(fvote_kernel, dim3((unsigned)p.B), dim3(64), 0, st, p);
    return hipGetLastError();
}

}  // namespace isr
