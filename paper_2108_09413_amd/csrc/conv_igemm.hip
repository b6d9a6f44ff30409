// int8 implicit-GEMM convolution on CDNA4 MFMA with the requantisation epilogue.
//
// GEMM view of one convolution layer over a chunk of noisy copies:
//   rows    M = output channels            (A operand: weights, [Mp][Kp], K contiguous)
//   columns N = B*Ho*Wo output pixels      (B operand: activations gathered on the fly)
//   depth   K = taps x input channels      (channel-contiguous NHWC, so a 16-byte
//                                           K chunk is 16 channels of one tap)
// acc (int32) starts at bias - z_in * sum(w) so that the kernel can multiply raw
// int8 activations; out-of-image taps are filled with z_in and so contribute 0.
// Epilogue: q = clamp(z_out + RHA(acc * M0, 31 + shift), relu ? z_out : -128, 127),
// one rounding, half away from zero, written as int8 NHWC.
//
// Two kernels share the arithmetic:
//  * conv_dma_kernel (layers with at least 64 output channels and the single-multiply
//    epilogue): a workgroup of BM/64 x BN/64 waves, each wave a 64 x 64 output block of
//    2 x 2 v_mfma_i32_32x32x32_i8 tiles.  K is consumed in steps of KB bytes; the
//    operand tiles of a step go from global memory straight into LDS
//    (global_load_lds_dwordx4, no staging registers) NST steps deep, tracked by hand
//    with s_waitcnt vmcnt and one s_barrier per step.  Large tiles cut the bytes that
//    cross the L1 per multiply, which is what bounds the K loop on this chip.
//  * conv_igemm_kernel (few output channels, the RGB stem, the two-multiply epilogue):
//    256 threads, operands staged through registers into LDS.  KB = 64: two LDS
//    buffers, one barrier per step.  KB = 128: one buffer, two barriers per step.
//    MT = 32 uses v_mfma_i32_32x32x32_i8, MT = 16 uses v_mfma_i32_16x16x64_i8.
#include <cstdlib>

#include "conv_dma.h"

namespace isr {

template <int MT, int BM, int BN, int WGM, bool FAST, int MINW, bool FUSE, int KB, bool TF>
__global__ __launch_bounds__(256, MINW) void conv_igemm_kernel(const ConvParams p) {
    constexpr int WGN = 4 / WGM;
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int FM = WM / MT, FN = WN / MT;
    constexpr int CPR = KB / 16;            // 16-byte chunks per tile row
    constexpr int RPP = 256 / CPR;          // rows covered by one pass of the 256 threads
    constexpr int NBUF = KB == 64 ? 2 : 1;
    constexpr int NA = (BM * CPR + 255) / 256, NB = BN * CPR / 256;
    constexpr int ACC = MT == 32 ? 16 : 4;
    static_assert(WM % MT == 0 && WN % MT == 0 && BN % 64 == 0 && (KB == 64 || KB == 128), "tile shape");

    __shared__ __attribute__((aligned(16))) int8_t As[NBUF][BM * KB];
    __shared__ __attribute__((aligned(16))) int8_t Bs[NBUF][BN * KB];
    __shared__ uint32_t ktg_s[512];   // per 16-byte K chunk: ky | kx << 8, 0xFFFFFFFF = padding chunk
    __shared__ int kto_s[512];        // per 16-byte K chunk: byte offset of its tap and channel from the window origin
    __shared__ __attribute__((aligned(16))) int prm_s[4][BM];   // bias, M0, chi, shift-1 of this M tile

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WGM, wn = wave / WGM;
    // Workgroup ids are dealt round-robin to the 8 XCDs; give each XCD a contiguous
    // range of logical tiles, M tile fastest, so that the workgroups sharing an
    // activation tile run on the same XCD (same L2) close together in time.
    const int nblk = gridDim.x, mt = (p.Cout_p + BM - 1) / BM;
    const int xcd = blockIdx.x & 7, per = nblk >> 3, extra = nblk & 7;
    const int logical = xcd * per + (xcd < extra ? xcd : extra) + (blockIdx.x >> 3);
    const int m0 = (logical % mt) * BM;
    const long n0 = (long)(logical / mt) * BN;
    const int nk = p.Kp / KB;
    const int col = tid % CPR, row0 = tid / CPR;
    const bool flat = p.ktab == nullptr;   // 1x1, stride 1, no padding: pixel n reads input pixel n

    if (!flat)
        for (int i = tid; i < nk * CPR; i += 256) { ktg_s[i] = p.ktab[i]; kto_s[i] = p.ktoff[i]; }
    for (int i = tid; i < BM; i += 256) {
        prm_s[0][i] = p.bias[m0 + i];
        if constexpr (FAST) { prm_s[1][i] = p.m0s[m0 + i]; prm_s[2][i] = p.chi[m0 + i]; prm_s[3][i] = p.shm1[m0 + i]; }
    }

    // per-thread gather state for its NB activation rows: byte offset of the window
    // origin (may be negative inside the padding; a chunk's tensor is below 2 GiB)
    int pixoff[NB];
    int iy0[NB], ix0[NB];
    bool rvalid[NB];
    const int HoWo = p.Ho * p.Wo;
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        long n = n0 + row0 + RPP * j;
        rvalid[j] = n < p.npix;
        if (flat) {
            // rows past the end re-read the last pixel; their results are never stored
            pixoff[j] = (int)((rvalid[j] ? n : (long)p.npix - 1) * p.Cin_p) + col * 16;
            iy0[j] = ix0[j] = 0;
        } else {
            int nn = rvalid[j] ? (int)n : 0;
            int b = nn / HoWo;
            int rem = nn - b * HoWo;
            int oy = rem / p.Wo, ox = rem - oy * p.Wo;
            iy0[j] = oy * p.stride - p.pad;
            ix0[j] = ox * p.stride - p.pad;
            pixoff[j] = ((b * p.H + iy0[j]) * p.W + ix0[j]) * p.Cin_p;
        }
    }
    const uint32_t zb = (uint32_t)(p.zp_in & 0xFF) * 0x01010101u;
    const v4i zfill = {(int)zb, (int)zb, (int)zb, (int)zb};
    const int8_t *wrow[NA];
#pragma unroll
    for (int j = 0; j < NA; ++j) wrow[j] = p.w + (long)(m0 + row0 + RPP * j) * p.Kp + col * 16;

    v4i ra[NA], rb[NB];   // the next K step, in flight while the current one is computed

    auto load_global = [&](int ks) {
#pragma unroll
        for (int j = 0; j < NA; ++j)
            if (BM * CPR >= 256 || row0 + RPP * j < BM) ra[j] = *(const v4i *)(wrow[j] + (long)ks * KB);
        if (flat) {
#pragma unroll
            for (int j = 0; j < NB; ++j) rb[j] = *(const v4i *)(p.in + (uint32_t)(pixoff[j] + ks * KB));
        } else if (!p.c4) {
            const uint32_t g = ktg_s[ks * CPR + col];
            const int toff = kto_s[ks * CPR + col];
            const int ky = g & 0xFF, kx = (g >> 8) & 0xFF;
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                int iy = iy0[j] + ky, ix = ix0[j] + kx;
                bool ok = rvalid[j] && g != 0xFFFFFFFFu && (unsigned)iy < (unsigned)p.H && (unsigned)ix < (unsigned)p.W;
                uint32_t off = ok ? (uint32_t)(pixoff[j] + toff) : 0u;   // offset 0 is always readable
                v4i v = *(const v4i *)(p.in + off);
                rb[j] = ok ? v : zfill;
            }
        } else {
            const uint32_t g = ktg_s[ks * CPR + col];
            const int toff = kto_s[ks * CPR + col];
            const int ky = g & 0xFF, kx = (g >> 8) & 0xFF;
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                int iy = iy0[j] + ky;
                bool rowok = rvalid[j] && g != 0xFFFFFFFFu && (unsigned)iy < (unsigned)p.H;
                v4i v;
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    int ix = ix0[j] + kx + t;
                    bool ok = rowok && (unsigned)ix < (unsigned)p.W;
                    uint32_t off = ok ? (uint32_t)(pixoff[j] + toff + 4 * t) : 0u;
                    int w = *(const int *)(p.in + off);
                    v[t] = ok ? w : (int)zb;
                }
                rb[j] = v;
            }
        }
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int j = 0; j < NA; ++j) {
            int r = row0 + RPP * j;
            if (BM * CPR >= 256 || r < BM) *(v4i *)(&As[buf][r * KB + ((col ^ swz<CPR>(r)) << 4)]) = ra[j];
        }
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            int r = row0 + RPP * j;
            *(v4i *)(&Bs[buf][r * KB + ((col ^ swz<CPR>(r)) << 4)]) = rb[j];
        }
    };

    typedef int acc_t __attribute__((ext_vector_type(ACC)));
    acc_t acc[FM][FN];
    // first channel (within the M tile) held by this lane for fragment fm
    auto lane_oc = [&](int fm) { return wm * WM + fm * MT + (MT == 32 ? 16 * (lane >> 5) : 4 * (lane >> 4)); };

    // residual operand of a fused add: fetched up front, consumed in the epilogue
    int rres[FUSE ? FM : 1][FUSE ? FN : 1][ACC / 4];
    if constexpr (FUSE) {
#pragma unroll
        for (int fm = 0; fm < FM; ++fm)
#pragma unroll
            for (int fn = 0; fn < FN; ++fn) {
                long n = n0 + wn * WN + fn * MT + (lane & (MT - 1));
                if (n >= p.npix) n = p.npix - 1;
                int occ = m0 + lane_oc(fm);
                if (occ >= p.Cout_p) occ = 0;
                const int8_t *src = p.res + n * p.Cout_p + occ;
                if constexpr (MT == 32) {
                    v4i rv = *(const v4i *)src;
#pragma unroll
                    for (int d = 0; d < 4; ++d) rres[fm][fn][d] = rv[d];
                } else {
                    rres[fm][fn][0] = *(const int *)src;
                }
            }
    }

    __syncthreads();   // ktab_s, prm_s visible
    // accumulators start at the folded bias
#pragma unroll
    for (int fm = 0; fm < FM; ++fm) {
        acc_t init;
#pragma unroll
        for (int i = 0; i < ACC; ++i) init[i] = prm_s[0][lane_oc(fm) + i];
#pragma unroll
        for (int fn = 0; fn < FN; ++fn) acc[fm][fn] = init;
    }
    load_global(0);
    if constexpr (NBUF == 2) {
        store_lds(0);
        __syncthreads();
    }

    for (int ks = 0; ks < nk; ++ks) {
        const int buf = NBUF == 2 ? (ks & 1) : 0;
        if constexpr (NBUF == 1) {
            if (ks) __syncthreads();   // every wave is done reading the previous step
            store_lds(0);
            __syncthreads();
        }
        if (ks + 1 < nk) load_global(ks + 1);
        if constexpr (MT == 32) {
#pragma unroll
            for (int ksub = 0; ksub < KB / 32; ++ksub) {
                const int c = ksub * 2 + (lane >> 5);
                v4i fa[FM], fb[FN];
#pragma unroll
                for (int fm = 0; fm < FM; ++fm) {
                    int r = wm * WM + fm * 32 + (lane & 31);
                    fa[fm] = *(const v4i *)(&As[buf][r * KB + ((c ^ swz<CPR>(r)) << 4)]);
                }
#pragma unroll
                for (int fn = 0; fn < FN; ++fn) {
                    int r = wn * WN + fn * 32 + (lane & 31);
                    fb[fn] = *(const v4i *)(&Bs[buf][r * KB + ((c ^ swz<CPR>(r)) << 4)]);
                }
#pragma unroll
                for (int fm = 0; fm < FM; ++fm)
#pragma unroll
                    for (int fn = 0; fn < FN; ++fn)
                        acc[fm][fn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[fm], fb[fn], acc[fm][fn], 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int ksub = 0; ksub < KB / 64; ++ksub) {
                const int c = ksub * 4 + (lane >> 4);
                v4i fa[FM], fb[FN];
#pragma unroll
                for (int fm = 0; fm < FM; ++fm) {
                    int r = wm * WM + fm * 16 + (lane & 15);
                    fa[fm] = *(const v4i *)(&As[buf][r * KB + ((c ^ swz<CPR>(r)) << 4)]);
                }
#pragma unroll
                for (int fn = 0; fn < FN; ++fn) {
                    int r = wn * WN + fn * 16 + (lane & 15);
                    fb[fn] = *(const v4i *)(&Bs[buf][r * KB + ((c ^ swz<CPR>(r)) << 4)]);
                }
#pragma unroll
                for (int fm = 0; fm < FM; ++fm)
#pragma unroll
                    for (int fn = 0; fn < FN; ++fn)
                        acc[fm][fn] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa[fm], fb[fn], acc[fm][fn], 0, 0, 0);
            }
        }
        if constexpr (NBUF == 2) {
            if (ks + 1 < nk) store_lds(buf ^ 1);
            __syncthreads();
        }
    }

    // epilogue: requantise, clamp, pack, store (NHWC)
    const int lo = p.relu ? p.zp_out : -128;
#pragma unroll
    for (int fm = 0; fm < FM; ++fm) {
        const int oc = m0 + wm * WM + fm * MT + (MT == 32 ? 16 * (lane >> 5) : 4 * (lane >> 4));
        if (oc >= p.Cout_p) continue;
        if constexpr (FAST) {
            int mm[ACC], ch[ACC], ss[ACC];
#pragma unroll
            for (int i = 0; i < ACC; ++i) {
                mm[i] = prm_s[1][oc - m0 + i]; ch[i] = prm_s[2][oc - m0 + i]; ss[i] = prm_s[3][oc - m0 + i];
            }
            {
#pragma unroll
                for (int fn = 0; fn < FN; ++fn) {
                    long n = n0 + wn * WN + fn * MT + (lane & (MT - 1));
                    if (n >= p.npix) continue;
                    int q[ACC];
#pragma unroll
                    for (int i = 0; i < ACC; ++i) q[i] = clamp3(requant_q<TF>(acc[fm][fn][i], mm[i], ch[i], ss[i]), lo, 127);
                    if constexpr (FUSE) {
                        // second requantisation: the residual add on the int8 result
#pragma unroll
                        for (int i = 0; i < ACC; ++i) {
                            int r8 = (int)(int8_t)((uint32_t)rres[fm][fn][i >> 2] >> (8 * (i & 3)));
                            q[i] = fused_add<TF>(q[i], r8, p);
                        }
                    }
                    int8_t *dst = p.out + n * p.Cout_p + oc;
                    if constexpr (MT == 32) {
                        v4i v = {(int)pack4(q[0], q[1], q[2], q[3]), (int)pack4(q[4], q[5], q[6], q[7]),
                                 (int)pack4(q[8], q[9], q[10], q[11]), (int)pack4(q[12], q[13], q[14], q[15])};
                        *(v4i *)dst = v;
                    } else {
                        *(uint32_t *)dst = pack4(q[0], q[1], q[2], q[3]);
                    }
                }
            }
        } else {
            uint32_t mm[ACC], rl[ACC], rh[ACC], ss[ACC];
#pragma unroll
            for (int i = 0; i < ACC; ++i) {
                mm[i] = p.m0x2[oc + i]; rl[i] = p.rnd_lo[oc + i]; rh[i] = p.rnd_hi[oc + i]; ss[i] = p.shift[oc + i];
            }
#pragma unroll
            for (int fn = 0; fn < FN; ++fn) {
                long n = n0 + wn * WN + fn * MT + (lane & (MT - 1));
                if (n >= p.npix) continue;
                int q[ACC];
#pragma unroll
                for (int i = 0; i < ACC; ++i) {
                    int r = p.zp_out + requant(acc[fm][fn][i], mm[i], rl[i], rh[i], ss[i]);
                    q[i] = r < lo ? lo : (r > 127 ? 127 : r);
                }
                int8_t *dst = p.out + n * p.Cout_p + oc;
                if constexpr (MT == 32) {
                    v4i v = {(int)pack4(q[0], q[1], q[2], q[3]), (int)pack4(q[4], q[5], q[6], q[7]),
                             (int)pack4(q[8], q[9], q[10], q[11]), (int)pack4(q[12], q[13], q[14], q[15])};
                    *(v4i *)dst = v;
                } else {
                    *(uint32_t *)dst = pack4(q[0], q[1], q[2], q[3]);
                }
            }
        }
    }
}


int conv_tile_m(int cout_p) { return cout_p <= 16 ? 16 : (cout_p <= 32 ? 32 : (cout_p <= 64 ? 64 : 128)); }

template <int MT, int BM, int BN, int WGM, int MINW, int MINW_FUSED>
static hipError_t launch_staged(const ConvParams &p, hipStream_t st) {
    dim3 grid((unsigned)(((p.npix + BN - 1) / BN) * ((p.Cout_p + BM - 1) / BM)));
    if (p.kb != 64 || (p.fuse_add && !p.fast_requant) || p.fuse_add == 2) return hipErrorInvalidValue;
    static const std::string name = "conv_igemm_kernel<" + std::to_string(MT) + ", " + std::to_string(BM) + ", " + std::to_string(BN) + ">";
    set_kernel_name(name.c_str());
    // TF: the rounding of this layer (and of its fused add) never meets an exact half -> shorter epilogue
    const bool tf = p.tie_free && (!p.fuse_add || p.add_tie_free);
    if (p.fuse_add && tf)
        hipLaunchKernelGGL((conv_igemm_kernel<MT, BM, BN, WGM, true, MINW_FUSED, true, 64, true>), grid, dim3(256), 0, st, p);
    else if (p.fuse_add)
        hipLaunchKernelGGL((conv_igemm_kernel<MT, BM, BN, WGM, true, MINW_FUSED, true, 64, false>), grid, dim3(256), 0, st, p);
    else if (p.fast_requant && tf)
        hipLaunchKernelGGL((conv_igemm_kernel<MT, BM, BN, WGM, true, MINW, false, 64, true>), grid, dim3(256), 0, st, p);
    else if (p.fast_requant)
        hipLaunchKernelGGL((conv_igemm_kernel<MT, BM, BN, WGM, true, MINW, false, 64, false>), grid, dim3(256), 0, st, p);
    else
        hipLaunchKernelGGL((conv_igemm_kernel<MT, BM, BN, WGM, false, 2, false, 64, false>), grid, dim3(256), 0, st, p);
    return hipGetLastError();
}

template <int BM, int BN, int KB, int NST, int MINB>
static hipError_t launch_dma(const ConvParams &p, hipStream_t st) {
    constexpr int NT = (BM / 64) * (BN / 64) * 64;
    dim3 grid((unsigned)(((p.npix + BN - 1) / BN) * ((p.Cout_p + BM - 1) / BM)));
    set_kernel_name(conv_dma_name<BM, BN, KB, NST, 0, MINB, 64, 64>());
    if (p.tie_free)
        hipLaunchKernelGGL((conv_dma_kernel<BM, BN, KB, NST, 0, MINB, true>), grid, dim3(NT), 0, st, p);
    else
        hipLaunchKernelGGL((conv_dma_kernel<BM, BN, KB, NST, 0, MINB, false>), grid, dim3(NT), 0, st, p);
    return hipGetLastError();
}

// With a fused residual add: 64-byte K steps in two buffers (any Kp is a multiple of 64),
// the second of which also receives the residual tile; small tiles, 3-4 workgroups per CU.
template <int BM, int BN, int MINB, int MINB2>
static hipError_t launch_dma_fused(const ConvParams &p, hipStream_t st) {
    constexpr int NT = (BM / 64) * (BN / 64) * 64;
    dim3 grid((unsigned)(((p.npix + BN - 1) / BN) * ((p.Cout_p + BM - 1) / BM)));
    if (p.fuse_add == 2) {
        if (!p.in2 || !p.w2 || p.Cin2_p < 64 || p.Cin2_p % 64 != 0) return hipErrorInvalidValue;
        set_kernel_name(conv_dma_name<BM, BN, 64, 2, 2, MINB2, 64, 64>());
        // the tie-free forms are chosen separately for the two convolutions and for the add: an add that can
        // meet an exact half costs two more instructions per output, a convolution that can costs a 64-bit multiply
        if (p.tie_free && p.tie_free2 && p.add_tie_free)
            hipLaunchKernelGGL((conv_dma_kernel<BM, BN, 64, 2, 2, MINB2, true>), grid, dim3(NT), 0, st, p);
        else if (p.tie_free && p.tie_free2)
            hipLaunchKernelGGL((conv_dma_kernel<BM, BN, 64, 2, 2, MINB2, true, 64, 64, false>), grid, dim3(NT), 0, st, p);
        else
            hipLaunchKernelGGL((conv_dma_kernel<BM, BN, 64, 2, 2, MINB2, false>), grid, dim3(NT), 0, st, p);
    } else if (BM == 128 && p.Kp == 128) {
        // two K steps: with a third buffer the residual tile is fetched at the start instead of
        // during the last step, which measured faster than the fourth workgroup per CU
        if constexpr (BM == 128) {
            set_kernel_name(conv_dma_name<BM, BN, 64, 3, 1, 3, 64, 64>());
            if (p.tie_free && p.add_tie_free)
                hipLaunchKernelGGL((conv_dma_kernel<BM, BN, 64, 3, 1, 3, true>), grid, dim3(NT), 0, st, p);
            else if (p.tie_free)
                hipLaunchKernelGGL((conv_dma_kernel<BM, BN, 64, 3, 1, 3, true, 64, 64, false>), grid, dim3(NT), 0, st, p);
            else
                hipLaunchKernelGGL((conv_dma_kernel<BM, BN, 64, 3, 1, 3, false>), grid, dim3(NT), 0, st, p);
        }
    } else {
        set_kernel_name(conv_dma_name<BM, BN, 64, 2, 1, MINB, 64, 64>());
        if (p.tie_free && p.add_tie_free)
            hipLaunchKernelGGL((conv_dma_kernel<BM, BN, 64, 2, 1, MINB, true>), grid, dim3(NT), 0, st, p);
        else if (p.tie_free)
            hipLaunchKernelGGL((conv_dma_kernel<BM, BN, 64, 2, 1, MINB, true, 64, 64, false>), grid, dim3(NT), 0, st, p);
        else
            hipLaunchKernelGGL((conv_dma_kernel<BM, BN, 64, 2, 1, MINB, false>), grid, dim3(NT), 0, st, p);
    }
    return hipGetLastError();
}

// The direct-to-LDS kernel serves layers with at least 64 stored output channels,
// the single-multiply epilogue and 16-channel-aligned input (not the RGB stem).
static bool dma_path(int cout_p, int fast_requant, int c4) { return fast_requant && !c4 && cout_p >= 64; }

// K bytes per step for a layer whose unpadded depth is `kreal` bytes (cin_p == 0 marks
// the RGB stem): 128 for deep layers of the direct-to-LDS kernel with at least 256
// output channels, where two 128-byte steps in flight measured faster than three
// 64-byte ones and no extra K padding is needed; else 64.
int conv_k_step(int kreal, int cin_p, int cout_p, int fast_requant) {
    return (dma_path(cout_p, fast_requant, cin_p == 0) && cout_p >= 256 && kreal % 128 == 0 && kreal >= 1024) ? 128 : 64;
}

// Output tile of the direct-to-LDS kernel for this launch.  Larger tiles move fewer
// bytes per multiply, so their K loop runs faster, but a layer with few tiles then
// leaves CUs idle or pays for a mostly empty last round; the epilogue of a shallow
// (small K) layer hides better behind several small workgroups.
// W: four waves of 128 x 128 (conv_deep.hip); H: eight of 128 x 64; P: 3x3 stride-1 layers with a tile's pixel rows
// staged once per channel slice (conv_patch.hip)
enum DmaTile { T64x256, T128x128, T128x256, T256x128, T256x256, T256x256W, T256x256H, T256x256P };

static DmaTile pick_tile(const ConvParams &p) {
    const int forced = p.force_tile;
    if (p.Cout_p <= 64) return T64x256;
    if (forced >= T128x128 && forced <= T256x256H && !(p.Cout_p <= 128 && forced >= T256x128))
        return (DmaTile)forced;
    if (forced == T256x256P && conv_patch_supported(p)) return T256x256P;
    static const char *deep = std::getenv("ISR_DEEP_TILE");   // A/B switch for tuning: W, H, N (no conv_patch.hip) or unset
    // 3x3 layers: the staged-rows kernel moves about 40 % fewer bytes into LDS per multiply (measured 7-10 % faster on
    // the 14 x 14 and 28 x 28 layers of a ResNet-50); its tile is 256 pixels wide, so it wants launches that give
    // at least half of the CUs a tile
    if (!(deep && deep[0] == 'N') && conv_patch_supported(p) &&
        ((long)(p.npix + 255) / 256) * ((p.Cout_p + 255) / 256) >= 128)
        return T256x256P;
    if (p.Cout_p > 128 && p.Kp < 1024) return T128x128;
    // cost of a candidate: workgroups per CU (rounded up: the last round costs a full
    // one) x tile area / relative K-loop throughput of the tile, as measured
    struct Cand { DmaTile t; int bm, bn; double rate64, rate128; };
    static const Cand cands[] = {{T128x128, 128, 128, 1.00, 1.00}, {T128x256, 128, 256, 1.12, 1.15},
                                 {T256x128, 256, 128, 1.12, 1.15}, {T256x256, 256, 256, 1.20, 1.35}};
    constexpr long CUS = 256;
    DmaTile best = T128x128;
    double best_cost = 0;
    for (const Cand &c : cands) {
        if (c.bm > 128 && p.Cout_p <= 128) continue;
        const long wgs = ((long)(p.npix + c.bn - 1) / c.bn) * ((p.Cout_p + c.bm - 1) / c.bm);
        const double cost = (double)((wgs + CUS - 1) / CUS) * c.bm * c.bn / (p.kb == 128 ? c.rate128 : c.rate64);
        if (best_cost == 0 || cost < best_cost) { best_cost = cost; best = c.t; }
    }
    // deep layers on whole 256 x 256 tiles: four waves of 128 x 128 read half the LDS bytes per multiply
    if (best == T256x256 && p.kb == 128 && deep) best = deep[0] == 'W' ? T256x256W : deep[0] == 'H' ? T256x256H : best;
    return best;
}

hipError_t launch_conv(const ConvParams &p, hipStream_t st) {
    if (p.npix <= 0) return hipSuccess;
    if ((p.kb != 64 && p.kb != 128) || p.Kp % p.kb != 0 || p.Kp > 8192 || p.Cout_p % 16 != 0 || p.Mp % 128 != 0 ||
        p.Mp < p.Cout_p)
        return hipErrorInvalidValue;
    if (dma_path(p.Cout_p, p.fast_requant, p.c4)) {
        if (!p.zpad) return hipErrorInvalidValue;
        const bool k128 = p.kb == 128;
        if (p.fuse_add) return p.Cout_p <= 64 ? launch_dma_fused<64, 256, 3, 3>(p, st) : launch_dma_fused<128, 128, 4, 3>(p, st);
        switch (pick_tile(p)) {
        case T64x256:
            // two steps in flight and three workgroups per CU measured faster than three and two
            if (k128) return hipErrorInvalidValue;
            return launch_dma<64, 256, 64, 2, 3>(p, st);
        case T128x128:
            // shallow layers are epilogue-bound: two steps in flight suffice and a fourth
            // workgroup per CU hides more of the epilogue's memory latency
            if (!p.fuse_add && p.Kp < 1024 && !k128) return launch_dma<128, 128, 64, 2, 4>(p, st);
            return k128 ? launch_dma<128, 128, 128, 2, 2>(p, st) : launch_dma<128, 128, 64, 3, 3>(p, st);
        case T128x256:
            return k128 ? launch_dma<128, 256, 128, 2, 1>(p, st) : launch_dma<128, 256, 64, 3, 2>(p, st);
        case T256x128:
            return k128 ? launch_dma<256, 128, 128, 2, 1>(p, st) : launch_dma<256, 128, 64, 3, 2>(p, st);
        case T256x256: return k128 ? launch_dma<256, 256, 128, 2, 1>(p, st) : launch_dma<256, 256, 64, 3, 1>(p, st);
        case T256x256W: return launch_conv_deep(p, st);
        case T256x256P: return launch_conv_patch(p, st);
        case T256x256H: {
            const dim3 grid((unsigned)(((p.npix + 255) / 256) * ((p.Cout_p + 255) / 256)));
            set_kernel_name(k128 ? conv_dma_name<256, 256, 128, 2, 0, 1, 128, 64>() : conv_dma_name<256, 256, 64, 3, 0, 1, 128, 64>());
            if (k128) {
                if (p.tie_free) hipLaunchKernelGGL((conv_dma_kernel<256, 256, 128, 2, 0, 1, true, 128, 64>), grid, dim3(512), 0, st, p);
                else hipLaunchKernelGGL((conv_dma_kernel<256, 256, 128, 2, 0, 1, false, 128, 64>), grid, dim3(512), 0, st, p);
            } else {
                if (p.tie_free) hipLaunchKernelGGL((conv_dma_kernel<256, 256, 64, 3, 0, 1, true, 128, 64>), grid, dim3(512), 0, st, p);
                else hipLaunchKernelGGL((conv_dma_kernel<256, 256, 64, 3, 0, 1, false, 128, 64>), grid, dim3(512), 0, st, p);
            }
            return hipGetLastError();
        }
        }
        return hipErrorInvalidValue;
    }
    switch (conv_tile_m(p.Cout_p)) {
    case 16: return launch_staged<16, 16, 256, 1, 4, 4>(p, st);
    case 32: return launch_staged<32, 32, 256, 1, 3, 3>(p, st);
    case 64: return launch_staged<32, 64, 256, 1, 3, 3>(p, st);
    default: return launch_staged<32, 128, 128, 2, 4, 3>(p, st);
    }
}

}  // namespace isr
