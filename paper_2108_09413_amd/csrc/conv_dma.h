// The direct-to-LDS implicit-GEMM convolution kernel (see conv_igemm.hip for the GEMM view and the
// epilogue arithmetic).  A template in a header because its instances are compiled in two
// translation units with different register policies: wave tiles of 64 x 64 keep their 64
// accumulator registers among the ordinary VGPRs (conv_igemm.hip), wave tiles of 128 x 128 need the
// 256 accumulation registers next to the 256 ordinary ones (conv_deep.hip).
#ifndef ISR_CONV_DMA_H
#define ISR_CONV_DMA_H

#include <string>

#include "conv_device.h"

namespace isr {

// "conv_dma_kernel<BM, BN, KB, stages, fused add, min blocks, wave tile>" of an instance, for the timing report
template <int BM, int BN, int KB, int NST, int FUSE, int MINB, int WTM, int WTN>
inline const char *conv_dma_name() {
    static const std::string s = "conv_dma_kernel<" + std::to_string(BM) + ", " + std::to_string(BN) + ", " + std::to_string(KB) + ", " +
                                 std::to_string(NST) + ", " + std::to_string(FUSE) + ", " + std::to_string(MINB) + ", " +
                                 std::to_string(WTM) + "x" + std::to_string(WTN) + ">";
    return s.c_str();
}

// FUSE: 0 plain, 1 residual add with the residual read from memory, 2 residual add with the
// residual computed here by a second (1x1, stride 1) convolution.
// WTM x WTN: output block of one wave (channels x pixels): 64 x 64 = 2 x 2 MFMA tiles, 128 x 64 = 4 x 2,
// 128 x 128 = 4 x 4.  A larger block reads fewer operand bytes from LDS per multiply.
// TF: the convolutions' requantisations are free of rounding ties (single-multiply form); TFA: so is the fused add.
template <int BM, int BN, int KB, int NST, int FUSE, int MINB, bool TF, int WTM = 64, int WTN = 64, bool TFA = TF>
__global__ __launch_bounds__((BM / WTM) * (BN / WTN) * 64, MINB) void conv_dma_kernel(const ConvParams p) {
    constexpr int MT = 32;
    constexpr int WGM = BM / WTM, WGN = BN / WTN, NT = WGM * WGN * 64;
    constexpr int FM = WTM / 32, FN = WTN / 32;
    constexpr bool PIPELINED = WTM == 128 && WTN == 128;   // one wave per SIMD: the wave hides its own LDS latency
    constexpr int CPR = KB / 16;             // 16-byte chunks per tile row
    constexpr int RPP = NT / CPR;            // rows covered by one pass of all threads
    constexpr int NA = BM / RPP, NB = BN / RPP;
    constexpr int L = NA + NB;               // loads per lane per step
    constexpr int ACC = 16;
    constexpr int STAGE = (BM + BN) * KB;
    constexpr int KS = KB / 32;
    static_assert(BM % WTM == 0 && BN % WTN == 0 && (WTM == 64 || WTM == 128) && (WTN == 64 || WTN == 128) && BM % RPP == 0 && BN % RPP == 0 && RPP % 32 == 0 && NST >= 2 &&
                      NST <= 3 && (KB == 64 || KB == 128),
                  "tile shape");

    __shared__ __attribute__((aligned(16))) int8_t Ls[NST][STAGE];   // per step: A rows, then B rows
    __shared__ uint32_t ktg_s[512];   // per 16-byte K chunk: ky | kx << 8 | channel byte offset << 16; ~0 = padding
    __shared__ __attribute__((aligned(16))) int prm_s[4][BM];   // bias, M0, chi, shift-1 of this M tile
    // A fused residual add fetches the residual tile as whole pixel
    // rows, [pixel][BM channels] with the 16-byte chunks XOR-swizzled per pixel, into the
    // operand buffer that is idle during the last K step.
    constexpr int RCH = BM / 16;                    // chunks per pixel row
    constexpr int RPB = BM >= 256 ? 1 : 256 / BM;   // pixel rows per 256 bytes (one pass over the 64 banks)
    static_assert(FUSE != 1 || (STAGE >= BM * BN && BM * BN / 16 % NT == 0), "residual tile fits a buffer");
    __shared__ __attribute__((aligned(16))) int prm2_s[4][FUSE == 2 ? BM : 1];   // the same for the residual convolution
    auto rswz = [](int pixel) { return (pixel / RPB) & (RCH - 1); };

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WGM, wn = wave / WGM;
    // same XCD-aware tile order as conv_igemm_kernel
    const int nblk = gridDim.x, mt = (p.Cout_p + BM - 1) / BM;
    const int xcd = blockIdx.x & 7, per = nblk >> 3, extra = nblk & 7;
    const int logical = xcd * per + (xcd < extra ? xcd : extra) + (blockIdx.x >> 3);
    const int m0 = (logical % mt) * BM;
    const long n0 = (long)(logical / mt) * BN;
    const int nk = p.Kp / KB;
    const bool flat = p.ktab == nullptr;
    const int col = tid % CPR, row0 = tid / CPR;
    // LDS position (row, col) holds K chunk col ^ swz(row); RPP is a multiple of 32, so
    // the chunk a lane fetches is the same for all of its rows
    const int cl = col ^ swz<CPR>(row0);

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
            pixoff[j] = (int)((rvalid[j] ? n : (long)p.npix - 1) * p.Cin_p) + cl * 16;
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
    // weight rows past Mp (tile taller than the padded matrix) re-read row 0; never stored
    const int8_t *wrow[NA];
#pragma unroll
    for (int j = 0; j < NA; ++j) {
        int r = m0 + row0 + RPP * j;
        wrow[j] = p.w + (long)(r < p.Mp ? r : 0) * p.Kp + cl * 16;
    }

    // Enqueues the loads of K step ks into LDS buffer `buf`: L per lane.  A pass of all
    // threads fills NT * 16 contiguous bytes, a wave 1 KiB of it.  Out-of-image taps read
    // the 16 zero-point bytes at p.zpad, so they contribute 0 like everywhere else.
    auto issue = [&](int ks, int buf) {
        int8_t *sa = &Ls[buf][wave * 1024];
#pragma unroll
        for (int j = 0; j < NA; ++j) ISR_GLOBAL_TO_LDS16(wrow[j] + (long)ks * KB, sa + j * (NT * 16));
        int8_t *sb = sa + BM * KB;
        if (flat) {
#pragma unroll
            for (int j = 0; j < NB; ++j) ISR_GLOBAL_TO_LDS16(p.in + (uint32_t)(pixoff[j] + ks * KB), sb + j * (NT * 16));
        } else {
            const uint32_t g = ktg_s[ks * CPR + cl];
            const int ky = g & 0xFF, kx = (g >> 8) & 0xFF;
            const int toff = (ky * p.W + kx) * p.Cin_p + (int)(g >> 16);
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                int iy = iy0[j] + ky, ix = ix0[j] + kx;
                const bool ok = (int)rvalid[j] & (int)(g != 0xFFFFFFFFu) & (int)((unsigned)iy < (unsigned)p.H) &
                                (int)((unsigned)ix < (unsigned)p.W);
                const int8_t *real = p.in + (uint32_t)(pixoff[j] + toff);
                const int8_t *src = ok ? real : p.zpad;
                ISR_GLOBAL_TO_LDS16(src, sb + j * (NT * 16));
            }
        }
    };

    // the residual convolution's operands: pixel n of the output reads pixel n of in2
    int pixoff2[FUSE == 2 ? NB : 1];
    const int8_t *wrow2[FUSE == 2 ? NA : 1];
    if constexpr (FUSE == 2) {
#pragma unroll
        for (int j = 0; j < NB; ++j) pixoff2[j] = (int)((rvalid[j] ? n0 + row0 + RPP * j : (long)p.npix - 1) * p.Cin2_p) + cl * 16;
#pragma unroll
        for (int j = 0; j < NA; ++j) {
            int r = m0 + row0 + RPP * j;
            wrow2[j] = p.w2 + (long)(r < p.Mp ? r : 0) * p.Cin2_p + cl * 16;
        }
    }
    auto issue2 = [&](int ks, int buf) {
        if constexpr (FUSE == 2) {
            int8_t *sa = &Ls[buf][wave * 1024];
#pragma unroll
            for (int j = 0; j < NA; ++j) ISR_GLOBAL_TO_LDS16(wrow2[j] + (long)ks * KB, sa + j * (NT * 16));
            int8_t *sb = sa + BM * KB;
#pragma unroll
            for (int j = 0; j < NB; ++j) ISR_GLOBAL_TO_LDS16(p.in2 + (uint32_t)(pixoff2[j] + ks * KB), sb + j * (NT * 16));
        }
    };

    typedef int acc_t __attribute__((ext_vector_type(ACC)));
    acc_t acc[FM][FN];
    auto lane_oc = [&](int fm) { return wm * WTM + fm * MT + 16 * (lane >> 5); };

    int res_buf = -1;   // buffer that receives the residual tile
    auto issue_residual = [&](int buf) {
#pragma unroll
        for (int j = 0; j < BM * BN / 16 / NT; ++j) {
            const int c = j * NT + tid, pixel = c / RCH, chunk = (c % RCH) ^ rswz(pixel);
            long n = n0 + pixel;
            if (n >= p.npix) n = p.npix - 1;
            int oc = m0 + chunk * 16;
            if (oc >= p.Cout_p) oc = 0;
            ISR_GLOBAL_TO_LDS16(p.res + n * p.Cout_p + oc, &Ls[buf][(j * NT + wave * 64) * 16]);
        }
    };
    if constexpr (FUSE == 1)
        if (nk < NST) { res_buf = NST - 1; issue_residual(res_buf); }   // the last buffer is never used by a K step

    // The first GEMM's first steps are fetched before the per-channel constants are staged, when
    // their addresses need nothing from LDS (plain 1x1 GEMM; the residual convolution always is one):
    // the two memory latencies then overlap.  Every buffer is free at the start.
    bool prefetched = false;
    if constexpr (FUSE == 2) {
#pragma unroll
        for (int s = 0; s < NST; ++s)
            if (s < p.Cin2_p / KB) issue2(s, s);
        prefetched = true;
    } else if (flat) {
#pragma unroll
        for (int s = 0; s < NST; ++s)
            if (s < nk) issue(s, s);
        prefetched = true;
    }

    if (!flat)
        for (int i = tid; i < nk * CPR; i += NT) {
            const uint32_t g = p.ktab[i];
            const int chan = p.ktoff[i] - (int)((g & 0xFF) * p.W + ((g >> 8) & 0xFF)) * p.Cin_p;
            ktg_s[i] = g == 0xFFFFFFFFu ? g : (g | ((uint32_t)chan << 16));
        }
    for (int i = tid; i < BM; i += NT) {
        const bool in = m0 + i < p.Mp;
        prm_s[0][i] = in ? p.bias[m0 + i] : 0;
        prm_s[1][i] = in ? p.m0s[m0 + i] : 0;
        prm_s[2][i] = in ? p.chi[m0 + i] : 0;
        prm_s[3][i] = in ? p.shm1[m0 + i] : 1;
        if constexpr (FUSE == 2) {
            prm2_s[0][i] = in ? p.bias2[m0 + i] : 0;
            prm2_s[1][i] = in ? p.m0s2[m0 + i] : 0;
            prm2_s[2][i] = in ? p.chi2[m0 + i] : 0;
            prm2_s[3][i] = in ? p.shm12[m0 + i] : 1;
        }
    }

    __syncthreads();   // ktg_s, prm_s visible
    // per-lane fragment offsets inside a step's buffer
    int aoff[KS][FM], boff[KS][FN];
#pragma unroll
    for (int ksub = 0; ksub < KS; ++ksub) {
        const int c = ksub * 2 + (lane >> 5);
#pragma unroll
        for (int fm = 0; fm < FM; ++fm) {
            int r = wm * WTM + fm * 32 + (lane & 31);
            aoff[ksub][fm] = r * KB + ((c ^ swz<CPR>(r)) << 4);
        }
#pragma unroll
        for (int fn = 0; fn < FN; ++fn) {
            int r = wn * WTN + fn * 32 + (lane & 31);
            boff[ksub][fn] = BM * KB + r * KB + ((c ^ swz<CPR>(r)) << 4);
        }
    }

    // One GEMM over `steps` K steps fetched by `fetch(step, buffer)`; accumulators start at `bias_s`.
    auto gemm = [&](int steps, const int *bias_s, auto fetch, bool with_residual_tile, bool fetched) {
#pragma unroll
        for (int fm = 0; fm < FM; ++fm) {
            acc_t init;
#pragma unroll
            for (int i = 0; i < ACC; ++i) init[i] = bias_s[lane_oc(fm) + i];
#pragma unroll
            for (int fn = 0; fn < FN; ++fn) acc[fm][fn] = init;
        }
        // every buffer is free at the start: the first NST steps are all fetched at once
        if (!fetched) {
#pragma unroll
            for (int s = 0; s < NST; ++s)
                if (s < steps) fetch(s, s);
        }
        int cur = 0, fill = 0;   // buffer computed on now / buffer refilled next (the one of step ks - 1)
        for (int ks = 0; ks < steps; ++ks) {
            // This wave's loads of step ks have landed once at most the loads of the steps after it
            // (L each) are still in flight: min(steps, NST) - 1 of them at step 0, then
            // min(steps - 1 - ks, NST - 2).
            if (ks == 0) {
                if (NST == 3 && steps >= 3) wait_vmcnt<2 * L>();
                else if (steps >= 2) wait_vmcnt<L>();
                else wait_vmcnt<0>();
            } else if (NST == 3 && ks + 1 < steps) wait_vmcnt<L>();
            else wait_vmcnt<0>();
            __builtin_amdgcn_s_barrier();   // every wave's loads of step ks landed; every wave is done with step ks - 1
            if (ks >= 1) {
                if (ks + NST - 1 < steps) fetch(ks + NST - 1, fill);
                else if (FUSE == 1 && with_residual_tile && ks + 1 == steps && res_buf < 0) { res_buf = fill; issue_residual(fill); }
                fill = fill + 1 == NST ? 0 : fill + 1;
            }
            const int8_t *base = Ls[cur];
#pragma unroll
            for (int ksub = 0; ksub < KS; ++ksub) {
                v4i fa[FM], fb[FN];
#pragma unroll
                for (int fm = 0; fm < FM; ++fm) fa[fm] = *(const v4i *)(base + aoff[ksub][fm]);
#pragma unroll
                for (int fn = 0; fn < FN; ++fn) fb[fn] = *(const v4i *)(base + boff[ksub][fn]);
#pragma unroll
                for (int fm = 0; fm < FM; ++fm)
#pragma unroll
                    for (int fn = 0; fn < FN; ++fn)
                        acc[fm][fn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[fm], fb[fn], acc[fm][fn], 0, 0, 0);
            }
            cur = cur + 1 == NST ? 0 : cur + 1;
        }
    };

    // The same GEMM for the 128 x 128 wave tile, which runs one wave per SIMD: no other wave hides the
    // latency of the fragment reads, so the wave pipelines them itself.  The fragments of K sub-step
    // k + 1 are read (into a second register set) before the 16 MFMAs of sub-step k are issued; at the
    // last sub-step of a K step the wave waits for the next step's operands, synchronises, refills the
    // buffer it has just finished, and reads the next step's first fragments -- all in front of that
    // sub-step's MFMAs.  Two stages, no fused residual.
    auto gemm_pipelined = [&](int steps, const int *bias_s, auto fetch, bool fetched) {
        static_assert(!PIPELINED || (NST == 2 && FUSE == 0 && KS % 2 == 0), "pipelined loop: two stages, plain epilogue");
#pragma unroll
        for (int fm = 0; fm < FM; ++fm) {
            acc_t init;
#pragma unroll
            for (int i = 0; i < ACC; ++i) init[i] = bias_s[lane_oc(fm) + i];
#pragma unroll
            for (int fn = 0; fn < FN; ++fn) acc[fm][fn] = init;
        }
        if (!fetched) {
#pragma unroll
            for (int s = 0; s < NST; ++s)
                if (s < steps) fetch(s, s);
        }
        if (steps >= 2) wait_vmcnt<L>();
        else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();   // every wave's loads of step 0 landed
        v4i fa[2][FM], fb[2][FN];
        auto read_fragments = [&](const int8_t *base, int ksub, int slot) {
#pragma unroll
            for (int fm = 0; fm < FM; ++fm) fa[slot][fm] = *(const v4i *)(base + aoff[ksub][fm]);
#pragma unroll
            for (int fn = 0; fn < FN; ++fn) fb[slot][fn] = *(const v4i *)(base + boff[ksub][fn]);
        };
        read_fragments(Ls[0], 0, 0);
        int cur = 0;
        for (int ks = 0; ks < steps; ++ks) {
            const int8_t *base = Ls[cur];
            const int nxt = cur ^ 1;
#pragma unroll
            for (int ksub = 0; ksub < KS; ++ksub) {
                const int slot = ksub & 1;
                if (ksub + 1 < KS) {
                    read_fragments(base, ksub + 1, slot ^ 1);
                } else if (ks + 1 < steps) {
                    // only the loads of step ks + 1 are in flight (those of step ks + 2 are issued below);
                    // this wave's reads of the current buffer are complete before any wave refills it
                    wait_vmcnt<0>();
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                    __builtin_amdgcn_s_barrier();
                    if (ks + 2 < steps) fetch(ks + 2, cur);
                    read_fragments(Ls[nxt], 0, slot ^ 1);
                }
#pragma unroll
                for (int fm = 0; fm < FM; ++fm)
#pragma unroll
                    for (int fn = 0; fn < FN; ++fn)
                        acc[fm][fn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[slot][fm], fb[slot][fn], acc[fm][fn], 0, 0, 0);
            }
            cur = nxt;
        }
    };

    // residual convolution first: its int8 result stays packed in registers (16 channels per dword group)
    v4i rq[FUSE == 2 ? FM : 1][FUSE == 2 ? FN : 1];
    if constexpr (FUSE == 2) {
        gemm(p.Cin2_p / KB, prm2_s[0], issue2, false, prefetched);
#pragma unroll
        for (int fm = 0; fm < FM; ++fm)
#pragma unroll
            for (int fn = 0; fn < FN; ++fn) {
                int q[ACC];
#pragma unroll
                for (int i = 0; i < ACC; ++i) {
                    const int c = lane_oc(fm) + i;
                    q[i] = clamp3(requant_q<TF>(acc[fm][fn][i], prm2_s[1][c], prm2_s[2][c], prm2_s[3][c]), p.lo2, 127);
                }
                rq[fm][fn] = v4i{(int)pack4(q[0], q[1], q[2], q[3]), (int)pack4(q[4], q[5], q[6], q[7]),
                                 (int)pack4(q[8], q[9], q[10], q[11]), (int)pack4(q[12], q[13], q[14], q[15])};
            }
        __syncthreads();   // every wave is done with the operand buffers before the main GEMM refills them
    }
    if constexpr (PIPELINED) gemm_pipelined(nk, prm_s[0], issue, prefetched);
    else gemm(nk, prm_s[0], issue, true, FUSE != 2 && prefetched);

    // epilogue: requantise, clamp, optional residual add, pack, store (NHWC)
    const int8_t *resbuf = nullptr;
    if constexpr (FUSE == 1) {
        wait_vmcnt<0>();
        __syncthreads();   // the residual tile is in LDS
        resbuf = Ls[res_buf];
    }
    const int lo = p.relu ? p.zp_out : -128;
#pragma unroll
    for (int fm = 0; fm < FM; ++fm) {
        const int oc = m0 + lane_oc(fm);
        if (oc >= p.Cout_p) continue;
        int mm[ACC], ch[ACC], ss[ACC];
#pragma unroll
        for (int i = 0; i < ACC; ++i) {
            mm[i] = prm_s[1][oc - m0 + i]; ch[i] = prm_s[2][oc - m0 + i]; ss[i] = prm_s[3][oc - m0 + i];
        }
        {
#pragma unroll
            for (int fn = 0; fn < FN; ++fn) {
                long n = n0 + wn * WTN + fn * MT + (lane & (MT - 1));
                if (n >= p.npix) continue;
                int q[ACC];
#pragma unroll
                for (int i = 0; i < ACC; ++i) q[i] = clamp3(requant_q<TF>(acc[fm][fn][i], mm[i], ch[i], ss[i]), lo, 127);
                if constexpr (FUSE != 0) {
                    const int pixel = wn * WTN + fn * MT + (lane & (MT - 1));
                    v4i rv;
                    if constexpr (FUSE == 2) rv = rq[fm][fn];
                    else rv = *(const v4i *)(resbuf + (pixel * RCH + ((lane_oc(fm) >> 4) ^ rswz(pixel))) * 16);
#pragma unroll
                    for (int i = 0; i < ACC; ++i) {
                        int r8 = (int)(int8_t)((uint32_t)rv[i >> 2] >> (8 * (i & 3)));
                        q[i] = fused_add<TFA>(q[i], r8, p);
                    }
                }
                int8_t *dst = p.out + n * p.Cout_p + oc;
                v4i v = {(int)pack4(q[0], q[1], q[2], q[3]), (int)pack4(q[4], q[5], q[6], q[7]),
                         (int)pack4(q[8], q[9], q[10], q[11]), (int)pack4(q[12], q[13], q[14], q[15])};
                *(v4i *)dst = v;
            }
        }
    }
}

}  // namespace isr

#endif
