// Bottleneck residual block with 64 middle channels in one kernel:
//   t1 = clamp(requant(conv1x1(x)))                     Cin -> 64
//   t2 = clamp(requant(conv3x3(t1)))                    64 -> 64, stride 1, pad 1
//   y  = add_requant(clamp(requant(conv1x1(t2))), x)    64 -> Cout = Cin   (TAIL only)
// A workgroup of four waves makes an 8 x 28 pixel tile of one image: 224 output pixels = seven full
// 32-pixel MFMA fragments (no padding columns in the two later convolutions, whose requantisation
// arithmetic is what bounds this kernel), 10 x 30 = 300 halo pixels = ten fragments for the first.
//   1. The first convolution runs as a GEMM over the halo pixels (wave = 32 channels x 5 fragments):
//      K steps of 64 input channels go from global memory straight into two LDS stages.
//      Recomputing the halo costs a third more of this (cheap) GEMM and saves writing and
//      re-reading t1.
//   2. Its int8 result goes into an LDS tile [halo pixel][64 channels]; halo pixels outside the
//      image get t1's zero-point, the padding value of the 3x3 convolution.
//   3. The 3x3 convolution reads its pixel operands from that tile at tap-shifted addresses
//      (no gather from memory) and its weights from LDS (fetched while step 2 runs, into
//      the space of the two operand stages): 18 K steps of 32, no barrier inside
//      (wave = 32 channels x 4 or 3 fragments).
//   4. HEAD: t2 is requantised and stored.  TAIL: t2 replaces t1 in LDS, and the last 1x1
//      convolution + residual add is split over the waves by OUTPUT CHANNEL: each wave owns 64 of
//      every 256 channels for all seven pixel fragments, so the four waves (one per SIMD) carry
//      the same load; its weight fragments and per-channel constants are loaded once per 32
//      channels, the pixel operands come from the t2 tile (held in registers), and the residual --
//      x at the wave's own 64 channels, which are the input channels of one K step of step 1 -- was
//      copied from that step's LDS stage into registers: x is read from memory once.
// x is read once (plus halo, mostly cache hits), t1 and t2 never leave the CU.
#include "conv_device.h"

namespace isr {

namespace {

constexpr int TH = 8, TW = 28;                 // output tile
constexpr int HH = TH + 2, HW = TW + 2;        // halo tile: 10 x 30 = 300 pixels
constexpr int NHALO = HH * HW;                 // 300
constexpr int NH_FR = 10;                      // fragments (of 32 GEMM columns) covering the halo: 320 columns
constexpr int NP_FR = 7;                       // fragments covering the 224 output pixels, all full
constexpr int W2_CHUNKS = 37;                  // 16-byte chunks per 3x3 weight row in LDS: 36 + 1 pad (bank spread)

// MODE 0: head (t2 stored); 1: whole identity block (residual = x); 2: whole first block of a stage --
// the residual is itself a 1x1 convolution of x (projection shortcut, Cin = 64), computed here as well.
template <int MODE, bool TF>
__global__ __launch_bounds__(256, 2) void bottleneck_kernel(const BneckParams p) {
    constexpr bool TAIL = MODE != 0, PROJ = MODE == 2;
    constexpr int KB = 64, STAGE = (64 + 32 * NH_FR) * KB;            // 64 weight rows + 320 pixel rows per stage
    static_assert(64 * W2_CHUNKS * 16 <= 2 * STAGE, "3x3 weights fit the operand stages");
    __shared__ __attribute__((aligned(16))) int8_t Ls[2 * STAGE];     // step 1: two stages (A rows, then B rows); step 3: 3x3 weights
    __shared__ __attribute__((aligned(16))) int8_t T[32 * NH_FR * 64]; // t1: [halo pixel][channel chunk ^ swizzle]; later t2: [output pixel][...]
    __shared__ int prm[2][4][64];                                     // bias, M0, chi, shift-1 of the first two convolutions
    __shared__ __attribute__((aligned(16))) int prm3[TAIL ? 4 : 1][TAIL ? 256 : 4];
    __shared__ __attribute__((aligned(16))) int prmp[PROJ ? 4 : 1][PROJ ? 256 : 4];   // the same for the projection

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l = lane & 31, half = lane >> 5;
    const int wm = wave & 1, wn = wave >> 1;   // first two convolutions: 32 channels x one half of the fragments
    // tiles that share halo rows run on the same XCD (workgroup ids are dealt round-robin over 8 XCDs)
    const int nblk = gridDim.x;
    const int xcd = blockIdx.x & 7, per = nblk >> 3, extra = nblk & 7;
    const int logical = xcd * per + (xcd < extra ? xcd : extra) + (blockIdx.x >> 3);
    const int tiles_x = (p.W + TW - 1) / TW, tiles_y = (p.H + TH - 1) / TH;
    const int b = logical / (tiles_x * tiles_y), t = logical % (tiles_x * tiles_y);
    const int oy0 = (t / tiles_x) * TH, ox0 = (t % tiles_x) * TW;     // first output pixel of the tile
    const int y0 = oy0 - 1, x0 = ox0 - 1;                            // image position of halo pixel (0, 0)

    for (int i = tid; i < 2 * 64; i += 256) {
        const int cv = i >> 6, c = i & 63;
        prm[cv][0][c] = (cv ? p.bias2 : p.bias1)[c];
        prm[cv][1][c] = (cv ? p.m0s2 : p.m0s1)[c];
        prm[cv][2][c] = (cv ? p.chi2 : p.chi1)[c];
        prm[cv][3][c] = (cv ? p.shm12 : p.shm11)[c];
    }
    if constexpr (TAIL)
        for (int i = tid; i < p.Cout_p; i += 256) {
            prm3[0][i] = p.bias3[i]; prm3[1][i] = p.m0s3[i]; prm3[2][i] = p.chi3[i]; prm3[3][i] = p.shm13[i];
            if constexpr (PROJ) { prmp[0][i] = p.biasp[i]; prmp[1][i] = p.m0sp[i]; prmp[2][i] = p.chip[i]; prmp[3][i] = p.shm1p[i]; }
        }

    // ---- step 1: t1 accumulators over the halo, K = Cin_p in steps of 64 ----
    // LDS position (row, col) of a stage holds K chunk col ^ swz(row); a lane fetches the same
    // chunk `cl` for all its rows (their numbers differ by multiples of 64)
    const int col = tid & 3, row0 = tid >> 2, cl = col ^ swz<4>(row0);
    const int8_t *wrow = p.w1 + (long)row0 * p.Cin_p + cl * 16;
    uint32_t boff[5];
    bool bok[5];
#pragma unroll
    for (int j = 0; j < 5; ++j) {
        const int h = row0 + 64 * j, hy = h / HW, hx = h - hy * HW, y = y0 + hy, x = x0 + hx;
        bok[j] = h < NHALO && (unsigned)y < (unsigned)p.H && (unsigned)x < (unsigned)p.W;
        boff[j] = bok[j] ? (uint32_t)((((long)b * p.H + y) * p.W + x) * p.Cin_p + cl * 16) : 0u;
    }
    auto issue = [&](int ks, int buf) {
        int8_t *sa = &Ls[buf * STAGE + wave * 1024];
        ISR_GLOBAL_TO_LDS16(wrow + ks * KB, sa);
        int8_t *sb = sa + 64 * KB;
#pragma unroll
        for (int j = 0; j < 5; ++j) {
            // halo pixels outside the image (and the 20 columns past the halo): any readable bytes,
            // their results are replaced in step 2 or never used
            const int8_t *src = bok[j] ? p.in + (boff[j] + (uint32_t)(ks * KB)) : p.zpad;
            ISR_GLOBAL_TO_LDS16(src, sb + j * 4096);
        }
    };
    const int nk = p.Cin_p / KB;
    issue(0, 0);
    if (nk > 1) issue(1, 1);            // both stages are free at the start
    __syncthreads();                    // prm visible

    const int c16 = wm * 32 + 16 * half;   // first of the lane's 16 channels in the first two convolutions
    v16i acc[5];
    {
        v16i init;
#pragma unroll
        for (int i = 0; i < 16; ++i) init[i] = prm[0][0][c16 + i];
#pragma unroll
        for (int f = 0; f < 5; ++f) acc[f] = init;
    }
    // TAIL: the residual of the closing add is x itself.  Wave w will own output channels [64 w, 64 w + 64) there,
    // which are exactly the input channels of K step w of this GEMM: while that step's pixel rows sit in the
    // LDS stage the wave copies its residual values (its 64 channels of the seven fragments' pixels) into
    // registers, so x is not read from memory a second time.
    // (With a projection shortcut x has only 64 channels and is the pixel operand of a second GEMM: it is
    // read again from memory -- cache hits, a fifth of the block's traffic at most -- rather than held in 56 registers.)
    v4i resid[MODE == 1 ? NP_FR : 1][2];
    {
        int aoff[2], boffs[2][5];   // [K half of the step][fragment]
#pragma unroll
        for (int ksub = 0; ksub < 2; ++ksub) {
            const int c = ksub * 2 + half;
            const int ra = wm * 32 + l;
            aoff[ksub] = ra * KB + ((c ^ swz<4>(ra)) << 4);
#pragma unroll
            for (int f = 0; f < 5; ++f) {
                const int rb = (wn * 5 + f) * 32 + l;
                boffs[ksub][f] = 64 * KB + rb * KB + ((c ^ swz<4>(rb)) << 4);
            }
        }
        for (int ks = 0; ks < nk; ++ks) {
            if (ks == 0 && nk > 1) wait_vmcnt<6>();   // step 0 landed; the 6 loads of step 1 may still be in flight
            else wait_vmcnt<0>();
            __builtin_amdgcn_s_barrier();   // every wave's loads of step ks landed; every wave is done with step ks - 1
            if (ks >= 1 && ks + 1 < nk) issue(ks + 1, (ks + 1) & 1);
            const int8_t *base = &Ls[(ks & 1) * STAGE];
            if constexpr (MODE == 1) {
                if (ks == wave) {   // wave-uniform
#pragma unroll
                    for (int f = 0; f < NP_FR; ++f) {
                        const int o = f * 32 + l, oy = o / TW, ox = o - oy * TW, hp = (oy + 1) * HW + ox + 1;   // the output pixel's own halo position
#pragma unroll
                        for (int mi = 0; mi < 2; ++mi)
                            resid[f][mi] = *(const v4i *)(base + 64 * KB + hp * KB + (((mi * 2 + half) ^ swz<4>(hp)) << 4));
                    }
                }
            }
#pragma unroll
            for (int ksub = 0; ksub < 2; ++ksub) {
                const v4i fa = *(const v4i *)(base + aoff[ksub]);
                v4i fb[5];
#pragma unroll
                for (int f = 0; f < 5; ++f) fb[f] = *(const v4i *)(base + boffs[ksub][f]);
#pragma unroll
                for (int f = 0; f < 5; ++f) acc[f] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa, fb[f], acc[f], 0, 0, 0);
            }
        }
    }
    __syncthreads();   // every wave is done with the operand stages

    // 3x3 weights -> LDS (the space of the stages): row r at chunk r * 37, 36 chunks + 1 pad
    {
        constexpr int TOTAL = 64 * W2_CHUNKS;            // 2368 = 9 * 256 + 64: the last pass is wave 0 alone
#pragma unroll
        for (int pass = 0; pass < (TOTAL + 255) / 256; ++pass) {
            if (pass * 256 + wave * 64 < TOTAL) {        // wave-uniform
                const int q = pass * 256 + tid, r = q / W2_CHUNKS, c = q % W2_CHUNKS;
                ISR_GLOBAL_TO_LDS16(p.w2 + (long)r * 576 + (c < 36 ? c : 0) * 16, &Ls[(pass * 256 + wave * 64) * 16]);
            }
        }
    }

    // ---- step 2: requantise t1 into the LDS tile ----
    {
        const uint32_t zt = (uint32_t)(p.zp_t1 & 0xFF) * 0x01010101u;
        int mm[16], ch[16], ss[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) { mm[i] = prm[0][1][c16 + i]; ch[i] = prm[0][2][c16 + i]; ss[i] = prm[0][3][c16 + i]; }
#pragma unroll
        for (int f = 0; f < 5; ++f) {
            const int h = (wn * 5 + f) * 32 + l, hy = h / HW, hx = h - hy * HW, y = y0 + hy, x = x0 + hx;
            const bool inside = h < NHALO && (unsigned)y < (unsigned)p.H && (unsigned)x < (unsigned)p.W;
            int q[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) q[i] = clamp3(requant_q<TF>(acc[f][i], mm[i], ch[i], ss[i]), p.lo1, 127);
            v4i v = {(int)pack4(q[0], q[1], q[2], q[3]), (int)pack4(q[4], q[5], q[6], q[7]),
                     (int)pack4(q[8], q[9], q[10], q[11]), (int)pack4(q[12], q[13], q[14], q[15])};
            if (!inside) v = v4i{(int)zt, (int)zt, (int)zt, (int)zt};
            *(v4i *)(&T[h * 64 + (((wm * 2 + half) ^ swz<4>(h)) << 4)]) = v;
        }
    }
    wait_vmcnt<0>();
    __syncthreads();   // t1 tile and 3x3 weights in LDS

    // ---- step 3: 3x3 convolution from LDS: this wave's 32 channels x its 4 (wn = 0) or 3 (wn = 1) fragments ----
    const int nfr = wn ? NP_FR - 4 : 4;   // wave-uniform
    int hb[4];                            // halo pixel of tap (0, 0) of the lane's output pixel in fragment f
#pragma unroll
    for (int f = 0; f < 4; ++f) {
        const int o = (wn * 4 + f) * 32 + l;
        const int oo = o < TH * TW ? o : 0, oy = oo / TW, ox = oo - oy * TW;
        hb[f] = oy * HW + ox;
    }
    {
        v16i init;
#pragma unroll
        for (int i = 0; i < 16; ++i) init[i] = prm[1][0][c16 + i];
#pragma unroll
        for (int f = 0; f < 4; ++f) acc[f] = init;
    }
#pragma unroll
    for (int ks = 0; ks < 18; ++ks) {
        const int tap = ks >> 1, ky = tap / 3, kx = tap % 3, cc = (ks & 1) * 2 + half;
        const v4i fa = *(const v4i *)(&Ls[((wm * 32 + l) * W2_CHUNKS + 2 * ks + half) * 16]);
        v4i fb[4];
#pragma unroll
        for (int f = 0; f < 4; ++f) {
            const int hp = hb[f] + ky * HW + kx;
            fb[f] = *(const v4i *)(&T[hp * 64 + ((cc ^ swz<4>(hp)) << 4)]);
        }
#pragma unroll
        for (int f = 0; f < 4; ++f)
            if (f < 3 || nfr == 4) acc[f] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa, fb[f], acc[f], 0, 0, 0);
    }

    // ---- step 4: requantise t2 ----
    v4i t2[4];
    {
        int mm[16], ch[16], ss[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) { mm[i] = prm[1][1][c16 + i]; ch[i] = prm[1][2][c16 + i]; ss[i] = prm[1][3][c16 + i]; }
#pragma unroll
        for (int f = 0; f < 4; ++f) {
            if (f == 3 && nfr != 4) { t2[f] = v4i{0, 0, 0, 0}; continue; }
            int q[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) q[i] = clamp3(requant_q<TF>(acc[f][i], mm[i], ch[i], ss[i]), p.lo2, 127);
            t2[f] = v4i{(int)pack4(q[0], q[1], q[2], q[3]), (int)pack4(q[4], q[5], q[6], q[7]),
                        (int)pack4(q[8], q[9], q[10], q[11]), (int)pack4(q[12], q[13], q[14], q[15])};
        }
    }
    if constexpr (!TAIL) {
#pragma unroll
        for (int f = 0; f < 4; ++f) {
            if (f == 3 && nfr != 4) continue;
            const int o = (wn * 4 + f) * 32 + l, oy = o / TW, ox = o - oy * TW;
            if (oy0 + oy < p.H && ox0 + ox < p.W)
                *(v4i *)(p.out + (((long)b * p.H + oy0 + oy) * p.W + ox0 + ox) * 64 + c16) = t2[f];
        }
    } else {
        __syncthreads();   // every wave is done reading the t1 tile: t2 takes its place, [output pixel][64 channels]
#pragma unroll
        for (int f = 0; f < 4; ++f) {
            if (f == 3 && nfr != 4) continue;
            const int o = (wn * 4 + f) * 32 + l;
            *(v4i *)(&T[o * 64 + (((wm * 2 + half) ^ swz<4>(o)) << 4)]) = t2[f];
        }
        __syncthreads();   // the t2 tile is complete

        // ---- last 1x1 convolution + residual add: this wave's output channels, all seven pixel fragments ----
        ConvParams ap{};   // the fused add reads its constants from here
        ap.add_mul_self = p.add_mul_self; ap.add_mul_res = p.add_mul_res; ap.add_c0 = p.add_c0; ap.add_k = p.add_k;
        ap.add_sh = p.add_sh; ap.add_lo = p.add_lo;
        int opix[NP_FR];    // index (image, row, column) of the lane's pixel of fragment f; -1: outside the image
        v4i fbt[PROJ ? 1 : NP_FR][2];  // the lane's pixel operands (64 channels of t2 = two K halves) of every fragment
#pragma unroll
        for (int f = 0; f < NP_FR; ++f) {
            const int o = f * 32 + l, oy = o / TW, ox = o - oy * TW;
            const bool st = oy0 + oy < p.H && ox0 + ox < p.W;
            opix[f] = st ? ((b * p.H + oy0 + oy) * p.W + ox0 + ox) : -1;
            if constexpr (!PROJ) {
#pragma unroll
                for (int ksub = 0; ksub < 2; ++ksub) fbt[f][ksub] = *(const v4i *)(&T[o * 64 + (((ksub * 2 + half) ^ swz<4>(o)) << 4)]);
            }
        }
        // this wave's 64 output channels (Cout <= 256 = four waves x 64): two groups of 32
        const int nmf = p.Cout_p >> 5;   // 32-channel groups of the output
        // weight fragments of both groups, fetched before the first group's stores: a load issued behind stores
        // waits for them as well (loads and stores share one counter)
        v4i fa_pre[2][2];
        if (2 * wave < nmf) {
#pragma unroll
            for (int g = 0; g < 2; ++g)
#pragma unroll
                for (int ksub = 0; ksub < 2; ++ksub) {
                    fa_pre[g][ksub] = *(const v4i *)(p.w3 + (long)((2 * wave + g) * 32 + l) * 64 + ksub * 32 + half * 16);
                }
        }
        // one group of 32 output channels; mi is a compile-time constant for the identity block (it selects
        // registers of the residual copy) and a loop variable for the projection block
        auto channel_group = [&](auto mi) {
            {
                const int m0 = (2 * wave + (int)mi) * 32, c0 = m0 + 16 * half;   // the lane's 16 channels
                v4i rpack[NP_FR];   // the residual of every fragment, packed int8
                if constexpr (PROJ) {
                    // projection shortcut first: r = clamp(requant(Wp x)), kept packed
                    v4i fp[2];
#pragma unroll
                    for (int ksub = 0; ksub < 2; ++ksub) fp[ksub] = *(const v4i *)(p.wp + (long)(m0 + l) * 64 + ksub * 32 + half * 16);
                    int mm[16], ch[16], ss[16];
                    v16i init;
#pragma unroll
                    for (int i = 0; i < 16; ++i) { init[i] = prmp[0][c0 + i]; mm[i] = prmp[1][c0 + i]; ch[i] = prmp[2][c0 + i]; ss[i] = prmp[3][c0 + i]; }
                    v4i xn[2];   // x at the lane's pixel of the next fragment (pixels outside the image read pixel 0: in bounds, unused)
#pragma unroll
                    for (int ksub = 0; ksub < 2; ++ksub) xn[ksub] = *(const v4i *)(p.in + (long)(opix[0] >= 0 ? opix[0] : 0) * 64 + ksub * 32 + half * 16);
#pragma unroll
                    for (int f = 0; f < NP_FR; ++f) {
                        const v4i x0 = xn[0], x1 = xn[1];
                        if (f + 1 < NP_FR) {
#pragma unroll
                            for (int ksub = 0; ksub < 2; ++ksub) xn[ksub] = *(const v4i *)(p.in + (long)(opix[f + 1] >= 0 ? opix[f + 1] : 0) * 64 + ksub * 32 + half * 16);
                        }
                        v16i a = __builtin_amdgcn_mfma_i32_32x32x32_i8(fp[0], x0, init, 0, 0, 0);
                        a = __builtin_amdgcn_mfma_i32_32x32x32_i8(fp[1], x1, a, 0, 0, 0);
                        int q[16];
#pragma unroll
                        for (int i = 0; i < 16; ++i) q[i] = clamp3(requant_q<TF>(a[i], mm[i], ch[i], ss[i]), p.lop, 127);
                        rpack[f] = v4i{(int)pack4(q[0], q[1], q[2], q[3]), (int)pack4(q[4], q[5], q[6], q[7]),
                                       (int)pack4(q[8], q[9], q[10], q[11]), (int)pack4(q[12], q[13], q[14], q[15])};
                    }
                } else {
#pragma unroll
                    for (int f = 0; f < NP_FR; ++f) rpack[f] = resid[f][decltype(mi)::value];
                }
                v4i fa[2];
#pragma unroll
                for (int ksub = 0; ksub < 2; ++ksub) fa[ksub] = mi == 0 ? fa_pre[0][ksub] : fa_pre[1][ksub];
                int mm[16], ch[16], ss[16];
                v16i init;
#pragma unroll
                for (int i = 0; i < 16; ++i) { init[i] = prm3[0][c0 + i]; mm[i] = prm3[1][c0 + i]; ch[i] = prm3[2][c0 + i]; ss[i] = prm3[3][c0 + i]; }
#pragma unroll
                for (int f = 0; f < NP_FR; ++f) {
                    const v4i res = rpack[f];
                    v4i fb[2];
                    if constexpr (PROJ) {   // the pixel operands are re-read from the t2 tile: the registers hold x
                        const int o = f * 32 + l;
#pragma unroll
                        for (int ksub = 0; ksub < 2; ++ksub) fb[ksub] = *(const v4i *)(&T[o * 64 + (((ksub * 2 + half) ^ swz<4>(o)) << 4)]);
                    } else {
                        fb[0] = fbt[f][0]; fb[1] = fbt[f][1];
                    }
                    v16i a = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[0], fb[0], init, 0, 0, 0);
                    a = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[1], fb[1], a, 0, 0, 0);
                    int q[16];
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int qc = clamp3(requant_q<TF>(a[i], mm[i], ch[i], ss[i]), p.lo3, 127);
                        const int r8 = (int)(int8_t)((uint32_t)res[i >> 2] >> (8 * (i & 3)));
                        q[i] = fused_add<TF>(qc, r8, ap);
                    }
                    if (opix[f] >= 0)
                        *(v4i *)(p.out + (long)opix[f] * p.Cout_p + c0) = v4i{(int)pack4(q[0], q[1], q[2], q[3]), (int)pack4(q[4], q[5], q[6], q[7]),
                                                            (int)pack4(q[8], q[9], q[10], q[11]), (int)pack4(q[12], q[13], q[14], q[15])};
                }
            }
        };
        if (2 * wave < nmf) {
            if constexpr (PROJ) {
#pragma unroll 1
                for (int mi = 0; mi < 2; ++mi) channel_group(mi);
            } else {
                channel_group(std::integral_constant<int, 0>{});
                channel_group(std::integral_constant<int, 1>{});
            }
        }
    }
}

}  // namespace

// Geometry with a kernel: first convolution 1x1 (stride 1) from a multiple of 64 stored channels
// into 64; second 3x3 stride 1 pad 1, 64 -> 64; optional tail 1x1 from 64 back to the input's
// channel count (at most 256) with the block input as residual.
bool bottleneck_supported(int cin_p, int cmid_p, int cout_p, int tail) {
    if (cin_p % 64 != 0 || cin_p < 64 || cin_p > 1024 || cmid_p != 64) return false;
    if (tail == 2) return cin_p == 64 && cout_p % 64 == 0 && cout_p >= 64 && cout_p <= 256;   // projection shortcut from 64 channels
    return !tail || (cout_p == cin_p && cout_p <= 256);
}

hipError_t launch_bottleneck(const BneckParams &p, hipStream_t st) {
    if (p.B <= 0) return hipSuccess;
    if (!p.in || !p.out || !p.w1 || !p.w2 || !p.zpad || p.H < 1 || p.W < 1 ||
        !bottleneck_supported(p.Cin_p, 64, p.Cout_p, p.tail ? (p.proj ? 2 : 1) : 0) || (p.tail && !p.w3) ||
        (p.proj && (!p.tail || !p.wp || !p.biasp || !p.m0sp || !p.chip || !p.shm1p)))
        return hipErrorInvalidValue;
    const long tiles = (long)p.B * ((p.H + TH - 1) / TH) * ((p.W + TW - 1) / TW);
    if (tiles > 0x7fffffffL || (long)p.B * p.H * p.W * (p.Cin_p > 64 ? p.Cin_p : 64) >= (1L << 31)) return hipErrorInvalidValue;
    const dim3 grid((unsigned)tiles), block(256);
    const int mode = p.tail ? (p.proj ? 2 : 1) : 0;
    static const char *const names[3][2] = {{"bottleneck_kernel<head, false>", "bottleneck_kernel<head, true>"},
                                            {"bottleneck_kernel<block, false>", "bottleneck_kernel<block, true>"},
                                            {"bottleneck_kernel<block + projection, false>", "bottleneck_kernel<block + projection, true>"}};
    set_kernel_name(names[mode][p.tie_free ? 1 : 0]);
    if (mode == 2) {
        if (p.tie_free) hipLaunchKernelGGL((bottleneck_kernel<2, true>), grid, block, 0, st, p);
        else hipLaunchKernelGGL((bottleneck_kernel<2, false>), grid, block, 0, st, p);
    } else if (mode == 1) {
        if (p.tie_free) hipLaunchKernelGGL((bottleneck_kernel<1, true>), grid, block, 0, st, p);
        else hipLaunchKernelGGL((bottleneck_kernel<1, false>), grid, block, 0, st, p);
    } else {
        if (p.tie_free) hipLaunchKernelGGL((bottleneck_kernel<0, true>), grid, block, 0, st, p);
        else hipLaunchKernelGGL((bottleneck_kernel<0, false>), grid, block, 0, st, p);
    }
    return hipGetLastError();
}

}  // namespace isr
