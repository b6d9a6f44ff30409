// Identity bottleneck block with 128 middle channels in one kernel (the 28 x 28 stage of the
// deep bottleneck net, where a 512-channel tensor of a chunk is far larger than the caches and
// every layer of the block is bound by its memory traffic when run alone):
//   t1 = clamp(requant(conv1x1(x)))                     Cin -> 128
//   t2 = clamp(requant(conv3x3(t1)))                    128 -> 128, stride 1, pad 1
//   y  = add_requant(clamp(requant(conv1x1(t2))), x)    128 -> Cout = Cin
// x is read once (plus the halo) and y written once; t1 and t2 never leave the CU.
// A workgroup of four waves makes a 14 x 14 pixel tile of one image:
//   1. first convolution as a GEMM over the 16 x 16 halo pixels of the tile (128 x 256 outputs, each
//      wave 64 channels x 128 pixels = 2 x 4 MFMA tiles); K steps of 64 input channels go from global
//      memory straight into two LDS stages;
//   2. its int8 result goes to an LDS tile [halo pixel][128 channels] that takes the place of the
//      stages; halo pixels outside the image get t1's zero-point, the padding value of the 3x3;
//   3. the 3x3 convolution reads its pixel operands from that tile at tap-shifted addresses; its
//      weights (144 KB) stream through three small LDS stages, 64 K-bytes (half a tap) per step;
//   4. t2 replaces t1 in LDS ([output pixel][128 channels]): the last convolution needs all 128
//      channels of a pixel, which two waves hold between them;
//   5. last 1x1 convolution + residual add, split over the waves by output channel (each wave 128
//      of every 512 channels, all 196 pixels): its weight fragments and per-channel constants come
//      from global memory once per 32 channels, the pixel operands from the t2 tile, the residual x
//      from global memory at the tile's own pixels.
#include "conv_device.h"

namespace isr {

namespace {

constexpr int BT = 14;              // output tile edge
constexpr int BH = BT + 2;          // halo tile edge: 16 x 16 = 256 GEMM columns
constexpr int CM = 128;             // middle channels
constexpr int NFR = 7;              // 32-pixel fragments covering the 196 output pixels

template <bool TF>
__global__ __launch_bounds__(256, 2) void bottleneck128_kernel(const BneckParams p) {
    constexpr int KB = 64;
    constexpr int STAGE1 = (CM + 256) * KB;        // one stage of the first GEMM: 128 weight rows, 256 pixel rows
    constexpr int T_BYTES = 256 * CM;              // t1 tile; later the t2 tile (224 x 128)
    constexpr int W2_STAGE = CM * KB;              // one K step of the 3x3 weights
    constexpr int LDS_BYTES = T_BYTES + 3 * W2_STAGE;
    static_assert(2 * STAGE1 <= LDS_BYTES, "the first GEMM's stages fit the space of the tile and the 3x3 weight stages");
    __shared__ __attribute__((aligned(16))) int8_t Ls[LDS_BYTES];
    __shared__ int prm[2][4][CM];                  // bias, M0, chi, shift-1 of the first two convolutions
    int8_t *const T = Ls;                          // [pixel][16-byte channel chunk ^ (pixel & 7)]
    int8_t *const W2s = Ls + T_BYTES;              // three stages of [128 rows][64 bytes]

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l = lane & 31, half = lane >> 5;
    const int wm = wave & 1, wn = wave >> 1;
    // tiles that share halo rows run on the same XCD (workgroup ids are dealt round-robin over 8 XCDs)
    const int nblk = gridDim.x;
    const int xcd = blockIdx.x & 7, per = nblk >> 3, extra = nblk & 7;
    const int logical = xcd * per + (xcd < extra ? xcd : extra) + (blockIdx.x >> 3);
    const int tiles_x = (p.W + BT - 1) / BT, tiles_y = (p.H + BT - 1) / BT;
    const int b = logical / (tiles_x * tiles_y), t = logical % (tiles_x * tiles_y);
    const int oy0 = (t / tiles_x) * BT, ox0 = (t % tiles_x) * BT;     // first output pixel of the tile
    const int y0 = oy0 - 1, x0 = ox0 - 1;                            // image position of halo pixel (0, 0)

    for (int i = tid; i < 2 * CM; i += 256) {
        const int cv = i >> 7, c = i & (CM - 1);
        prm[cv][0][c] = (cv ? p.bias2 : p.bias1)[c];
        prm[cv][1][c] = (cv ? p.m0s2 : p.m0s1)[c];
        prm[cv][2][c] = (cv ? p.chi2 : p.chi1)[c];
        prm[cv][3][c] = (cv ? p.shm12 : p.shm11)[c];
    }

    // ---- step 1: t1 accumulators over the halo, K = Cin_p in steps of 64 ----
    // LDS position (row, col) of a stage holds K chunk col ^ swz(row); a lane fetches the same chunk
    // `cl` for all its rows (their numbers differ by multiples of 64)
    const int col = tid & 3, row0 = tid >> 2, cl = col ^ swz<4>(row0);
    const int8_t *wrow1 = p.w1 + (long)row0 * p.Cin_p + cl * 16;
    uint32_t xoff[4];
    bool xok[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int h = row0 + 64 * j, y = y0 + (h >> 4), x = x0 + (h & 15);
        xok[j] = (unsigned)y < (unsigned)p.H && (unsigned)x < (unsigned)p.W;
        xoff[j] = xok[j] ? (uint32_t)((((long)b * p.H + y) * p.W + x) * p.Cin_p + cl * 16) : 0u;
    }
    auto issue1 = [&](int ks, int buf) {
        int8_t *sa = &Ls[buf * STAGE1 + wave * 1024];
#pragma unroll
        for (int j = 0; j < 2; ++j) ISR_GLOBAL_TO_LDS16(wrow1 + (long)(64 * j) * p.Cin_p + ks * KB, sa + j * 4096);
        int8_t *sb = sa + CM * KB;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            // halo pixels outside the image: any readable bytes, their results are replaced in step 2
            const int8_t *src = xok[j] ? p.in + (xoff[j] + (uint32_t)(ks * KB)) : p.zpad;
            ISR_GLOBAL_TO_LDS16(src, sb + j * 4096);
        }
    };
    const int nk = p.Cin_p / KB;
    issue1(0, 0);
    if (nk > 1) issue1(1, 1);           // both stages are free at the start
    __syncthreads();                    // prm visible

    auto lane_c = [&](int fm) { return wm * 64 + fm * 32 + 16 * half; };   // first of the lane's 16 channels in M fragment fm
    v16i acc[2][4];
#pragma unroll
    for (int fm = 0; fm < 2; ++fm) {
        v16i init;
#pragma unroll
        for (int i = 0; i < 16; ++i) init[i] = prm[0][0][lane_c(fm) + i];
#pragma unroll
        for (int fn = 0; fn < 4; ++fn) acc[fm][fn] = init;
    }
    {
        int aoff[2][2], boff[2][4];   // [K half of the step][fragment]
#pragma unroll
        for (int ksub = 0; ksub < 2; ++ksub) {
            const int c = ksub * 2 + half;
#pragma unroll
            for (int f = 0; f < 2; ++f) {
                const int ra = wm * 64 + f * 32 + l;
                aoff[ksub][f] = ra * KB + ((c ^ swz<4>(ra)) << 4);
            }
#pragma unroll
            for (int f = 0; f < 4; ++f) {
                const int rb = wn * 128 + f * 32 + l;
                boff[ksub][f] = CM * KB + rb * KB + ((c ^ swz<4>(rb)) << 4);
            }
        }
        for (int ks = 0; ks < nk; ++ks) {
            if (ks == 0 && nk > 1) wait_vmcnt<6>();   // step 0 landed; the 6 loads of step 1 may still be in flight
            else wait_vmcnt<0>();
            __builtin_amdgcn_s_barrier();   // every wave's loads of step ks landed; every wave is done with step ks - 1
            if (ks >= 1 && ks + 1 < nk) issue1(ks + 1, (ks + 1) & 1);
            const int8_t *base = &Ls[(ks & 1) * STAGE1];
#pragma unroll
            for (int ksub = 0; ksub < 2; ++ksub) {
                v4i fa[2], fb[4];
#pragma unroll
                for (int f = 0; f < 2; ++f) fa[f] = *(const v4i *)(base + aoff[ksub][f]);
#pragma unroll
                for (int f = 0; f < 4; ++f) fb[f] = *(const v4i *)(base + boff[ksub][f]);
#pragma unroll
                for (int fm = 0; fm < 2; ++fm)
#pragma unroll
                    for (int fn = 0; fn < 4; ++fn)
                        acc[fm][fn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[fm], fb[fn], acc[fm][fn], 0, 0, 0);
            }
        }
    }
    __syncthreads();   // every wave is done with the operand stages: their space becomes the t1 tile and the 3x3 weight stages

    // 3x3 weight steps: 128 rows x 64 bytes, two loads per lane; row r of step ks at chunk (r, col ^ swz(r))
    const int8_t *wrow2 = p.w2 + (long)row0 * (9 * CM) + cl * 16;
    auto issue2 = [&](int ks, int buf) {
        int8_t *sa = &W2s[buf * W2_STAGE + wave * 1024];
#pragma unroll
        for (int j = 0; j < 2; ++j) ISR_GLOBAL_TO_LDS16(wrow2 + (long)(64 * j) * (9 * CM) + ks * KB, sa + j * 4096);
    };
    issue2(0, 0);
    issue2(1, 1);
    issue2(2, 2);

    // ---- step 2: requantise t1 into the LDS tile ----
    {
        const uint32_t zt = (uint32_t)(p.zp_t1 & 0xFF) * 0x01010101u;
#pragma unroll
        for (int fm = 0; fm < 2; ++fm) {
            int mm[16], ch[16], ss[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int c = lane_c(fm) + i;
                mm[i] = prm[0][1][c]; ch[i] = prm[0][2][c]; ss[i] = prm[0][3][c];
            }
#pragma unroll
            for (int fn = 0; fn < 4; ++fn) {
                const int h = wn * 128 + fn * 32 + l, y = y0 + (h >> 4), x = x0 + (h & 15);
                const bool inside = (unsigned)y < (unsigned)p.H && (unsigned)x < (unsigned)p.W;
                int q[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) q[i] = clamp3(requant_q<TF>(acc[fm][fn][i], mm[i], ch[i], ss[i]), p.lo1, 127);
                v4i v = {(int)pack4(q[0], q[1], q[2], q[3]), (int)pack4(q[4], q[5], q[6], q[7]),
                         (int)pack4(q[8], q[9], q[10], q[11]), (int)pack4(q[12], q[13], q[14], q[15])};
                if (!inside) v = v4i{(int)zt, (int)zt, (int)zt, (int)zt};
                *(v4i *)(&T[h * CM + (((lane_c(fm) >> 4) ^ (h & 7)) << 4)]) = v;
            }
        }
    }

    // ---- step 3: 3x3 convolution, pixel operands from the t1 tile, weights through the three stages ----
    const int nfr = wn ? NFR - 4 : 4;   // fragments of this wave: output pixels [128 wn, 128 wn + 32 nfr); wave-uniform
    int hb[4];                          // halo pixel of tap (0, 0) of the lane's output pixel in fragment fn
#pragma unroll
    for (int fn = 0; fn < 4; ++fn) {
        const int o = wn * 128 + fn * 32 + l;
        const int oo = o < BT * BT ? o : 0, oy = oo / BT, ox = oo % BT;
        hb[fn] = oy * BH + ox;
    }
#pragma unroll
    for (int fm = 0; fm < 2; ++fm) {
        v16i init;
#pragma unroll
        for (int i = 0; i < 16; ++i) init[i] = prm[1][0][lane_c(fm) + i];
#pragma unroll
        for (int fn = 0; fn < 4; ++fn) acc[fm][fn] = init;
    }
    {
        int aoff[2][2];
#pragma unroll
        for (int ksub = 0; ksub < 2; ++ksub)
#pragma unroll
            for (int f = 0; f < 2; ++f) {
                const int ra = wm * 64 + f * 32 + l;
                aoff[ksub][f] = ra * KB + (((ksub * 2 + half) ^ swz<4>(ra)) << 4);
            }
        constexpr int STEPS = 18;       // 9 taps x 2 halves of the 128 channels
        int cur = 0;
        for (int ks = 0; ks < STEPS; ++ks) {
            // this wave's 2 loads of step ks have landed once only those of later steps are in flight: steps 1
            // and 2 at the start, afterwards step ks + 1 alone (step ks + 2 is issued below, after the barrier)
            if (ks == 0) wait_vmcnt<4>();
            else if (ks + 1 < STEPS) wait_vmcnt<2>();
            else wait_vmcnt<0>();
            if (ks == 0) __syncthreads();           // also: every wave's part of the t1 tile is written
            else __builtin_amdgcn_s_barrier();      // every wave's loads of step ks landed; every wave is done with step ks - 1
            if (ks >= 1 && ks + 2 < STEPS) issue2(ks + 2, cur == 0 ? 2 : cur - 1);   // into the stage of step ks - 1
            const int tap = ks >> 1, ky = tap / 3, kx = tap - 3 * ky, chalf = (ks & 1) * 4;
            const int8_t *wbase = &W2s[cur * W2_STAGE];
#pragma unroll
            for (int ksub = 0; ksub < 2; ++ksub) {
                const int cc = chalf + ksub * 2 + half;
                v4i fa[2], fb[4];
#pragma unroll
                for (int f = 0; f < 2; ++f) fa[f] = *(const v4i *)(wbase + aoff[ksub][f]);
#pragma unroll
                for (int fn = 0; fn < 4; ++fn) {
                    const int hp = hb[fn] + ky * BH + kx;
                    fb[fn] = *(const v4i *)(&T[hp * CM + ((cc ^ (hp & 7)) << 4)]);
                }
#pragma unroll
                for (int fm = 0; fm < 2; ++fm)
#pragma unroll
                    for (int fn = 0; fn < 4; ++fn)
                        if (fn < 3 || nfr == 4)
                            acc[fm][fn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[fm], fb[fn], acc[fm][fn], 0, 0, 0);
            }
            cur = cur == 2 ? 0 : cur + 1;
        }
    }
    __syncthreads();   // every wave is done reading the t1 tile: t2 takes its place

    // ---- step 4: requantise t2 into the LDS tile, [output pixel][channel chunk ^ (pixel & 7)] ----
#pragma unroll
    for (int fm = 0; fm < 2; ++fm) {
        int mm[16], ch[16], ss[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int c = lane_c(fm) + i;
            mm[i] = prm[1][1][c]; ch[i] = prm[1][2][c]; ss[i] = prm[1][3][c];
        }
#pragma unroll
        for (int fn = 0; fn < 4; ++fn) {
            if (fn == 3 && nfr != 4) continue;
            const int o = wn * 128 + fn * 32 + l;
            int q[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) q[i] = clamp3(requant_q<TF>(acc[fm][fn][i], mm[i], ch[i], ss[i]), p.lo2, 127);
            *(v4i *)(&T[o * CM + (((lane_c(fm) >> 4) ^ (o & 7)) << 4)]) =
                v4i{(int)pack4(q[0], q[1], q[2], q[3]), (int)pack4(q[4], q[5], q[6], q[7]),
                    (int)pack4(q[8], q[9], q[10], q[11]), (int)pack4(q[12], q[13], q[14], q[15])};
        }
    }
    __syncthreads();   // the t2 tile is complete

    // ---- step 5: last 1x1 convolution + residual add; this wave's output channels, every pixel ----
    ConvParams ap{};   // the fused add reads its constants from here
    ap.add_mul_self = p.add_mul_self; ap.add_mul_res = p.add_mul_res; ap.add_c0 = p.add_c0; ap.add_k = p.add_k;
    ap.add_sh = p.add_sh; ap.add_lo = p.add_lo;
    long opix[NFR];    // element offset of the lane's pixel of fragment fn in x and y; -1: not stored
#pragma unroll
    for (int fn = 0; fn < NFR; ++fn) {
        const int o = fn * 32 + l;
        const int oo = o < BT * BT ? o : 0, oy = oo / BT, ox = oo % BT;
        const bool st = o < BT * BT && oy0 + oy < p.H && ox0 + ox < p.W;
        opix[fn] = st ? (((long)b * p.H + oy0 + oy) * p.W + ox0 + ox) * p.Cout_p : -1;
    }
    // the weight fragments of a pass and the residual x at the lane's seven pixels are fetched one pass
    // ahead, so that no pass starts by waiting for them; the per-channel constants (cache hits after the
    // first workgroups) at the start of their pass
    struct PassOperands {
        v4i fa[4], res[NFR];
    };
    auto load_pass = [&](int m0, PassOperands &o) {
        const int c0 = m0 + 16 * half;
#pragma unroll
        for (int ksub = 0; ksub < 4; ++ksub) o.fa[ksub] = *(const v4i *)(p.w3 + (long)(m0 + l) * CM + ksub * 32 + half * 16);
#pragma unroll
        for (int fn = 0; fn < NFR; ++fn) o.res[fn] = opix[fn] >= 0 ? *(const v4i *)(p.in + opix[fn] + c0) : v4i{0, 0, 0, 0};
    };
    PassOperands cur;
    if (wave * 32 < p.Cout_p) load_pass(wave * 32, cur);
    for (int m0 = wave * 32; m0 < p.Cout_p; m0 += 128) {   // 32 output channels per pass, passes dealt round-robin to the waves
        const int c0 = m0 + 16 * half;                      // the lane's 16 channels
        v4i cbias[4], cmul[4], cchi[4], cshm[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            cbias[i] = *(const v4i *)(p.bias3 + c0 + 4 * i); cmul[i] = *(const v4i *)(p.m0s3 + c0 + 4 * i);
            cchi[i] = *(const v4i *)(p.chi3 + c0 + 4 * i); cshm[i] = *(const v4i *)(p.shm13 + c0 + 4 * i);
        }
        PassOperands nxt;
        load_pass(m0 + 128 < p.Cout_p ? m0 + 128 : m0, nxt);   // the last pass fetches itself again
        v16i init;
#pragma unroll
        for (int i = 0; i < 16; ++i) init[i] = cbias[i >> 2][i & 3];
#pragma unroll
        for (int fn = 0; fn < NFR; ++fn) {
            const int o = fn * 32 + l;
            v16i a = init;
#pragma unroll
            for (int ksub = 0; ksub < 4; ++ksub) {
                const v4i fb = *(const v4i *)(&T[o * CM + (((ksub * 2 + half) ^ (o & 7)) << 4)]);
                a = __builtin_amdgcn_mfma_i32_32x32x32_i8(cur.fa[ksub], fb, a, 0, 0, 0);
            }
            int q[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int qc = clamp3(requant_q<TF>(a[i], cmul[i >> 2][i & 3], cchi[i >> 2][i & 3], cshm[i >> 2][i & 3]), p.lo3, 127);
                const int r8 = (int)(int8_t)((uint32_t)cur.res[fn][i >> 2] >> (8 * (i & 3)));
                q[i] = fused_add<TF>(qc, r8, ap);
            }
            if (opix[fn] >= 0)
                *(v4i *)(p.out + opix[fn] + c0) = v4i{(int)pack4(q[0], q[1], q[2], q[3]), (int)pack4(q[4], q[5], q[6], q[7]),
                                                     (int)pack4(q[8], q[9], q[10], q[11]), (int)pack4(q[12], q[13], q[14], q[15])};
        }
        cur = nxt;
    }
}

}  // namespace

// Geometry with this kernel: first convolution 1x1 (stride 1) from a multiple of 64 stored channels
// into 128; second 3x3 stride 1 pad 1, 128 -> 128; closing 1x1 from 128 back to the input's channel
// count (a multiple of 32) with the block input as residual.
bool bottleneck128_supported(int cin_p, int cmid_p, int cout_p) {
    return cmid_p == CM && cin_p % 64 == 0 && cin_p >= 64 && cin_p <= 2048 && cout_p == cin_p && cout_p % 32 == 0;
}

hipError_t launch_bottleneck128(const BneckParams &p, hipStream_t st) {
    if (p.B <= 0) return hipSuccess;
    if (!p.in || !p.out || !p.w1 || !p.w2 || !p.w3 || !p.zpad || p.H < 1 || p.W < 1 || !p.tail ||
        !bottleneck128_supported(p.Cin_p, CM, p.Cout_p))
        return hipErrorInvalidValue;
    const long tiles = (long)p.B * ((p.H + BT - 1) / BT) * ((p.W + BT - 1) / BT);
    if (tiles > 0x7fffffffL || (long)p.B * p.H * p.W * p.Cin_p >= (1L << 31)) return hipErrorInvalidValue;
    const dim3 grid((unsigned)tiles), block(256);
    set_kernel_name(p.tie_free ? "bottleneck128_kernel<true>" : "bottleneck128_kernel<false>");
    if (p.tie_free) hipLaunchKernelGGL((bottleneck128_kernel<true>), grid, block, 0, st, p);
    else hipLaunchKernelGGL((bottleneck128_kernel<false>), grid, block, 0, st, p);
    return hipGetLastError();
}

}  // namespace isr
