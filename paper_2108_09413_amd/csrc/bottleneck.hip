// Bottleneck residual block with 64 middle channels in one kernel:
//   t1 = clamp(requant(conv1x1(x)))                     Cin -> 64
//   t2 = clamp(requant(conv3x3(t1)))                    64 -> 64, stride 1, pad 1
//   y  = add_requant(clamp(requant(conv1x1(t2))), x)    64 -> Cout = Cin   (TAIL only)
// A workgroup of four waves makes a 14 x 14 pixel tile of one image.
//   1. The first convolution runs as a GEMM over the 16 x 16 halo pixels of the tile (each
//      wave 64 channels x 64 pixels = 2 x 2 v_mfma_i32_32x32x32_i8 tiles): K steps of 64
//      input channels go from global memory straight into two LDS stages.  Recomputing the
//      halo costs 31 % more of this (cheap) GEMM and saves writing and re-reading t1.
//   2. Its int8 result goes into an LDS tile [halo pixel][64 channels]; halo pixels outside
//      the image get t1's zero-point, the padding value of the 3x3 convolution.
//   3. The 3x3 convolution reads its pixel operands from that tile at tap-shifted addresses
//      (no gather from memory) and its weights from LDS (fetched while step 2 runs, into
//      the space of the two operand stages): 18 K steps of 32, no barrier inside.
//   4. HEAD: t2 is requantised and stored.  TAIL: the packed int8 t2 of a lane is exactly the
//      pixel operand of the last 1x1 convolution (16 consecutive channels per register
//      group), so each wave goes on alone: 64 output channels at a time, weights from
//      global memory (L1/L2 resident), residual x read at the tile's own pixels, y stored.
// x is read once (plus halo, mostly cache hits), t1 and t2 never leave the CU.
#include "conv_device.h"

namespace isr {

namespace {

constexpr int BT = 14;              // output tile edge
constexpr int BH = BT + 2;          // halo tile edge: 16 x 16 = 256 GEMM columns
constexpr int W2_CHUNKS = 37;       // 16-byte chunks per 3x3 weight row in LDS: 36 + 1 pad (bank spread)

template <bool TAIL, bool TF>
__global__ __launch_bounds__(256, 2) void bottleneck_kernel(const BneckParams p) {
    constexpr int KB = 64, STAGE = (64 + 256) * KB;
    static_assert(64 * W2_CHUNKS * 16 <= 2 * STAGE, "3x3 weights fit the operand stages");
    __shared__ __attribute__((aligned(16))) int8_t Ls[2 * STAGE];     // step 1: two stages (A rows, then B rows); step 3: 3x3 weights
    __shared__ __attribute__((aligned(16))) int8_t T1[BH * BH * 64];  // [halo pixel][channel chunk ^ swizzle]
    __shared__ int prm[2][4][64];                                     // bias, M0, chi, shift-1 of the first two convolutions
    __shared__ int prm3[TAIL ? 4 : 1][TAIL ? 256 : 1];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l = lane & 31, half = lane >> 5;
    // tiles that share halo rows run on the same XCD (workgroup ids are dealt round-robin over 8 XCDs)
    const int nblk = gridDim.x;
    const int xcd = blockIdx.x & 7, per = nblk >> 3, extra = nblk & 7;
    const int logical = xcd * per + (xcd < extra ? xcd : extra) + (blockIdx.x >> 3);
    const int tiles_x = (p.W + BT - 1) / BT, tiles_y = (p.H + BT - 1) / BT;
    const int b = logical / (tiles_x * tiles_y), t = logical % (tiles_x * tiles_y);
    const int oy0 = (t / tiles_x) * BT, ox0 = (t % tiles_x) * BT;     // first output pixel of the tile
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
        }

    // ---- step 1: t1 accumulators over the halo, K = Cin_p in steps of 64 ----
    // LDS position (row, col) of a stage holds K chunk col ^ swz(row); a lane fetches the same
    // chunk `cl` for all its rows (their numbers differ by multiples of 64)
    const int col = tid & 3, row0 = tid >> 2, cl = col ^ swz<4>(row0);
    const int8_t *wrow = p.w1 + (long)row0 * p.Cin_p + cl * 16;
    uint32_t boff[4];
    bool bok[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int h = row0 + 64 * j, y = y0 + (h >> 4), x = x0 + (h & 15);
        bok[j] = (unsigned)y < (unsigned)p.H && (unsigned)x < (unsigned)p.W;
        boff[j] = bok[j] ? (uint32_t)((((long)b * p.H + y) * p.W + x) * p.Cin_p + cl * 16) : 0u;
    }
    auto issue = [&](int ks, int buf) {
        int8_t *sa = &Ls[buf * STAGE + wave * 1024];
        ISR_GLOBAL_TO_LDS16(wrow + ks * KB, sa);
        int8_t *sb = sa + 64 * KB;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            // halo pixels outside the image: any readable bytes, their results are replaced in step 2
            const int8_t *src = bok[j] ? p.in + (boff[j] + (uint32_t)(ks * KB)) : p.zpad;
            ISR_GLOBAL_TO_LDS16(src, sb + j * 4096);
        }
    };
    __syncthreads();   // prm visible

    auto lane_c = [&](int fm) { return fm * 32 + 16 * half; };   // first of the lane's 16 channels in M fragment fm
    v16i acc[2][2];
#pragma unroll
    for (int fm = 0; fm < 2; ++fm) {
        v16i init;
#pragma unroll
        for (int i = 0; i < 16; ++i) init[i] = prm[0][0][lane_c(fm) + i];
        acc[fm][0] = acc[fm][1] = init;
    }
    int aoff[2][2], boffs[2][2];   // [K half of the step][fragment]
#pragma unroll
    for (int ksub = 0; ksub < 2; ++ksub) {
        const int c = ksub * 2 + half;
#pragma unroll
        for (int f = 0; f < 2; ++f) {
            const int ra = f * 32 + l, rb = wave * 64 + f * 32 + l;
            aoff[ksub][f] = ra * KB + ((c ^ swz<4>(ra)) << 4);
            boffs[ksub][f] = 64 * KB + rb * KB + ((c ^ swz<4>(rb)) << 4);
        }
    }
    const int nk = p.Cin_p / KB;
    issue(0, 0);
    if (nk > 1) issue(1, 1);            // both stages are free at the start
    for (int ks = 0; ks < nk; ++ks) {
        if (ks == 0 && nk > 1) wait_vmcnt<5>();   // step 0 landed; the 5 loads of step 1 may still be in flight
        else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();   // every wave's loads of step ks landed; every wave is done with step ks - 1
        if (ks >= 1 && ks + 1 < nk) issue(ks + 1, (ks + 1) & 1);
        const int8_t *base = &Ls[(ks & 1) * STAGE];
#pragma unroll
        for (int ksub = 0; ksub < 2; ++ksub) {
            v4i fa[2], fb[2];
#pragma unroll
            for (int f = 0; f < 2; ++f) {
                fa[f] = *(const v4i *)(base + aoff[ksub][f]);
                fb[f] = *(const v4i *)(base + boffs[ksub][f]);
            }
#pragma unroll
            for (int fm = 0; fm < 2; ++fm)
#pragma unroll
                for (int fn = 0; fn < 2; ++fn)
                    acc[fm][fn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[fm], fb[fn], acc[fm][fn], 0, 0, 0);
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
#pragma unroll
        for (int fn = 0; fn < 2; ++fn) {
            const int h = wave * 64 + fn * 32 + l, y = y0 + (h >> 4), x = x0 + (h & 15);
            const bool inside = (unsigned)y < (unsigned)p.H && (unsigned)x < (unsigned)p.W;
#pragma unroll
            for (int fm = 0; fm < 2; ++fm) {
                int q[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int c = lane_c(fm) + i;
                    q[i] = clamp3(requant_q<TF>(acc[fm][fn][i], prm[0][1][c], prm[0][2][c], prm[0][3][c]), p.lo1, 127);
                }
                v4i v = {(int)pack4(q[0], q[1], q[2], q[3]), (int)pack4(q[4], q[5], q[6], q[7]),
                         (int)pack4(q[8], q[9], q[10], q[11]), (int)pack4(q[12], q[13], q[14], q[15])};
                if (!inside) v = v4i{(int)zt, (int)zt, (int)zt, (int)zt};
                *(v4i *)(&T1[h * 64 + (((2 * fm + half) ^ swz<4>(h)) << 4)]) = v;
            }
        }
    }
    wait_vmcnt<0>();
    __syncthreads();   // t1 tile and 3x3 weights in LDS

    // ---- step 3: 3x3 convolution from LDS ----
    int hb[2];         // halo pixel of tap (0, 0) of the lane's output pixel in N fragment fn
    bool ostore[2];
    int opix[2];
#pragma unroll
    for (int fn = 0; fn < 2; ++fn) {
        const int o = wave * 64 + fn * 32 + l;
        const bool real = o < BT * BT;
        const int oo = real ? o : 0, oy = oo / BT, ox = oo % BT;
        hb[fn] = oy * BH + ox;
        ostore[fn] = real && oy0 + oy < p.H && ox0 + ox < p.W;
        opix[fn] = ostore[fn] ? ((b * p.H + oy0 + oy) * p.W + ox0 + ox) : 0;
    }
    // tail operands of 64 output channels from m0 on: residual x at the lane's pixels, weight fragments.
    // Fetched one pass ahead (the first before the 3x3 convolution) so that the loads' latency is covered.
    auto load_pass = [&](int m0, v4i (&res)[2][2], v4i (&fa)[2][2]) {
#pragma unroll
        for (int fm = 0; fm < 2; ++fm)
#pragma unroll
            for (int fn = 0; fn < 2; ++fn)   // pixels that are not stored read pixel 0 of the tensor: in bounds, unused
                res[fm][fn] = *(const v4i *)(p.in + (long)opix[fn] * p.Cin_p + m0 + lane_c(fm));
#pragma unroll
        for (int ksub = 0; ksub < 2; ++ksub)
#pragma unroll
            for (int fm = 0; fm < 2; ++fm)
                fa[ksub][fm] = *(const v4i *)(p.w3 + (long)(m0 + fm * 32 + l) * 64 + ksub * 32 + half * 16);
    };
    v4i res_cur[2][2], fa_cur[2][2];
    if constexpr (TAIL) load_pass(0, res_cur, fa_cur);
    // the 196 output pixels fill 6 1/8 fragments of 32: the last wave's second fragment holds none
    const bool two = wave * 64 + 32 < BT * BT;   // wave-uniform
#pragma unroll
    for (int fm = 0; fm < 2; ++fm) {
        v16i init;
#pragma unroll
        for (int i = 0; i < 16; ++i) init[i] = prm[1][0][lane_c(fm) + i];
        acc[fm][0] = acc[fm][1] = init;
    }
#pragma unroll
    for (int ks = 0; ks < 18; ++ks) {
        const int tap = ks >> 1, ky = tap / 3, kx = tap % 3, cc = (ks & 1) * 2 + half;
        v4i fa[2], fb[2];
#pragma unroll
        for (int fm = 0; fm < 2; ++fm) fa[fm] = *(const v4i *)(&Ls[((fm * 32 + l) * W2_CHUNKS + 2 * ks + half) * 16]);
#pragma unroll
        for (int fn = 0; fn < 2; ++fn) {
            const int hp = hb[fn] + ky * BH + kx;
            fb[fn] = *(const v4i *)(&T1[hp * 64 + ((cc ^ swz<4>(hp)) << 4)]);
        }
#pragma unroll
        for (int fm = 0; fm < 2; ++fm) {
            acc[fm][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[fm], fb[0], acc[fm][0], 0, 0, 0);
            if (two) acc[fm][1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[fm], fb[1], acc[fm][1], 0, 0, 0);
        }
    }

    // ---- step 4: requantise t2 ----
    v4i t2[2][2];
#pragma unroll
    for (int fm = 0; fm < 2; ++fm)
#pragma unroll
        for (int fn = 0; fn < 2; ++fn) {
            if (fn == 1 && !two) { t2[fm][fn] = v4i{0, 0, 0, 0}; continue; }
            int q[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int c = lane_c(fm) + i;
                q[i] = clamp3(requant_q<TF>(acc[fm][fn][i], prm[1][1][c], prm[1][2][c], prm[1][3][c]), p.lo2, 127);
            }
            t2[fm][fn] = v4i{(int)pack4(q[0], q[1], q[2], q[3]), (int)pack4(q[4], q[5], q[6], q[7]),
                             (int)pack4(q[8], q[9], q[10], q[11]), (int)pack4(q[12], q[13], q[14], q[15])};
        }
    if constexpr (!TAIL) {
#pragma unroll
        for (int fm = 0; fm < 2; ++fm)
#pragma unroll
            for (int fn = 0; fn < 2; ++fn)
                if (ostore[fn]) *(v4i *)(p.out + (long)opix[fn] * 64 + lane_c(fm)) = t2[fm][fn];
    } else {
        // ---- last 1x1 convolution + residual add, 64 output channels per pass; this wave's 64 pixels ----
        ConvParams ap{};   // the fused add reads its constants from here
        ap.add_mul_self = p.add_mul_self; ap.add_mul_res = p.add_mul_res; ap.add_c0 = p.add_c0; ap.add_k = p.add_k;
        ap.add_sh = p.add_sh; ap.add_lo = p.add_lo;
        for (int m0 = 0; m0 < p.Cout_p; m0 += 64) {
            v4i res[2][2], fa[2][2], res_next[2][2], fa_next[2][2];
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int v = 0; v < 2; ++v) { res[u][v] = res_cur[u][v]; fa[u][v] = fa_cur[u][v]; }
            load_pass(m0 + 64 < p.Cout_p ? m0 + 64 : m0, res_next, fa_next);   // the last pass fetches itself again
#pragma unroll
            for (int fm = 0; fm < 2; ++fm) {
                v16i init;
#pragma unroll
                for (int i = 0; i < 16; ++i) init[i] = prm3[0][m0 + lane_c(fm) + i];
                acc[fm][0] = acc[fm][1] = init;
            }
#pragma unroll
            for (int ksub = 0; ksub < 2; ++ksub)
#pragma unroll
                for (int fm = 0; fm < 2; ++fm)
#pragma unroll
                    for (int fn = 0; fn < 2; ++fn)
                        if (fn == 0 || two)
                            acc[fm][fn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[ksub][fm], t2[ksub][fn], acc[fm][fn], 0, 0, 0);
#pragma unroll
            for (int fm = 0; fm < 2; ++fm) {
                int mm[16], ch[16], ss[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int c = m0 + lane_c(fm) + i;
                    mm[i] = prm3[1][c]; ch[i] = prm3[2][c]; ss[i] = prm3[3][c];
                }
#pragma unroll
                for (int fn = 0; fn < 2; ++fn) {
                    if (fn == 1 && !two) continue;
                    int q[16];
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int qc = clamp3(requant_q<TF>(acc[fm][fn][i], mm[i], ch[i], ss[i]), p.lo3, 127);
                        const int r8 = (int)(int8_t)((uint32_t)res[fm][fn][i >> 2] >> (8 * (i & 3)));
                        q[i] = fused_add<TF>(qc, r8, ap);
                    }
                    if (ostore[fn])
                        *(v4i *)(p.out + (long)opix[fn] * p.Cout_p + m0 + lane_c(fm)) =
                            v4i{(int)pack4(q[0], q[1], q[2], q[3]), (int)pack4(q[4], q[5], q[6], q[7]),
                                (int)pack4(q[8], q[9], q[10], q[11]), (int)pack4(q[12], q[13], q[14], q[15])};
                }
            }
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int v = 0; v < 2; ++v) { res_cur[u][v] = res_next[u][v]; fa_cur[u][v] = fa_next[u][v]; }
        }
    }
}

}  // namespace

// Geometry with a kernel: first convolution 1x1 (stride 1) from a multiple of 64 stored channels
// into 64; second 3x3 stride 1 pad 1, 64 -> 64; optional tail 1x1 from 64 back to the input's
// channel count (at most 256) with the block input as residual.
bool bottleneck_supported(int cin_p, int cmid_p, int cout_p, int tail) {
    if (cin_p % 64 != 0 || cin_p < 64 || cin_p > 1024 || cmid_p != 64) return false;
    return !tail || (cout_p == cin_p && cout_p <= 256);
}

hipError_t launch_bottleneck(const BneckParams &p, hipStream_t st) {
    if (p.B <= 0) return hipSuccess;
    if (!p.in || !p.out || !p.w1 || !p.w2 || !p.zpad || p.H < 1 || p.W < 1 ||
        !bottleneck_supported(p.Cin_p, 64, p.Cout_p, p.tail) || (p.tail && !p.w3))
        return hipErrorInvalidValue;
    const long tiles = (long)p.B * ((p.H + BT - 1) / BT) * ((p.W + BT - 1) / BT);
    if (tiles > 0x7fffffffL || (long)p.B * p.H * p.W * (p.Cin_p > 64 ? p.Cin_p : 64) >= (1L << 31)) return hipErrorInvalidValue;
    const dim3 grid((unsigned)tiles), block(256);
    set_kernel_name(p.tail ? (p.tie_free ? "bottleneck_kernel<true, true>" : "bottleneck_kernel<true, false>")
                           : (p.tie_free ? "bottleneck_kernel<false, true>" : "bottleneck_kernel<false, false>"));
    if (p.tail) {
        if (p.tie_free) hipLaunchKernelGGL((bottleneck_kernel<true, true>), grid, block, 0, st, p);
        else hipLaunchKernelGGL((bottleneck_kernel<true, false>), grid, block, 0, st, p);
    } else {
        if (p.tie_free) hipLaunchKernelGGL((bottleneck_kernel<false, true>), grid, block, 0, st, p);
        else hipLaunchKernelGGL((bottleneck_kernel<false, false>), grid, block, 0, st, p);
    }
    return hipGetLastError();
}

}  // namespace isr
