// The closing 1x1 convolution + residual add of a bottleneck block with 128 middle channels and the opening
// 1x1 convolution of the NEXT block in one kernel: y = add(requant(W3 t2), x) is written once and the next
// block's t1' = relu(requant(W1' y)) is computed from the copy of y that is still in LDS, so the 512-channel
// tensor is not read back from memory by a second kernel.
//
// A workgroup of eight waves owns 32 consecutive pixels with ALL 512 channels and walks over such tiles
// (persistent grid).  Per tile:
//   * x (32 x 512 bytes) and t2 (32 x 128 bytes) arrive by direct-to-LDS loads two tiles ahead (three buffers);
//   * expand: wave w computes channels 64 w .. 64 w + 63 of the 32 pixels (two 32x32x32 MFMA tiles, K = 128);
//     its weight fragments stay in registers for the whole launch (fragment-major copy of the weights, made
//     when the model is loaded), the pixel fragments come from the t2 tile;
//   * the epilogue requantises, reads the residual from the x tile, adds, writes y to memory AND over x in LDS;
//   * reduce: wave w computes output channels 16 w .. 16 w + 15 of the 32 pixels with v_mfma_i32_16x16x64_i8
//     over K = 512 channels of the y tile (its weight fragments, too, stay in registers), requantises and
//     stores t1'.
// Two barriers per tile.  LDS rows of the x / y tile are 512 bytes: 16-byte chunk c of pixel p sits at chunk
// c ^ (p & 15), so that 16 consecutive pixels reading one logical chunk cover the 64 banks exactly once, for the
// epilogue's 32x32 layout and for the 16x16x64 fragment reads alike.
//
// A second kernel does the same for a stage's FIRST block, whose residual is not a stored tensor but a projection
// 1x1 convolution (256 -> 512 channels) of the block input: y = add(requant(W3 t2), requant(Wp x0)).  Sixteen waves,
// 32 channels each, hold the fragments of all three weight matrices; x0 (32 x 256 bytes) takes the place of x
// among the loads and the y tile is written, not overwritten.
#include "conv_device.h"

namespace isr {

namespace {

constexpr int XK1 = 128, XC = 512, XN2 = 128, XPX = 32, XNW = 8, XNT = XNW * 64;
constexpr int XNB = 3;   // tile buffers: loads run two tiles ahead
typedef int v4acc __attribute__((ext_vector_type(4)));

template <bool TFA>
__global__ __launch_bounds__(XNT, 4) void expand_reduce_kernel(const XrParams p) {
    __shared__ __attribute__((aligned(256))) int8_t XY[XNB][XPX * XC];
    __shared__ __attribute__((aligned(16))) int8_t T2[XNB][XPX * XK1];
    __shared__ __attribute__((aligned(16))) int prm1[4][XC];    // bias, M0, chi, shift-1 of the expanding convolution
    __shared__ __attribute__((aligned(16))) int prm2[4][XN2];   // the same of the reducing convolution

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ntiles = (p.npix + XPX - 1) / XPX, G = gridDim.x;
    const uint32_t xy_lds = lds_address(&XY[0][0]), t2_lds = lds_address(&T2[0][0]);

    // direct-to-LDS loads of a tile: wave-load q of the x tile covers pixels 2 q, 2 q + 1 (wave w issues q = 2 w,
    // 2 w + 1); wave-load q of the t2 tile covers pixels 8 q .. 8 q + 7 (waves 0 .. 3).  Pixels past the end
    // re-read the last pixel; their results are never stored.
    auto issue_tile = [&](int tile, int buf) {
        const int n0 = tile * XPX;
        int l = lane;
        asm volatile("" : "+v"(l));   // recompute the per-lane offsets per call: kept across the tile loop they would be spilled
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int q = 2 * wave + j, px = 2 * q + (l >> 5), c = (l & 31) ^ (px & 15);
            int n = n0 + px;
            n = n < p.npix ? n : p.npix - 1;
            ISR_GLOBAL_TO_LDS16_AT(p.x + ((uint32_t)n * (uint32_t)XC + (uint32_t)(c * 16)), xy_lds + buf * (XPX * XC) + q * 1024);
        }
        if (wave < 4) {
            const int row = 8 * wave + (l >> 3), c = (l & 7) ^ swz<8>(row);
            int n = n0 + row;
            n = n < p.npix ? n : p.npix - 1;
            ISR_GLOBAL_TO_LDS16_AT(p.t2 + ((uint32_t)n * (uint32_t)XK1 + (uint32_t)(c * 16)), t2_lds + buf * (XPX * XK1) + wave * 1024);
        }
    };

    int tile = blockIdx.x;
    if (tile < ntiles) issue_tile(tile, 0);
    if (tile + G < ntiles) issue_tile(tile + G, 1);
    for (int i = tid; i < XC; i += XNT) {
        prm1[0][i] = p.bias1[i]; prm1[1][i] = p.m0s1[i]; prm1[2][i] = p.chi1[i]; prm1[3][i] = p.shm11[i];
    }
    if (tid < XN2) {
        prm2[0][tid] = p.bias2[tid]; prm2[1][tid] = p.m0s2[tid]; prm2[2][tid] = p.chi2[tid]; prm2[3][tid] = p.shm12[tid];
    }
    // weight fragments, kept in registers for the whole launch: expand [fm][ksub] (32 output channels x 32 K bytes
    // each), reduce [kstep] (16 output channels x 64 K bytes each)
    const uint32_t lane16 = (uint32_t)lane * 16;
    v4i a1[2][XK1 / 32], a2[XC / 64];
#pragma unroll
    for (int fm = 0; fm < 2; ++fm)
#pragma unroll
        for (int ks = 0; ks < XK1 / 32; ++ks)
            a1[fm][ks] = *(const v4i *)(p.a1 + (size_t)wave * (2 * (XK1 / 32) * 1024) + (lane16 + (uint32_t)((fm * (XK1 / 32) + ks) * 1024)));
#pragma unroll
    for (int ks = 0; ks < XC / 64; ++ks) a2[ks] = *(const v4i *)(p.a2 + (size_t)wave * (XC / 64) * 1024 + (lane16 + (uint32_t)(ks * 1024)));
    wait_vmcnt<0>();
    __syncthreads();   // the constants are in LDS, the first tile has landed

    int buf = 0;
    for (int it = 0; tile < ntiles; tile += G, ++it) {
        const int n0 = tile * XPX;
        // per-lane positions, recomputed per tile (a handful of instructions) instead of held in registers next to the
        // 64 registers of weight fragments
        int l = lane;
        asm volatile("" : "+v"(l));
        const int half = l >> 5, px1 = l & 31;            // expand: the lane's pixel and channel half
        const int g = l >> 4, px2 = l & 15;               // reduce: the lane's K / channel group and pixel
        const int b_off1 = px1 * XK1 + ((half ^ swz<8>(px1)) << 4);   // t2 fragment of K sub-step 0; sub-step k flips bits 5..6 by k
        const bool prefetch = tile + 2 * G < ntiles;
        if (it > 0) {
            // The loads of this tile were issued two tiles ago.  Vector memory operations complete in issue order, so
            // they have landed once at most the operations issued after them are outstanding: the four stores of each of
            // the two tiles since, and the loads of the tile issued one tile ago (three for waves 0 .. 3, two for the
            // others).  Where the sequence differs (the second tile, which has one tile of stores behind it) the wave
            // waits for everything.
            if (it >= 2 && tile + G < ntiles) {
                if (wave < 4) wait_vmcnt<11>();
                else wait_vmcnt<10>();
            } else {
                wait_vmcnt<0>();
            }
            __builtin_amdgcn_s_barrier();    // every wave's loads of this tile landed; every wave is done with the previous tile's buffers
        }
        if (prefetch) issue_tile(tile + 2 * G, buf >= 1 ? buf - 1 : XNB - 1);   // the buffer of the previous tile

        // ---- expand: 64 channels x 32 pixels per wave, 32 channels at a time ----
        const int8_t *t2b = T2[buf];
        int8_t *xyb = XY[buf];
        const long n1 = (long)n0 + px1;
#pragma unroll
        for (int fm = 0; fm < 2; ++fm) {
            const int oc = wave * 64 + fm * 32 + half * 16;
            v16i acc;
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = prm1[0][oc + i];
#pragma unroll
            for (int ks = 0; ks < XK1 / 32; ++ks) {
                const v4i fb = *(const v4i *)(t2b + (b_off1 ^ (ks << 5)));
                acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1[fm][ks], fb, acc, 0, 0, 0);
            }
            int8_t *cell = xyb + px1 * XC + ((((oc >> 4)) ^ (px1 & 15)) << 4);
            const v4i rv = *(const v4i *)cell;
            v4i yv;
            // four channels at a time: their constants are three 16-byte LDS reads, the results one packed dword
#pragma unroll
            for (int gi = 0; gi < 4; ++gi) {
                const v4i mm = *(const v4i *)&prm1[1][oc + 4 * gi], ch = *(const v4i *)&prm1[2][oc + 4 * gi], ss = *(const v4i *)&prm1[3][oc + 4 * gi];
                int q[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int v = clamp3(requant_tie_free(acc[4 * gi + i], mm[i], ch[i], ss[i]), p.lo1, 127);
                    const int r8 = (int)(int8_t)((uint32_t)rv[gi] >> (8 * i));
                    if constexpr (TFA) {
                        const int s = __mul24(v, p.add_mul_self) + (p.add_c0 + p.add_k) + __mul24(r8, p.add_mul_res);
                        q[i] = clamp3(s >> p.add_sh, p.add_lo, 127);
                    } else {
                        const int s = __mul24(v, p.add_mul_self) + p.add_c0 + __mul24(r8, p.add_mul_res);
                        q[i] = clamp3((s + p.add_k + (s >> 31)) >> p.add_sh, p.add_lo, 127);
                    }
                }
                yv[gi] = (int)pack4(q[0], q[1], q[2], q[3]);
            }
            *(v4i *)cell = yv;
            if (n1 < p.npix) *(v4i *)(p.y + n1 * XC + oc) = yv;
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // this wave's part of the y tile is in LDS (its stores to memory may still be under way)
        __builtin_amdgcn_s_barrier();                         // the y tile is complete
        asm volatile("" ::: "memory");

        // ---- reduce: 16 channels x 32 pixels per wave, K = 512 channels of the y tile ----
        v4acc acc2[2];
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc2[nb][i] = prm2[0][wave * 16 + g * 4 + i];
#pragma unroll
        for (int ks = 0; ks < XC / 64; ++ks) {
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                const int px = px2 + 16 * nb;
                const v4i fb = *(const v4i *)(xyb + px * XC + (((4 * ks + g) ^ px2) << 4));
                acc2[nb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a2[ks], fb, acc2[nb], 0, 0, 0);
            }
        }
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
            const long n2 = (long)n0 + px2 + 16 * nb;
            int q[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int c = wave * 16 + g * 4 + i;
                q[i] = clamp3(requant_tie_free(acc2[nb][i], prm2[1][c], prm2[2][c], prm2[3][c]), p.lo2, 127);
            }
            if (n2 < p.npix) *(uint32_t *)(p.t1n + n2 * XN2 + wave * 16 + g * 4) = pack4(q[0], q[1], q[2], q[3]);
        }
        buf = buf + 1 == XNB ? 0 : buf + 1;
    }
}

// ---- the same with the residual computed by a projection convolution of the block input ----

constexpr int XPK = 256, XNW2 = 16, XNT2 = XNW2 * 64;

template <bool TFA>
__global__ __launch_bounds__(XNT2, 4) void proj_expand_reduce_kernel(const XrParams p) {
    __shared__ __attribute__((aligned(256))) int8_t Y[XPX * XC];
    __shared__ __attribute__((aligned(256))) int8_t X0[XNB][XPX * XPK];
    __shared__ __attribute__((aligned(16))) int8_t T2[XNB][XPX * XK1];
    __shared__ __attribute__((aligned(16))) int prm1[4][XC];    // bias, M0, chi, shift-1 of the expanding convolution
    __shared__ __attribute__((aligned(16))) int prmp[4][XC];    // of the projection
    __shared__ __attribute__((aligned(16))) int prm2[4][XN2];   // of the reducing convolution

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ntiles = (p.npix + XPX - 1) / XPX, G = gridDim.x;
    const uint32_t x0_lds = lds_address(&X0[0][0]), t2_lds = lds_address(&T2[0][0]);

    // direct-to-LDS loads of a tile: wave-load q of the x0 tile covers pixels 4 q .. 4 q + 3 (waves 0 .. 7), wave-load q
    // of the t2 tile pixels 8 q .. 8 q + 7 (waves 8 .. 11)
    auto issue_tile = [&](int tile, int buf) {
        const int n0 = tile * XPX;
        int l = lane;
        asm volatile("" : "+v"(l));   // recompute the per-lane offsets per call: kept across the tile loop they would be spilled
        if (wave < 8) {
            const int px = 4 * wave + (l >> 4), c = (l & 15) ^ (px & 15);
            int n = n0 + px;
            n = n < p.npix ? n : p.npix - 1;
            // the projection may be strided: output pixel (b, y, x) reads input pixel (b, s y, s x)
            const int HoWo = p.Ho * p.Wo, b = n / HoWo, rem = n - b * HoWo, y = rem / p.Wo, x = rem - y * p.Wo;
            const uint32_t src = (uint32_t)((b * p.Hin + y * p.pstride) * p.Win + x * p.pstride);
            ISR_GLOBAL_TO_LDS16_AT(p.in2 + (src * (uint32_t)XPK + (uint32_t)(c * 16)), x0_lds + buf * (XPX * XPK) + wave * 1024);
        } else if (wave < 12) {
            const int q = wave - 8, row = 8 * q + (l >> 3), c = (l & 7) ^ swz<8>(row);
            int n = n0 + row;
            n = n < p.npix ? n : p.npix - 1;
            ISR_GLOBAL_TO_LDS16_AT(p.t2 + ((uint32_t)n * (uint32_t)XK1 + (uint32_t)(c * 16)), t2_lds + buf * (XPX * XK1) + q * 1024);
        }
    };

    int tile = blockIdx.x;
    if (tile < ntiles) issue_tile(tile, 0);
    if (tile + G < ntiles) issue_tile(tile + G, 1);
    for (int i = tid; i < XC; i += XNT2) {
        prm1[0][i] = p.bias1[i]; prm1[1][i] = p.m0s1[i]; prm1[2][i] = p.chi1[i]; prm1[3][i] = p.shm11[i];
        prmp[0][i] = p.biasp[i]; prmp[1][i] = p.m0sp[i]; prmp[2][i] = p.chip[i]; prmp[3][i] = p.shm1p[i];
    }
    if (tid < XN2) {
        prm2[0][tid] = p.bias2[tid]; prm2[1][tid] = p.m0s2[tid]; prm2[2][tid] = p.chi2[tid]; prm2[3][tid] = p.shm12[tid];
    }
    // weight fragments, kept in registers for the whole launch: wave w owns channels 32 w .. 32 w + 31 of the expanding
    // convolution [ksub] and of the projection [ksub], and 16 channels x 16 pixels of the reducing convolution [kstep]
    const uint32_t lane16 = (uint32_t)lane * 16;
    v4i a1[XK1 / 32], ap[XPK / 32], a2[XC / 64];
#pragma unroll
    for (int ks = 0; ks < XK1 / 32; ++ks) a1[ks] = *(const v4i *)(p.a1 + (size_t)wave * (XK1 / 32) * 1024 + (lane16 + (uint32_t)(ks * 1024)));
#pragma unroll
    for (int ks = 0; ks < XPK / 32; ++ks) ap[ks] = *(const v4i *)(p.ap + (size_t)wave * (XPK / 32) * 1024 + (lane16 + (uint32_t)(ks * 1024)));
#pragma unroll
    for (int ks = 0; ks < XC / 64; ++ks) a2[ks] = *(const v4i *)(p.a2 + (size_t)(wave >> 1) * (XC / 64) * 1024 + (lane16 + (uint32_t)(ks * 1024)));
    wait_vmcnt<0>();
    __syncthreads();   // the constants are in LDS, the first tile has landed

    int buf = 0;
    for (int it = 0; tile < ntiles; tile += G, ++it) {
        const int n0 = tile * XPX;
        const bool prefetch = tile + 2 * G < ntiles;
        if (it > 0) {
            // as in expand_reduce_kernel: since this tile's loads, a wave has issued two stores per tile for two tiles and
            // the load of the next tile (waves 0 .. 11)
            if (it >= 2 && tile + G < ntiles) {
                if (wave < 12) wait_vmcnt<5>();
                else wait_vmcnt<4>();
            } else {
                wait_vmcnt<0>();
            }
            __builtin_amdgcn_s_barrier();    // every wave's loads of this tile landed; every wave is done with the previous tile
        }
        if (prefetch) issue_tile(tile + 2 * G, buf >= 1 ? buf - 1 : XNB - 1);

        int l = lane;
        asm volatile("" : "+v"(l));
        const int half = l >> 5, px1 = l & 31;
        const int g = l >> 4, px2 = l & 15;
        const int oc = wave * 32 + half * 16;

        // ---- projection of the block input: the residual, 32 channels x 32 pixels per wave, kept packed ----
        v4i rq;
        {
            v16i acc;
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = prmp[0][oc + i];
            const int8_t *xb = X0[buf];
            const int x_off = px1 * XPK + ((half ^ (px1 & 15)) << 4);   // chunk (2 k + half) ^ (px & 15): sub-step k flips bits 5..7 by k
#pragma unroll
            for (int ks = 0; ks < XPK / 32; ++ks) {
                const v4i fb = *(const v4i *)(xb + (x_off ^ (ks << 5)));
                acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(ap[ks], fb, acc, 0, 0, 0);
            }
#pragma unroll
            for (int gi = 0; gi < 4; ++gi) {
                __builtin_amdgcn_sched_barrier(0);   // one group's constants at a time: the registers are needed for weight fragments
                const v4i mm = *(const v4i *)&prmp[1][oc + 4 * gi], ch = *(const v4i *)&prmp[2][oc + 4 * gi], ss = *(const v4i *)&prmp[3][oc + 4 * gi];
                int q[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) q[i] = clamp3(requant_tie_free(acc[4 * gi + i], mm[i], ch[i], ss[i]), p.lop, 127);
                rq[gi] = (int)pack4(q[0], q[1], q[2], q[3]);
            }
        }
        // ---- expand + add ----
        {
            v16i acc;
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = prm1[0][oc + i];
            const int8_t *t2b = T2[buf];
            const int b_off1 = px1 * XK1 + ((half ^ swz<8>(px1)) << 4);
#pragma unroll
            for (int ks = 0; ks < XK1 / 32; ++ks) {
                const v4i fb = *(const v4i *)(t2b + (b_off1 ^ (ks << 5)));
                acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1[ks], fb, acc, 0, 0, 0);
            }
            v4i yv;
#pragma unroll
            for (int gi = 0; gi < 4; ++gi) {
                __builtin_amdgcn_sched_barrier(0);
                const v4i mm = *(const v4i *)&prm1[1][oc + 4 * gi], ch = *(const v4i *)&prm1[2][oc + 4 * gi], ss = *(const v4i *)&prm1[3][oc + 4 * gi];
                int q[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int v = clamp3(requant_tie_free(acc[4 * gi + i], mm[i], ch[i], ss[i]), p.lo1, 127);
                    const int r8 = (int)(int8_t)((uint32_t)rq[gi] >> (8 * i));
                    if constexpr (TFA) {
                        const int s = __mul24(v, p.add_mul_self) + (p.add_c0 + p.add_k) + __mul24(r8, p.add_mul_res);
                        q[i] = clamp3(s >> p.add_sh, p.add_lo, 127);
                    } else {
                        const int s = __mul24(v, p.add_mul_self) + p.add_c0 + __mul24(r8, p.add_mul_res);
                        q[i] = clamp3((s + p.add_k + (s >> 31)) >> p.add_sh, p.add_lo, 127);
                    }
                }
                yv[gi] = (int)pack4(q[0], q[1], q[2], q[3]);
            }
            *(v4i *)(Y + px1 * XC + (((oc >> 4) ^ (px1 & 15)) << 4)) = yv;
            const long n1 = (long)n0 + px1;
            if (n1 < p.npix) *(v4i *)(p.y + n1 * XC + oc) = yv;
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // this wave's part of the y tile is in LDS
        __builtin_amdgcn_s_barrier();                         // the y tile is complete
        asm volatile("" ::: "memory");

        // ---- reduce: wave w computes channels 16 (w / 2) .. + 15 of pixels 16 (w % 2) .. + 15 ----
        {
            const int mb = wave >> 1, px = px2 + 16 * (wave & 1);
            v4acc acc2;
#pragma unroll
            for (int i = 0; i < 4; ++i) acc2[i] = prm2[0][mb * 16 + g * 4 + i];
#pragma unroll
            for (int ks = 0; ks < XC / 64; ++ks) {
                const v4i fb = *(const v4i *)(Y + px * XC + (((4 * ks + g) ^ px2) << 4));
                acc2 = __builtin_amdgcn_mfma_i32_16x16x64_i8(a2[ks], fb, acc2, 0, 0, 0);
            }
            int q[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int c = mb * 16 + g * 4 + i;
                q[i] = clamp3(requant_tie_free(acc2[i], prm2[1][c], prm2[2][c], prm2[3][c]), p.lo2, 127);
            }
            const long n2 = (long)n0 + px;
            if (n2 < p.npix) *(uint32_t *)(p.t1n + n2 * XN2 + mb * 16 + g * 4) = pack4(q[0], q[1], q[2], q[3]);
        }
        buf = buf + 1 == XNB ? 0 : buf + 1;
    }
}

// ---- identity block followed by a block with 256 middle channels (the first block of the next stage) ----
// As expand_reduce_kernel, but the reducing convolution has 256 outputs: sixteen waves, wave w owns channels
// 32 w .. 32 w + 31 of the expanding convolution and channels 16 w .. 16 w + 15 (all 32 pixels) of the reducing one.

constexpr int XN2W = 256;

template <bool TFA>
__global__ __launch_bounds__(XNT2, 4) void expand_reduce256_kernel(const XrParams p) {
    __shared__ __attribute__((aligned(256))) int8_t XY[XNB][XPX * XC];
    __shared__ __attribute__((aligned(16))) int8_t T2[XNB][XPX * XK1];
    __shared__ __attribute__((aligned(16))) int prm1[4][XC];     // bias, M0, chi, shift-1 of the expanding convolution
    __shared__ __attribute__((aligned(16))) int prm2[4][XN2W];   // of the reducing convolution

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ntiles = (p.npix + XPX - 1) / XPX, G = gridDim.x;
    const uint32_t xy_lds = lds_address(&XY[0][0]), t2_lds = lds_address(&T2[0][0]);

    // direct-to-LDS loads of a tile: wave w fetches pixels 2 w, 2 w + 1 of the x tile, waves 0 .. 3 also pixels
    // 8 w .. 8 w + 7 of the t2 tile
    auto issue_tile = [&](int tile, int buf) {
        const int n0 = tile * XPX;
        int l = lane;
        asm volatile("" : "+v"(l));   // recompute the per-lane offsets per call: kept across the tile loop they would be spilled
        {
            const int px = 2 * wave + (l >> 5), c = (l & 31) ^ (px & 15);
            int n = n0 + px;
            n = n < p.npix ? n : p.npix - 1;
            ISR_GLOBAL_TO_LDS16_AT(p.x + ((uint32_t)n * (uint32_t)XC + (uint32_t)(c * 16)), xy_lds + buf * (XPX * XC) + wave * 1024);
        }
        if (wave < 4) {
            const int row = 8 * wave + (l >> 3), c = (l & 7) ^ swz<8>(row);
            int n = n0 + row;
            n = n < p.npix ? n : p.npix - 1;
            ISR_GLOBAL_TO_LDS16_AT(p.t2 + ((uint32_t)n * (uint32_t)XK1 + (uint32_t)(c * 16)), t2_lds + buf * (XPX * XK1) + wave * 1024);
        }
    };

    int tile = blockIdx.x;
    if (tile < ntiles) issue_tile(tile, 0);
    if (tile + G < ntiles) issue_tile(tile + G, 1);
    for (int i = tid; i < XC; i += XNT2) {
        prm1[0][i] = p.bias1[i]; prm1[1][i] = p.m0s1[i]; prm1[2][i] = p.chi1[i]; prm1[3][i] = p.shm11[i];
    }
    if (tid < XN2W) {
        prm2[0][tid] = p.bias2[tid]; prm2[1][tid] = p.m0s2[tid]; prm2[2][tid] = p.chi2[tid]; prm2[3][tid] = p.shm12[tid];
    }
    const uint32_t lane16 = (uint32_t)lane * 16;
    v4i a1[XK1 / 32], a2[XC / 64];   // weight fragments, kept in registers for the whole launch
#pragma unroll
    for (int ks = 0; ks < XK1 / 32; ++ks) a1[ks] = *(const v4i *)(p.a1 + (size_t)wave * (XK1 / 32) * 1024 + (lane16 + (uint32_t)(ks * 1024)));
#pragma unroll
    for (int ks = 0; ks < XC / 64; ++ks) a2[ks] = *(const v4i *)(p.a2 + (size_t)wave * (XC / 64) * 1024 + (lane16 + (uint32_t)(ks * 1024)));
    wait_vmcnt<0>();
    __syncthreads();   // the constants are in LDS, the first tile has landed

    int buf = 0;
    for (int it = 0; tile < ntiles; tile += G, ++it) {
        const int n0 = tile * XPX;
        const bool prefetch = tile + 2 * G < ntiles;
        if (it > 0) {
            // as in expand_reduce_kernel: since this tile's loads, a wave has issued three stores per tile for two tiles and
            // the loads of the next tile (two for waves 0 .. 3, one for the others)
            if (it >= 2 && tile + G < ntiles) {
                if (wave < 4) wait_vmcnt<8>();
                else wait_vmcnt<7>();
            } else {
                wait_vmcnt<0>();
            }
            __builtin_amdgcn_s_barrier();    // every wave's loads of this tile landed; every wave is done with the previous tile
        }
        if (prefetch) issue_tile(tile + 2 * G, buf >= 1 ? buf - 1 : XNB - 1);

        int l = lane;
        asm volatile("" : "+v"(l));
        const int half = l >> 5, px1 = l & 31;
        const int g = l >> 4, px2 = l & 15;
        const int oc = wave * 32 + half * 16;
        int8_t *xyb = XY[buf];

        // ---- expand + add: 32 channels x 32 pixels per wave ----
        {
            v16i acc;
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = prm1[0][oc + i];
            const int8_t *t2b = T2[buf];
            const int b_off1 = px1 * XK1 + ((half ^ swz<8>(px1)) << 4);
#pragma unroll
            for (int ks = 0; ks < XK1 / 32; ++ks) {
                const v4i fb = *(const v4i *)(t2b + (b_off1 ^ (ks << 5)));
                acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1[ks], fb, acc, 0, 0, 0);
            }
            int8_t *cell = xyb + px1 * XC + (((oc >> 4) ^ (px1 & 15)) << 4);
            const v4i rv = *(const v4i *)cell;
            v4i yv;
#pragma unroll
            for (int gi = 0; gi < 4; ++gi) {
                __builtin_amdgcn_sched_barrier(0);
                const v4i mm = *(const v4i *)&prm1[1][oc + 4 * gi], ch = *(const v4i *)&prm1[2][oc + 4 * gi], ss = *(const v4i *)&prm1[3][oc + 4 * gi];
                int q[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int v = clamp3(requant_tie_free(acc[4 * gi + i], mm[i], ch[i], ss[i]), p.lo1, 127);
                    const int r8 = (int)(int8_t)((uint32_t)rv[gi] >> (8 * i));
                    if constexpr (TFA) {
                        const int s = __mul24(v, p.add_mul_self) + (p.add_c0 + p.add_k) + __mul24(r8, p.add_mul_res);
                        q[i] = clamp3(s >> p.add_sh, p.add_lo, 127);
                    } else {
                        const int s = __mul24(v, p.add_mul_self) + p.add_c0 + __mul24(r8, p.add_mul_res);
                        q[i] = clamp3((s + p.add_k + (s >> 31)) >> p.add_sh, p.add_lo, 127);
                    }
                }
                yv[gi] = (int)pack4(q[0], q[1], q[2], q[3]);
            }
            *(v4i *)cell = yv;
            const long n1 = (long)n0 + px1;
            if (n1 < p.npix) *(v4i *)(p.y + n1 * XC + oc) = yv;
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // this wave's part of the y tile is in LDS
        __builtin_amdgcn_s_barrier();                         // the y tile is complete
        asm volatile("" ::: "memory");

        // ---- reduce: wave w computes channels 16 w .. 16 w + 15 of the 32 pixels ----
        {
            v4acc acc2[2];
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int i = 0; i < 4; ++i) acc2[nb][i] = prm2[0][wave * 16 + g * 4 + i];
#pragma unroll
            for (int ks = 0; ks < XC / 64; ++ks) {
#pragma unroll
                for (int nb = 0; nb < 2; ++nb) {
                    const v4i fb = *(const v4i *)(xyb + (px2 + 16 * nb) * XC + (((4 * ks + g) ^ px2) << 4));
                    acc2[nb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a2[ks], fb, acc2[nb], 0, 0, 0);
                }
            }
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                const long n2 = (long)n0 + px2 + 16 * nb;
                int q[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int c = wave * 16 + g * 4 + i;
                    q[i] = clamp3(requant_tie_free(acc2[nb][i], prm2[1][c], prm2[2][c], prm2[3][c]), p.lo2, 127);
                }
                if (n2 < p.npix) *(uint32_t *)(p.t1n + n2 * XN2W + wave * 16 + g * 4) = pack4(q[0], q[1], q[2], q[3]);
            }
        }
        buf = buf + 1 == XNB ? 0 : buf + 1;
    }
}

// ---- the 14x14 stage: 256 middle and 1024 block channels ----
// Same scheme, sixteen waves: wave w owns channels 64 w .. 64 w + 63 of the expanding convolution (K = 256: 64 registers
// of fragments, kept for the whole launch) and channels 16 w .. 16 w + 15 of the reducing one, whose K = 1024 no longer
// fits next to them: its fragments are re-read from L2 per tile, two K steps at a time, one group ahead of the MFMAs
// (256 KB per tile and workgroup, contiguous 1 KB wave-loads).  Rows of the x / y tile are 1024 bytes, of the t2 tile
// 256 bytes; chunk c of pixel p sits at chunk c ^ (p & 15) in both.

constexpr int DK1 = 256, DC = 1024, DN2 = 256;

template <bool TFA>
__global__ __launch_bounds__(XNT2, 4) void expand_reduce1024_kernel(const XrParams p) {
    __shared__ __attribute__((aligned(256))) int8_t XY[XNB][XPX * DC];
    __shared__ __attribute__((aligned(256))) int8_t T2[XNB][XPX * DK1];
    __shared__ __attribute__((aligned(16))) int prm1[4][DC];     // bias, M0, chi, shift-1 of the expanding convolution
    __shared__ __attribute__((aligned(16))) int prm2[4][DN2];    // of the reducing convolution

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ntiles = (p.npix + XPX - 1) / XPX, G = gridDim.x;
    const uint32_t xy_lds = lds_address(&XY[0][0]), t2_lds = lds_address(&T2[0][0]);

    // direct-to-LDS loads of a tile: wave w fetches pixels 2 w and 2 w + 1 of the x tile (one 1024-byte row per load),
    // waves 0 .. 7 also pixels 4 w .. 4 w + 3 of the t2 tile
    auto issue_tile = [&](int tile, int buf) {
        const int n0 = tile * XPX;
        int l = lane;
        asm volatile("" : "+v"(l));   // recompute the per-lane offsets per call: kept across the tile loop they would be spilled
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int px = 2 * wave + j, c = l ^ (px & 15);
            int n = n0 + px;
            n = n < p.npix ? n : p.npix - 1;
            ISR_GLOBAL_TO_LDS16_AT(p.x + ((uint32_t)n * (uint32_t)DC + (uint32_t)(c * 16)), xy_lds + buf * (XPX * DC) + px * 1024);
        }
        if (wave < 8) {
            const int px = 4 * wave + (l >> 4), c = (l & 15) ^ (px & 15);
            int n = n0 + px;
            n = n < p.npix ? n : p.npix - 1;
            ISR_GLOBAL_TO_LDS16_AT(p.t2 + ((uint32_t)n * (uint32_t)DK1 + (uint32_t)(c * 16)), t2_lds + buf * (XPX * DK1) + wave * 1024);
        }
    };

    int tile = blockIdx.x;
    if (tile < ntiles) issue_tile(tile, 0);
    if (tile + G < ntiles) issue_tile(tile + G, 1);
    for (int i = tid; i < DC; i += XNT2) {
        prm1[0][i] = p.bias1[i]; prm1[1][i] = p.m0s1[i]; prm1[2][i] = p.chi1[i]; prm1[3][i] = p.shm11[i];
    }
    if (tid < DN2) {
        prm2[0][tid] = p.bias2[tid]; prm2[1][tid] = p.m0s2[tid]; prm2[2][tid] = p.chi2[tid]; prm2[3][tid] = p.shm12[tid];
    }
    const uint32_t lane16 = (uint32_t)lane * 16;
    // expand fragments [fm][ksub], kept in registers for the whole launch
    const int8_t *a1w = p.a1 + (size_t)wave * (2 * (DK1 / 32) * 1024);
    v4i a1[2 * (DK1 / 32)];
#pragma unroll
    for (int f = 0; f < 2 * (DK1 / 32); ++f) a1[f] = *(const v4i *)(a1w + (lane16 + (uint32_t)(f * 1024)));
    const int8_t *a2w = p.a2 + (size_t)wave * ((DC / 64) * 1024);   // this wave's reduce fragments [kstep]
    // the fragments are in their registers before the tile loop starts (else the compiler carries "load pending" into the
    // loop and waits for every outstanding memory operation at their first use in each tile)
#pragma unroll
    for (int f = 0; f < 2 * (DK1 / 32); ++f) asm volatile("" : "+v"(a1[f]));
    wait_vmcnt<0>();
    __syncthreads();   // the constants are in LDS, the first tile has landed

    int buf = 0;
    for (int it = 0; tile < ntiles; tile += G, ++it) {
        const int n0 = tile * XPX;
        const bool prefetch = tile + 2 * G < ntiles;
        if (it > 0) {
            // Vector memory operations complete in issue order and the reduce below has already waited for its own fragment
            // loads, which were issued after the loads of this tile: all that may still be under way are the two stores that
            // ended the previous tile.
            wait_vmcnt<2>();
            __builtin_amdgcn_s_barrier();    // every wave's loads of this tile landed; every wave is done with the previous tile
        }
        if (prefetch) issue_tile(tile + 2 * G, buf >= 1 ? buf - 1 : XNB - 1);
        int l = lane;
        asm volatile("" : "+v"(l));   // per-lane values below are recomputed per tile, loads from them are not hoisted out of the loop
        const int half = l >> 5, px1 = l & 31;
        const int g = l >> 4, px2 = l & 15;
        int8_t *xyb = XY[buf];

        // ---- expand + add: 64 channels x 32 pixels per wave, 32 channels at a time ----
        const int8_t *t2b = T2[buf];
        const int b_off1 = px1 * DK1 + ((half ^ (px1 & 15)) << 4);   // chunk (2 k + half) ^ (px & 15): sub-step k flips bits 5..7 by k
        const long n1 = (long)n0 + px1;
#pragma unroll
        for (int fm = 0; fm < 2; ++fm) {
            const int oc = wave * 64 + fm * 32 + half * 16;
            v16i acc;
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = prm1[0][oc + i];
#pragma unroll
            for (int ks = 0; ks < DK1 / 32; ++ks) {
                const v4i fb = *(const v4i *)(t2b + (b_off1 ^ (ks << 5)));
                acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1[fm * (DK1 / 32) + ks], fb, acc, 0, 0, 0);
            }
            int8_t *cell = xyb + px1 * DC + (((oc >> 4) ^ (px1 & 15)) << 4);
            const v4i rv = *(const v4i *)cell;
            v4i yv;
#pragma unroll
            for (int gi = 0; gi < 4; ++gi) {
                __builtin_amdgcn_sched_barrier(0);   // one group's constants at a time: the registers are needed for weight fragments
                const v4i mm = *(const v4i *)&prm1[1][oc + 4 * gi], ch = *(const v4i *)&prm1[2][oc + 4 * gi], ss = *(const v4i *)&prm1[3][oc + 4 * gi];
                int q[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int v = clamp3(requant_tie_free(acc[4 * gi + i], mm[i], ch[i], ss[i]), p.lo1, 127);
                    const int r8 = (int)(int8_t)((uint32_t)rv[gi] >> (8 * i));
                    if constexpr (TFA) {
                        const int s = __mul24(v, p.add_mul_self) + (p.add_c0 + p.add_k) + __mul24(r8, p.add_mul_res);
                        q[i] = clamp3(s >> p.add_sh, p.add_lo, 127);
                    } else {
                        const int s = __mul24(v, p.add_mul_self) + p.add_c0 + __mul24(r8, p.add_mul_res);
                        q[i] = clamp3((s + p.add_k + (s >> 31)) >> p.add_sh, p.add_lo, 127);
                    }
                }
                yv[gi] = (int)pack4(q[0], q[1], q[2], q[3]);
            }
            *(v4i *)cell = yv;
            if (n1 < p.npix) *(v4i *)(p.y + n1 * DC + oc) = yv;
        }
        // the first group of reduce fragments is on its way while the workgroup meets at the barrier
        constexpr int GK = 2;   // K steps per group of reduce fragments (four measured no faster)
        v4i a2c[2][GK];
#pragma unroll
        for (int i = 0; i < GK; ++i) a2c[0][i] = *(const v4i *)(a2w + ((uint32_t)l * 16 + (uint32_t)(i * 1024)));
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // this wave's part of the y tile is in LDS
        __builtin_amdgcn_s_barrier();                         // the y tile is complete
        asm volatile("" ::: "memory");

        // ---- reduce: wave w computes channels 16 w .. 16 w + 15 of the 32 pixels, K = 1024 ----
        {
            v4acc acc2[2];
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int i = 0; i < 4; ++i) acc2[nb][i] = prm2[0][wave * 16 + g * 4 + i];
#pragma unroll
            for (int j = 0; j < DC / 64 / GK; ++j) {
                if (j + 1 < DC / 64 / GK) {
#pragma unroll
                    for (int i = 0; i < GK; ++i) a2c[(j + 1) & 1][i] = *(const v4i *)(a2w + ((uint32_t)l * 16 + (uint32_t)(((j + 1) * GK + i) * 1024)));
                }
#pragma unroll
                for (int i = 0; i < GK; ++i) {
                    const int ks = GK * j + i;
#pragma unroll
                    for (int nb = 0; nb < 2; ++nb) {
                        const v4i fb = *(const v4i *)(xyb + (px2 + 16 * nb) * DC + (((4 * ks + g) ^ px2) << 4));
                        acc2[nb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a2c[j & 1][i], fb, acc2[nb], 0, 0, 0);
                    }
                }
            }
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                const long n2 = (long)n0 + px2 + 16 * nb;
                int q[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int c = wave * 16 + g * 4 + i;
                    q[i] = clamp3(requant_tie_free(acc2[nb][i], prm2[1][c], prm2[2][c], prm2[3][c]), p.lo2, 127);
                }
                if (n2 < p.npix) *(uint32_t *)(p.t1n + n2 * DN2 + wave * 16 + g * 4) = pack4(q[0], q[1], q[2], q[3]);
            }
        }
        buf = buf + 1 == XNB ? 0 : buf + 1;
    }
}

}  // namespace

// Which of the two convolutions of a fuse_add == 2 descriptor is the projection: the main one (256 input channels, may be
// strided; the expanding convolution is then the second, w2) or the second one.
static bool projection_is_main(const ConvParams &e) { return e.fuse_add == 2 && e.Cin_p == XPK; }

// expand: 1x1, 128 -> 512 channels, with a fused residual add (the residual a stored tensor, or the 1x1 projection of a
// 256-channel tensor computed alongside); reduce: 1x1 stride 1, 512 -> 128, reading the sum; single-multiply tie-free
// requantisations (the add may meet ties); fragment-major weight copies present
bool expand_reduce_supported(const ConvParams &e, const ConvParams &r) {
    if (e.fuse_add == 1 && e.Cin_p == DK1)   // the 14 x 14 stage: 256 -> 1024 + add, then 1024 -> 256
        return e.k == 1 && e.stride == 1 && e.pad == 0 && e.Kp == DK1 && e.Cout_p == DC && e.fast_requant && e.tie_free && !e.c4 && e.wfrag &&
               r.k == 1 && r.stride == 1 && r.pad == 0 && r.Cin_p == DC && r.Kp == DC && r.Cout_p == DN2 && !r.fuse_add && r.fast_requant &&
               r.tie_free && !r.c4 && r.wfrag && e.Ho == r.H && e.Wo == r.W && r.Ho == r.H && r.Wo == r.W;
    bool expand = e.k == 1 && e.pad == 0 && e.Cout_p == XC && e.fast_requant && e.tie_free && !e.c4 && e.wfrag;
    if (e.fuse_add == 1) expand = expand && e.stride == 1 && e.Cin_p == XK1 && e.Kp == XK1;
    else if (projection_is_main(e))   // main: projection 256 -> 512, stride 1 or 2; second: the expanding convolution on the output pixels
        expand = expand && (e.stride == 1 || e.stride == 2) && e.Kp == XPK && e.Cin2_p == XK1 && e.tie_free2 && e.wfrag2 &&
                 (long)e.H * e.W * XPK < (1l << 31);
    else
        expand = expand && e.fuse_add == 2 && e.stride == 1 && e.Cin_p == XK1 && e.Kp == XK1 && e.Cin2_p == XPK && e.tie_free2 && e.wfrag2;
    const bool reduce = r.k == 1 && r.stride == 1 && r.pad == 0 && r.Cin_p == XC && r.Kp == XC &&
                        (r.Cout_p == XN2 || (r.Cout_p == XN2W && e.fuse_add == 1)) && !r.fuse_add && r.fast_requant && r.tie_free &&
                        !r.c4 && r.wfrag;
    return expand && reduce && e.Ho == r.H && e.Wo == r.W && r.Ho == r.H && r.Wo == r.W;
}

// The kernel's arguments from the descriptors of the expanding (+ add) and the reducing convolution and their tensors:
// `a` is the main convolution's input, `b` the add's other operand (fuse_add == 1) or the second convolution's input.
void expand_reduce_params(const ConvParams &e, const ConvParams &r, const int8_t *a, const int8_t *b, int8_t *y, int8_t *t1n,
                          int32_t copies, XrParams &xp) {
    xp = XrParams{};
    xp.y = y; xp.t1n = t1n;
    xp.a2 = r.wfrag; xp.bias2 = r.bias; xp.m0s2 = r.m0s; xp.chi2 = r.chi; xp.shm12 = r.shm1;
    xp.lo2 = r.relu ? r.zp_out : -128;
    xp.add_c0 = e.add_c0; xp.add_k = e.add_k; xp.add_sh = e.add_sh; xp.add_lo = e.add_lo;
    xp.npix = copies * e.Ho * e.Wo;
    xp.n2 = r.Cout_p;
    xp.k1 = e.fuse_add == 1 ? e.Cin_p : XK1;
    xp.Hin = e.H; xp.Win = e.W; xp.Ho = e.Ho; xp.Wo = e.Wo; xp.pstride = 1;
    const int lo_main = e.relu ? e.zp_out : -128;
    if (projection_is_main(e)) {
        xp.in2 = a; xp.pstride = e.stride;
        xp.ap = e.wfrag; xp.biasp = e.bias; xp.m0sp = e.m0s; xp.chip = e.chi; xp.shm1p = e.shm1; xp.lop = lo_main;
        xp.t2 = b;
        xp.a1 = e.wfrag2; xp.bias1 = e.bias2; xp.m0s1 = e.m0s2; xp.chi1 = e.chi2; xp.shm11 = e.shm12; xp.lo1 = e.lo2;
        xp.add_mul_self = e.add_mul_res; xp.add_mul_res = e.add_mul_self;   // "self" in the kernel = the expanding convolution
    } else {
        xp.t2 = a;
        xp.a1 = e.wfrag; xp.bias1 = e.bias; xp.m0s1 = e.m0s; xp.chi1 = e.chi; xp.shm11 = e.shm1; xp.lo1 = lo_main;
        xp.add_mul_self = e.add_mul_self; xp.add_mul_res = e.add_mul_res;
        if (e.fuse_add == 2) {
            xp.in2 = b;
            xp.ap = e.wfrag2; xp.biasp = e.bias2; xp.m0sp = e.m0s2; xp.chip = e.chi2; xp.shm1p = e.shm12; xp.lop = e.lo2;
        } else {
            xp.x = b;
        }
    }
}

hipError_t launch_expand_reduce(const XrParams &p, int add_tie_free, hipStream_t st) {
    if (p.npix <= 0) return hipSuccess;
    if ((long)p.npix * DC >= (1l << 32)) return hipErrorInvalidValue;   // 32-bit byte offsets inside the tensors
    const int ntiles = (p.npix + XPX - 1) / XPX;
    if (p.k1 == DK1) {
        const dim3 grid((unsigned)(ntiles < 256 ? ntiles : 256));
        set_kernel_name("expand_reduce_kernel<256, 1024, 256>");
        if (add_tie_free) hipLaunchKernelGGL((expand_reduce1024_kernel<true>), grid, dim3(XNT2), 0, st, p);
        else hipLaunchKernelGGL((expand_reduce1024_kernel<false>), grid, dim3(XNT2), 0, st, p);
        return hipGetLastError();
    }
    if (p.in2) {
        const dim3 grid((unsigned)(ntiles < 256 ? ntiles : 256));   // one workgroup of sixteen waves per CU
        set_kernel_name("proj_expand_reduce_kernel<256, 128, 512, 128>");
        if (add_tie_free) hipLaunchKernelGGL((proj_expand_reduce_kernel<true>), grid, dim3(XNT2), 0, st, p);
        else hipLaunchKernelGGL((proj_expand_reduce_kernel<false>), grid, dim3(XNT2), 0, st, p);
        return hipGetLastError();
    }
    if (p.n2 == XN2W) {
        const dim3 grid((unsigned)(ntiles < 256 ? ntiles : 256));
        set_kernel_name("expand_reduce_kernel<128, 512, 256>");
        if (add_tie_free) hipLaunchKernelGGL((expand_reduce256_kernel<true>), grid, dim3(XNT2), 0, st, p);
        else hipLaunchKernelGGL((expand_reduce256_kernel<false>), grid, dim3(XNT2), 0, st, p);
        return hipGetLastError();
    }
    const dim3 grid((unsigned)(ntiles < 512 ? ntiles : 512));
    set_kernel_name("expand_reduce_kernel<128, 512, 128>");
    if (add_tie_free) hipLaunchKernelGGL((expand_reduce_kernel<true>), grid, dim3(XNT), 0, st, p);
    else hipLaunchKernelGGL((expand_reduce_kernel<false>), grid, dim3(XNT), 0, st, p);
    return hipGetLastError();
}

}  // namespace isr
