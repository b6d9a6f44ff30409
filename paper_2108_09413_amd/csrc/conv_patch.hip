// 3x3 stride-1 pad-1 convolutions of the deeper layers (at least 128 output channels, input channels a
// multiple of the K step) with the activations staged ONCE per channel slice instead of once per tap.
//
// The implicit-GEMM kernel of conv_dma.h gathers, for each of the nine taps, the channel bytes of every
// pixel of its tile again: per 128 input channels a 256 x 256 tile moves 9 x (32 KB of weights + 32 KB of
// activations) from L2 into LDS, and issuing and awaiting that transfer is what its K step spends most of
// its time on.  In the flat pixel order of an NHWC tensor the neighbour (dy, dx) of pixel n is pixel
// n + dy W + dx whenever it lies in the image, so the nine shifted views of a tile of 256 consecutive pixels
// all lie in the 256 + 2 (W + 1) pixel rows around it.  This kernel stages those rows once per slice of KB
// channels and lets the fragment reads of tap (dy, dx) address row  i + (W + 1) + dy W + dx,  or zero
// points for a neighbour outside the image: with KB = 128, 9 x 32 KB + 40 KB instead of 9 x 64 KB per
// slice.  The weights stream as before, one [BM channels][KB bytes] block per (slice, tap); integer
// accumulation makes the changed K order (slice-major, tap-minor) exact.
//
// LDS: two weight buffers, two activation buffers of 320 rows + 256 bytes of zero points, the per-channel
// constants.  <256 channels, 128-byte slices>: 148 KB, sixteen waves of 64 x 64, one workgroup per CU;
// <128, 64>: 58 KB, eight waves, two workgroups per CU.  Chunk swizzle and epilogue as in conv_dma.h.
#include "conv_device.h"

namespace isr {

namespace {

constexpr int PBN = 256;                         // pixels per tile
constexpr int PROWS = 320;                       // staged pixel rows per buffer: 256 + 2 (W + 1) <= 320 for W <= 31
constexpr int PZBYTES = 256;                     // zero points behind them: one pass over the 64 LDS banks

template <int BM, int KB, int MINB, bool TF, bool DUTY>
__global__ __launch_bounds__((BM / 64) * (PBN / 64) * 64, MINB) void conv_patch_kernel(const ConvParams p) {
    constexpr int WGM = BM / 64, NW = WGM * (PBN / 64), NT = NW * 64;
    constexpr int CPR = KB / 16;                 // 16-byte chunks per row
    constexpr int RPP = NT / CPR;                // rows covered by one pass of all threads
    constexpr int NA = BM / RPP;                 // weight loads per lane per step
    constexpr int KS = KB / 32;
    constexpr int ABUF = BM * KB, ZOFF = PROWS * KB, BBUF = ZOFF + PZBYTES;
    static_assert(RPP == 128 && BM % RPP == 0 && (KB == 64 || KB == 128) && ZOFF % 256 == 0, "tile shape");

    __shared__ __attribute__((aligned(256))) int8_t Bs[2][BBUF];
    __shared__ __attribute__((aligned(16))) int8_t As[2][ABUF];
    __shared__ __attribute__((aligned(16))) int prm_s[4][BM];   // bias, M0, chi, shift-1 of this M tile

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WGM, wn = wave / WGM;
    // same XCD-aware tile order as the other convolution kernels
    const int nblk = gridDim.x, mt = (p.Cout_p + BM - 1) / BM;
    const int xcd = blockIdx.x & 7, per = nblk >> 3, extra = nblk & 7;
    const int logical = xcd * per + (xcd < extra ? xcd : extra) + (blockIdx.x >> 3);
    const int m0 = (logical % mt) * BM;
    const int n0 = (logical / mt) * PBN;
    const int W = p.W, halo = W + 1;
    const int nslice = p.Cin_p / KB, nk = 9 * nslice;

    // ---- loader side ----
    // A wave-load moves 1 KB = RW rows of KB bytes; lane (lrow, lcol) of it fetches chunk lcol ^ swz(row) of its row.
    // DUTY: in every step the loads of the whole workgroup are issued by ONE wave per SIMD (the group t mod NG of
    // waves 4 g .. 4 g + 3), the other waves go straight to their fragment reads and MFMAs.  A wave is held about
    // 200 cycles at each direct-to-LDS load it issues (in-kernel timestamps), whoever else issues; the other waves of
    // its SIMD, and the second workgroup of the CU, keep the matrix pipe busy meanwhile.
    constexpr int RW = 1024 / KB, NG = NW / 4, LA = BM / RW / 4, LB = 128 / RW / 4;
    static_assert(!DUTY || (NW % 4 == 0 && LA >= 1 && LB >= 2), "duty groups");
    const int sigma = wave & 3, grp = wave >> 2;
    const int lrow = lane / CPR, lcol = lane % CPR;
    const uint32_t a_lds0 = lds_address(&As[0][0]), b_lds0 = lds_address(&Bs[0][0]);
    uint32_t aofs[DUTY ? LA : 1];   // DUTY: byte offset in the weight matrix of the lane's 16 bytes of wave-load sigma LA + j
    if constexpr (DUTY) {
#pragma unroll
        for (int j = 0; j < LA; ++j) {
            const int row = (sigma * LA + j) * RW + lrow, r = m0 + row;
            aofs[j] = (uint32_t)(r < p.Mp ? r : 0) * (uint32_t)p.Kp + ((lcol ^ swz<CPR>(row)) << 4);   // rows past Mp re-read row 0
        }
    }
    auto issue_a_duty = [&](int slice, int tap, int buf) {
        const int8_t *src = p.w + ((long)tap * p.Cin_p + slice * KB);
        const uint32_t dst = a_lds0 + buf * ABUF + sigma * LA * 1024;
#pragma unroll
        for (int j = 0; j < LA; ++j) ISR_GLOBAL_TO_LDS16_AT(src + aofs[j], dst + j * 1024);
    };
    auto issue_b_duty = [&](int slice, int jb, int buf) {
        const int cnt = jb < 2 ? LB : LB / 2;   // the third pass covers rows 256..319
#pragma unroll
        for (int i = 0; i < LB; ++i) {
            if (i < cnt) {
                const int q = sigma * cnt + i, rho = 128 * jb + q * RW + lrow;
                int g = n0 - halo + rho;
                g = g < 0 ? 0 : (g >= p.npix ? p.npix - 1 : g);
                const uint32_t off = (uint32_t)g * (uint32_t)p.Cin_p + ((lcol ^ swz<CPR>(rho)) << 4) + (uint32_t)(slice * KB);
                ISR_GLOBAL_TO_LDS16_AT(p.in + off, b_lds0 + buf * BBUF + (128 * jb / RW + q) * 1024);
            }
        }
    };

    // every wave its share: lane (row0, col) of a pass of all threads fetches chunk col ^ swz(row0) of row row0 + 128 j
    const int col = tid % CPR, row0 = tid / CPR;
    const int cl = col ^ swz<CPR>(row0);
    const int8_t *wrow[DUTY ? 1 : NA];
    uint32_t prow[DUTY ? 1 : 3];
    if constexpr (!DUTY) {
#pragma unroll
        for (int j = 0; j < NA; ++j) {
            const int r = m0 + row0 + RPP * j;
            wrow[j] = p.w + (long)(r < p.Mp ? r : 0) * p.Kp + cl * 16;   // rows past Mp re-read row 0; never stored
        }
        // staged row rho holds pixel n0 - halo + rho; pixels outside the tensor are clamped (only taps outside the image would read them)
#pragma unroll
        for (int j = 0; j < 3; ++j) {
            int g = n0 - halo + row0 + RPP * j;
            g = g < 0 ? 0 : (g >= p.npix ? p.npix - 1 : g);
            prow[j] = (uint32_t)g * (uint32_t)p.Cin_p + cl * 16;
        }
    }
    // weights of step t = (slice, tap) into buffer t & 1
    auto issue_a = [&](int slice, int tap, int buf) {
        if constexpr (DUTY) issue_a_duty(slice, tap, buf);
        else {
            const uint32_t sa = a_lds0 + wave * 1024 + buf * ABUF;
            const long koff = (long)tap * p.Cin_p + slice * KB;
#pragma unroll
            for (int j = 0; j < NA; ++j) ISR_GLOBAL_TO_LDS16_AT(wrow[j] + koff, sa + j * (NT * 16));
        }
    };
    // pass j (128 rows; the third pass covers rows 256..319 with the first half of the waves) of a slice's pixel rows
    auto issue_b = [&](int slice, int j, int buf) {
        if constexpr (DUTY) issue_b_duty(slice, j, buf);
        else if (j < 2 || wave < NW / 2)
            ISR_GLOBAL_TO_LDS16_AT(p.in + (prow[j] + (uint32_t)(slice * KB)), b_lds0 + wave * 1024 + buf * BBUF + j * (NT * 16));
    };

    if constexpr (DUTY) {
        // the first loads, spread over the groups
        if (grp == 0) issue_a(0, 0, 0);
        if (grp == (NG == 4 ? 1 : 0)) { issue_b(0, 0, 0); issue_b(0, 2, 0); }
        if (grp == (NG == 4 ? 2 : 1)) issue_b(0, 1, 0);
        if (grp == NG - 1) issue_a(0, 1, 1);   // step 1 is tap 1 of slice 0
    } else {
        issue_b(0, 0, 0); issue_b(0, 1, 0); issue_b(0, 2, 0);
        issue_a(0, 0, 0);
        issue_a(0, 1, 1);   // step 1 is tap 1 of slice 0
    }

    for (int i = tid; i < BM; i += NT) {
        const bool in = m0 + i < p.Mp;
        prm_s[0][i] = in ? p.bias[m0 + i] : 0;
        prm_s[1][i] = in ? p.m0s[m0 + i] : 0;
        prm_s[2][i] = in ? p.chi[m0 + i] : 0;
        prm_s[3][i] = in ? p.shm1[m0 + i] : 1;
    }
    if (tid < 2 * (PZBYTES / 4)) *(int *)(&Bs[tid / (PZBYTES / 4)][ZOFF + (tid % (PZBYTES / 4)) * 4]) = (p.zp_in & 0xFF) * 0x01010101;
    __syncthreads();   // prm_s and the zero points visible

    // ---- compute side ----
    // byte offset of the lane's first weight fragment (K sub-step 0) in a weight buffer; sub-step k reads chunk
    // (2 k + half) ^ swz = (half ^ swz) ^ 2 k, i.e. the offset with bits 5..6 flipped by k
    const int half = (lane >> 5);
    int aoff[2];
#pragma unroll
    for (int fm = 0; fm < 2; ++fm) {
        const int r = wm * 64 + fm * 32 + (lane & 31);
        aoff[fm] = r * KB + ((half ^ swz<CPR>(r)) << 4);
    }
    // pixel i of the tile sits in staged row i + halo; bit (dy + 1) * 3 + (dx + 1) of `inside` says that its neighbour
    // (dy, dx) lies in the image
    int rho0[2];
    uint32_t inside[2];
    {
        const int HW = p.H * W;
#pragma unroll
        for (int fn = 0; fn < 2; ++fn) {
            const int i = wn * 64 + fn * 32 + (lane & 31);
            const int n = n0 + i, rem = n % HW, y = rem / W, x = rem - y * W;
            const uint32_t rowok = (y > 0 ? 1u : 0u) | 2u | (y + 1 < p.H ? 4u : 0u);
            const uint32_t colok = (x > 0 ? 1u : 0u) | 2u | (x + 1 < W ? 4u : 0u);
            uint32_t m = 0;
#pragma unroll
            for (int ty = 0; ty < 3; ++ty)
                if (rowok >> ty & 1) m |= colok << (3 * ty);
            inside[fn] = m;
            rho0[fn] = i + halo;
        }
    }
    auto lane_oc = [&](int fm) { return wm * 64 + fm * 32 + 16 * (lane >> 5); };
    v16i acc[2][2];
#pragma unroll
    for (int fm = 0; fm < 2; ++fm) {
        v16i init;
#pragma unroll
        for (int i = 0; i < 16; ++i) init[i] = prm_s[0][lane_oc(fm) + i];
        acc[fm][0] = init;
        acc[fm][1] = init;
    }

    // Byte offset of the lane's first fragment of a tap in an activation buffer.  A neighbour outside the image
    // reads the zero points at the same offset modulo 256, i.e. from the banks its in-image read would have used:
    // the 16 lanes that the LDS serves together then still cover the 64 banks exactly once.
    auto tap_rows = [&](int tap, int (&brow)[2]) {
        const int ty = tap / 3, tx = tap - 3 * ty;
        const int shift = (ty - 1) * W + (tx - 1);
#pragma unroll
        for (int fn = 0; fn < 2; ++fn) {
            const int rho = rho0[fn] + shift;
            const int off = rho * KB + ((half ^ swz<CPR>(rho)) << 4);
            brow[fn] = (inside[fn] >> tap & 1) ? off : ZOFF + (off & (PZBYTES - 1));
        }
    };
    // the loads that follow the barrier of step u = (slice, tap): the weights of step u + 1 into the buffer that step
    // u - 1 used, and, during the first three taps of a slice, a pass of the next slice's pixel rows into the
    // activation buffer that was last read in the previous slice
    auto refill = [&](int u, int slice, int tap) {
        if (!DUTY || (u & (NG - 1)) == grp) {
            if (u >= 1 && u + 1 < nk) {
                const int nt = tap + 1 == 9 ? 0 : tap + 1;
                issue_a(slice + (tap + 1 == 9 ? 1 : 0), nt, (u + 1) & 1);
            }
            if (tap < 3 && slice + 1 < nslice) issue_b(slice + 1, tap, (slice + 1) & 1);
        }
    };

    // K loop with the fragment reads one sub-step ahead of the MFMAs (two register sets).  Before a step's barrier
    // a wave waits for its own loads of that step (step 1's weights, issued last before the loop, may still be in
    // flight at step 0).  At the last sub-step of a step the wave holds that sub-step's fragments already: it
    // passes the next step's barrier, issues its refill and reads the next step's first fragments BEFORE it issues
    // those four MFMAs, so the matrix pipe has work queued while the workgroup goes through barrier, refill and
    // the first fragment reads (measured +1 to +3 % over reading each sub-step's fragments right before its MFMAs).
    static_assert(KS % 2 == 0, "register sets alternate");
    v4i fa[2][2], fb[2][2];
    auto read_fragments = [&](const int8_t *abase, const int8_t *bbase, const int (&brow)[2], int ksub, int slot) {
#pragma unroll
        for (int fm = 0; fm < 2; ++fm) fa[slot][fm] = *(const v4i *)(abase + (aoff[fm] ^ (ksub << 5)));
#pragma unroll
        for (int fn = 0; fn < 2; ++fn) fb[slot][fn] = *(const v4i *)(bbase + (brow[fn] ^ (ksub << 5)));
    };
    int slice = 0, tap = 0;
    int brow[2];
    if (!DUTY) wait_vmcnt<NA>();
    else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();   // step 0 landed
    refill(0, 0, 0);
    tap_rows(0, brow);
    read_fragments(As[0], Bs[0], brow, 0, 0);
#pragma unroll 1
    for (int t = 0; t < nk; ++t) {
        const int8_t *abase = As[t & 1], *bbase = Bs[slice & 1];
#pragma unroll
        for (int ksub = 0; ksub < KS; ++ksub) {
            const int slot = ksub & 1;
            if (ksub + 1 < KS) {
                read_fragments(abase, bbase, brow, ksub + 1, slot ^ 1);
            } else if (t + 1 < nk) {
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // this wave's reads of step t are complete
                wait_vmcnt<0>();
                __builtin_amdgcn_s_barrier();   // every wave's loads of step t + 1 landed; every wave is done reading step t
                if (++tap == 9) { tap = 0; ++slice; }
                refill(t + 1, slice, tap);
                tap_rows(tap, brow);
                read_fragments(As[(t + 1) & 1], Bs[slice & 1], brow, 0, slot ^ 1);
            }
#pragma unroll
            for (int fm = 0; fm < 2; ++fm)
#pragma unroll
                for (int fn = 0; fn < 2; ++fn)
                    acc[fm][fn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[slot][fm], fb[slot][fn], acc[fm][fn], 0, 0, 0);
        }
    }

    // epilogue: requantise, clamp, pack, store (NHWC)
    const int lo = p.relu ? p.zp_out : -128;
#pragma unroll
    for (int fm = 0; fm < 2; ++fm) {
        const int oc = m0 + lane_oc(fm);
        if (oc >= p.Cout_p) continue;
        int mm[16], ch[16], ss[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            mm[i] = prm_s[1][oc - m0 + i]; ch[i] = prm_s[2][oc - m0 + i]; ss[i] = prm_s[3][oc - m0 + i];
        }
#pragma unroll
        for (int fn = 0; fn < 2; ++fn) {
            const long n = (long)n0 + wn * 64 + fn * 32 + (lane & 31);
            if (n >= p.npix) continue;
            int q[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) q[i] = clamp3(requant_q<TF>(acc[fm][fn][i], mm[i], ch[i], ss[i]), lo, 127);
            *(v4i *)(p.out + n * p.Cout_p + oc) = v4i{(int)pack4(q[0], q[1], q[2], q[3]), (int)pack4(q[4], q[5], q[6], q[7]),
                                                       (int)pack4(q[8], q[9], q[10], q[11]), (int)pack4(q[12], q[13], q[14], q[15])};
        }
    }
}

template <int BM, int KB, int MINB, bool DUTY>
hipError_t launch_patch(const ConvParams &p, hipStream_t st, const char *name) {
    const dim3 grid((unsigned)(((p.npix + PBN - 1) / PBN) * ((p.Cout_p + BM - 1) / BM)));
    const dim3 block((BM / 64) * (PBN / 64) * 64);
    set_kernel_name(name);
    if (p.tie_free) hipLaunchKernelGGL((conv_patch_kernel<BM, KB, MINB, true, DUTY>), grid, block, 0, st, p);
    else hipLaunchKernelGGL((conv_patch_kernel<BM, KB, MINB, false, DUTY>), grid, block, 0, st, p);
    return hipGetLastError();
}

}  // namespace

// 3x3, stride 1, pad 1, same-size output; whole channel slices; a tile's pixel rows fit the staging buffer;
// 256-channel tiles step through K in 128-byte slices, 128-channel tiles in 64-byte slices
bool conv_patch_supported(const ConvParams &p) {
    if (!(p.k == 3 && p.stride == 1 && p.pad == 1 && p.H == p.Ho && p.W == p.Wo && p.W >= 2 && 2 * (p.W + 1) + PBN <= PROWS))
        return false;
    if (p.fuse_add || !p.fast_requant || p.c4 || p.Kp != 9 * p.Cin_p || (long)p.npix * p.Cin_p >= (1l << 31)) return false;
    if (p.Cout_p >= 256) return p.kb == 128 && p.Cin_p % 128 == 0;
    return p.Cout_p == 128 && p.kb == 64 && p.Cin_p % 64 == 0;
}

hipError_t launch_conv_patch(const ConvParams &p, hipStream_t st) {
    if (p.npix <= 0) return hipSuccess;
    if (!conv_patch_supported(p) || p.Mp < p.Cout_p) return hipErrorInvalidValue;
    // One issuing wave per SIMD and step pays with two workgroups per CU (the other workgroup computes while that wave
    // is held at its loads: 1720 -> 1810 TOP/s on 3x3 128 -> 128 at 28 x 28); with one workgroup per CU the issuing
    // wave, which still has its own MFMAs to do, becomes the last to reach the barrier (2120 -> 2060).
    if (p.Cout_p >= 256) return launch_patch<256, 128, 1, false>(p, st, "conv_patch_kernel<256, 256, 128>");
    return launch_patch<128, 64, 2, true>(p, st, "conv_patch_kernel<128, 256, 64>");
}

}  // namespace isr
