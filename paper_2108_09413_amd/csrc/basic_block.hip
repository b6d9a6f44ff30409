// Identity residual block of the narrow, small-image nets in one kernel:
//   t = clamp(requant(conv3x3(x)));  y = add_requant(clamp(requant(conv3x3(t))), x)
// (both convolutions stride 1, pad 1, C -> C channels, S x S pixels).  A workgroup keeps
// NI whole images in LDS -- x and t as (S+2) x (S+2) x C int8 tiles whose border holds the
// tensor's zero-point, so taps need no bounds checks and contribute 0; t never leaves the
// CU and x is read from HBM once for both the first convolution and the residual.  The
// weight fragments a wave needs do not depend on the pixel fragment: it reads them from
// global memory (L2-resident, a few KiB) once per convolution into registers; with 64
// channels the two M fragments are split over the waves so that they fit.  The 16 K-bytes
// of an MFMA operand lane are 16 channels of one tap: one aligned 128-bit LDS read at
// (pixel + tap offset) * C, no gather through the texture path.  C = 16 uses v_mfma_i32_16x16x64_i8, C = 32 / 64 v_mfma_i32_32x32x32_i8.
// A launch runs a CHAIN of such blocks (same shape, each feeding the next): the output of a
// block overwrites x in LDS in place -- a lane reads the residual at its own pixel and writes
// the sum there, the second convolution itself reads only t -- so a run of identity blocks
// reads its input from HBM once and writes once.
#include <string>

#include "conv_device.h"

namespace isr {

namespace {

template <int C, int S, int NI, bool TF>
__global__ __launch_bounds__(256) void basic_block_kernel(const BlockParams p) {
    constexpr int P = S + 2;                         // padded tile edge
    constexpr int KP = (9 * C + 63) / 64 * 64;       // K bytes per weight row in global memory
    constexpr int MT = C == 16 ? 16 : 32;            // MFMA tile edge
    constexpr int MF = C / MT;                       // M fragments
    constexpr int MSPLIT = MF;                       // waves that share one pixel fragment, one M fragment each
    constexpr int NF = S * S / MT;                   // pixel fragments per image
    constexpr int KS = C == 16 ? KP / 64 : KP / 32;  // K steps
    constexpr int ACC = MT == 16 ? 4 : 16;
    constexpr int CH = C / 16;                       // 16-byte chunks per pixel
    static_assert(S * S % MT == 0 && (C == 16 || C == 32 || C == 64), "shape");
    typedef int acc_t __attribute__((ext_vector_type(ACC)));

    __shared__ __attribute__((aligned(16))) int8_t X[NI][P * P * C];
    __shared__ __attribute__((aligned(16))) int8_t T[NI][P * P * C];
    __shared__ int prm[2][4][C];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const long img0 = (long)blockIdx.x * NI;

    // ---- the images ----
    for (int i = tid; i < NI * S * S * CH; i += 256) {
        const int im = i / (S * S * CH), j = i % (S * S * CH), pix = j / CH, c = j % CH;
        const int y = pix / S, x = pix % S;
        long g = img0 + im;
        if (g >= p.B) g = p.B - 1;                   // images past the end repeat the last one; never stored
        *(v4i *)(&X[im][((y + 1) * P + x + 1) * C + c * 16]) = *(const v4i *)(p.in + (g * S * S + pix) * C + c * 16);
    }
    // per block: per-channel constants and the two padding rings (zero-points of x and t)
    auto stage_block = [&](const BlockDesc &d) {
        for (int i = tid; i < 2 * C; i += 256) {
            const int cv = i / C, c = i % C;
            prm[cv][0][c] = (cv ? d.bias2 : d.bias1)[c];
            prm[cv][1][c] = (cv ? d.m0s2 : d.m0s1)[c];
            prm[cv][2][c] = (cv ? d.chi2 : d.chi1)[c];
            prm[cv][3][c] = (cv ? d.shm12 : d.shm11)[c];
        }
        const uint32_t zx = (uint32_t)(d.zp_x & 0xFF) * 0x01010101u, zt = (uint32_t)(d.zp_t & 0xFF) * 0x01010101u;
        for (int i = tid; i < NI * (4 * P - 4) * CH; i += 256) {
            const int im = i / ((4 * P - 4) * CH), j = i % ((4 * P - 4) * CH), b = j / CH, c = j % CH;
            // border pixel b: top row, bottom row, then the left and right columns without the corners
            int y, x;
            if (b < P) { y = 0; x = b; }
            else if (b < 2 * P) { y = P - 1; x = b - P; }
            else if (b < 3 * P - 2) { y = b - 2 * P + 1; x = 0; }
            else { y = b - (3 * P - 2) + 1; x = P - 1; }
            const int off = (y * P + x) * C + c * 16;
            *(v4i *)(&X[im][off]) = v4i{(int)zx, (int)zx, (int)zx, (int)zx};
            *(v4i *)(&T[im][off]) = v4i{(int)zt, (int)zt, (int)zt, (int)zt};
        }
    };

    // lane's place in an MFMA operand: pixel / weight row `l`, 16-byte K chunk `kg` of the step
    const int l = lane & (MT - 1), kg = lane / MT;
    constexpr int CPS = 64 / MT == 4 ? 4 : 2;        // 16-byte chunks per K step (4 for 16x16x64, 2 for 32x32x32)
    const int ocl = MT == 16 ? 4 * kg : 16 * kg;     // first output channel (within an M fragment) this lane holds

    // One 3x3 convolution over all NI images from the padded tile `src`, weights `w`;
    // `emit(image, pixel, m fragment, accumulators)` consumes each fragment.
    const int mf = wave % MSPLIT;                    // this wave's M fragment
    auto conv = [&](const int8_t (*src)[P * P * C], int cv, const int8_t *w, auto emit) {
        acc_t binit;
#pragma unroll
        for (int i = 0; i < ACC; ++i) binit[i] = prm[cv][0][mf * MT + ocl + i];
        if constexpr (C == 16) {
            // 16 channels: a K step of v_mfma_i32_16x16x64_i8 is one kernel row -- lane group kg holds
            // tap (ky = step, kx = kg), the fourth group zero weights -- and a wave walks down 16 rows
            // of a 16-pixel column strip: the operands of rows y+1, y+2 of one output row are those of
            // rows y, y+1 of the next, so each output fragment costs one new LDS read instead of three.
            static_assert(S == 32 && NI == 1, "walk assumes two 16-pixel strips and one image");
            const int strip = wave & 1, row0 = (wave >> 1) * 16, kx = kg < 3 ? kg : 0;
            v4i fa[3];
#pragma unroll
            for (int ky = 0; ky < 3; ++ky) {
                fa[ky] = *(const v4i *)(w + (long)l * KP + (ky * 3 + kx) * 16);
                if (kg == 3) fa[ky] = v4i{0, 0, 0, 0};
            }
            const int x = 16 * strip + l;
            const int8_t *col = &src[0][(row0 * P + x + kx) * C];   // padded (row0, x + kx) = tap (0, kx) of output (row0, x)
            v4i b0 = *(const v4i *)col, b1 = *(const v4i *)(col + P * C);
#pragma unroll 4
            for (int r = 0; r < 16; ++r) {
                const v4i b2 = *(const v4i *)(col + (r + 2) * P * C);
                acc_t acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa[0], b0, binit, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa[1], b1, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa[2], b2, acc, 0, 0, 0);
                emit(0, (row0 + r) * S + x, 0, acc);
                b0 = b1;
                b1 = b2;
            }
        } else {
            v4i fa[KS];                                  // the wave's weight fragments, all K steps
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) fa[ks] = *(const v4i *)(w + (long)(mf * MT + l) * KP + (ks * CPS + kg) * 16);
            for (int f = wave / MSPLIT; f < NI * NF; f += 4 / MSPLIT) {
                const int im = f / NF, pix = (f % NF) * MT + l;
                const int y = pix / S, x = pix % S;
                const int8_t *base = &src[im][(y * P + x) * C];   // tap (0, 0) of this pixel in the padded tile
                acc_t acc = binit;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const int j = ks * CPS + kg;              // 16-byte K chunk: tap j / CH, channel chunk j % CH
                    int tap = j / CH;
                    const int cc = j % CH;
                    if (tap > 8) tap = 0;                     // K padding: zero weights, any readable address
                    const v4i fb = *(const v4i *)(base + ((tap / 3) * P + tap % 3) * C + cc * 16);
                    acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[ks], fb, acc, 0, 0, 0);
                }
                emit(im, pix, mf, acc);
            }
        }
    };

    // Per-channel requantisation constants of the lane's ACC output channels, held in registers
    // across the pixel loop (the lane's channels do not change): re-reading them from LDS for every
    // fragment would cost more LDS bandwidth than the operands.
    struct Req { int m0[ACC], chi[ACC], shm1[ACC]; };
    auto load_req = [&](int cv) {
        Req r;
#pragma unroll
        for (int i = 0; i < ACC; ++i) {
            r.m0[i] = prm[cv][1][mf * MT + ocl + i];
            r.chi[i] = prm[cv][2][mf * MT + ocl + i];
            r.shm1[i] = prm[cv][3][mf * MT + ocl + i];
        }
        return r;
    };

    for (int blk = 0; blk < p.nblocks; ++blk) {
        const BlockDesc d = p.blocks[blk];
        const bool last = blk + 1 == p.nblocks;
        if (blk) __syncthreads();   // every wave is done with the previous block's constants and has written its part of x
        stage_block(d);
        __syncthreads();

        // ---- first convolution: requantise, clamp, into the interior of T ----
        const int lo1 = d.relu1 ? d.zp_t : -128;
        {
            const Req rq = load_req(0);
            conv(X, 0, d.w1, [&](int im, int pix, int mf, const acc_t &a) {
                const int c0 = mf * MT + ocl;
                int q[ACC];
#pragma unroll
                for (int i = 0; i < ACC; ++i) q[i] = clamp3(requant_q<TF>(a[i], rq.m0[i], rq.chi[i], rq.shm1[i]), lo1, 127);
                int8_t *dst = &T[im][((pix / S + 1) * P + pix % S + 1) * C + c0];
                if constexpr (MT == 16) *(uint32_t *)dst = pack4(q[0], q[1], q[2], q[3]);
                else
                    *(v4i *)dst = v4i{(int)pack4(q[0], q[1], q[2], q[3]), (int)pack4(q[4], q[5], q[6], q[7]),
                                      (int)pack4(q[8], q[9], q[10], q[11]), (int)pack4(q[12], q[13], q[14], q[15])};
            });
        }
        __syncthreads();

        // ---- second convolution: requantise, clamp, add the residual x; the sum replaces x in LDS
        // (next block of the chain) or goes to memory (last block) ----
        const int lo2 = d.relu2 ? d.zp_u : -128;
        ConvParams ap{};   // the fused add reads its constants from here
        ap.add_mul_self = d.add_mul_self; ap.add_mul_res = d.add_mul_res; ap.add_c0 = d.add_c0; ap.add_k = d.add_k;
        ap.add_sh = d.add_sh; ap.add_lo = d.add_lo;
        const Req rq2 = load_req(1);
        conv(T, 1, d.w2, [&](int im, int pix, int mf, const acc_t &a) {
            const int c0 = mf * MT + ocl;
            const long g = img0 + im;
            int8_t *res = &X[im][((pix / S + 1) * P + pix % S + 1) * C + c0];
            int q[ACC];
            uint32_t rw[ACC / 4];
            if constexpr (MT == 16) rw[0] = *(const uint32_t *)res;
            else {
                const v4i rv = *(const v4i *)res;
#pragma unroll
                for (int d4 = 0; d4 < 4; ++d4) rw[d4] = (uint32_t)rv[d4];
            }
#pragma unroll
            for (int i = 0; i < ACC; ++i) {
                const int qc = clamp3(requant_q<TF>(a[i], rq2.m0[i], rq2.chi[i], rq2.shm1[i]), lo2, 127);
                const int r8 = (int)(int8_t)(rw[i >> 2] >> (8 * (i & 3)));
                q[i] = fused_add<TF>(qc, r8, ap);
            }
            if (last && g >= p.B) return;
            int8_t *dst = last ? p.out + (g * S * S + pix) * C + c0 : res;
            if constexpr (MT == 16) *(uint32_t *)dst = pack4(q[0], q[1], q[2], q[3]);
            else
                *(v4i *)dst = v4i{(int)pack4(q[0], q[1], q[2], q[3]), (int)pack4(q[4], q[5], q[6], q[7]),
                                  (int)pack4(q[8], q[9], q[10], q[11]), (int)pack4(q[12], q[13], q[14], q[15])};
        });
    }
}

template <int C, int S, int NI>
hipError_t launch_shape(const BlockParams &p, hipStream_t st) {
    const unsigned blocks = (unsigned)((p.B + NI - 1) / NI);
    static const std::string name = "basic_block_kernel<" + std::to_string(C) + ", " + std::to_string(S) + ", " + std::to_string(NI) + ">";
    set_kernel_name(name.c_str());
    if (p.tie_free) hipLaunchKernelGGL((basic_block_kernel<C, S, NI, true>), dim3(blocks), dim3(256), 0, st, p);
    else hipLaunchKernelGGL((basic_block_kernel<C, S, NI, false>), dim3(blocks), dim3(256), 0, st, p);
    return hipGetLastError();
}

}  // namespace

// Shapes with a kernel: 16 channels at 32 x 32, 32 at 16 x 16, 64 at 8 x 8 (the three stages of
// the CIFAR-style residual nets).
bool basic_block_supported(int channels, int size) {
    return (channels == 16 && size == 32) || (channels == 32 && size == 16) || (channels == 64 && size == 8);
}

hipError_t launch_basic_block(const BlockParams &p, hipStream_t st) {
    if (p.B <= 0) return hipSuccess;
    if (!p.in || !p.out || !p.blocks || p.nblocks < 1 || !basic_block_supported(p.C, p.S)) return hipErrorInvalidValue;
    if (p.C == 16) return launch_shape<16, 32, 1>(p, st);
    if (p.C == 32) return launch_shape<32, 16, 2>(p, st);
    return launch_shape<64, 8, 4>(p, st);
}

}  // namespace isr
