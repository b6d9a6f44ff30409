// Down-sampling residual block of the narrow small-image nets in one kernel:
//   t = clamp(requant(conv3x3 stride 2 (x)))     C/2 -> C channels, 2S x 2S -> S x S pixels
//   u = clamp(requant(conv3x3 stride 1 (t)))     C -> C
//   r = clamp(requant(conv1x1 stride 2 (x)))     C/2 -> C   (projection shortcut)
//   y = add_requant(r, u)
// Same scheme as the identity-block kernel: a workgroup keeps NI whole images in LDS -- x
// with a ring of its zero-point on top and to the left (the only padding a stride-2 window
// reaches), t with a full ring -- so every pixel operand of an MFMA is one aligned 128-bit
// LDS read at a tap-shifted address; t, u and r never leave the CU.  Weight fragments come
// from global memory (L2-resident) into registers once per convolution.
// (C, S) = (32, 16) and (64, 8); v_mfma_i32_32x32x32_i8 throughout.
#include <string>

#include "conv_device.h"

namespace isr {

namespace {

template <int C, int S, int NI, bool TF>
__global__ __launch_bounds__(256, C == 32 ? 3 : 2) void trans_block_kernel(const TransParams p) {
    constexpr int CI = C / 2, SI = 2 * S;            // input channels, input edge
    constexpr int PX = SI + 1;                       // padded input edge (ring on top / left)
    constexpr int PT = S + 2;                        // padded edge of t
    constexpr int MF = C / 32;                       // M fragments
    constexpr int NF = S * S / 32;                   // pixel fragments per image
    constexpr int KP1 = (9 * CI + 63) / 64 * 64;     // K bytes per weight row in global memory, first convolution
    constexpr int KS1 = (9 * CI + 31) / 32;          // its K steps of 32
    constexpr int KP2 = (9 * C + 63) / 64 * 64;
    constexpr int KS2 = KP2 / 32;
    constexpr int KPP = 64;                          // projection: CI channels padded to 64
    static_assert((C == 32 || C == 64) && S * S % 32 == 0 && 4 % MF == 0, "shape");

    __shared__ __attribute__((aligned(16))) int8_t X[NI][PX * PX * CI];
    __shared__ __attribute__((aligned(16))) int8_t T[NI][PT * PT * C];
    __shared__ int prm[3][4][C];                     // first, second convolution, projection: bias, M0, chi, shift-1

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const long img0 = (long)blockIdx.x * NI;

    for (int i = tid; i < 3 * C; i += 256) {
        const int cv = i / C, c = i % C;
        prm[cv][0][c] = (cv == 0 ? p.bias1 : cv == 1 ? p.bias2 : p.biasp)[c];
        prm[cv][1][c] = (cv == 0 ? p.m0s1 : cv == 1 ? p.m0s2 : p.m0sp)[c];
        prm[cv][2][c] = (cv == 0 ? p.chi1 : cv == 1 ? p.chi2 : p.chip)[c];
        prm[cv][3][c] = (cv == 0 ? p.shm11 : cv == 1 ? p.shm12 : p.shm1p)[c];
    }
    const uint32_t zx = (uint32_t)(p.zp_x & 0xFF) * 0x01010101u, zt = (uint32_t)(p.zp_t & 0xFF) * 0x01010101u;
    constexpr int XCH = CI / 16, TCH = C / 16;       // 16-byte chunks per pixel
    for (int i = tid; i < NI * SI * SI * XCH; i += 256) {
        const int im = i / (SI * SI * XCH), j = i % (SI * SI * XCH), pix = j / XCH, c = j % XCH;
        long g = img0 + im;
        if (g >= p.B) g = p.B - 1;                   // images past the end repeat the last one; never stored
        *(v4i *)(&X[im][((pix / SI + 1) * PX + pix % SI + 1) * CI + c * 16]) =
            *(const v4i *)(p.in + (g * SI * SI + pix) * CI + c * 16);
    }
    for (int i = tid; i < NI * (2 * PX - 1) * XCH; i += 256) {      // top row, then the left column below it
        const int im = i / ((2 * PX - 1) * XCH), j = i % ((2 * PX - 1) * XCH), b = j / XCH, c = j % XCH;
        const int y = b < PX ? 0 : b - PX + 1, x = b < PX ? b : 0;
        *(v4i *)(&X[im][(y * PX + x) * CI + c * 16]) = v4i{(int)zx, (int)zx, (int)zx, (int)zx};
    }
    for (int i = tid; i < NI * (4 * PT - 4) * TCH; i += 256) {
        const int im = i / ((4 * PT - 4) * TCH), j = i % ((4 * PT - 4) * TCH), b = j / TCH, c = j % TCH;
        int y, x;
        if (b < PT) { y = 0; x = b; }
        else if (b < 2 * PT) { y = PT - 1; x = b - PT; }
        else if (b < 3 * PT - 2) { y = b - 2 * PT + 1; x = 0; }
        else { y = b - (3 * PT - 2) + 1; x = PT - 1; }
        *(v4i *)(&T[im][(y * PT + x) * C + c * 16]) = v4i{(int)zt, (int)zt, (int)zt, (int)zt};
    }
    __syncthreads();

    const int l = lane & 31, half = lane >> 5;
    const int mf = wave % MF;                        // this wave's M fragment
    const int c0 = mf * 32 + 16 * half;              // first of the lane's 16 output channels
    auto requant16 = [&](const v16i &a, int cv, int lo, int (&q)[16]) {
#pragma unroll
        for (int i = 0; i < 16; ++i)
            q[i] = clamp3(requant_q<TF>(a[i], prm[cv][1][c0 + i], prm[cv][2][c0 + i], prm[cv][3][c0 + i]), lo, 127);
    };
    auto bias16 = [&](int cv) {
        v16i b;
#pragma unroll
        for (int i = 0; i < 16; ++i) b[i] = prm[cv][0][c0 + i];
        return b;
    };

    // ---- first convolution (stride 2) into the interior of T ----
    {
        v4i fa[KS1];
#pragma unroll
        for (int ks = 0; ks < KS1; ++ks) fa[ks] = *(const v4i *)(p.w1 + (long)(mf * 32 + l) * KP1 + ks * 32 + half * 16);
        const v16i binit = bias16(0);
        for (int f = wave / MF; f < NI * NF; f += 4 / MF) {
            const int im = f / NF, pix = (f % NF) * 32 + l, oy = pix / S, ox = pix % S;
            const int8_t *base = &X[im][((2 * oy) * PX + 2 * ox) * CI];      // tap (0, 0) in the padded tile
            v16i acc = binit;
#pragma unroll
            for (int ks = 0; ks < KS1; ++ks) {
                // CI = 16: a step is two taps, the lane half picks one; CI = 32: one tap, the half picks 16 channels
                int tap = CI == 16 ? 2 * ks + half : ks;
                const int cc = CI == 16 ? 0 : half * 16;
                if (tap > 8) tap = 0;                    // K padding: zero weights, any readable address
                const v4i fb = *(const v4i *)(base + ((tap / 3) * PX + tap % 3) * CI + cc);
                acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[ks], fb, acc, 0, 0, 0);
            }
            int q[16];
            requant16(acc, 0, p.lo1, q);
            *(v4i *)(&T[im][((oy + 1) * PT + ox + 1) * C + c0]) =
                v4i{(int)pack4(q[0], q[1], q[2], q[3]), (int)pack4(q[4], q[5], q[6], q[7]),
                    (int)pack4(q[8], q[9], q[10], q[11]), (int)pack4(q[12], q[13], q[14], q[15])};
        }
    }
    __syncthreads();

    // ---- second convolution and the projection, residual add, store ----
    {
        v4i fa[KS2];
#pragma unroll
        for (int ks = 0; ks < KS2; ++ks) fa[ks] = *(const v4i *)(p.w2 + (long)(mf * 32 + l) * KP2 + ks * 32 + half * 16);
        const v4i fp = *(const v4i *)(p.wp + (long)(mf * 32 + l) * KPP + half * 16);   // K step 0: channels 0..31 (zeros past CI)
        const v16i binit = bias16(1), binitp = bias16(2);
        ConvParams ap{};   // the fused add reads its constants from here
        ap.add_mul_self = p.add_mul_self; ap.add_mul_res = p.add_mul_res; ap.add_c0 = p.add_c0; ap.add_k = p.add_k;
        ap.add_sh = p.add_sh; ap.add_lo = p.add_lo;
        constexpr int CH = C / 16;
        for (int f = wave / MF; f < NI * NF; f += 4 / MF) {
            const int im = f / NF, pix = (f % NF) * 32 + l, oy = pix / S, ox = pix % S;
            const int8_t *base = &T[im][(oy * PT + ox) * C];
            v16i acc = binit;
#pragma unroll
            for (int ks = 0; ks < KS2; ++ks) {
                const int j = ks * 2 + half;             // 16-byte K chunk: tap j / CH, channel chunk j % CH
                int tap = j / CH;
                const int cc = j % CH;
                if (tap > 8) tap = 0;
                const v4i fb = *(const v4i *)(base + ((tap / 3) * PT + tap % 3) * C + cc * 16);
                acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[ks], fb, acc, 0, 0, 0);
            }
            // projection: input pixel (2 oy, 2 ox); with CI = 16 the upper lane half meets zero weights
            const v4i fx = *(const v4i *)(&X[im][((2 * oy + 1) * PX + 2 * ox + 1) * CI + (CI == 16 ? 0 : half * 16)]);
            const v16i accp = __builtin_amdgcn_mfma_i32_32x32x32_i8(fp, fx, binitp, 0, 0, 0);
            int u[16], r[16], q[16];
            requant16(acc, 1, p.lo2, u);
            requant16(accp, 2, p.lop, r);
#pragma unroll
            for (int i = 0; i < 16; ++i) q[i] = fused_add<TF>(r[i], u[i], ap);   // the add is attached to the projection: it is "self"
            const long g = img0 + im;
            if (g < p.B)
                *(v4i *)(p.out + (g * S * S + pix) * C + c0) =
                    v4i{(int)pack4(q[0], q[1], q[2], q[3]), (int)pack4(q[4], q[5], q[6], q[7]),
                        (int)pack4(q[8], q[9], q[10], q[11]), (int)pack4(q[12], q[13], q[14], q[15])};
        }
    }
}

template <int C, int S, int NI>
hipError_t launch_shape(const TransParams &p, hipStream_t st) {
    const unsigned blocks = (unsigned)((p.B + NI - 1) / NI);
    static const std::string name = "trans_block_kernel<" + std::to_string(C) + ", " + std::to_string(S) + ", " + std::to_string(NI) + ">";
    set_kernel_name(name.c_str());
    if (p.tie_free) hipLaunchKernelGGL((trans_block_kernel<C, S, NI, true>), dim3(blocks), dim3(256), 0, st, p);
    else hipLaunchKernelGGL((trans_block_kernel<C, S, NI, false>), dim3(blocks), dim3(256), 0, st, p);
    return hipGetLastError();
}

}  // namespace

// Shapes with a kernel: 16 -> 32 channels at 32 x 32 -> 16 x 16 and 32 -> 64 at 16 x 16 -> 8 x 8.
bool trans_block_supported(int cout, int size_out) { return (cout == 32 && size_out == 16) || (cout == 64 && size_out == 8); }

hipError_t launch_trans_block(const TransParams &p, hipStream_t st) {
    if (p.B <= 0) return hipSuccess;
    if (!p.in || !p.out || !p.w1 || !p.w2 || !p.wp || !trans_block_supported(p.C, p.S)) return hipErrorInvalidValue;
    return p.C == 32 ? launch_shape<32, 16, 1>(p, st) : launch_shape<64, 8, 3>(p, st);
}

}  // namespace isr
