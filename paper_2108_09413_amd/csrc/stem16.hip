// First layer of the narrow small-image nets: 3x3 convolution (stride 1, pad 1) of the
// noisy NHWC4 image into 16 channels.  A wave owns one image: the image goes into LDS
// once, padded with the input zero-point, and every output fragment (16 pixels of a row x
// 16 channels) is ONE v_mfma_i32_16x16x64_i8: lane group ky of the pixel operand reads the
// 16 contiguous bytes of kernel row ky -- 4 horizontally adjacent pixels x 4 stored
// channels, the fourth pixel and the fourth channel meeting zero weights -- and the fourth
// lane group meets an all-zero weight chunk.  No gather from global memory.
#include "conv_device.h"

namespace isr {

namespace {

constexpr int S16_MAXW = 64, S16_MAXH = 64;
constexpr int S16_LDS = 40 * 1024;             // bytes of padded images per workgroup (4 images)

__global__ __launch_bounds__(256) void stem16_kernel(const Stem16Params p) {
    __shared__ __attribute__((aligned(16))) int8_t img[S16_LDS];
    __shared__ int prm[4][16];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int PW = p.W + 4;                    // padded row in pixels: 1 left, 3 right (keeps rows 16-byte aligned)
    const int per = (p.H + 2) * PW * 4;        // bytes per padded image
    const long g = (long)blockIdx.x * 4 + wave;
    const long gi = g < p.B ? g : p.B - 1;     // waves past the end redo the last image and store nothing
    int8_t *my = &img[wave * per];
    if (tid < 64) { prm[0][tid & 15] = p.bias[tid & 15]; prm[1][tid & 15] = p.m0s[tid & 15]; prm[2][tid & 15] = p.chi[tid & 15]; prm[3][tid & 15] = p.shm1[tid & 15]; }
    const uint32_t zb = (uint32_t)(p.zp_in & 0xFF) * 0x01010101u;
    // interior: 16-byte chunks of 4 pixels; then the padding ring
    const int wch = p.W >> 2;
    for (int i = lane; i < p.H * wch; i += 64) {
        const int y = i / wch, c = i - y * wch;
        const v4i v = *(const v4i *)(p.in + ((gi * p.H + y) * p.W + 4 * c) * 4);
        int *dst = (int *)(my + ((y + 1) * PW + 1 + 4 * c) * 4);
        dst[0] = v[0]; dst[1] = v[1]; dst[2] = v[2]; dst[3] = v[3];
    }
    for (int i = lane; i < PW; i += 64) { ((int *)my)[i] = (int)zb; ((int *)my)[(p.H + 1) * PW + i] = (int)zb; }
    for (int i = lane; i < p.H * 4; i += 64) {
        const int y = 1 + (i >> 2), c = i & 3;
        ((int *)my)[y * PW + (c == 0 ? 0 : p.W + c)] = (int)zb;
    }
    __syncthreads();

    const int l = lane & 15, kg = lane >> 4;
    const v4i fa = *(const v4i *)(p.w + l * 64 + kg * 16);     // row = channel l, K chunk kg = kernel row kg (chunk 3: zeros)
    int m0[4], chi[4], sh[4];
    v4i binit;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        binit[i] = prm[0][4 * kg + i]; m0[i] = prm[1][4 * kg + i]; chi[i] = prm[2][4 * kg + i]; sh[i] = prm[3][4 * kg + i];
    }
    const int kr = kg < 3 ? kg : 0;            // the fourth lane group reads any valid row
    const int strips = p.W >> 4;
    for (int s = 0; s < strips; ++s) {
        const int x = 16 * s + l;
        const int *src = (const int *)(my + (kr * PW + x) * 4);   // padded (row y + kr, columns x .. x + 3) at y = 0
        int8_t *dst = p.out + ((gi * p.H) * p.W + x) * 16 + 4 * kg;
        for (int y = 0; y < p.H; ++y) {
            const v4i fb = {src[0], src[1], src[2], src[3]};
            const v4i acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa, fb, binit, 0, 0, 0);
            int q[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int r = p.tie_free ? requant_tie_free(acc[i], m0[i], chi[i], sh[i]) : requant_fast(acc[i], m0[i], chi[i], sh[i]);
                q[i] = clamp3(r, p.lo, 127);
            }
            if (g < p.B) *(uint32_t *)dst = pack4(q[0], q[1], q[2], q[3]);
            src += PW;
            dst += p.W * 16;
        }
    }
}

}  // namespace

bool stem16_supported(int k, int stride, int pad, int cout_p, int H, int W, int fast_requant) {
    return k == 3 && stride == 1 && pad == 1 && cout_p == 16 && fast_requant && W % 16 == 0 && W >= 16 && W <= S16_MAXW &&
           H >= 1 && H <= S16_MAXH && 4 * (H + 2) * (W + 4) * 4 <= S16_LDS;
}

hipError_t launch_stem16(const Stem16Params &p, hipStream_t st) {
    if (p.B <= 0) return hipSuccess;
    if (!p.in || !p.out || !p.w || !stem16_supported(3, 1, 1, 16, p.H, p.W, 1)) return hipErrorInvalidValue;
    set_kernel_name("stem16_kernel");
    hipLaunchKernelGGL(stem16_kernel, dim3((unsigned)((p.B + 3) / 4)), dim3(256), 0, st, p);
    return hipGetLastError();
}

}  // namespace isr
