// Deep convolution layers on 256 x 256 output tiles with four waves of 128 x 128 each: a wave's 4 x 4
// MFMA tiles take 16 MFMAs from 8 fragment reads per K sub-step (half the LDS bytes per
// multiply of the 64 x 64 wave tile, whose fragment reads alone saturate the LDS at the matrix
// pipe's peak).  The 256 accumulator registers of a wave live in the accumulation half of the
// register file, so this translation unit is compiled without the option that keeps MFMA
// results among the ordinary VGPRs; one wave per SIMD.
#include "conv_dma.h"

namespace isr {

template <int KB>
static hipError_t launch_deep(const ConvParams &p, hipStream_t st) {
    dim3 grid((unsigned)(((p.npix + 255) / 256) * ((p.Cout_p + 255) / 256)));
    set_kernel_name(conv_dma_name<256, 256, KB, 2, 0, 1, 128, 128>());
    if (p.tie_free)
        hipLaunchKernelGGL((conv_dma_kernel<256, 256, KB, 2, 0, 1, true, 128, 128>), grid, dim3(256), 0, st, p);
    else
        hipLaunchKernelGGL((conv_dma_kernel<256, 256, KB, 2, 0, 1, false, 128, 128>), grid, dim3(256), 0, st, p);
    return hipGetLastError();
}

hipError_t launch_conv_deep(const ConvParams &p, hipStream_t st) {
    if (p.npix <= 0) return hipSuccess;
    if (p.fuse_add || !p.zpad || !p.fast_requant || p.c4 || p.Cout_p <= 128 || (p.kb != 64 && p.kb != 128) || p.Kp % p.kb != 0 ||
        p.Kp > 8192 || p.Mp % 128 != 0 || p.Mp < p.Cout_p)
        return hipErrorInvalidValue;
    return p.kb == 128 ? launch_deep<128>(p, st) : launch_deep<64>(p, st);
}

}  // namespace isr
