// Internal declarations shared by the host code and the kernel launchers.
#ifndef ISR_INTERNAL_H
#define ISR_INTERNAL_H

#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>
#include <memory>
#include <string>
#include <vector>

#include "isr.h"

namespace isr {

// ---- noise table -----------------------------------------------------------
constexpr uint32_t NOISE_TABLE_MAX = 512;   // >= 510 thresholds between -255 and 255
constexpr uint32_t NOISE_GUIDE_BITS = 12;
constexpr uint32_t NOISE_GUIDE_SIZE = 1u << NOISE_GUIDE_BITS;

struct DeviceNoiseTable {
    uint32_t hi[NOISE_TABLE_MAX];
    uint32_t lo[NOISE_TABLE_MAX];
    uint16_t guide[NOISE_GUIDE_SIZE + 2];
    uint32_t n;      // thresholds in use
    int32_t dmin;    // delta = dmin + #{j < n : T[j] <= u}
};

bool build_noise_table(uint32_t sigma, std::vector<uint64_t> &T, uint32_t &R);
struct NoiseTable {
    std::vector<uint64_t> T;   // 2R ascending thresholds
    uint32_t R = 0;
};
// Shared, immutable table of a sigma (built on first use); null for sigma outside 1..1024.
std::shared_ptr<const NoiseTable> cached_noise_table(uint32_t sigma);
// Table of the stored-noise generator as one block of 32-bit words: n high words, n low words, guide table.
bool build_bank_table(uint32_t sigma, std::vector<uint32_t> &words, uint32_t &n_out, uint32_t &R_out);
// Records the hipError_t that isr_last_device_error() reports on this thread.
void set_last_device_error(int hip_error);
bool build_device_table(uint32_t sigma, DeviceNoiseTable &out);

// One (image, sigma) pair of a batched call.
struct NoiseItem {
    uint32_t image;          // index into the array of clean images
    uint32_t table_slot;     // index into the array of noise tables
    uint32_t image_id;       // counter word of the random stream
};

// Which image, table and sample index copy `copy` of a chunk draws from.  Single pair: the call's
// own; batch mode (items != null): copy s is slot slot_begin + s of a list in which item i owns
// the n_per_item slots from i * n_per_item on.
struct NoiseSource {
    const uint8_t *x;                // [C][H][W] clean image ([images][C][H][W] in batch mode)
    const DeviceNoiseTable *table;   // the table (batch mode: table 0 of the array indexed by table_slot)
    const NoiseItem *items;
    uint32_t key0, key1, image, phase, sample_begin, n_per_item;
    uint64_t slot_begin;
    int32_t C, H, W;
};

// ---- parsed model (host) ---------------------------------------------------
enum OpType : int32_t { OP_CONV = 1, OP_ADD = 2, OP_MAXPOOL = 3, OP_GAP = 4, OP_FC = 5 };

struct TensorDesc {
    int32_t C, H, W, zp;
    int32_t Cp;          // channels as stored on the device (multiple of 16; 4 for the input)
};

struct HostOp {
    OpType type;
    int32_t a = -1, b = -1, out = -1;
    int32_t k = 0, stride = 1, pad = 0, relu = 0;
    int32_t Ma = 0, Mb = 0, sh = 0;
    std::vector<int8_t> w;                  // CONV: OIHW, FC: [Cout][Cin]
    std::vector<int32_t> bias, M0, shift;
};

struct ParsedModel {
    int32_t C = 0, H = 0, W = 0, classes = 0;
    std::vector<TensorDesc> tensors;
    std::vector<HostOp> ops;
};

// Returns ISR_OK / ISR_ERR_FORMAT / ISR_ERR_UNSUPPORTED; `why` gets a short reason.
int parse_model(const void *blob, size_t bytes, ParsedModel &out, std::string &why);

// ---- device-side op descriptors -------------------------------------------
struct ConvParams {
    const int8_t *in;        // [B][H][W][Cin_p]
    int8_t *out;             // [B][Ho][Wo][Cout_p]
    const int8_t *w;         // [Mp][Kp] rows in MFMA row order, K = (tap, channel)
    const int32_t *bias;     // [Mp] bias - z_in * sum(w)
    const uint32_t *m0x2;    // [Mp] M0 << 1
    const uint32_t *rnd_lo;  // [Mp] low / high word of 2^(31 + shift)
    const uint32_t *rnd_hi;
    const uint32_t *shift;   // [Mp]
    const int32_t *m0s;      // [Mp] M0                                  } single-multiply path,
    const int32_t *chi;      // [Mp] 2^(shift-2) + z_out * 2^(shift-1)   } valid when every
    const int32_t *shm1;     // [Mp] shift - 1                           } shift is in [2, 22]
    int32_t fast_requant;
    // 1: no output channel can meet acc * M0 = (odd) * 2^(30 + shift) within its accumulator range, so RHA
    // never rounds an exact half and the sign correction of the rounding term is dead: the kernel then
    // takes (mulhi(acc, M0) + chi) >> (shift - 1) (decided per layer when the model is loaded)
    int32_t tie_free;
    // residual add folded into the epilogue (fuse_add != 0): with q the int8 result above,
    //   v = q * add_mul_self + res * add_mul_res + add_c0            (= (q-z)Ms + (res-zr)Mr)
    //   out = clamp((v + add_k + (v >> 31)) >> add_sh, add_lo, 127)  (add_k = 2^(sh-1) + z_o 2^sh)
    const int8_t *res;       // [B][Ho][Wo][Cout_p] other input of the add
    int32_t fuse_add, add_mul_self, add_mul_res, add_c0, add_k, add_sh, add_lo;
    int32_t add_tie_free;    // 1: no pair of int8 inputs makes v a negative exact half: out = clamp((v + add_k) >> add_sh)
    // fuse_add == 2: the residual is itself the output of a 1x1 stride-1 convolution (same pixels, same
    // channels) that has no other reader; the kernel computes it first, keeps it in registers and never
    // stores it.  Its operands:
    const int8_t *in2;       // [B][Ho][Wo][Cin2_p]
    const int8_t *w2;        // [Mp][Cin2_p] rows in MFMA row order
    const int32_t *bias2, *m0s2, *chi2, *shm12;   // as bias / m0s / chi / shm1
    int32_t Cin2_p, lo2, tie_free2;                // lo2: lower clamp of the residual tensor
    const uint32_t *ktab;    // [Kp/16] per 16-byte K chunk: ky | kx<<8, 0xFFFFFFFF = padding chunk; null = plain GEMM
    const int32_t *ktoff;    // [Kp/16] byte offset (ky*W + kx)*Cin_p + channel of the chunk
    const int8_t *zpad;      // 16 bytes of z_in: source of out-of-image taps for loads that go straight to LDS
    // 1x1 layers of the shapes expand_reduce.hip serves: the weights once more, one 1 KB block per MFMA operand
    // fragment (64 lanes x 16 bytes in lane order); null elsewhere
    const int8_t *wfrag;
    const int8_t *wfrag2;    // fuse_add == 2: the same of the residual convolution (w2)
    int32_t H, W, Cin_p, Ho, Wo, Cout_p;
    int32_t k, stride, pad, Kp, Mp;   // k: kernel size (k x k taps)
    int32_t force_tile;      // 0: the launcher picks the output tile; 1..7: 128x128, 128x256, 256x128, 256x256, 256x256 with 128x128 / 128x64 per wave, 256x256 of conv_patch.hip
    int32_t kb;              // K bytes per step of the kernel (64 or 128); Kp is a multiple of it
    int32_t zp_in, zp_out, relu;
    int32_t npix;            // B * Ho * Wo
    int32_t c4;              // 1: input is NHWC4 and a K chunk is 4 horizontal taps
};

// First convolution (7x7 stride 2 pad 3 on the NHWC4 image, 64 stored output channels)
// fused with the 3x3 stride-2 pad-1 max pooling that follows it.
struct StemPoolParams {
    const int8_t *in;        // [B][H][W][4] noisy image
    int8_t *out;             // [B][Hp][Wp][64] pooled activations
    const int8_t *w;         // [>= 64][256] rows in MFMA row order, K = (ky, kx padded to 8, channel padded to 4)
    const int32_t *bias, *m0s, *chi, *shm1;   // as in ConvParams (single-multiply requantisation)
    int32_t H, W, Ho, Wo, Hp, Wp;
    int32_t zp_in, zp_out, relu, tie_free, B;
    // fused_noise != 0: `in` is unused; the kernel draws the noisy input rows of its band itself (the
    // sampler of the noise stage on the same counter-based stream), copy b of the launch from `noise`
    int32_t fused_noise;
    NoiseSource noise;
};

// First convolution of the narrow small-image nets: 3x3 stride 1 pad 1 on the NHWC4 image
// into 16 stored channels (stem16.hip).
struct Stem16Params {
    const int8_t *in;        // [B][H][W][4]
    int8_t *out;             // [B][H][W][16]
    const int8_t *w;         // [16][64], K = (ky, kx padded to 4, channel padded to 4)
    const int32_t *bias, *m0s, *chi, *shm1;
    int32_t H, W, B, zp_in, lo, tie_free;
};

// Identity residual block in one kernel: t = conv3x3(x), y = add(conv3x3(t), x); both
// convolutions C -> C channels, stride 1, pad 1, on S x S images (basic_block.hip).
struct BlockDesc {           // one block of a chain, stored in device memory
    const int8_t *w1, *w2;   // [>= C][Kp] each, K = (tap, channel), Kp = 9 C rounded up to 64
    const int32_t *bias1, *m0s1, *chi1, *shm11;   // first convolution, as in ConvParams
    const int32_t *bias2, *m0s2, *chi2, *shm12;   // second convolution
    int32_t zp_x, zp_t, relu1;   // zero-points of x and t; lower clamp of t is zp_t when relu1
    int32_t zp_u, relu2;         // the same for the second convolution's own int8 result
    int32_t add_mul_self, add_mul_res, add_c0, add_k, add_sh, add_lo;   // as in ConvParams
    int32_t pad_;
};
struct BlockParams {
    const int8_t *in;        // [B][S][S][C] input x of the first block
    int8_t *out;             // [B][S][S][C] output of the last block
    const BlockDesc *blocks; // [nblocks] (device): a chain of blocks of one shape, each feeding the next
    int32_t nblocks;
    int32_t C, S, B;
    int32_t tie_free;        // every convolution and add of the chain is free of rounding ties
};

// Bottleneck block in one kernel: conv1x1 -> conv3x3 [-> conv1x1 + residual add with the block input
// when tail != 0]; 64 middle channels (bottleneck.hip) or 128 (bottleneck128.hip, tail only).
struct BneckParams {
    const int8_t *in;        // [B][H][W][Cin_p] block input x (also the residual of the tail)
    int8_t *out;             // tail: [B][H][W][Cout_p]; else the 3x3 output [B][H][W][64]
    const int8_t *w1;        // [>= Cmid][Cin_p] rows in MFMA row order
    const int8_t *w2;        // [>= Cmid][9 Cmid], K = (tap, channel)
    const int8_t *w3;        // [>= Cout_p][Cmid] (tail)
    const int32_t *bias1, *m0s1, *chi1, *shm11;   // as in ConvParams, per convolution
    const int32_t *bias2, *m0s2, *chi2, *shm12;
    const int32_t *bias3, *m0s3, *chi3, *shm13;
    // proj != 0 (with tail): the residual is not x but clamp(requant(conv1x1_p(x))), a projection shortcut
    // from 64 input channels computed in the same kernel; its weights [>= Cout_p][64] and constants:
    const int8_t *wp;
    const int32_t *biasp, *m0sp, *chip, *shm1p;
    int32_t proj, lop;       // lop: lower clamp of the projection's int8 result
    const int8_t *zpad;      // 16 readable bytes (source of halo pixels outside the image)
    int32_t Cin_p, Cout_p, H, W, B, tail;
    int32_t zp_t1;           // zero-point of the first convolution's output (padding value of the 3x3)
    int32_t lo1, lo2, lo3;   // lower clamps of the three int8 results
    int32_t add_mul_self, add_mul_res, add_c0, add_k, add_sh, add_lo;   // as in ConvParams
    int32_t tie_free;        // every requantisation (and the add) is free of rounding ties
};

// Closing 1x1 convolution + residual add of one bottleneck block and the opening 1x1 convolution of the next
// in one kernel (expand_reduce.hip): y = add(requant(W3 t2), x), t1n = requant(W1n y); 128 -> 512 -> 128 channels.
struct XrParams {
    const int8_t *t2;        // [npix][128] input of the expanding convolution
    const int8_t *x;         // [npix][512] residual
    int8_t *y;               // [npix][512] the sum (the next block's input and residual)
    int8_t *t1n;             // [npix][128] output of the reducing convolution
    const int8_t *a1, *a2;   // fragment-major weight copies (ConvParams::wfrag) of the two convolutions
    // in2 != null: the residual is not x but clamp(requant(Wp in2)), a projection from 256 channels computed in the kernel
    const int8_t *in2;       // [npix][256]
    const int8_t *ap;        // fragment-major copy of the projection weights
    const int32_t *biasp, *m0sp, *chip, *shm1p;   // [512]
    int32_t lop;             // lower clamp of the projection's int8 result
    int32_t Hin, Win, Ho, Wo, pstride;   // the projection reads pixel (pstride y, pstride x) of its Hin x Win input for output pixel (y, x)
    const int32_t *bias1, *m0s1, *chi1, *shm11;   // as in ConvParams, expanding convolution [512]
    const int32_t *bias2, *m0s2, *chi2, *shm12;   // reducing convolution [128]
    int32_t lo1, lo2;        // lower clamps of the two convolutions' int8 results
    int32_t add_mul_self, add_mul_res, add_c0, add_k, add_sh, add_lo;   // as in ConvParams
    int32_t npix;
    int32_t n2;              // output channels of the reducing convolution: 128, or 256 (stored residual only)
    int32_t k1;              // input channels of the expanding convolution: 128 (512 block channels) or 256 (1024; stored residual, n2 = 256)
};

// Down-sampling residual block in one kernel (trans_block.hip): t = conv3x3/2(x), u = conv3x3(t),
// r = conv1x1/2(x), y = add(r, u); x has C/2 channels on 2S x 2S pixels.
struct TransParams {
    const int8_t *in;        // [B][2S][2S][C/2]
    int8_t *out;             // [B][S][S][C]
    const int8_t *w1, *w2, *wp;   // weight rows in MFMA row order: [C][9 C/2 -> 64-multiple], [C][9 C -> 64-multiple], [C][64]
    const int32_t *bias1, *m0s1, *chi1, *shm11;   // as in ConvParams, per convolution
    const int32_t *bias2, *m0s2, *chi2, *shm12;
    const int32_t *biasp, *m0sp, *chip, *shm1p;
    int32_t C, S, B;
    int32_t zp_x, zp_t;      // zero-points of x and t (their padding values)
    int32_t lo1, lo2, lop;   // lower clamps of t, u, r
    int32_t add_mul_self, add_mul_res, add_c0, add_k, add_sh, add_lo;   // as in ConvParams; "self" is the projection r
    int32_t tie_free;
};

struct AddParams {
    const int8_t *a, *b;
    int8_t *out;
    int32_t za, zb, zo, Ma, Mb, sh, relu;
    int64_t n16;             // number of 16-byte groups
};

struct PoolParams {
    const int8_t *in;
    int8_t *out;
    int32_t H, W, Cp, Ho, Wo, k, stride, pad;
    int32_t B;
};

struct GapParams {
    const int8_t *in;        // [B][HW][Cp]
    int8_t *out;             // [B][Cp]
    int32_t HW, Cp, zp_in, zp_out, M0, sh, B;
};

struct FcParams {
    const int8_t *in;        // [B][Kp]
    const int8_t *w;         // [Kp / 16][classes_p][16]: 16-byte K chunks, class-contiguous
    const int32_t *bias;     // [classes], bias - z_in * sum(w)
    int32_t Kp, classes, classes_p, B;   // classes_p: classes rounded up to a multiple of 4
    int32_t *logits;         // [B][classes] or null
    int32_t *argmax;         // [B] or null
    uint32_t *counts;        // [classes] (accumulated) or null; [items][classes] in batch mode
    // batch mode (n_per_item != 0): copy s of the chunk is slot slot_begin + s of a list in which
    // every item owns n_per_item consecutive slots; its vote goes to counts[slot / n_per_item]
    uint32_t n_per_item;
    uint64_t slot_begin;
};


struct NoiseParams {
    const uint8_t *x;        // [C][H][W] clean image ([images][C][H][W] in batch mode)
    const DeviceNoiseTable *table;   // the table (batch mode: table 0 of the array indexed by table_slot)
    int8_t *out;             // [B][H][W][4]
    int32_t C, H, W;
    uint32_t key0, key1, image, phase, sample_begin, count;
    // batch mode (items != null): copy s of the chunk is slot slot_begin + s; item i owns slots
    // [i * n_per_item, (i + 1) * n_per_item) and sample index = slot - i * n_per_item; the
    // launch covers items item_first .. item_first + item_count - 1 (one grid row each)
    const NoiseItem *items;
    uint32_t n_per_item, item_first, item_count;
    uint64_t slot_begin;
};

// Stored-noise generator: count tensors of d draws each, int16.
struct NoiseBankParams {
    const uint32_t *thi, *tlo;   // [n] high / low words of the ascending thresholds (device)
    const uint16_t *guide;       // [NOISE_GUIDE_SIZE + 2]: #{j : thi[j] < (b << (32 - NOISE_GUIDE_BITS))} (device)
    int32_t n, R;                // n = 2R thresholds; draw = #{j : T[j] <= u} - R
    int16_t *out;                // [count][d]
    uint32_t d;                  // draws per tensor, a multiple of 4
    uint32_t key0, key1, bank, first, count;
};

// ---- floating-point comparison systems (float_path.hip) ------------------------------------
// Continuous Gaussian noise: copy s, logical element p = (c*H + y)*W + x gets x[p] + sigma z with z the
// standard-normal draw of counter (p >> 2, sample_begin + s, image, 8 + phase), element p & 3.
struct FloatNoiseParams {
    const uint8_t *x;        // [C][H][W] clean image
    void *out;               // quant: int8 [B][H][W][4], clamp(round(v), 0, 255) - 128; else float [B][H][W][4], v - center
    int32_t C, H, W;
    uint32_t key0, key1, image, phase, sample_begin, count;
    float sigma, center;
    int32_t quant;
};

// fp32 convolution as an implicit GEMM on the fp32 MFMA, NHWC activations:
//   t = act((bias + sum over in-bounds taps of in * w) * scale);  out = res ? act_add(ma * t + mb * res) : t
struct FConvParams {
    const float *in;         // [B][H][W][Cin_p]
    float *out;              // [B][Ho][Wo][Cout_p]
    const float *res;        // [B][Ho][Wo][Cout_p] or null
    const float *w;          // [Kq][Cout_pp][4]: quad kq holds k = 4 kq .. 4 kq + 3 of K = (tap, channel); rows in MFMA row order per 32 channels
    const float *bias, *scale;   // [Cout_pp], by channel
    const int32_t *ktab;     // [Kq]: dy << 24 | dx << 16 | channel offset of the quad; -1 = padding quad
    int32_t H, W, Cin_p, Ho, Wo, Cout_p, Cout_pp, stride, pad, Kq;   // Kq a multiple of 4
    int32_t npix;            // B * Ho * Wo
    int32_t relu, add_relu;
    float ma, mb;
};
struct FAddParams { const float *a, *b; float *out; float ma, mb; int32_t relu; int64_t n4; };
struct FPoolParams { const float *in; float *out; int32_t H, W, Cp, Ho, Wo, k, stride, pad, B; };
struct FGapParams { const float *in; float *out; int32_t HW, Cp, B; float scale; };
struct FVoteParams { const float *logits; int32_t classes, stride, B; int32_t *argmax; uint32_t *counts; };
hipError_t launch_float_noise(const FloatNoiseParams &p, hipStream_t st);
hipError_t launch_fconv(const FConvParams &p, hipStream_t st);
int fconv_tile_m(int cout_p);   // channels per output tile chosen for a layer (Cout_pp is a multiple of it)
hipError_t launch_fadd(const FAddParams &p, hipStream_t st);
hipError_t launch_fmaxpool(const FPoolParams &p, hipStream_t st);
hipError_t launch_fgap(const FGapParams &p, hipStream_t st);
hipError_t launch_fvote(const FVoteParams &p, hipStream_t st);

// Name of the kernel instance the last launcher call on this thread enqueued (template arguments
// included, as a profiler prints them); the per-kernel timing report is keyed by it.
void set_kernel_name(const char *name);
const char *last_kernel_name();

// Kernel launchers (kernels.hip / conv_igemm.hip).  All asynchronous on `st`.
hipError_t launch_noise_bank(const NoiseBankParams &p, hipStream_t st);
hipError_t launch_noise(const NoiseParams &p, hipStream_t st);
hipError_t launch_conv(const ConvParams &p, hipStream_t st);
bool conv_patch_supported(const ConvParams &p);
hipError_t launch_conv_patch(const ConvParams &p, hipStream_t st);   // deep 3x3 layers, pixel rows staged once per channel slice (conv_patch.hip)
hipError_t launch_conv_deep(const ConvParams &p, hipStream_t st);   // 256 x 256 tiles, 128 x 128 per wave (conv_deep.hip)
hipError_t launch_stem_pool(const StemPoolParams &p, hipStream_t st);
bool stem_pool_supported(int k, int stride, int pad, int cout_p, int H, int W, int fast_requant, int pool_k,
                         int pool_stride, int pool_pad);
hipError_t launch_stem16(const Stem16Params &p, hipStream_t st);
bool stem16_supported(int k, int stride, int pad, int cout_p, int H, int W, int fast_requant);
hipError_t launch_basic_block(const BlockParams &p, hipStream_t st);
bool basic_block_supported(int channels, int size);
hipError_t launch_bottleneck(const BneckParams &p, hipStream_t st);
bool bottleneck_supported(int cin_p, int cmid_p, int cout_p, int tail);
hipError_t launch_bottleneck128(const BneckParams &p, hipStream_t st);
bool expand_reduce_supported(const ConvParams &expand, const ConvParams &reduce);
void expand_reduce_params(const ConvParams &expand, const ConvParams &reduce, const int8_t *a, const int8_t *b, int8_t *y,
                          int8_t *t1n, int32_t copies, XrParams &xp);
hipError_t launch_expand_reduce(const XrParams &p, int add_tie_free, hipStream_t st);   // expand_reduce.hip   // 128 middle channels, identity blocks (bottleneck128.hip)
bool bottleneck128_supported(int cin_p, int cmid_p, int cout_p);
hipError_t launch_trans_block(const TransParams &p, hipStream_t st);
bool trans_block_supported(int cout, int size_out);
hipError_t launch_add(const AddParams &p, hipStream_t st);
hipError_t launch_maxpool(const PoolParams &p, hipStream_t st);
hipError_t launch_gap(const GapParams &p, hipStream_t st);
hipError_t launch_fc(const FcParams &p, hipStream_t st);
hipError_t launch_fill_u32(uint32_t *p, uint32_t value, size_t n, hipStream_t st);
// Tile geometry of the convolution kernel chosen for (Cout_p): rows per M tile.
int conv_tile_m(int cout_p);
// K bytes per step chosen for a layer (see conv_igemm.hip).
int conv_k_step(int kreal, int cin_p, int cout_p, int fast_requant);

}  // namespace isr

#endif
