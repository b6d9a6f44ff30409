/*
 * isr.h -- C ABI of the MI355X integer-randomized-smoothing library.
 *
 * The library runs the Monte-Carlo loop behind the paper's certification
 * procedure (Alg. 1) and prediction procedure (Alg. 2, appendix "Practical
 * Prediction"): for every sample index it adds discrete-Gaussian noise
 * (Def. 3.3) to the quantized image on the integer pixel grid, runs the
 * int8 base classifier with integer-only arithmetic (Thm. 3.2, step 1) and
 * tallies the predicted class; the tallies then give the one-sided lower
 * confidence bound and the l2 radius sigma * Phi^-1(p_A) (Alg. 1) or the
 * binomial test (Alg. 2).  Every step of the loop runs in HIP kernels on the
 * GPU; only the O(classes) decision on the tallies runs on the host in fp64.
 *
 * Conventions
 *   - "host" / "device" on a pointer says which memory it must point to.
 *   - All functions return ISR_OK or an ISR_ERR_* code; abstention is not an
 *     error (cls == ISR_ABSTAIN, radius == 0, status ISR_OK).
 *   - sigma and radius are in grid units of the uint8 pixel lattice (one unit
 *     = one step of the 8-bit grid); 1 <= sigma <= 1024.
 *   - Results are a pure function of (model, x, sigma, n0, n, alpha, seed,
 *     image_id): independent of the chunk size and of kernel choices.
 *   - Calls on one isr_model must not overlap in time (one workspace).
 */
#ifndef ISR_H
#define ISR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ISR_OK 0
#define ISR_ERR_ARG 1          /* null pointer or value outside the documented domain */
#define ISR_ERR_FORMAT 2       /* model blob malformed or fails validation */
#define ISR_ERR_UNSUPPORTED 3  /* well-formed, but a shape/op the kernels do not cover */
#define ISR_ERR_WORKSPACE 4    /* no workspace set, or too small for the chunk size */
#define ISR_ERR_DEVICE 5       /* a HIP call failed; isr_last_device_error() has the code */

#define ISR_ABSTAIN (-1)

typedef struct isr_model isr_model; /* opaque; owned by the library until isr_free_model */

typedef struct isr_result {
    int32_t cls;      /* predicted class 0..classes-1, or ISR_ABSTAIN */
    double radius;    /* certified l2 radius in grid units (Alg. 1); 0 on abstain / for predict */
    double p_lower;   /* certify: Clopper-Pearson lower bound of p_A; predict: binomial p-value */
    uint32_t n_top;   /* certify: estimation votes of the selected class; predict: n_A */
    uint32_t n_second;/* predict: n_B (runner-up votes); certify: 0 */
    /* certify, integer-only tail (Thm 3.2, proof steps 2-3), for integer sigma in 1..1024 when a
     * class is returned: the radius with the discrete law's own quantile in place of Phi^-1 --
     * radius_int = the largest lattice point t (grid units) with floor(2^64 P[delta <= t]) <=
     * floor(2^64 p_lower), delta ~ N_Z(0, sigma^2), by lookup in the sampler's cdf table (may be
     * <= 0 when p_lower is barely above 1/2), and radius_sq_int = t * t for t > 0, else 0 (squared
     * grid units).  t <= radius always (t lies in [radius - 3/2, radius - 1/2] up to the table's
     * resolution).  Both 0 on abstain, for predict, and for a non-integer sigma.  The bound
     * p_lower itself stays float64: the paper gives no integer form of the confidence bound. */
    int32_t radius_int;
    uint64_t radius_sq_int;
} isr_result;

/* ---- model ------------------------------------------------------------- */

/* ISRM model blob (little-endian 32-bit fields):
 *   header : 'ISRM', version 1, in_C, in_H, in_W, classes, n_tensors, n_ops
 *   tensors: n_tensors x {C, H, W, zero_point}; tensor 0 = input (pixel - 128, zp 0)
 *   ops    : n_ops x {type, payload_bytes, payload}, executed in order:
 *     1 CONV    in, out, k, stride, pad, relu, w int8[Cout][Cin][k][k] (padded
 *               to 4 bytes), bias i32[Cout], M0 i32[Cout] in [2^30,2^31), shift i32[Cout] in [0,31]
 *               acc = bias + sum over in-bounds taps (q - z_in) w;
 *               q_out = clamp(z_out + RHA(acc * M0, 31 + shift), relu ? z_out : -128, 127)
 *     2 ADD     a, b, out, Ma, Mb, shift, relu:  RHA((qa-za) Ma + (qb-zb) Mb, shift), same clamp
 *     3 MAXPOOL in, out, k, stride, pad (max over in-bounds taps)
 *     4 GAP     in, out, M0, shift: requantised sum over H x W of (q - z_in)
 *     5 FC      in, out, w int8[Cout][Cin], bias i32[Cout]: int32 logits, no requantisation
 *   RHA(v, s) = round-half-away-from-zero of v / 2^s (one rounding).
 *
 * isr_load_model parses and validates a blob (host memory), re-lays the weights
 * for the MFMA kernels and uploads them to the current HIP device.  The blob is
 * not referenced after the call returns. */
int isr_load_model(const void *blob_host, size_t bytes, isr_model **out);
int isr_free_model(isr_model *m);
/* Host-only structural validation of a blob (no GPU needed). */
int isr_validate_model(const void *blob_host, size_t bytes);
int isr_model_info(const isr_model *m, int *C, int *H, int *W, int *num_classes);

/* Device scratch for activations of `chunk_samples` noisy copies processed at a
 * time.  The caller allocates it (e.g. a torch uint8 tensor), keeps it alive
 * while the model uses it, and passes the HIP stream all work is enqueued on
 * (NULL = the default stream). */
size_t isr_workspace_bytes(const isr_model *m, uint32_t chunk_samples);
int isr_set_workspace(isr_model *m, void *workspace_device, size_t bytes, uint32_t chunk_samples,
                      void *hip_stream);

/* ---- the two procedures -------------------------------------------------- */

/* Alg. 1 (certification).  x_device: uint8 [C][H][W] image in device memory.
 * Runs n0 selection samples (phase 0) and n estimation samples (phase 1),
 * takes c_A = the most voted class of phase 0 (lowest index on ties), the
 * one-sided (1-alpha) Clopper-Pearson lower bound p_A from phase-1 votes of
 * c_A, and returns (c_A, sigma * Phi^-1(p_A)) if p_A > 1/2, else abstains.
 * counts0_host / counts1_host: optional uint32[classes] outputs (host). */
int isr_certify(isr_model *m, const uint8_t *x_device, uint32_t sigma, uint32_t n0, uint32_t n,
                double alpha, uint64_t seed, uint32_t image_id, isr_result *out,
                uint32_t *counts0_host, uint32_t *counts1_host);

/* Alg. 2 (prediction).  Runs n samples (phase 0), takes the two most voted
 * classes (n_A >= n_B) and returns c_A if the two-sided binomial p-value of
 * n_A out of n_A + n_B at 1/2 is <= alpha, else abstains. */
int isr_predict(isr_model *m, const uint8_t *x_device, uint32_t sigma, uint32_t n, double alpha,
                uint64_t seed, uint32_t image_id, isr_result *out, uint32_t *counts_host);

/* ---- the two procedures over many (image, sigma) pairs at once ------------- */

/* One pair of a batched call: which image of the array, which noise level, and
 * the image_id word of its random stream. */
typedef struct isr_item {
    uint32_t image;    /* index into x_device, < n_images */
    uint32_t sigma;    /* 1..1024 grid units */
    uint32_t image_id;
} isr_item;

/* Alg. 1 / Alg. 2 for n_items (image, sigma) pairs in one pass -- the sweeps of the
 * paper's evaluation (many test images, certification sigma varied against the
 * training sigma, prediction with small n as in the appendix table of Alg. 2's
 * sample sizes).  x_device: uint8 [n_images][C][H][W] in device memory;
 * items_host: n_items descriptors (host); at most 8 distinct sigma values per
 * call.  All pairs share n0, n, alpha and seed.  out_host[i], and row i of the
 * optional uint32 [n_items][classes] vote arrays (host), are exactly what
 * isr_certify / isr_predict return for (x[items[i].image], items[i].sigma, n0, n,
 * alpha, seed, items[i].image_id).  The sample slots of all pairs form one list
 * that is cut into chunks of chunk_samples regardless of pair boundaries, so a
 * call with small n per pair still launches full chunks.  ISR_ERR_ARG for an
 * image index or sigma out of range, more than 8 distinct sigmas, n_items == 0. */
int isr_certify_batch(isr_model *m, const uint8_t *x_device, uint32_t n_images, const isr_item *items_host,
                      uint32_t n_items, uint32_t n0, uint32_t n, double alpha, uint64_t seed,
                      isr_result *out_host, uint32_t *counts0_host, uint32_t *counts1_host);
int isr_predict_batch(isr_model *m, const uint8_t *x_device, uint32_t n_images, const isr_item *items_host,
                      uint32_t n_items, uint32_t n, double alpha, uint64_t seed, isr_result *out_host,
                      uint32_t *counts_host);

/* ---- noise stored ahead of training ---------------------------------------- */

/* Training with discrete-Gaussian data augmentation (section "Quantization Aware Training
 * with ...": noise for a batch is sampled once, stored, then shuffled and added to inputs):
 * fills out_device with count tensors of d draws each from N_Z(0, sigma^2) (Def. 3.3), int16,
 * [count][d], device memory.  Draw p of tensor first + t is the table sampler of
 * isr_noise_table applied to the uniform 64-bit word of counter (p >> 2, first + t, bank_id,
 * 4 | half), word p & 3, key = seed: the inference sampler's stream with phase 2, unsaturated
 * (|draw| <= R <= 9216).  Needs no model; enqueued on hip_stream (NULL = default) and
 * synchronised before returning.  ISR_ERR_ARG unless 1 <= sigma <= 1024, d a positive
 * multiple of 4, first + count <= 2^32. */
int isr_noise_bank(uint32_t sigma, uint64_t seed, uint32_t bank_id, uint32_t first, uint32_t count, uint32_t d,
                   int16_t *out_device, void *hip_stream);

/* isr_noise_bank for callers that cannot allocate device memory: code under HIP graph capture
 * set-up, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same draws, same
 * error behaviour as isr_noise_bank, but the sampler's table goes into a fixed array in device
 * memory that is part of the library's code object (isr_noise_bank_static_capacity() bytes, 64 KiB:
 * room for every sigma up to about 420; each GPU the library runs on holds its own copy for the
 * life of the process) and the call performs no hipMalloc / hipFree.  ISR_ERR_WORKSPACE when the
 * table of this sigma does not fit the array.  All calls on one GPU share that array: calls that
 * overlap in time on one GPU, from any thread or stream, race -- serialise them.  A call leaves
 * its table in the array; the next call overwrites it before its kernel runs. */
int isr_noise_bank_static(uint32_t sigma, uint64_t seed, uint32_t bank_id, uint32_t first, uint32_t count,
                          uint32_t d, int16_t *out_device, void *hip_stream);
size_t isr_noise_bank_static_capacity(void);

/* ---- the paper's floating-point comparison systems ------------------------- */

/* Section "Experiments" compares integer randomized smoothing with standard randomized smoothing
 * (continuous Gaussian noise N(0, sigma^2 I), radius sigma * Phi^-1(p_A)) in two forms:
 *   ISR_FLOATRS_QUANT  the noisy image is rounded back onto the 8-bit pixel grid (nearest level,
 *                      ties to even, saturated to [0, 255]) and classified by the int8 network;
 *   ISR_FLOATRS_FP     the noisy image is classified by the fp32 network behind the quantized one:
 *                      every tensor holds the real values r = q - z that the int8 codes stand for
 *                      and every op is the blob's op without its rounding and without saturation at
 *                      the ends of the int8 range (a ReLU clamp at the zero-point stays as r >= 0):
 *                      CONV r_out = act(M (bias + sum r_in w)), M = M0 2^-(31 + shift);
 *                      ADD act((Ma r_a + Mb r_b) 2^-shift); MAXPOOL; GAP M sum r_in; FC bias + sum r_in w;
 *                      input r_0 = x + sigma z - 128 - z_0.  Arithmetic: fp32, accumulation on the
 *                      fp32 matrix cores.
 * Both run Alg. 1 as isr_certify does (same two loops, same decision on the tallies).  The noise of
 * copy s, logical element p = (c*H + y)*W + x, is sigma * z with z the binary32 standard-normal draw
 * of Philox4x32-10 counter (p >> 2, s, image_id, 8 + phase), key = seed, element p & 3: words
 * (w0, w1) give elements 0 and 1, (w2, w3) elements 2 and 3 by the Box-Muller transform with
 * u = ((w_a >> 8) + 1) / 2^24, v = (w_b >> 8) / 2^24, every step one IEEE binary32 operation, so
 * the draws -- and with them the rounded inputs and the int8 logits of ISR_FLOATRS_QUANT -- are
 * reproducible bit for bit; the fp32 logits of ISR_FLOATRS_FP are reproducible up to the rounding
 * of fp32 sums.  sigma: any float in [0, 4096] (grid units).  radius_int / radius_sq_int of the
 * result are 0.  ISR_FLOATRS_FP keeps fp32 copies of all weights on the device from its first use
 * and processes isr_float_chunk() copies at a time inside the workspace of isr_set_workspace, which
 * must hold isr_float_workspace_bytes() bytes (ISR_ERR_WORKSPACE otherwise); ISR_ERR_UNSUPPORTED
 * for a model whose FC layer reads a non-square tensor. */
#define ISR_FLOATRS_QUANT 1
#define ISR_FLOATRS_FP 2
size_t isr_float_workspace_bytes(isr_model *m, uint32_t chunk_samples, int system);
uint32_t isr_float_chunk(const isr_model *m, int system);
int isr_float_certify(isr_model *m, const uint8_t *x_device, float sigma, uint32_t n0, uint32_t n, double alpha,
                      uint64_t seed, uint32_t image_id, int system, isr_result *out, uint32_t *counts0_host,
                      uint32_t *counts1_host);
/* Parity hooks of the comparison systems, as isr_debug_noisy / isr_debug_forward / isr_debug_tensor:
 * out_host of isr_float_debug_noisy is int8 [count][C][H][W] (ISR_FLOATRS_QUANT: the rounded,
 * recentred input) or float [count][C][H][W] (ISR_FLOATRS_FP: x + sigma z itself), count <=
 * isr_float_chunk(); logits_host of isr_float_debug_forward is int32 resp. float [count][classes];
 * isr_float_debug_tensor returns one tensor of the fp32 network as float [C][H][W]
 * (ISR_ERR_UNSUPPORTED for a convolution output that only feeds a residual add: the add runs in
 * that convolution's kernel and the tensor is never stored). */
int isr_float_debug_noisy(isr_model *m, const uint8_t *x_device, float sigma, uint64_t seed, uint32_t image_id,
                          uint32_t phase, uint32_t sample_begin, uint32_t count, int system, void *out_host);
int isr_float_debug_forward(isr_model *m, const uint8_t *x_device, float sigma, uint64_t seed, uint32_t image_id,
                            uint32_t phase, uint32_t sample_begin, uint32_t count, int system, void *logits_host,
                            int32_t *argmax_host, uint32_t *counts_host);
int isr_float_debug_tensor(isr_model *m, const uint8_t *x_device, float sigma, uint64_t seed, uint32_t image_id,
                           uint32_t phase, uint32_t sample, int32_t tensor_id, float *out_host);

/* ---- parity / resume hooks (sample-index ranges are reproducible) -------- */

/* Noisy copies for sample indices [sample_begin, sample_begin+count) of one
 * phase: out_host gets count * C*H*W int8 values in [C][H][W] order, each
 * clamp(x + delta, 0, 255) - 128.  count <= chunk_samples. */
int isr_debug_noisy(isr_model *m, const uint8_t *x_device, uint32_t sigma, uint64_t seed,
                    uint32_t image_id, uint32_t phase, uint32_t sample_begin, uint32_t count,
                    int8_t *out_host);

/* Full forward for a sample-index range: any of logits_host (count*classes
 * int32), argmax_host (count int32), counts_host (classes uint32, accumulated
 * into) may be NULL.  Votes are additive over ranges.  Any count >= 1. */
int isr_debug_forward(isr_model *m, const uint8_t *x_device, uint32_t sigma, uint64_t seed,
                      uint32_t image_id, uint32_t phase, uint32_t sample_begin, uint32_t count,
                      int32_t *logits_host, int32_t *argmax_host, uint32_t *counts_host);

/* One intermediate tensor (id as in the blob's tensor table; not the logits)
 * of ONE noisy copy, converted to int8 [C][H][W] on the host. */
int isr_debug_tensor(isr_model *m, const uint8_t *x_device, uint32_t sigma, uint64_t seed,
                     uint32_t image_id, uint32_t phase, uint32_t sample, int32_t tensor_id,
                     int8_t *out_host);

/* Which plan isr_debug_tensor serves a tensor from while fusion is enabled: *from_fused_out = 1 when the
 * fused kernels store that tensor themselves (the bytes returned are the fused kernel's own output),
 * 0 when no fused kernel stores it and the op-by-op kernels produce it for the hook.  Lets a parity
 * test say which kernels a tensor comparison exercises.  ISR_ERR_ARG for an id outside the table. */
int isr_debug_tensor_source(const isr_model *m, int32_t tensor_id, int *from_fused_out);

/* ---- host-only pieces (no GPU needed) ------------------------------------ */

/* Inverse-CDF thresholds of the discrete Gaussian N_Z(0, sigma^2) (Def. 3.3):
 * T[i] = floor(2^64 P[delta <= i - R]) for i in [0, 2R); a uniform 64-bit u
 * gives delta = -R + #{i : T[i] <= u}.  Writes min(cap, 2R) entries to T_host
 * (may be NULL with cap 0) and R to R_out. */
int isr_noise_table(uint32_t sigma, uint64_t *T_host, size_t cap, uint32_t *R_out);

/* One-sided (1-alpha) Clopper-Pearson lower bound after k successes in n trials (Alg. 1). */
int isr_cp_lower(uint32_t k, uint32_t n, double alpha, double *p_lower);
/* Standard normal quantile Phi^-1(p), 0 < p < 1 (radius factor of Alg. 1). */
int isr_normal_quantile(double p, double *z);
/* Integer-only tail of the certification (Thm 3.2, proof steps 2 and 3): the inverse cdf of
 * the one-dimensional discrete Gaussian N_Z(0, sigma^2) by lookup in the table of
 * isr_noise_table -- t_out = the largest lattice point t (input grid units) with
 * floor(2^64 P[delta <= t]) <= floor(2^64 p_lower), -R - 1 if there is none -- and the squared
 * radius radius_sq_out = t * t for t > 0, else 0 (squared grid units).  With the discrete
 * law's Phi^-1 the radius sigma * Phi^-1(p) of Alg. 1 is t itself.  Host only, integers but
 * for the conversion of p_lower; either output pointer may be NULL.  ISR_ERR_ARG unless
 * 1 <= sigma <= 1024 and 0 <= p_lower <= 1. */
int isr_discrete_quantile(uint32_t sigma, double p_lower, int32_t *t_out, uint64_t *radius_sq_out);
/* Two-sided binomial p-value min(1, 2 P[Bin(n_a+n_b, 1/2) >= n_a]) (Alg. 2). */
int isr_binom_pvalue(uint32_t n_a, uint32_t n_b, double *pvalue);
/* Decisions of Alg. 1 / Alg. 2 on tallies already on the host. */
int isr_decide_certify(const uint32_t *counts0, const uint32_t *counts1, uint32_t classes,
                       double sigma, uint32_t n, double alpha, isr_result *out);
int isr_decide_predict(const uint32_t *counts, uint32_t classes, double alpha, isr_result *out);

/* The paper's two evaluation metrics (section "Evaluation Metrics") over `count`
 * certification results with ground-truth labels (host arrays):
 *   certified percentage  CP    = #{i : not abstained} / count
 *   certified accuracy    CA(r) = #{i : not abstained, cls_i == label_i, radius_i >= r} / #{i : not abstained}
 * (the denominator of CA as in the paper's formula; CA(r) * CP is the fraction of
 * the whole set; CA = 0 when every result abstained).  cp_out may be NULL; ca_out
 * gets n_radii values for the thresholds radii[] (same unit as isr_result.radius);
 * n_radii may be 0, then labels, radii and ca_out may be NULL. */
int isr_certified_metrics(const isr_result *results, const int32_t *labels, uint32_t count, const double *radii,
                          uint32_t n_radii, double *cp_out, double *ca_out);

/* Kernel-variant switch for parity checks: enable = 1 (the default) lets the
 * library fuse ops of the blob into one kernel where that is faster (a residual add
 * into the convolution before it; the first convolution with the max pooling after
 * it; a 1x1 convolution that only feeds a residual add into that add's kernel;
 * whole residual blocks of the narrow nets; the convolutions of a bottleneck block
 * with 64 middle channels; the closing 1x1 convolution + add of a bottleneck block
 * with 128 or 256 middle channels together with the opening 1x1 convolution of the
 * next block, which still writes the sum but does not read it back); 2 also folds identity bottleneck blocks with 128 middle
 * channels into one kernel (correct, at present slower than their three kernels);
 * 0 runs every op of the blob as its own kernel.  Results are identical in every
 * mode; tensors that a fused kernel never stores are served by the unfused plan
 * in isr_debug_tensor.  ISR_ERR_ARG for other values. */
int isr_set_fusion(isr_model *m, int enable);

/* Kernel-variant switch for parity checks and tuning: output tile of the
 * direct-to-LDS convolution kernel for layers with more than 64 stored output
 * channels.  0 (the default) lets the library choose per launch; 1..4 force
 * 128x128, 128x256, 256x128, 256x256 (channels x pixels; the 256-channel tiles
 * only where a layer has more than 128 channels); 5 forces 256x256 computed by
 * four waves of 128x128 each instead of sixteen of 64x64, 6 by eight waves of
 * 128x64; 7 forces, on 3x3 stride-1 layers with at least 256 output channels and
 * a multiple of 128 input channels, the kernel that stages a tile's pixel rows
 * once per channel slice (automatic choice elsewhere).  Results are identical for
 * every choice.  ISR_ERR_ARG for other values. */
int isr_set_conv_tile(isr_model *m, int tile);

/* ---- per-kernel timing (HIP events on the model's stream) ------------------ */

typedef struct isr_kernel_stat {
    char name[80];        /* kernel instance as a profiler prints it, template arguments included:
                             "conv_dma_kernel<BM, BN, KB, stages, fused add, min blocks, wave tile>",
                             "bottleneck_kernel<tail, tie-free>", "stem_pool_kernel", "noise_kernel", ... */
    int32_t is_conv;      /* 1: the kernel executes convolution ops of the model (S3/S4 of the path) */
    uint64_t launches;    /* launches timed so far */
    double total_ms;      /* sum of their durations */
    double alg_ops;       /* algorithmic integer ops of those launches (2 per multiply-accumulate,
                             real channel counts, no padding); 0 for the memory-bound kernels */
    double alg_bytes;     /* algorithmic bytes read + written by those launches */
} isr_kernel_stat;

/* every_chunks > 0: bracket every kernel launch of each every_chunks-th chunk
 * with HIP events and accumulate per kernel instance (the chunk is followed by a
 * stream synchronisation); 0 switches timing off.  Either call resets the
 * accumulators. */
int isr_profile(isr_model *m, uint32_t every_chunks);
/* Copies up to cap accumulated entries to out_host and their number to n_out. */
int isr_profile_read(const isr_model *m, isr_kernel_stat *out_host, uint32_t cap, uint32_t *n_out);

const char *isr_strerror(int status);
int isr_last_device_error(void); /* hipError_t of the last failing HIP call on this thread */

#ifdef __cplusplus
}
#endif
#endif /* ISR_H */
