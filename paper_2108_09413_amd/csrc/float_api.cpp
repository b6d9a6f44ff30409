// C ABI of the two floating-point comparison systems of the paper's evaluation (section "Experiments"):
// FloatRS-quant -- continuous Gaussian noise rounded back onto the pixel grid, then the int8 network
// (the integer path's loop with another input stage, api.cpp) -- and FloatRS-fp -- continuous Gaussian
// noise, then the fp32 network derived from the quantized one: every tensor holds the real values
// r = q - z behind the int8 codes and every op is the quantized op without its rounding and without
// the saturation at the ends of the int8 range.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <vector>

#include "isr_internal.h"
#include "model.h"

using namespace isr;

#define HIP_TRY(expr)                                     \
    do {                                                  \
        hipError_t e_ = (expr);                           \
        if (e_ != hipSuccess) {                           \
            set_last_device_error((int)e_);               \
            return ISR_ERR_DEVICE;                        \
        }                                                 \
    } while (0)

namespace isr {

struct FloatOp {
    OpType type;
    int a = -1, b = -1, out = -1;
    FConvParams conv{};            // CONV and FC (an FC layer is a convolution over the whole input)
    int res = -1;                  // tensor read by the residual add folded into the convolution, or -1
    float ma = 0.f, mb = 0.f;      // ADD
    int relu = 0;
    FPoolParams pool{};
    float gap_scale = 0.f;
    double flops = 0.0, bytes = 0.0;   // per copy: 2 per multiply-accumulate on real channels; fp32 bytes in + out
};

struct FloatNet {
    std::vector<FloatOp> ops;
    Plan plan;                     // tensor placement: the ops' tensor ids with the int8 planner, whose bytes for B copies hold B / 4 fp32 copies
    uint32_t planned_chunk = 0;
    uint8_t *dconst = nullptr;
    int status = ISR_OK;           // ISR_ERR_UNSUPPORTED when an op has no float kernel
};

void free_float_net(FloatNet *net) {
    if (!net) return;
    if (net->dconst) (void)hipFree(net->dconst);
    delete net;
}

}  // namespace isr

namespace {

// MFMA 32x32 accumulator: register i of lane half h is row 8 (i / 4) + 4 h + i % 4; the weights of
// channel 16 h + i go to that row so that a lane ends up with 16 consecutive channels.
int mfma_row_of_channel(int c) {
    const int h = c >> 4, a = (c & 15) >> 2, b = c & 3;
    return 8 * a + 4 * h + b;
}

size_t put(std::vector<uint8_t> &arena, const void *src, size_t bytes) {
    const size_t off = (arena.size() + 255) & ~(size_t)255;
    arena.resize(off + bytes);
    std::memcpy(arena.data() + off, src, bytes);
    return off;
}

// Weights, per-channel constants and the K table of one convolution (k x k taps over a [H][W][Cin_p] input).
int build_conv(const ParsedModel &pm, const HostOp &o, int k, int stride, int pad, bool fc, std::vector<uint8_t> &arena,
               FloatOp &f) {
    const TensorDesc &ti = pm.tensors[o.a], &to = pm.tensors[o.out];
    if (k > 127) return ISR_ERR_UNSUPPORTED;
    FConvParams &c = f.conv;
    c.H = ti.H; c.W = ti.W; c.Cin_p = ti.Cp; c.Ho = to.H; c.Wo = to.W; c.Cout_p = to.Cp;
    const int bm = fconv_tile_m(c.Cout_p);
    c.Cout_pp = (c.Cout_p + bm - 1) / bm * bm;
    c.stride = stride; c.pad = pad;
    const int kq_real = k * k * ti.Cp / 4;
    c.Kq = (kq_real + 3) & ~3;
    c.relu = fc ? 0 : o.relu;
    std::vector<float> w((size_t)c.Kq * c.Cout_pp * 4, 0.f), bias(c.Cout_pp, 0.f), scale(c.Cout_pp, 0.f);
    std::vector<int32_t> ktab(c.Kq, -1);
    for (int kq = 0; kq < kq_real; ++kq) {
        const int tap = 4 * kq / ti.Cp, coff = 4 * kq % ti.Cp;
        ktab[kq] = ((tap / k) << 24) | ((tap % k) << 16) | coff;
    }
    for (int oc = 0; oc < to.C; ++oc) {
        const int row = (oc / 32) * 32 + mfma_row_of_channel(oc % 32);
        for (int ic = 0; ic < ti.C; ++ic)
            for (int t = 0; t < k * k; ++t) {
                const int kidx = t * ti.Cp + ic;
                w[((size_t)(kidx / 4) * c.Cout_pp + row) * 4 + kidx % 4] = (float)o.w[((size_t)oc * ti.C + ic) * k * k + t];
            }
        bias[oc] = (float)o.bias[oc];
        scale[oc] = fc ? 1.f : (float)std::ldexp((double)o.M0[oc], -(31 + o.shift[oc]));
    }
    // offsets now, pointers after the upload
    c.w = (const float *)put(arena, w.data(), w.size() * 4);
    c.bias = (const float *)put(arena, bias.data(), bias.size() * 4);
    c.scale = (const float *)put(arena, scale.data(), scale.size() * 4);
    c.ktab = (const int32_t *)put(arena, ktab.data(), ktab.size() * 4);
    f.flops = 2.0 * to.C * to.H * to.W * ti.C * k * k;
    f.bytes = 4.0 * ((double)ti.C * ti.H * ti.W + (double)to.C * to.H * to.W);
    return ISR_OK;
}

int build_float_net(isr_model *m) {
    if (m->fnet) return m->fnet->status;
    FloatNet *net = new FloatNet();
    m->fnet = net;
    const ParsedModel &pm = m->pm;
    std::vector<int> uses(pm.tensors.size(), 0);
    for (const HostOp &o : pm.ops) {
        if (o.a >= 0) uses[o.a]++;
        if (o.b >= 0) uses[o.b]++;
    }
    std::vector<uint8_t> arena(256, 0);
    for (const HostOp &o : pm.ops) {
        FloatOp f;
        f.type = o.type; f.a = o.a; f.b = o.b; f.out = o.out;
        const TensorDesc &ti = pm.tensors[o.a], &to = pm.tensors[o.out];
        switch (o.type) {
        case OP_CONV:
            if ((net->status = build_conv(pm, o, o.k, o.stride, o.pad, false, arena, f)) != ISR_OK) return net->status;
            break;
        case OP_FC:
            if (ti.H != ti.W) return net->status = ISR_ERR_UNSUPPORTED;
            if ((net->status = build_conv(pm, o, ti.H, 1, 0, true, arena, f)) != ISR_OK) return net->status;
            break;
        case OP_ADD: {
            f.ma = (float)std::ldexp((double)o.Ma, -o.sh);
            f.mb = (float)std::ldexp((double)o.Mb, -o.sh);
            f.relu = o.relu;
            f.bytes = 12.0 * to.C * to.H * to.W;
            // the convolution issued right before, read by this add alone: the add moves into its epilogue
            FloatOp *prev = net->ops.empty() ? nullptr : &net->ops.back();
            if (prev && prev->type == OP_CONV && prev->res < 0 && o.a != o.b && (prev->out == o.a || prev->out == o.b) &&
                uses[prev->out] == 1) {
                const bool conv_is_a = prev->out == o.a;
                prev->res = conv_is_a ? o.b : o.a;
                prev->conv.ma = conv_is_a ? f.ma : f.mb;
                prev->conv.mb = conv_is_a ? f.mb : f.ma;
                prev->conv.add_relu = o.relu;
                prev->out = o.out;
                prev->bytes += 4.0 * to.C * to.H * to.W;
                continue;
            }
            break; }
        case OP_MAXPOOL:
            f.pool.H = ti.H; f.pool.W = ti.W; f.pool.Cp = ti.Cp; f.pool.Ho = to.H; f.pool.Wo = to.W;
            f.pool.k = o.k; f.pool.stride = o.stride; f.pool.pad = o.pad;
            f.bytes = 4.0 * ((double)ti.C * ti.H * ti.W + (double)to.C * to.H * to.W);
            break;
        case OP_GAP:
            f.gap_scale = (float)std::ldexp((double)o.Ma, -(31 + o.sh));
            f.bytes = 4.0 * ((double)ti.C * ti.H * ti.W + to.C);
            break;
        }
        net->ops.push_back(f);
    }
    hipError_t e = hipMalloc((void **)&net->dconst, arena.size());
    if (e == hipSuccess) e = hipMemcpy(net->dconst, arena.data(), arena.size(), hipMemcpyHostToDevice);
    if (e != hipSuccess) { set_last_device_error((int)e); return net->status = ISR_ERR_DEVICE; }
    for (FloatOp &f : net->ops)
        if (f.type == OP_CONV || f.type == OP_FC) {
            FConvParams &c = f.conv;
            c.w = (const float *)(net->dconst + (size_t)c.w);
            c.bias = (const float *)(net->dconst + (size_t)c.bias);
            c.scale = (const float *)(net->dconst + (size_t)c.scale);
            c.ktab = (const int32_t *)(net->dconst + (size_t)c.ktab);
        }
    for (const FloatOp &f : net->ops) {   // what the planner looks at: op type and tensor ids
        DevOp d{};
        d.type = f.type; d.a = f.a; d.b = f.res >= 0 ? f.res : f.b; d.out = f.out;
        net->plan.ops.push_back(d);
    }
    return net->status = ISR_OK;
}

// Places the float network's tensors for chunks of m->chunk int8-sized copies (a quarter as many fp32 copies).
int plan_float_net(isr_model *m, uint32_t chunk_samples) {
    FloatNet &net = *m->fnet;
    if (net.planned_chunk != chunk_samples) {
        plan_workspace(m->pm, chunk_samples, net.plan);
        net.planned_chunk = chunk_samples;
    }
    return ISR_OK;
}

// Copies per chunk of the fp32 network: tensors sit at the offsets of the op-by-op int8 plan, four
// bytes per element, so a quarter of the int8 chunk fits (less when the padded logits need more).
uint32_t float_chunk(const isr_model *m) {
    const TensorDesc &tl = m->pm.tensors[m->pm.ops.back().out];
    const uint64_t by_logits = (uint64_t)m->chunk * m->pm.classes / (uint64_t)tl.Cp;
    return (uint32_t)std::min<uint64_t>(m->chunk / 4, by_logits);
}

// The Monte-Carlo loop of FloatRS-fp over sample indices [begin, begin + count) of one phase.
// raw_noise: stop after the noise stage and leave x + sigma z itself (not recentred) in tensor 0;
// stop_tensor >= 0 ends each forward right after the op that writes that tensor (0: after the noise stage).
int run_fp_range(isr_model *m, const uint8_t *x, float sigma, uint64_t seed, uint32_t image, uint32_t phase, uint32_t begin,
                 uint64_t count, float *logits_host, int32_t *argmax_host, uint32_t *dcounts, bool raw_noise, int stop_tensor = -1) {
    const ParsedModel &pm = m->pm;
    const Plan &pl = m->fnet->plan;
    const FloatNet &net = *m->fnet;
    const uint32_t chunk = float_chunk(m);
    if (chunk == 0) return ISR_ERR_WORKSPACE;
    auto tptr = [&](int t) { return (float *)(m->ws + pl.toff[t]); };
    const TensorDesc &tl = pm.tensors[pm.ops.back().out];
    float *dlogits = (float *)(m->ws + pl.logits_off);
    int32_t *dargmax = (int32_t *)(m->ws + pl.argmax_off);
    std::vector<float> stage;
    for (uint64_t done = 0; done < count;) {
        const uint32_t bn = (uint32_t)std::min<uint64_t>(chunk, count - done);
        const bool timed = m->profile_every && (m->chunk_counter++ % m->profile_every) == 0;
        size_t ev = 0;
        struct Work { const char *kernel; int conv; double ops, bytes; };
        std::vector<Work> work;
        auto mark = [&]() -> int {
            if (!timed) return ISR_OK;
            if (ev == m->events.size()) {
                hipEvent_t e;
                HIP_TRY(hipEventCreate(&e));
                m->events.push_back(e);
            }
            HIP_TRY(hipEventRecord(m->events[ev++], m->stream));
            return ISR_OK;
        };
        int rc;
        if ((rc = mark()) != ISR_OK) return rc;
        FloatNoiseParams np{};
        np.x = x; np.out = tptr(0); np.C = pm.C; np.H = pm.H; np.W = pm.W;
        np.key0 = (uint32_t)seed; np.key1 = (uint32_t)(seed >> 32); np.image = image; np.phase = phase;
        np.sample_begin = begin + (uint32_t)done; np.count = bn; np.sigma = sigma;
        np.center = raw_noise ? 0.f : 128.f + (float)pm.tensors[0].zp;
        np.quant = 0;
        HIP_TRY(launch_float_noise(np, m->stream));
        work.push_back({last_kernel_name(), 0, 0.0, (double)bn * pm.H * pm.W * 16});
        bool whole = !raw_noise && stop_tensor != 0;
        if (whole) {
            for (const FloatOp &f : net.ops) {
                if ((rc = mark()) != ISR_OK) return rc;
                const TensorDesc &ti = pm.tensors[f.a], &to = pm.tensors[f.out];
                switch (f.type) {
                case OP_CONV:
                case OP_FC: {
                    FConvParams c = f.conv;
                    c.in = tptr(f.a);
                    c.out = f.type == OP_FC ? dlogits : tptr(f.out);
                    c.res = f.res >= 0 ? tptr(f.res) : nullptr;
                    c.npix = (int32_t)(bn * c.Ho * c.Wo);
                    HIP_TRY(launch_fconv(c, m->stream));
                    break; }
                case OP_ADD: {
                    FAddParams a{tptr(f.a), tptr(f.b), tptr(f.out), f.ma, f.mb, f.relu, (int64_t)bn * to.H * to.W * to.Cp / 4};
                    HIP_TRY(launch_fadd(a, m->stream));
                    break; }
                case OP_MAXPOOL: {
                    FPoolParams q = f.pool;
                    q.in = tptr(f.a); q.out = tptr(f.out); q.B = (int32_t)bn;
                    HIP_TRY(launch_fmaxpool(q, m->stream));
                    break; }
                case OP_GAP: {
                    FGapParams g{tptr(f.a), tptr(f.out), ti.H * ti.W, ti.Cp, (int32_t)bn, f.gap_scale};
                    HIP_TRY(launch_fgap(g, m->stream));
                    break; }
                }
                work.push_back({last_kernel_name(), f.type == OP_CONV || f.type == OP_FC, f.flops * bn, f.bytes * bn});
                if (f.out == stop_tensor) { whole = false; break; }
            }
        }
        if (whole) {
            if ((rc = mark()) != ISR_OK) return rc;
            FVoteParams v{dlogits, pm.classes, tl.Cp, (int32_t)bn, dargmax, dcounts};
            HIP_TRY(launch_fvote(v, m->stream));
            work.push_back({last_kernel_name(), 0, 0.0, (double)bn * pm.classes * 4});
        }
        if (timed) {
            if ((rc = mark()) != ISR_OK) return rc;
            HIP_TRY(hipStreamSynchronize(m->stream));
            for (size_t i = 0; i + 1 < ev && i < work.size(); ++i) {
                float ms = 0.f;
                HIP_TRY(hipEventElapsedTime(&ms, m->events[i], m->events[i + 1]));
                isr_kernel_stat &st = m->stats[work[i].kernel];
                if (st.launches == 0) {
                    std::strncpy(st.name, work[i].kernel, sizeof(st.name) - 1);
                    st.is_conv = work[i].conv;
                }
                st.launches += 1;
                st.total_ms += ms;
                st.alg_ops += work[i].ops;
                st.alg_bytes += work[i].bytes;
            }
        }
        if (logits_host) {   // device rows are padded to the stored channel count
            stage.resize((size_t)bn * tl.Cp);
            HIP_TRY(hipMemcpyAsync(stage.data(), dlogits, stage.size() * 4, hipMemcpyDeviceToHost, m->stream));
            HIP_TRY(hipStreamSynchronize(m->stream));
            for (uint32_t s = 0; s < bn; ++s)
                std::memcpy(logits_host + (done + s) * pm.classes, stage.data() + (size_t)s * tl.Cp, (size_t)pm.classes * 4);
        }
        if (argmax_host) {
            HIP_TRY(hipMemcpyAsync(argmax_host + done, dargmax, (size_t)bn * 4, hipMemcpyDeviceToHost, m->stream));
            HIP_TRY(hipStreamSynchronize(m->stream));
        }
        done += bn;
    }
    return ISR_OK;
}

int check_float_call(isr_model *m, const void *x, float sigma, int system) {
    if (!m || !x) return ISR_ERR_ARG;
    if (system != ISR_FLOATRS_QUANT && system != ISR_FLOATRS_FP) return ISR_ERR_ARG;
    if (!(sigma >= 0.f) || !(sigma <= 4096.f)) return ISR_ERR_ARG;
    if (!m->ws || m->chunk == 0) return ISR_ERR_WORKSPACE;
    if (system == ISR_FLOATRS_FP) {
        const int rc = build_float_net(m);
        if (rc != ISR_OK) return rc;
        plan_float_net(m, m->chunk);
        if (float_chunk(m) == 0 || m->fnet->plan.bytes > m->ws_bytes) return ISR_ERR_WORKSPACE;
    }
    return ISR_OK;
}

int run_system(isr_model *m, const uint8_t *x, float sigma, uint64_t seed, uint32_t image, uint32_t phase, uint32_t begin,
               uint64_t count, int system, void *logits_host, int32_t *argmax_host, uint32_t *dcounts) {
    if (system == ISR_FLOATRS_QUANT)
        return run_quant_range(m, x, sigma, seed, image, phase, begin, count, (int32_t *)logits_host, argmax_host, dcounts, -1);
    return run_fp_range(m, x, sigma, seed, image, phase, begin, count, (float *)logits_host, argmax_host, dcounts, false);
}

}  // namespace

extern "C" {

size_t isr_float_workspace_bytes(isr_model *m, uint32_t chunk_samples, int system) {
    if (!m || chunk_samples == 0) return 0;
    if (system == ISR_FLOATRS_QUANT) return isr_workspace_bytes(m, chunk_samples);
    if (system != ISR_FLOATRS_FP || build_float_net(m) != ISR_OK) return 0;
    plan_float_net(m, chunk_samples);
    return std::max(m->fnet->plan.bytes, isr_workspace_bytes(m, chunk_samples));
}

uint32_t isr_float_chunk(const isr_model *m, int system) {
    if (!m || !m->ws || m->chunk == 0) return 0;
    if (system == ISR_FLOATRS_QUANT) return m->chunk;
    return system == ISR_FLOATRS_FP ? float_chunk(m) : 0;
}

int isr_float_certify(isr_model *m, const uint8_t *x_device, float sigma, uint32_t n0, uint32_t n, double alpha,
                      uint64_t seed, uint32_t image_id, int system, isr_result *out, uint32_t *counts0_host,
                      uint32_t *counts1_host) {
    int rc = check_float_call(m, x_device, sigma, system);
    if (rc != ISR_OK) return rc;
    if (!out || n0 == 0 || n == 0 || !(alpha > 0.0 && alpha < 1.0)) return ISR_ERR_ARG;
    const uint32_t C = (uint32_t)m->pm.classes;
    HIP_TRY(launch_fill_u32(m->dcounts, 0, 2 * C, m->stream));
    if ((rc = run_system(m, x_device, sigma, seed, image_id, 0, 0, n0, system, nullptr, nullptr, m->dcounts)) != ISR_OK) return rc;
    if ((rc = run_system(m, x_device, sigma, seed, image_id, 1, 0, n, system, nullptr, nullptr, m->dcounts + C)) != ISR_OK) return rc;
    HIP_TRY(hipMemcpyAsync(m->hcounts, m->dcounts, sizeof(uint32_t) * 2 * C, hipMemcpyDeviceToHost, m->stream));
    HIP_TRY(hipStreamSynchronize(m->stream));
    if (counts0_host) std::memcpy(counts0_host, m->hcounts, sizeof(uint32_t) * C);
    if (counts1_host) std::memcpy(counts1_host, m->hcounts + C, sizeof(uint32_t) * C);
    rc = isr_decide_certify(m->hcounts, m->hcounts + C, C, (double)sigma, n, alpha, out);
    out->radius_int = 0;          // the lattice quantile belongs to the discrete law of the integer path
    out->radius_sq_int = 0;
    return rc;
}

int isr_float_debug_noisy(isr_model *m, const uint8_t *x_device, float sigma, uint64_t seed, uint32_t image_id,
                          uint32_t phase, uint32_t sample_begin, uint32_t count, int system, void *out_host) {
    int rc = check_float_call(m, x_device, sigma, system);
    if (rc != ISR_OK) return rc;
    if (!out_host || count == 0 || phase > 1 || count > isr_float_chunk(m, system)) return ISR_ERR_ARG;
    const ParsedModel &pm = m->pm;
    const size_t hw = (size_t)pm.H * pm.W;
    if (system == ISR_FLOATRS_QUANT) {
        if ((rc = run_quant_range(m, x_device, sigma, seed, image_id, phase, sample_begin, count, nullptr, nullptr, nullptr, 0)) != ISR_OK) return rc;
        std::vector<int8_t> tmp(count * hw * 4);
        HIP_TRY(hipMemcpyAsync(tmp.data(), m->ws + m->plan[m->use_fused].toff[0], tmp.size(), hipMemcpyDeviceToHost, m->stream));
        HIP_TRY(hipStreamSynchronize(m->stream));
        int8_t *o = (int8_t *)out_host;
        for (uint32_t s = 0; s < count; ++s)
            for (int c = 0; c < pm.C; ++c)
                for (size_t i = 0; i < hw; ++i) o[((size_t)s * pm.C + c) * hw + i] = tmp[((size_t)s * hw + i) * 4 + c];
        return ISR_OK;
    }
    if ((rc = run_fp_range(m, x_device, sigma, seed, image_id, phase, sample_begin, count, nullptr, nullptr, nullptr, true)) != ISR_OK) return rc;
    std::vector<float> tmp(count * hw * 4);
    HIP_TRY(hipMemcpyAsync(tmp.data(), m->ws + m->fnet->plan.toff[0], tmp.size() * 4, hipMemcpyDeviceToHost, m->stream));
    HIP_TRY(hipStreamSynchronize(m->stream));
    float *o = (float *)out_host;
    for (uint32_t s = 0; s < count; ++s)
        for (int c = 0; c < pm.C; ++c)
            for (size_t i = 0; i < hw; ++i) o[((size_t)s * pm.C + c) * hw + i] = tmp[((size_t)s * hw + i) * 4 + c];
    return ISR_OK;
}

int isr_float_debug_forward(isr_model *m, const uint8_t *x_device, float sigma, uint64_t seed, uint32_t image_id,
                            uint32_t phase, uint32_t sample_begin, uint32_t count, int system, void *logits_host,
                            int32_t *argmax_host, uint32_t *counts_host) {
    int rc = check_float_call(m, x_device, sigma, system);
    if (rc != ISR_OK) return rc;
    if (count == 0 || phase > 1) return ISR_ERR_ARG;
    const uint32_t C = (uint32_t)m->pm.classes;
    if (counts_host) HIP_TRY(launch_fill_u32(m->dcounts, 0, C, m->stream));
    rc = run_system(m, x_device, sigma, seed, image_id, phase, sample_begin, count, system, logits_host, argmax_host,
                    counts_host ? m->dcounts : nullptr);
    if (rc != ISR_OK) return rc;
    if (counts_host) {
        HIP_TRY(hipMemcpyAsync(m->hcounts, m->dcounts, sizeof(uint32_t) * C, hipMemcpyDeviceToHost, m->stream));
        HIP_TRY(hipStreamSynchronize(m->stream));
        for (uint32_t i = 0; i < C; ++i) counts_host[i] += m->hcounts[i];
    } else {
        HIP_TRY(hipStreamSynchronize(m->stream));
    }
    return ISR_OK;
}

int isr_float_debug_tensor(isr_model *m, const uint8_t *x_device, float sigma, uint64_t seed, uint32_t image_id,
                           uint32_t phase, uint32_t sample, int32_t tensor_id, float *out_host) {
    int rc = check_float_call(m, x_device, sigma, ISR_FLOATRS_FP);
    if (rc != ISR_OK) return rc;
    const ParsedModel &pm = m->pm;
    if (!out_host || phase > 1 || tensor_id < 0 || tensor_id >= (int)pm.tensors.size() || tensor_id == pm.ops.back().out)
        return ISR_ERR_ARG;
    bool stored = tensor_id == 0;   // an add folded into a convolution leaves that convolution's own output unstored
    for (const FloatOp &f : m->fnet->ops) stored = stored || f.out == tensor_id;
    if (!stored) return ISR_ERR_UNSUPPORTED;
    if ((rc = run_fp_range(m, x_device, sigma, seed, image_id, phase, sample, 1, nullptr, nullptr, nullptr, false, tensor_id)) != ISR_OK) return rc;
    const TensorDesc &t = pm.tensors[tensor_id];
    const size_t hw = (size_t)t.H * t.W;
    std::vector<float> tmp(hw * t.Cp);
    HIP_TRY(hipMemcpyAsync(tmp.data(), m->ws + m->fnet->plan.toff[tensor_id], tmp.size() * 4, hipMemcpyDeviceToHost, m->stream));
    HIP_TRY(hipStreamSynchronize(m->stream));
    for (int c = 0; c < t.C; ++c)
        for (size_t i = 0; i < hw; ++i) out_host[(size_t)c * hw + i] = tmp[i * t.Cp + c];
    return ISR_OK;
}

}  // extern "C"
