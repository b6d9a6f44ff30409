// C ABI: model loading, workspace planning and the Monte-Carlo driver that
// enqueues noise -> layers -> vote kernels for chunks of sample indices.
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <map>
#include <new>
#include <string>

#include "isr_internal.h"
#include "model.h"
#include "plan.h"

using namespace isr;

namespace {

thread_local int g_last_hip_error = 0;

#define HIP_TRY(expr)                                     \
    do {                                                  \
        hipError_t e_ = (expr);                           \
        if (e_ != hipSuccess) {                           \
            g_last_hip_error = (int)e_;                   \
            return ISR_ERR_DEVICE;                        \
        }                                                 \
    } while (0)

}  // namespace

void isr::set_last_device_error(int hip_error) { g_last_hip_error = hip_error; }

namespace { thread_local const char *g_kernel_name = ""; }
void isr::set_kernel_name(const char *name) { g_kernel_name = name; }
const char *isr::last_kernel_name() { return g_kernel_name; }


namespace {

int get_table(isr_model *m, uint32_t sigma, const DeviceNoiseTable **out) {
    for (int i = 0; i < TABLE_SLOTS; ++i)
        if (m->table_sigma[i] == sigma) { *out = m->dtables + i; return ISR_OK; }
    int slot = m->table_next;
    m->table_next = (slot + 1) % TABLE_SLOTS;
    // the staging slot may still be in flight from an earlier call on this stream
    HIP_TRY(hipStreamSynchronize(m->stream));
    if (!build_device_table(sigma, m->htables[slot])) return ISR_ERR_ARG;
    HIP_TRY(hipMemcpyAsync(m->dtables + slot, m->htables + slot, sizeof(DeviceNoiseTable), hipMemcpyHostToDevice, m->stream));
    m->table_sigma[slot] = sigma;
    *out = m->dtables + slot;
    return ISR_OK;
}

// A batched call: items (device array) that own n_per_item consecutive slots each.
struct BatchCtx {
    const NoiseItem *items;
    uint32_t n_items, n_per_item;
};

// Enqueues the Monte-Carlo loop for sample indices [begin, begin+count) of one
// phase.  Optional outputs: per-sample logits / argmax (device buffers inside
// the workspace, copied to the host pointers chunk by chunk) and the device
// vote counters.  stop_tensor >= 0 ends each forward right after that tensor.
// With `bc` the loop runs over the n_items * n_per_item slots of a batch instead
// (x = the image array, table = the table array, dcounts = [items][classes];
// image / begin / count are ignored): chunks are cut from the slot list without
// regard to item boundaries, so short per-item runs still fill the device.
int run_range(isr_model *m, const Plan &pl, const uint8_t *x, const DeviceNoiseTable *table, uint64_t seed,
              uint32_t image, uint32_t phase, uint32_t begin, uint64_t count, int32_t *logits_host,
              int32_t *argmax_host, uint32_t *dcounts, int stop_tensor, const BatchCtx *bc = nullptr) {
    const ParsedModel &pm = m->pm;
    uint8_t *ws = m->ws;
    if (bc) count = (uint64_t)bc->n_items * bc->n_per_item;
    // bytes of one copy of a tensor: copies are contiguous, so a range of copies of a chunk is a sub-chunk
    auto tptr = [&](int t, uint32_t first_copy) -> uint8_t * {
        const TensorDesc &d = pm.tensors[t];
        return ws + pl.toff[t] + (size_t)first_copy * d.H * d.W * d.Cp;
    };
    for (uint64_t done = 0; done < count;) {
        uint32_t cnt = (uint32_t)std::min<uint64_t>(m->chunk, count - done);
        if (bc) cnt = (uint32_t)std::min<uint64_t>(cnt, (uint64_t)bc->n_per_item * 65534);   // one grid row per item
        const bool timed = m->profile_every && (m->chunk_counter++ % m->profile_every) == 0;
        size_t ev = 0;
        auto mark = [&]() -> int {   // event before a launch / after the last one
            if (!timed) return ISR_OK;
            if (ev == m->events.size()) {
                hipEvent_t e;
                HIP_TRY(hipEventCreate(&e));
                m->events.push_back(e);
            }
            HIP_TRY(hipEventRecord(m->events[ev++], m->stream));
            return ISR_OK;
        };
        struct Work { const char *kernel; int conv; double ops, bytes; };
        std::vector<Work> ev_work;   // per timed launch: the kernel instance and its algorithmic work
        int prc;

        // copies [j0, j0 + bn) of the chunk through the noise stage
        auto run_noise = [&](uint32_t j0, uint32_t bn) -> int {
            NoiseParams np;
            np.x = x; np.table = table; np.out = (int8_t *)tptr(0, j0);
            np.C = pm.C; np.H = pm.H; np.W = pm.W;
            np.key0 = (uint32_t)seed; np.key1 = (uint32_t)(seed >> 32);
            np.image = image; np.phase = phase; np.sample_begin = begin + (uint32_t)done + j0; np.count = bn;
            np.items = nullptr; np.n_per_item = 0; np.item_first = 0; np.item_count = 0; np.slot_begin = 0;
            if (bc) {
                const uint64_t s0 = done + j0;
                np.items = bc->items; np.n_per_item = bc->n_per_item; np.slot_begin = s0;
                np.item_first = (uint32_t)(s0 / bc->n_per_item);
                np.item_count = (uint32_t)((s0 + bn - 1) / bc->n_per_item) - np.item_first + 1;
            }
            if ((prc = mark()) != ISR_OK) return prc;
            if (m->quant_sigma >= 0.f) {   // FloatRS-quant: continuous noise rounded onto the pixel grid (single pair only)
                FloatNoiseParams fp{};
                fp.x = x; fp.out = np.out; fp.C = pm.C; fp.H = pm.H; fp.W = pm.W;
                fp.key0 = np.key0; fp.key1 = np.key1; fp.image = image; fp.phase = phase;
                fp.sample_begin = np.sample_begin; fp.count = bn; fp.sigma = m->quant_sigma; fp.center = 0.f; fp.quant = 1;
                HIP_TRY(launch_float_noise(fp, m->stream));
            } else {
                HIP_TRY(launch_noise(np, m->stream));
            }
            ev_work.push_back({last_kernel_name(), 0, 0.0, (double)bn * pm.H * pm.W * 4});
            return ISR_OK;
        };
        // copies [j0, j0 + bn) of the chunk through one op of the plan
        auto run_op = [&](const DevOp &d, uint32_t j0, uint32_t bn) -> int {
            if ((prc = mark()) != ISR_OK) return prc;
            set_kernel_name("");
            switch (d.type) {
            case OP_CONV: {
                if (d.stem_pool) {
                    const TensorDesc &to = pm.tensors[d.out];
                    StemPoolParams sp;
                    sp.in = (const int8_t *)tptr(d.a, j0);
                    sp.out = (int8_t *)tptr(d.out, j0);
                    sp.w = d.conv.w; sp.bias = d.conv.bias; sp.m0s = d.conv.m0s; sp.chi = d.conv.chi; sp.shm1 = d.conv.shm1;
                    sp.H = d.conv.H; sp.W = d.conv.W; sp.Ho = d.conv.Ho; sp.Wo = d.conv.Wo; sp.Hp = to.H; sp.Wp = to.W;
                    sp.zp_in = d.conv.zp_in; sp.zp_out = d.conv.zp_out; sp.relu = d.conv.relu; sp.tie_free = d.conv.tie_free; sp.B = (int32_t)bn;
                    sp.fused_noise = d.noise_fused && m->quant_sigma < 0.f;
                    sp.noise = NoiseSource{};
                    if (sp.fused_noise) {
                        NoiseSource &ns = sp.noise;
                        ns.x = x; ns.table = table; ns.items = nullptr;
                        ns.key0 = (uint32_t)seed; ns.key1 = (uint32_t)(seed >> 32);
                        ns.image = image; ns.phase = phase; ns.sample_begin = begin + (uint32_t)done + j0;
                        ns.n_per_item = 0; ns.slot_begin = 0;
                        ns.C = pm.C; ns.H = pm.H; ns.W = pm.W;
                        if (bc) { ns.items = bc->items; ns.n_per_item = bc->n_per_item; ns.slot_begin = done + j0; }
                    }
                    HIP_TRY(launch_stem_pool(sp, m->stream));
                    break;
                }
                if (d.stem16) {
                    const ConvParams &c = d.conv;
                    Stem16Params sp;
                    sp.in = (const int8_t *)tptr(d.a, j0);
                    sp.out = (int8_t *)tptr(d.out, j0);
                    sp.w = c.w; sp.bias = c.bias; sp.m0s = c.m0s; sp.chi = c.chi; sp.shm1 = c.shm1;
                    sp.H = c.H; sp.W = c.W; sp.B = (int32_t)bn; sp.zp_in = c.zp_in;
                    sp.lo = c.relu ? c.zp_out : -128; sp.tie_free = c.tie_free;
                    HIP_TRY(launch_stem16(sp, m->stream));
                    break;
                }
                if (d.block) {
                    BlockParams bp{};
                    bp.in = (const int8_t *)tptr(d.a, j0);
                    bp.out = (int8_t *)tptr(d.out, j0);
                    bp.blocks = m->dblocks + d.chain_off;
                    bp.nblocks = (int32_t)d.chain.size();
                    bp.C = d.conv.Cout_p; bp.S = d.conv.H; bp.B = (int32_t)bn;
                    bp.tie_free = d.conv.tie_free && d.conv2.tie_free && d.conv2.add_tie_free;
                    HIP_TRY(launch_basic_block(bp, m->stream));
                    break;
                }
                if (d.trans) {
                    const ConvParams &c1 = d.conv, &c2 = d.conv2, &cp = d.conv3;
                    TransParams tp{};
                    tp.in = (const int8_t *)tptr(d.a, j0);
                    tp.out = (int8_t *)tptr(d.out, j0);
                    tp.w1 = c1.w; tp.bias1 = c1.bias; tp.m0s1 = c1.m0s; tp.chi1 = c1.chi; tp.shm11 = c1.shm1;
                    tp.w2 = c2.w; tp.bias2 = c2.bias; tp.m0s2 = c2.m0s; tp.chi2 = c2.chi; tp.shm12 = c2.shm1;
                    tp.wp = cp.w; tp.biasp = cp.bias; tp.m0sp = cp.m0s; tp.chip = cp.chi; tp.shm1p = cp.shm1;
                    tp.C = c1.Cout_p; tp.S = c1.Ho; tp.B = (int32_t)bn;
                    tp.zp_x = c1.zp_in; tp.zp_t = c1.zp_out;
                    tp.lo1 = c1.relu ? c1.zp_out : -128;
                    tp.lo2 = c2.relu ? c2.zp_out : -128;
                    tp.lop = cp.relu ? cp.zp_out : -128;
                    tp.add_mul_self = cp.add_mul_self; tp.add_mul_res = cp.add_mul_res; tp.add_c0 = cp.add_c0;
                    tp.add_k = cp.add_k; tp.add_sh = cp.add_sh; tp.add_lo = cp.add_lo;
                    tp.tie_free = c1.tie_free && c2.tie_free && cp.tie_free && cp.add_tie_free;
                    HIP_TRY(launch_trans_block(tp, m->stream));
                    break;
                }
                if (d.bneck) {
                    const ConvParams &c1 = d.conv, &c2 = d.conv2, &c3 = d.conv3;
                    BneckParams bp{};
                    bp.in = (const int8_t *)tptr(d.a, j0);
                    bp.out = (int8_t *)tptr(d.out, j0);
                    bp.w1 = c1.w; bp.bias1 = c1.bias; bp.m0s1 = c1.m0s; bp.chi1 = c1.chi; bp.shm11 = c1.shm1;
                    bp.w2 = c2.w; bp.bias2 = c2.bias; bp.m0s2 = c2.m0s; bp.chi2 = c2.chi; bp.shm12 = c2.shm1;
                    bp.zpad = c1.zpad;
                    bp.Cin_p = c1.Cin_p; bp.H = c1.H; bp.W = c1.W; bp.B = (int32_t)bn; bp.tail = d.bneck >= 2;
                    bp.zp_t1 = c1.zp_out;
                    bp.lo1 = c1.relu ? c1.zp_out : -128;
                    bp.lo2 = c2.relu ? c2.zp_out : -128;
                    bp.tie_free = c1.tie_free && c2.tie_free;
                    if (bp.tail) {
                        // the closing 1x1 convolution; with a projection shortcut (bneck == 4) conv3 carries two
                        // convolutions, and either of them may be the one that reads the block input
                        const bool swap = d.bneck == 4 && d.proj_is_main;
                        bp.w3 = swap ? c3.w2 : c3.w; bp.bias3 = swap ? c3.bias2 : c3.bias; bp.m0s3 = swap ? c3.m0s2 : c3.m0s;
                        bp.chi3 = swap ? c3.chi2 : c3.chi; bp.shm13 = swap ? c3.shm12 : c3.shm1;
                        bp.Cout_p = c3.Cout_p;
                        const int lo_main = c3.relu ? c3.zp_out : -128;
                        bp.lo3 = swap ? c3.lo2 : lo_main;
                        bp.add_mul_self = swap ? c3.add_mul_res : c3.add_mul_self;   // "self" in the kernel = the closing convolution
                        bp.add_mul_res = swap ? c3.add_mul_self : c3.add_mul_res;
                        bp.add_c0 = c3.add_c0; bp.add_k = c3.add_k; bp.add_sh = c3.add_sh; bp.add_lo = c3.add_lo;
                        bp.tie_free = bp.tie_free && c3.tie_free && c3.add_tie_free && (d.bneck != 4 || c3.tie_free2);
                        if (d.bneck == 4) {
                            bp.proj = 1;
                            bp.wp = swap ? c3.w : c3.w2; bp.biasp = swap ? c3.bias : c3.bias2; bp.m0sp = swap ? c3.m0s : c3.m0s2;
                            bp.chip = swap ? c3.chi : c3.chi2; bp.shm1p = swap ? c3.shm1 : c3.shm12;
                            bp.lop = swap ? lo_main : c3.lo2;
                        }
                    }
                    if (d.bneck == 3) HIP_TRY(launch_bottleneck128(bp, m->stream));
                    else HIP_TRY(launch_bottleneck(bp, m->stream));
                    break;
                }
                if (d.xr) {
                    XrParams xp;
                    expand_reduce_params(d.conv, d.conv2, (const int8_t *)tptr(d.a, j0), (const int8_t *)tptr(d.b, j0),
                                         (int8_t *)tptr(d.out, j0), (int8_t *)tptr(d.out2, j0), (int32_t)bn, xp);
                    HIP_TRY(launch_expand_reduce(xp, d.conv.add_tie_free, m->stream));
                    break;
                }
                ConvParams c = d.conv;
                c.in = (const int8_t *)tptr(d.a, j0);
                c.out = (int8_t *)tptr(d.out, j0);
                c.res = c.fuse_add == 1 ? (const int8_t *)tptr(d.b, j0) : nullptr;
                c.in2 = c.fuse_add == 2 ? (const int8_t *)tptr(d.b, j0) : nullptr;
                c.npix = (int32_t)(bn * c.Ho * c.Wo);
                c.force_tile = m->conv_tile;
                HIP_TRY(launch_conv(c, m->stream));
                break; }
            case OP_ADD: {
                AddParams a = d.add;
                const TensorDesc &t = pm.tensors[d.out];
                a.a = (const int8_t *)tptr(d.a, j0);
                a.b = (const int8_t *)tptr(d.b, j0);
                a.out = (int8_t *)tptr(d.out, j0);
                a.n16 = (int64_t)bn * t.H * t.W * t.Cp / 16;
                HIP_TRY(launch_add(a, m->stream));
                break; }
            case OP_MAXPOOL: {
                PoolParams p = d.pool;
                p.in = (const int8_t *)tptr(d.a, j0);
                p.out = (int8_t *)tptr(d.out, j0);
                p.B = (int32_t)bn;
                HIP_TRY(launch_maxpool(p, m->stream));
                break; }
            case OP_GAP: {
                GapParams g = d.gap;
                g.in = (const int8_t *)tptr(d.a, j0);
                g.out = (int8_t *)tptr(d.out, j0);
                g.B = (int32_t)bn;
                HIP_TRY(launch_gap(g, m->stream));
                break; }
            case OP_FC: {
                FcParams f = d.fc;
                f.in = (const int8_t *)tptr(d.a, j0);
                f.B = (int32_t)bn;
                f.logits = logits_host ? (int32_t *)(ws + pl.logits_off) + (size_t)j0 * pm.classes : nullptr;
                f.argmax = argmax_host ? (int32_t *)(ws + pl.argmax_off) + j0 : nullptr;
                f.counts = dcounts;
                if (bc) { f.n_per_item = bc->n_per_item; f.slot_begin = done + j0; }
                HIP_TRY(launch_fc(f, m->stream));
                break; }
            }
            ev_work.push_back({last_kernel_name(), d.type == OP_CONV ? 1 : 0, d.ops_per_sample * bn, d.bytes_per_sample * bn});
            return ISR_OK;
        };

        // The plan is walked in segments (plan.h): the ops of a segment run back to back on one
        // sub-chunk of copies after the other, so that what an op writes is still in the caches
        // when the next op of the segment reads it.  Segment 0 starts with the noise stage.
        size_t nops = pl.ops.size();
        if (stop_tensor == 0) nops = 0;
        else if (stop_tensor > 0)
            for (size_t i = 0; i < pl.ops.size(); ++i)
                if (pl.ops[i].out == stop_tensor || pl.ops[i].out2 == stop_tensor) { nops = i + 1; break; }
        size_t op0 = 0;
        bool noise_done = false;
        for (size_t sg = 0; sg <= pl.segments.size() && (op0 < nops || !noise_done); ++sg) {
            // ops [op0, op1) in sub-chunks of `sub` copies; past the last segment: the rest, whole chunk
            size_t op1 = nops;
            uint32_t sub = cnt;
            if (sg < pl.segments.size()) {
                op1 = std::min(nops, pl.segments[sg].end);
                sub = std::max<uint32_t>(1, std::min(cnt, pl.segments[sg].sub));
            }
            if (op1 < op0) op1 = op0;
            // no noise launch when the first op of the plan draws its own input (and runs at all)
            const bool own_noise = nops > 0 && !pl.ops.empty() && pl.ops[0].noise_fused && m->quant_sigma < 0.f;
            for (uint32_t j0 = 0; j0 < cnt; j0 += sub) {
                const uint32_t bn = std::min(sub, cnt - j0);
                if (!noise_done && !own_noise && (prc = run_noise(j0, bn)) != ISR_OK) return prc;
                for (size_t i = op0; i < op1; ++i)
                    if ((prc = run_op(pl.ops[i], j0, bn)) != ISR_OK) return prc;
            }
            noise_done = true;
            op0 = op1;
        }
        if (timed) {
            if ((prc = mark()) != ISR_OK) return prc;
            HIP_TRY(hipStreamSynchronize(m->stream));
            for (size_t i = 0; i + 1 < ev && i < ev_work.size(); ++i) {
                float ms = 0.f;
                HIP_TRY(hipEventElapsedTime(&ms, m->events[i], m->events[i + 1]));
                isr_kernel_stat &st = m->stats[ev_work[i].kernel];
                if (st.launches == 0) {
                    std::strncpy(st.name, ev_work[i].kernel, sizeof(st.name) - 1);
                    st.is_conv = ev_work[i].conv;
                }
                st.launches += 1;
                st.total_ms += ms;
                st.alg_ops += ev_work[i].ops;
                st.alg_bytes += ev_work[i].bytes;
            }
        }
        if (logits_host) {
            HIP_TRY(hipMemcpyAsync(logits_host + (size_t)done * pm.classes, ws + pl.logits_off,
                                   (size_t)cnt * pm.classes * 4, hipMemcpyDeviceToHost, m->stream));
        }
        if (argmax_host) {
            HIP_TRY(hipMemcpyAsync(argmax_host + done, ws + pl.argmax_off, (size_t)cnt * 4,
                                   hipMemcpyDeviceToHost, m->stream));
        }
        if (logits_host || argmax_host) HIP_TRY(hipStreamSynchronize(m->stream));
        done += cnt;
    }
    return ISR_OK;
}

}  // namespace

int isr::run_quant_range(isr_model *m, const uint8_t *x, float sigma, uint64_t seed, uint32_t image, uint32_t phase,
                         uint32_t begin, uint64_t count, int32_t *logits_host, int32_t *argmax_host, uint32_t *dcounts,
                         int stop_tensor) {
    m->quant_sigma = sigma;
    const int rc = run_range(m, m->plan[m->use_fused], x, nullptr, seed, image, phase, begin, count, logits_host, argmax_host,
                             dcounts, stop_tensor);
    m->quant_sigma = -1.f;
    return rc;
}

namespace {

// Makes the tables of every sigma in `sigmas` resident at once (at most TABLE_SLOTS
// distinct values) and returns the slot of each.
int get_tables(isr_model *m, const std::vector<uint32_t> &sigmas, std::vector<uint32_t> &slots) {
    std::vector<uint32_t> distinct;
    for (uint32_t s : sigmas)
        if (std::find(distinct.begin(), distinct.end(), s) == distinct.end()) distinct.push_back(s);
    if ((int)distinct.size() > TABLE_SLOTS) return ISR_ERR_ARG;
    bool synced = false;
    for (uint32_t s : distinct) {
        bool have = false;
        for (int i = 0; i < TABLE_SLOTS; ++i) have = have || m->table_sigma[i] == s;
        if (have) continue;
        int slot = -1;   // a slot whose table this batch does not need
        for (int k = 0; k < TABLE_SLOTS && slot < 0; ++k) {
            const int c = (m->table_next + k) % TABLE_SLOTS;
            if (std::find(distinct.begin(), distinct.end(), m->table_sigma[c]) == distinct.end()) slot = c;
        }
        if (slot < 0) return ISR_ERR_ARG;   // cannot happen: fewer needed tables than slots
        m->table_next = (slot + 1) % TABLE_SLOTS;
        if (!synced) { HIP_TRY(hipStreamSynchronize(m->stream)); synced = true; }   // staging slots may be in flight
        if (!build_device_table(s, m->htables[slot])) return ISR_ERR_ARG;
        HIP_TRY(hipMemcpyAsync(m->dtables + slot, m->htables + slot, sizeof(DeviceNoiseTable), hipMemcpyHostToDevice, m->stream));
        m->table_sigma[slot] = s;
    }
    slots.resize(sigmas.size());
    for (size_t i = 0; i < sigmas.size(); ++i)
        for (int k = 0; k < TABLE_SLOTS; ++k)
            if (m->table_sigma[k] == sigmas[i]) slots[i] = (uint32_t)k;
    return ISR_OK;
}

// Validates a batch, uploads its item descriptors and clears its vote counters
// (phases * n_items * classes words).
int prepare_batch(isr_model *m, const void *x, uint32_t n_images, const isr_item *items, uint32_t n_items, double alpha,
                  int phases) {
    if (!m || !x || !items || n_images == 0 || n_items == 0) return ISR_ERR_ARG;
    if (!(alpha > 0.0 && alpha < 1.0)) return ISR_ERR_ARG;
    if (!m->ws || m->chunk == 0) return ISR_ERR_WORKSPACE;
    std::vector<uint32_t> sigmas(n_items), slots;
    for (uint32_t i = 0; i < n_items; ++i) {
        if (items[i].image >= n_images || items[i].sigma < 1 || items[i].sigma > 1024) return ISR_ERR_ARG;
        sigmas[i] = items[i].sigma;
    }
    const size_t C = (size_t)m->pm.classes;
    if (n_items > m->items_cap) {
        HIP_TRY(hipStreamSynchronize(m->stream));
        if (m->ditems) (void)hipFree(m->ditems);
        if (m->hitems) (void)hipHostFree(m->hitems);
        if (m->dcounts_b) (void)hipFree(m->dcounts_b);
        if (m->hcounts_b) (void)hipHostFree(m->hcounts_b);
        m->ditems = m->hitems = nullptr;
        m->dcounts_b = m->hcounts_b = nullptr;
        m->items_cap = 0;
        const uint32_t cap = std::max<uint32_t>(n_items, 64);
        HIP_TRY(hipMalloc((void **)&m->ditems, sizeof(NoiseItem) * cap));
        HIP_TRY(hipHostMalloc((void **)&m->hitems, sizeof(NoiseItem) * cap, hipHostMallocDefault));
        HIP_TRY(hipMalloc((void **)&m->dcounts_b, sizeof(uint32_t) * 2 * cap * C));
        HIP_TRY(hipHostMalloc((void **)&m->hcounts_b, sizeof(uint32_t) * 2 * cap * C, hipHostMallocDefault));
        m->items_cap = cap;
    }
    int rc = get_tables(m, sigmas, slots);
    if (rc != ISR_OK) return rc;
    HIP_TRY(hipStreamSynchronize(m->stream));   // the pinned descriptors of an earlier call may still be in flight
    for (uint32_t i = 0; i < n_items; ++i) m->hitems[i] = NoiseItem{items[i].image, slots[i], items[i].image_id};
    HIP_TRY(hipMemcpyAsync(m->ditems, m->hitems, sizeof(NoiseItem) * n_items, hipMemcpyHostToDevice, m->stream));
    HIP_TRY(launch_fill_u32(m->dcounts_b, 0, (size_t)phases * n_items * C, m->stream));
    return ISR_OK;
}

int check_call(const isr_model *m, const void *x, uint32_t sigma, double alpha, bool need_alpha) {
    if (!m || !x) return ISR_ERR_ARG;
    if (sigma < 1 || sigma > 1024) return ISR_ERR_ARG;
    if (need_alpha && !(alpha > 0.0 && alpha < 1.0)) return ISR_ERR_ARG;
    if (!m->ws || m->chunk == 0) return ISR_ERR_WORKSPACE;
    return ISR_OK;
}

}  // namespace

extern "C" {

int isr_load_model(const void *blob_host, size_t bytes, isr_model **out) {
    if (!blob_host || !out) return ISR_ERR_ARG;
    *out = nullptr;
    isr_model *m = new (std::nothrow) isr_model();
    if (!m) return ISR_ERR_ARG;
    std::string why;
    int rc = parse_model(blob_host, bytes, m->pm, why);
    if (rc != ISR_OK) { delete m; return rc; }
    ConstArena arena;
    arena.put(nullptr, 256);  // offset 0 is never a valid table
    rc = build_device_ops(m->pm, m->ops, arena);
    if (rc != ISR_OK) { delete m; return rc; }
    auto cleanup = [&](int code) { isr_free_model(m); return code; };
    hipError_t e = hipMalloc((void **)&m->dconst, arena.host.size());
    if (e == hipSuccess) e = hipMemcpy(m->dconst, arena.host.data(), arena.host.size(), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMalloc((void **)&m->dtables, sizeof(DeviceNoiseTable) * TABLE_SLOTS);
    if (e == hipSuccess) e = hipHostMalloc((void **)&m->htables, sizeof(DeviceNoiseTable) * TABLE_SLOTS, hipHostMallocDefault);
    if (e == hipSuccess) e = hipMalloc((void **)&m->dcounts, sizeof(uint32_t) * 2 * m->pm.classes);
    if (e == hipSuccess) e = hipHostMalloc((void **)&m->hcounts, sizeof(uint32_t) * 2 * m->pm.classes, hipHostMallocDefault);
    if (e != hipSuccess) { g_last_hip_error = (int)e; return cleanup(ISR_ERR_DEVICE); }
    rebase_device_ops(m->ops, m->dconst);
    m->plan[0].ops = m->ops;
    build_fused_plan(m->pm, m->ops, m->plan[1].ops, false);
    build_fused_plan(m->pm, m->ops, m->plan[2].ops, true);
    {   // descriptors of the identity-block chains, in device memory
        std::vector<BlockDesc> descs;
        for (int pi = 1; pi <= 2; ++pi)
        for (DevOp &d : m->plan[pi].ops) {
            if (!d.block) continue;
            d.chain_off = descs.size();
            for (const auto &blk : d.chain) {
                const ConvParams &c1 = blk.first, &c2 = blk.second;
                BlockDesc b{};
                b.w1 = c1.w; b.bias1 = c1.bias; b.m0s1 = c1.m0s; b.chi1 = c1.chi; b.shm11 = c1.shm1;
                b.w2 = c2.w; b.bias2 = c2.bias; b.m0s2 = c2.m0s; b.chi2 = c2.chi; b.shm12 = c2.shm1;
                b.zp_x = c1.zp_in; b.zp_t = c1.zp_out; b.relu1 = c1.relu;
                b.zp_u = c2.zp_out; b.relu2 = c2.relu;
                b.add_mul_self = c2.add_mul_self; b.add_mul_res = c2.add_mul_res; b.add_c0 = c2.add_c0;
                b.add_k = c2.add_k; b.add_sh = c2.add_sh; b.add_lo = c2.add_lo;
                descs.push_back(b);
            }
        }
        if (!descs.empty()) {
            e = hipMalloc((void **)&m->dblocks, descs.size() * sizeof(BlockDesc));
            if (e == hipSuccess) e = hipMemcpy(m->dblocks, descs.data(), descs.size() * sizeof(BlockDesc), hipMemcpyHostToDevice);
            if (e != hipSuccess) { g_last_hip_error = (int)e; return cleanup(ISR_ERR_DEVICE); }
        }
    }
    *out = m;
    return ISR_OK;
}

int isr_set_fusion(isr_model *m, int enable) {
    if (!m) return ISR_ERR_ARG;
    if (enable < 0 || enable > 2) return ISR_ERR_ARG;
    m->use_fused = enable;
    return ISR_OK;
}

int isr_noise_bank(uint32_t sigma, uint64_t seed, uint32_t bank_id, uint32_t first, uint32_t count, uint32_t d,
                   int16_t *out_device, void *hip_stream) {
    if (sigma < 1 || sigma > 1024 || !out_device || d == 0 || (d & 3) != 0) return ISR_ERR_ARG;
    if ((uint64_t)first + count > (1ull << 32)) return ISR_ERR_ARG;
    if (count == 0) return ISR_OK;
    std::vector<uint32_t> host;
    uint32_t n = 0, R = 0;
    if (!build_bank_table(sigma, host, n, R)) return ISR_ERR_ARG;
    hipStream_t st = (hipStream_t)hip_stream;
    uint32_t *dev = nullptr;
    HIP_TRY(hipMalloc((void **)&dev, host.size() * 4));
    hipError_t e = hipMemcpyAsync(dev, host.data(), host.size() * 4, hipMemcpyHostToDevice, st);
    if (e == hipSuccess) {
        NoiseBankParams p;
        p.thi = dev; p.tlo = dev + n; p.guide = (const uint16_t *)(dev + 2 * n);
        p.n = (int32_t)n; p.R = (int32_t)R; p.out = out_device; p.d = d;
        p.key0 = (uint32_t)seed; p.key1 = (uint32_t)(seed >> 32); p.bank = bank_id; p.first = first; p.count = count;
        e = launch_noise_bank(p, st);
    }
    if (e == hipSuccess) e = hipStreamSynchronize(st);   // the staging vector and the table die with this call
    (void)hipFree(dev);
    if (e != hipSuccess) { g_last_hip_error = (int)e; return ISR_ERR_DEVICE; }
    return ISR_OK;
}

int isr_set_conv_tile(isr_model *m, int tile) {
    if (!m || tile < 0 || tile > 7) return ISR_ERR_ARG;
    m->conv_tile = tile;
    return ISR_OK;
}

int isr_profile(isr_model *m, uint32_t every_chunks) {
    if (!m) return ISR_ERR_ARG;
    m->profile_every = every_chunks;
    m->chunk_counter = 0;
    m->stats.clear();
    return ISR_OK;
}

int isr_profile_read(const isr_model *m, isr_kernel_stat *out_host, uint32_t cap, uint32_t *n_out) {
    if (!m || !n_out || (cap && !out_host)) return ISR_ERR_ARG;
    uint32_t n = 0;
    for (const auto &kv : m->stats) {
        if (n < cap) out_host[n] = kv.second;
        ++n;
    }
    *n_out = n;
    return ISR_OK;
}

int isr_free_model(isr_model *m) {
    if (!m) return ISR_OK;
    for (hipEvent_t e : m->events) (void)hipEventDestroy(e);
    if (m->dconst) (void)hipFree(m->dconst);
    if (m->dtables) (void)hipFree(m->dtables);
    if (m->htables) (void)hipHostFree(m->htables);
    if (m->dcounts) (void)hipFree(m->dcounts);
    if (m->hcounts) (void)hipHostFree(m->hcounts);
    if (m->dblocks) (void)hipFree(m->dblocks);
    if (m->ditems) (void)hipFree(m->ditems);
    if (m->hitems) (void)hipHostFree(m->hitems);
    if (m->dcounts_b) (void)hipFree(m->dcounts_b);
    if (m->hcounts_b) (void)hipHostFree(m->hcounts_b);
    free_float_net(m->fnet);
    delete m;
    return ISR_OK;
}

int isr_model_info(const isr_model *m, int *C, int *H, int *W, int *num_classes) {
    if (!m) return ISR_ERR_ARG;
    if (C) *C = m->pm.C;
    if (H) *H = m->pm.H;
    if (W) *W = m->pm.W;
    if (num_classes) *num_classes = m->pm.classes;
    return ISR_OK;
}

size_t isr_workspace_bytes(const isr_model *m, uint32_t chunk_samples) {
    if (!m || chunk_samples == 0) return 0;
    size_t need = 0;
    for (int i = 0; i < 3; ++i) {
        Plan pl;
        pl.ops = m->plan[i].ops;
        if (i >= 1) plan_segments(m->pm, chunk_samples, pl);
        plan_workspace(m->pm, chunk_samples, pl);
        need = std::max(need, pl.bytes);
    }
    return need;
}

int isr_set_workspace(isr_model *m, void *workspace_device, size_t bytes, uint32_t chunk_samples, void *hip_stream) {
    if (!m || !workspace_device || chunk_samples == 0) return ISR_ERR_ARG;
    if ((uintptr_t)workspace_device % 256 != 0) return ISR_ERR_ARG;
    // pixel counts of a chunk are kept in 32 bits inside the kernels
    for (const TensorDesc &t : m->pm.tensors)
        if ((uint64_t)chunk_samples * t.H * t.W * std::max(t.Cp, 16) >= (1ull << 31)) return ISR_ERR_ARG;
    if (bytes < isr_workspace_bytes(m, chunk_samples)) return ISR_ERR_WORKSPACE;
    plan_segments(m->pm, chunk_samples, m->plan[1]);
    plan_segments(m->pm, chunk_samples, m->plan[2]);
    for (int i = 0; i < 3; ++i) plan_workspace(m->pm, chunk_samples, m->plan[i]);
    m->ws = (uint8_t *)workspace_device;
    m->ws_bytes = bytes;
    m->chunk = chunk_samples;
    m->stream = (hipStream_t)hip_stream;
    return ISR_OK;
}

int isr_certify(isr_model *m, const uint8_t *x_device, uint32_t sigma, uint32_t n0, uint32_t n, double alpha,
                uint64_t seed, uint32_t image_id, isr_result *out, uint32_t *counts0_host, uint32_t *counts1_host) {
    int rc = check_call(m, x_device, sigma, alpha, true);
    if (rc != ISR_OK) return rc;
    if (!out || n0 == 0 || n == 0) return ISR_ERR_ARG;
    const uint32_t C = (uint32_t)m->pm.classes;
    const DeviceNoiseTable *table = nullptr;
    if ((rc = get_table(m, sigma, &table)) != ISR_OK) return rc;
    HIP_TRY(launch_fill_u32(m->dcounts, 0, 2 * C, m->stream));
    if ((rc = run_range(m, m->plan[m->use_fused], x_device, table, seed, image_id, 0, 0, n0, nullptr, nullptr, m->dcounts, -1)) != ISR_OK) return rc;
    if ((rc = run_range(m, m->plan[m->use_fused], x_device, table, seed, image_id, 1, 0, n, nullptr, nullptr, m->dcounts + C, -1)) != ISR_OK) return rc;
    HIP_TRY(hipMemcpyAsync(m->hcounts, m->dcounts, sizeof(uint32_t) * 2 * C, hipMemcpyDeviceToHost, m->stream));
    HIP_TRY(hipStreamSynchronize(m->stream));
    if (counts0_host) std::memcpy(counts0_host, m->hcounts, sizeof(uint32_t) * C);
    if (counts1_host) std::memcpy(counts1_host, m->hcounts + C, sizeof(uint32_t) * C);
    return isr_decide_certify(m->hcounts, m->hcounts + C, C, (double)sigma, n, alpha, out);
}

int isr_predict(isr_model *m, const uint8_t *x_device, uint32_t sigma, uint32_t n, double alpha, uint64_t seed,
                uint32_t image_id, isr_result *out, uint32_t *counts_host) {
    int rc = check_call(m, x_device, sigma, alpha, true);
    if (rc != ISR_OK) return rc;
    if (!out || n == 0) return ISR_ERR_ARG;
    const uint32_t C = (uint32_t)m->pm.classes;
    const DeviceNoiseTable *table = nullptr;
    if ((rc = get_table(m, sigma, &table)) != ISR_OK) return rc;
    HIP_TRY(launch_fill_u32(m->dcounts, 0, C, m->stream));
    if ((rc = run_range(m, m->plan[m->use_fused], x_device, table, seed, image_id, 0, 0, n, nullptr, nullptr, m->dcounts, -1)) != ISR_OK) return rc;
    HIP_TRY(hipMemcpyAsync(m->hcounts, m->dcounts, sizeof(uint32_t) * C, hipMemcpyDeviceToHost, m->stream));
    HIP_TRY(hipStreamSynchronize(m->stream));
    if (counts_host) std::memcpy(counts_host, m->hcounts, sizeof(uint32_t) * C);
    return isr_decide_predict(m->hcounts, C, alpha, out);
}

int isr_certify_batch(isr_model *m, const uint8_t *x_device, uint32_t n_images, const isr_item *items_host,
                      uint32_t n_items, uint32_t n0, uint32_t n, double alpha, uint64_t seed, isr_result *out_host,
                      uint32_t *counts0_host, uint32_t *counts1_host) {
    if (!out_host || n0 == 0 || n == 0) return ISR_ERR_ARG;
    int rc = prepare_batch(m, x_device, n_images, items_host, n_items, alpha, 2);
    if (rc != ISR_OK) return rc;
    const size_t C = (size_t)m->pm.classes, per_phase = (size_t)n_items * C;
    const Plan &pl = m->plan[m->use_fused];
    BatchCtx bc{m->ditems, n_items, n0};
    if ((rc = run_range(m, pl, x_device, m->dtables, seed, 0, 0, 0, 0, nullptr, nullptr, m->dcounts_b, -1, &bc)) != ISR_OK) return rc;
    bc.n_per_item = n;
    if ((rc = run_range(m, pl, x_device, m->dtables, seed, 0, 1, 0, 0, nullptr, nullptr, m->dcounts_b + per_phase, -1, &bc)) != ISR_OK) return rc;
    HIP_TRY(hipMemcpyAsync(m->hcounts_b, m->dcounts_b, sizeof(uint32_t) * 2 * per_phase, hipMemcpyDeviceToHost, m->stream));
    HIP_TRY(hipStreamSynchronize(m->stream));
    if (counts0_host) std::memcpy(counts0_host, m->hcounts_b, sizeof(uint32_t) * per_phase);
    if (counts1_host) std::memcpy(counts1_host, m->hcounts_b + per_phase, sizeof(uint32_t) * per_phase);
    for (uint32_t i = 0; i < n_items; ++i) {
        rc = isr_decide_certify(m->hcounts_b + i * C, m->hcounts_b + per_phase + i * C, (uint32_t)C, (double)items_host[i].sigma, n,
                                alpha, out_host + i);
        if (rc != ISR_OK) return rc;
    }
    return ISR_OK;
}

int isr_predict_batch(isr_model *m, const uint8_t *x_device, uint32_t n_images, const isr_item *items_host,
                      uint32_t n_items, uint32_t n, double alpha, uint64_t seed, isr_result *out_host,
                      uint32_t *counts_host) {
    if (!out_host || n == 0) return ISR_ERR_ARG;
    int rc = prepare_batch(m, x_device, n_images, items_host, n_items, alpha, 1);
    if (rc != ISR_OK) return rc;
    const size_t C = (size_t)m->pm.classes, per_phase = (size_t)n_items * C;
    BatchCtx bc{m->ditems, n_items, n};
    if ((rc = run_range(m, m->plan[m->use_fused], x_device, m->dtables, seed, 0, 0, 0, 0, nullptr, nullptr, m->dcounts_b, -1, &bc)) != ISR_OK) return rc;
    HIP_TRY(hipMemcpyAsync(m->hcounts_b, m->dcounts_b, sizeof(uint32_t) * per_phase, hipMemcpyDeviceToHost, m->stream));
    HIP_TRY(hipStreamSynchronize(m->stream));
    if (counts_host) std::memcpy(counts_host, m->hcounts_b, sizeof(uint32_t) * per_phase);
    for (uint32_t i = 0; i < n_items; ++i) {
        rc = isr_decide_predict(m->hcounts_b + i * C, (uint32_t)C, alpha, out_host + i);
        if (rc != ISR_OK) return rc;
    }
    return ISR_OK;
}

int isr_debug_noisy(isr_model *m, const uint8_t *x_device, uint32_t sigma, uint64_t seed, uint32_t image_id,
                    uint32_t phase, uint32_t sample_begin, uint32_t count, int8_t *out_host) {
    int rc = check_call(m, x_device, sigma, 0.5, false);
    if (rc != ISR_OK) return rc;
    if (!out_host || count == 0 || count > m->chunk || phase > 1) return ISR_ERR_ARG;
    const DeviceNoiseTable *table = nullptr;
    if ((rc = get_table(m, sigma, &table)) != ISR_OK) return rc;
    if ((rc = run_range(m, m->plan[m->use_fused], x_device, table, seed, image_id, phase, sample_begin, count, nullptr, nullptr, nullptr, 0)) != ISR_OK) return rc;
    const ParsedModel &pm = m->pm;
    const size_t hw = (size_t)pm.H * pm.W;
    std::vector<int8_t> tmp(count * hw * 4);
    HIP_TRY(hipMemcpyAsync(tmp.data(), m->ws + m->plan[m->use_fused].toff[0], tmp.size(), hipMemcpyDeviceToHost, m->stream));
    HIP_TRY(hipStreamSynchronize(m->stream));
    for (uint32_t s = 0; s < count; ++s)
        for (int c = 0; c < pm.C; ++c)
            for (size_t i = 0; i < hw; ++i) out_host[((size_t)s * pm.C + c) * hw + i] = tmp[((size_t)s * hw + i) * 4 + c];
    return ISR_OK;
}

int isr_debug_forward(isr_model *m, const uint8_t *x_device, uint32_t sigma, uint64_t seed, uint32_t image_id,
                      uint32_t phase, uint32_t sample_begin, uint32_t count, int32_t *logits_host,
                      int32_t *argmax_host, uint32_t *counts_host) {
    int rc = check_call(m, x_device, sigma, 0.5, false);
    if (rc != ISR_OK) return rc;
    if (count == 0 || phase > 1) return ISR_ERR_ARG;
    const uint32_t C = (uint32_t)m->pm.classes;
    const DeviceNoiseTable *table = nullptr;
    if ((rc = get_table(m, sigma, &table)) != ISR_OK) return rc;
    if (counts_host) HIP_TRY(launch_fill_u32(m->dcounts, 0, C, m->stream));
    rc = run_range(m, m->plan[m->use_fused], x_device, table, seed, image_id, phase, sample_begin, count, logits_host, argmax_host,
                   counts_host ? m->dcounts : nullptr, -1);
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

int isr_debug_tensor(isr_model *m, const uint8_t *x_device, uint32_t sigma, uint64_t seed, uint32_t image_id,
                     uint32_t phase, uint32_t sample, int32_t tensor_id, int8_t *out_host) {
    int rc = check_call(m, x_device, sigma, 0.5, false);
    if (rc != ISR_OK) return rc;
    const ParsedModel &pm = m->pm;
    if (!out_host || phase > 1 || tensor_id < 0 || tensor_id >= (int)pm.tensors.size() || tensor_id == pm.ops.back().out)
        return ISR_ERR_ARG;
    const DeviceNoiseTable *table = nullptr;
    if ((rc = get_table(m, sigma, &table)) != ISR_OK) return rc;
    // tensors that the fused plan never materialises come from the op-by-op plan
    const Plan &pl = (m->use_fused && m->plan[m->use_fused].has[tensor_id]) ? m->plan[m->use_fused] : m->plan[0];
    if ((rc = run_range(m, pl, x_device, table, seed, image_id, phase, sample, 1, nullptr, nullptr, nullptr, tensor_id)) != ISR_OK) return rc;
    const TensorDesc &t = pm.tensors[tensor_id];
    const size_t hw = (size_t)t.H * t.W;
    std::vector<int8_t> tmp(hw * t.Cp);
    HIP_TRY(hipMemcpyAsync(tmp.data(), m->ws + pl.toff[tensor_id], tmp.size(), hipMemcpyDeviceToHost, m->stream));
    HIP_TRY(hipStreamSynchronize(m->stream));
    for (int c = 0; c < t.C; ++c)
        for (size_t i = 0; i < hw; ++i) out_host[(size_t)c * hw + i] = tmp[i * t.Cp + c];
    return ISR_OK;
}

int isr_debug_tensor_source(const isr_model *m, int32_t tensor_id, int *from_fused_out) {
    if (!m || !from_fused_out || tensor_id < 0 || tensor_id >= (int)m->pm.tensors.size()) return ISR_ERR_ARG;
    if (m->plan[1].has.empty()) return ISR_ERR_WORKSPACE;   // plans are placed by isr_set_workspace
    *from_fused_out = (m->use_fused && m->plan[m->use_fused].has[tensor_id]) ? 1 : 0;
    return ISR_OK;
}

const char *isr_strerror(int status) {
    switch (status) {
    case ISR_OK: return "ok";
    case ISR_ERR_ARG: return "invalid argument";
    case ISR_ERR_FORMAT: return "malformed model blob";
    case ISR_ERR_UNSUPPORTED: return "model uses a shape or op the kernels do not cover";
    case ISR_ERR_WORKSPACE: return "workspace missing or too small";
    case ISR_ERR_DEVICE: return "HIP call failed";
    default: return "unknown status";
    }
}

int isr_last_device_error(void) { return g_last_hip_error; }

}  // extern "C"
