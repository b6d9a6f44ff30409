// C ABI: model loading, workspace planning and the Monte-Carlo driver that
// enqueues noise -> layers -> vote kernels for chunks of sample indices.
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <map>
#include <new>

#include "isr_internal.h"

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

constexpr int TABLE_SLOTS = 8;

enum KernelClass { KC_NOISE, KC_CONV16, KC_CONV32, KC_CONV64, KC_CONV128, KC_ADD, KC_POOL, KC_GAP, KC_FC, KC_COUNT };
const char *const KC_NAMES[KC_COUNT] = {"noise", "conv_m16", "conv_m32", "conv_m64", "conv_m128",
                                        "add", "maxpool", "gap", "fc_vote"};

struct DevOp {
    OpType type;
    int a = -1, b = -1, out = -1;
    int kclass = 0;
    double ops_per_sample = 0.0, bytes_per_sample = 0.0;   // algorithmic, for the timing report
    ConvParams conv{};
    int stem_pool = 0;                  // conv fused with the max pooling after it (out = the pooled tensor)
    int stem16 = 0;                     // first 3x3 convolution into 16 channels: the LDS-resident kernel
    int block = 0;                      // identity residual block: this conv, conv2 and the add in one kernel
    std::vector<std::pair<ConvParams, ConvParams>> chain;   // block != 0: the blocks of the chain this op runs (each feeds the next)
    size_t chain_off = 0;               // first BlockDesc of the chain in the model's device array
    int trans = 0;                      // down-sampling block: this conv (3x3/2), conv2 (3x3) and conv3 (1x1/2 + add) in one kernel
    int bneck = 0;                      // 1: this 1x1 conv and the 3x3 conv2 in one kernel; 2: plus conv3 (1x1 + residual add)
    ConvParams conv2{};
    ConvParams conv3{};
    AddParams add{};
    PoolParams pool{};
    GapParams gap{};
    FcParams fc{};
};

size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// MFMA 32x32 accumulator row r of lane half h, register i is 8*(i/4) + 4*h + i%4;
// weights of output channel 16*h + i go to that row so that a lane ends up
// holding 16 consecutive channels.
int mfma32_row_of_channel(int oc_local) {
    int h = oc_local >> 4, a = (oc_local & 15) >> 2, b = oc_local & 3;
    return 8 * a + 4 * h + b;
}

}  // namespace

// An executable op list plus where each tensor lives in the workspace.
struct Plan {
    std::vector<DevOp> ops;
    std::vector<size_t> toff;           // per tensor offset inside the workspace
    std::vector<char> has;              // tensor is produced by this plan
    size_t logits_off = 0, argmax_off = 0, bytes = 0;
};

struct isr_model {
    ParsedModel pm;
    std::vector<DevOp> ops;             // one descriptor per op of the blob
    Plan plan[2];                       // [0] op by op, [1] with every fusion the kernels cover
    int use_fused = 1;
    int conv_tile = 0;                  // forced conv output tile (0 = automatic)
    uint8_t *dconst = nullptr;          // weights and per-channel tables
    DeviceNoiseTable *dtables = nullptr;  // TABLE_SLOTS entries
    DeviceNoiseTable *htables = nullptr;  // pinned staging, TABLE_SLOTS entries
    uint32_t table_sigma[TABLE_SLOTS] = {0};
    int table_next = 0;
    uint32_t *dcounts = nullptr;        // 2 * classes
    uint32_t *hcounts = nullptr;        // pinned, 2 * classes
    BlockDesc *dblocks = nullptr;       // descriptors of the identity-block chains of plan[1]
    // batched calls: item descriptors and per-item vote counters, grown on demand
    NoiseItem *ditems = nullptr, *hitems = nullptr;
    uint32_t *dcounts_b = nullptr, *hcounts_b = nullptr;   // 2 * items_cap * classes each
    uint32_t items_cap = 0;
    // workspace
    uint8_t *ws = nullptr;
    size_t ws_bytes = 0;
    uint32_t chunk = 0;
    hipStream_t stream = nullptr;
    // per-kernel timing
    uint32_t profile_every = 0;
    uint64_t chunk_counter = 0;
    std::vector<hipEvent_t> events;
    isr_kernel_stat stats[KC_COUNT] = {};
};

namespace {

// Offsets of every tensor for a chunk of B samples; buffers are reused once the
// last op reading a tensor has been issued (stream order makes that safe).
void plan_workspace(const ParsedModel &pm, uint32_t B, Plan &pl) {
    const int nt = (int)pm.tensors.size();
    std::vector<int> last_use(nt, -1);
    for (int i = 0; i < (int)pl.ops.size(); ++i) {
        const DevOp &o = pl.ops[i];
        if (o.a >= 0) last_use[o.a] = i;
        if (o.b >= 0) last_use[o.b] = i;
    }
    auto tbytes = [&](int t) {
        const TensorDesc &d = pm.tensors[t];
        return round_up((size_t)B * d.H * d.W * d.Cp + 64, 256);
    };
    struct Block { size_t off, size; };
    std::vector<Block> freelist;
    size_t top = 0;
    auto alloc = [&](size_t n) {
        for (size_t i = 0; i < freelist.size(); ++i)
            if (freelist[i].size >= n) {
                size_t off = freelist[i].off;
                freelist[i].off += n;
                freelist[i].size -= n;
                if (freelist[i].size == 0) freelist.erase(freelist.begin() + i);
                return off;
            }
        size_t off = top;
        top += n;
        return off;
    };
    auto release = [&](size_t off, size_t n) {
        freelist.push_back({off, n});
        std::sort(freelist.begin(), freelist.end(), [](const Block &x, const Block &y) { return x.off < y.off; });
        for (size_t i = 0; i + 1 < freelist.size();)
            if (freelist[i].off + freelist[i].size == freelist[i + 1].off) {
                freelist[i].size += freelist[i + 1].size;
                freelist.erase(freelist.begin() + i + 1);
            } else {
                ++i;
            }
    };
    pl.toff.assign(nt, 0);
    pl.has.assign(nt, 0);
    pl.toff[0] = alloc(tbytes(0));
    pl.has[0] = 1;
    for (int i = 0; i < (int)pl.ops.size(); ++i) {
        const DevOp &o = pl.ops[i];
        if (o.type != OP_FC) { pl.toff[o.out] = alloc(tbytes(o.out)); pl.has[o.out] = 1; }
        for (int t : {o.a, o.b})
            if (t >= 0 && last_use[t] == i && !(t == o.b && o.a == o.b)) release(pl.toff[t], tbytes(t));
    }
    pl.logits_off = round_up(top, 256);
    pl.argmax_off = pl.logits_off + round_up((size_t)B * pm.classes * 4, 256);
    pl.bytes = pl.argmax_off + round_up((size_t)B * 4, 256);
}

// Folds each residual ADD into the convolution issued right before it when that
// convolution produces one of the add's inputs for the add alone and the sum
// fits 32 bits: the convolution then reads the other input in its epilogue and
// writes the add's output (the two roundings are kept).
void fuse_adds(const ParsedModel &pm, const std::vector<DevOp> &plain, std::vector<DevOp> &fused) {
    std::vector<int> uses(pm.tensors.size(), 0);
    for (const DevOp &d : plain) {
        if (d.a >= 0) uses[d.a]++;
        if (d.b >= 0) uses[d.b]++;
    }
    fused.clear();
    for (size_t i = 0; i < plain.size(); ++i) {
        const DevOp &d = plain[i];
        if (d.type == OP_ADD && !fused.empty() && fused.back().type == OP_CONV && !fused.back().conv.fuse_add &&
            fused.back().conv.fast_requant && d.a != d.b &&
            (fused.back().out == d.a || fused.back().out == d.b) && uses[fused.back().out] == 1) {
            DevOp &c = fused.back();
            const bool conv_is_a = c.out == d.a;
            const int res = conv_is_a ? d.b : d.a;
            const AddParams &a = d.add;
            const int64_t m_self = conv_is_a ? a.Ma : a.Mb, m_res = conv_is_a ? a.Mb : a.Ma;
            const int64_t z_self = conv_is_a ? a.za : a.zb, z_res = conv_is_a ? a.zb : a.za;
            const int64_t c0 = -z_self * m_self - z_res * m_res;
            const int64_t k = (a.sh >= 1 ? (1ll << (a.sh - 1)) : 0) + (int64_t)a.zo * (1ll << a.sh);
            auto mag = [](int64_t v) { return v < 0 ? -v : v; };
            const int64_t bound = 255 * (mag(m_self) + mag(m_res)) + mag(k) + 1;
            if (a.sh >= 1 && a.sh <= 30 && mag(m_self) < (1 << 23) && mag(m_res) < (1 << 23) && bound < (1ll << 31)) {
                c.conv.fuse_add = 1;
                c.conv.add_mul_self = (int32_t)m_self;
                c.conv.add_mul_res = (int32_t)m_res;
                c.conv.add_c0 = (int32_t)c0;
                c.conv.add_k = (int32_t)k;
                c.conv.add_sh = a.sh;
                c.conv.add_lo = a.relu ? a.zo : -128;
                // v = q Ms + r Mr + c0 over all int8 pairs: is a negative exact half of 2^sh ever met?
                bool add_ties = false;
                const int64_t halfbit = 1ll << (a.sh - 1), mask = (1ll << a.sh) - 1;
                for (int q = -128; q <= 127 && !add_ties; ++q)
                    for (int r = -128; r <= 127; ++r) {
                        const int64_t v = q * m_self + r * m_res + c0;
                        if (v < 0 && (v & mask) == halfbit) { add_ties = true; break; }
                    }
                c.conv.add_tie_free = add_ties ? 0 : 1;
                c.b = res;
                c.out = d.out;
                c.bytes_per_sample += d.bytes_per_sample / 3.0;   // the residual read
                // The residual is the output of the 1x1 convolution issued right before, read by this
                // add alone: compute it inside the same kernel instead of round-tripping it through memory.
                if (fused.size() >= 2) {
                    const DevOp &r = fused[fused.size() - 2];
                    const ConvParams &rc = r.conv;
                    const bool direct = c.conv.fast_requant && !c.conv.c4 && c.conv.Cout_p >= 64;
                    if (direct && r.type == OP_CONV && r.out == res && uses[res] == 1 && !rc.fuse_add && rc.fast_requant &&
                        !rc.c4 && rc.ktab == nullptr && rc.Cin_p % 64 == 0 && rc.Kp == rc.Cin_p &&
                        rc.Cout_p == c.conv.Cout_p && rc.Mp == c.conv.Mp && rc.Ho == c.conv.Ho && rc.Wo == c.conv.Wo) {
                        DevOp merged = c;
                        merged.conv.fuse_add = 2;
                        merged.conv.w2 = rc.w; merged.conv.bias2 = rc.bias; merged.conv.m0s2 = rc.m0s;
                        merged.conv.chi2 = rc.chi; merged.conv.shm12 = rc.shm1;
                        merged.conv.Cin2_p = rc.Cin_p;
                        merged.conv.lo2 = rc.relu ? rc.zp_out : -128;
                        merged.conv.tie_free2 = rc.tie_free;
                        merged.b = r.a;   // second input tensor (kept alive until this op is issued)
                        merged.ops_per_sample += r.ops_per_sample;
                        merged.bytes_per_sample += r.bytes_per_sample - 2.0 * d.bytes_per_sample / 3.0;   // no residual write + read
                        fused.pop_back();
                        fused.pop_back();
                        fused.push_back(merged);
                    }
                }
                continue;
            }
        }
        fused.push_back(d);
    }
}

// Folds conv3x3 -> conv3x3 -> add-with-the-block-input (identity residual block) into one
// kernel for the shapes that fit LDS whole.  Runs on the list in which the add is already
// folded into the second convolution.
void fuse_basic_blocks(const ParsedModel &pm, std::vector<DevOp> &ops) {
    std::vector<int> uses(pm.tensors.size(), 0);
    for (const DevOp &d : ops) {
        if (d.a >= 0) uses[d.a]++;
        if (d.b >= 0) uses[d.b]++;
    }
    for (size_t i = 0; i + 1 < ops.size(); ++i) {
        DevOp &a = ops[i];
        const DevOp &b = ops[i + 1];
        if (a.type != OP_CONV || b.type != OP_CONV || a.stem_pool || a.block || a.conv.fuse_add || b.conv.fuse_add != 1) continue;
        const ConvParams &ca = a.conv, &cb = b.conv;
        auto is3x3 = [](const ConvParams &c) { return c.k == 3 && c.stride == 1 && c.pad == 1 && !c.c4 && c.fast_requant; };
        if (!is3x3(ca) || !is3x3(cb) || b.a != a.out || b.b != a.a || uses[a.out] != 1) continue;
        if (ca.Cin_p != ca.Cout_p || cb.Cin_p != ca.Cout_p || cb.Cout_p != ca.Cout_p || ca.H != ca.W || ca.Ho != ca.H ||
            !basic_block_supported(ca.Cout_p, ca.H))
            continue;
        a.block = 1;
        a.conv2 = cb;
        a.chain.assign(1, {ca, cb});
        a.ops_per_sample += b.ops_per_sample;
        a.bytes_per_sample = (double)pm.tensors[a.a].C * ca.H * ca.W + (double)pm.tensors[b.out].C * ca.H * ca.W;
        a.out = b.out;
        ops.erase(ops.begin() + i + 1);
    }
}

// Joins consecutive identity-block ops of one shape, each read by the next alone, into one op:
// the kernel then keeps the images in LDS from the first block to the last.
void chain_basic_blocks(const ParsedModel &pm, std::vector<DevOp> &ops) {
    std::vector<int> uses(pm.tensors.size(), 0);
    for (const DevOp &d : ops) {
        if (d.a >= 0) uses[d.a]++;
        if (d.b >= 0) uses[d.b]++;
    }
    auto tf = [](const DevOp &d) { return d.conv.tie_free && d.conv2.tie_free && d.conv2.add_tie_free; };
    for (size_t i = 0; i + 1 < ops.size();) {
        DevOp &a = ops[i];
        const DevOp &b = ops[i + 1];
        if (a.block && b.block && b.a == a.out && uses[a.out] == 1 && a.conv.Cout_p == b.conv.Cout_p && a.conv.H == b.conv.H &&
            tf(a) == tf(b) && a.chain.size() < 64) {
            a.chain.insert(a.chain.end(), b.chain.begin(), b.chain.end());
            a.ops_per_sample += b.ops_per_sample;
            a.bytes_per_sample = (a.bytes_per_sample + b.bytes_per_sample) / 2;   // one read of the first input, one write of the last output
            a.out = b.out;
            ops.erase(ops.begin() + i + 1);
        } else {
            ++i;
        }
    }
}

// Folds the down-sampling block of the narrow nets -- conv3x3 stride 2, conv3x3, and the 1x1
// stride-2 projection that carries the residual add -- into one kernel for the shapes that fit LDS.
void fuse_trans_blocks(const ParsedModel &pm, std::vector<DevOp> &ops) {
    std::vector<int> uses(pm.tensors.size(), 0);
    for (const DevOp &d : ops) {
        if (d.a >= 0) uses[d.a]++;
        if (d.b >= 0) uses[d.b]++;
    }
    auto plain = [](const DevOp &d) {
        return d.type == OP_CONV && !d.stem_pool && !d.stem16 && !d.block && !d.bneck && !d.trans && !d.conv.c4 && d.conv.fast_requant;
    };
    for (size_t i = 0; i + 2 < ops.size(); ++i) {
        DevOp &a = ops[i];
        const DevOp &b = ops[i + 1], &c = ops[i + 2];
        if (!plain(a) || !plain(b) || !plain(c) || a.conv.fuse_add || b.conv.fuse_add || c.conv.fuse_add != 1) continue;
        const ConvParams &c1 = a.conv, &c2 = b.conv, &cp = c.conv;
        const int C = c1.Cout_p, S = c1.Ho;
        if (c1.k != 3 || c1.stride != 2 || c1.pad != 1 || c2.k != 3 || c2.stride != 1 || c2.pad != 1 || cp.k != 1 ||
            cp.stride != 2 || cp.pad != 0)
            continue;
        if (2 * c1.Cin_p != C || c2.Cin_p != C || c2.Cout_p != C || cp.Cin_p != c1.Cin_p || cp.Cout_p != C || c1.H != 2 * S ||
            c1.W != 2 * S || c1.Wo != S || cp.Ho != S || cp.Wo != S || !trans_block_supported(C, S))
            continue;
        if (c1.Kp != (9 * c1.Cin_p + 63) / 64 * 64 || c2.Kp != (9 * C + 63) / 64 * 64 || cp.Kp != 64) continue;
        if (b.a != a.out || c.a != a.a || c.b != b.out || uses[a.out] != 1 || uses[b.out] != 1) continue;
        a.trans = 1;
        a.conv2 = c2;
        a.conv3 = cp;
        a.ops_per_sample += b.ops_per_sample + c.ops_per_sample;
        a.bytes_per_sample = (double)pm.tensors[a.a].C * c1.H * c1.W + (double)pm.tensors[c.out].C * S * S;
        a.out = c.out;
        ops.erase(ops.begin() + i + 1, ops.begin() + i + 3);
    }
}

// Folds conv1x1 (-> 64 channels) -> conv3x3 (64 -> 64) of a bottleneck block into one kernel,
// and with them the closing conv1x1 + residual add when the residual is the block input.
// Runs on the list in which the adds are already folded into their convolutions.
void fuse_bottlenecks(const ParsedModel &pm, std::vector<DevOp> &ops) {
    std::vector<int> uses(pm.tensors.size(), 0);
    for (const DevOp &d : ops) {
        if (d.a >= 0) uses[d.a]++;
        if (d.b >= 0) uses[d.b]++;
    }
    auto plain = [](const DevOp &d) {
        return d.type == OP_CONV && !d.stem_pool && !d.stem16 && !d.block && !d.trans && !d.bneck && !d.conv.c4 && d.conv.fast_requant;
    };
    for (size_t i = 0; i + 1 < ops.size(); ++i) {
        DevOp &a = ops[i];
        const DevOp &b = ops[i + 1];
        if (!plain(a) || !plain(b) || a.conv.fuse_add || b.conv.fuse_add) continue;
        const ConvParams &c1 = a.conv, &c2 = b.conv;
        if (c1.k != 1 || c1.stride != 1 || c1.pad != 0 || c1.Kp != c1.Cin_p || c1.Cout_p != 64) continue;
        if (c2.k != 3 || c2.stride != 1 || c2.pad != 1 || c2.Cin_p != 64 || c2.Cout_p != 64 || c2.Kp != 576) continue;
        if (b.a != a.out || uses[a.out] != 1 || !bottleneck_supported(c1.Cin_p, 64, 0, 0)) continue;
        a.bneck = 1;
        a.conv2 = c2;
        a.ops_per_sample += b.ops_per_sample;
        a.bytes_per_sample = (double)pm.tensors[a.a].C * c1.H * c1.W + (double)pm.tensors[b.out].C * c1.H * c1.W;
        a.out = b.out;
        ops.erase(ops.begin() + i + 1);
        if (i + 1 < ops.size()) {
            const DevOp &c = ops[i + 1];
            const ConvParams &c3 = c.conv;
            if (plain(c) && c3.fuse_add == 1 && c3.k == 1 && c3.stride == 1 && c3.pad == 0 && c3.Cin_p == 64 && c3.Kp == 64 &&
                c.a == a.out && c.b == a.a && uses[a.out] == 1 && bottleneck_supported(c1.Cin_p, 64, c3.Cout_p, 1)) {
                a.bneck = 2;
                a.conv3 = c3;
                a.ops_per_sample += c.ops_per_sample;
                a.bytes_per_sample = 2.0 * pm.tensors[a.a].C * c1.H * c1.W;
                a.out = c.out;
                ops.erase(ops.begin() + i + 1);
            }
        }
    }
}

// Folds the max pooling that follows the first convolution into it when the fused
// kernel covers the geometry and the convolution output has no other reader.
void fuse_stem_pool(const ParsedModel &pm, std::vector<DevOp> &ops) {
    std::vector<int> uses(pm.tensors.size(), 0);
    for (const DevOp &d : ops) {
        if (d.a >= 0) uses[d.a]++;
        if (d.b >= 0) uses[d.b]++;
    }
    for (size_t i = 0; i + 1 < ops.size(); ++i) {
        DevOp &c = ops[i];
        const DevOp &q = ops[i + 1];
        if (c.type != OP_CONV || !c.conv.c4 || c.conv.fuse_add || q.type != OP_MAXPOOL || q.a != c.out || uses[c.out] != 1)
            continue;
        if (c.conv.Kp != 256) continue;   // K = 7 rows x 8 taps x 4 channels
        if (!stem_pool_supported(c.conv.k, c.conv.stride, c.conv.pad, c.conv.Cout_p, c.conv.H, c.conv.W, c.conv.fast_requant,
                                 q.pool.k, q.pool.stride, q.pool.pad))
            continue;
        c.stem_pool = 1;
        c.bytes_per_sample = (double)pm.tensors[c.a].C * c.conv.H * c.conv.W +
                             (double)pm.tensors[q.out].C * pm.tensors[q.out].H * pm.tensors[q.out].W;
        c.out = q.out;
        ops.erase(ops.begin() + i + 1);
        return;
    }
}

struct ConstArena {
    std::vector<uint8_t> host;
    size_t put(const void *src, size_t n) {
        size_t off = round_up(host.size(), 256);
        host.resize(off + round_up(n, 16), 0);
        if (src) std::memcpy(host.data() + off, src, n);
        return off;
    }
};

// Builds device descriptors; pointers into the constant arena are stored as
// offsets first and rebased after the upload.
int build_device_ops(isr_model *m, ConstArena &arena) {
    const ParsedModel &pm = m->pm;
    for (const HostOp &o : pm.ops) {
        DevOp d;
        d.type = o.type; d.a = o.a; d.b = o.b; d.out = o.out;
        switch (o.type) {
        case OP_CONV: {
            const TensorDesc &ti = pm.tensors[o.a], &to = pm.tensors[o.out];
            const bool c4 = o.a == 0;
            const int cin_p = ti.Cp, cout_p = to.Cp, k = o.k;
            const int kwp = (k + 3) & ~3;
            const int kreal = c4 ? k * kwp * 4 : k * k * cin_p;
            bool fast = true;
            for (int oc = 0; oc < to.C; ++oc) fast = fast && o.shift[oc] >= 2 && o.shift[oc] <= 22;
            const int kb = conv_k_step(kreal, c4 ? 0 : cin_p, cout_p, fast ? 1 : 0);
            const int Kp = (int)round_up((size_t)kreal, (size_t)kb), Mp = (int)round_up((size_t)cout_p, 128);
            const bool perm = conv_tile_m(cout_p) != 16;
            std::vector<int8_t> w((size_t)Mp * Kp, 0);
            std::vector<int32_t> bias(Mp, 0);
            bool tie_free = fast;
            const int64_t maxdev = std::max<int64_t>(127 - ti.zp, ti.zp + 128);   // |q - z_in| of an int8 input
            std::vector<uint32_t> m0x2(Mp, 0x80000000u), rlo(Mp, 0), rhi(Mp, 1), sh(Mp, 1);
            std::vector<int32_t> m0s(Mp, 1 << 30), chi(Mp, 1 + 2 * to.zp), shm1(Mp, 1);
            for (int oc = 0; oc < to.C; ++oc) {
                int row = perm ? (oc & ~31) + mfma32_row_of_channel(oc & 31) : oc;
                int64_t wsum = 0, wabs = 0;
                for (int ic = 0; ic < ti.C; ++ic)
                    for (int ky = 0; ky < k; ++ky)
                        for (int kx = 0; kx < k; ++kx) {
                            int8_t v = o.w[(((size_t)oc * ti.C + ic) * k + ky) * k + kx];
                            int kk = c4 ? (ky * kwp + kx) * 4 + ic : (ky * k + kx) * cin_p + ic;
                            w[(size_t)row * Kp + kk] = v;
                            wsum += v;
                            wabs += v < 0 ? -v : v;
                        }
                {
                    // acc * M0 is an exact half of 2^(31 + shift) only if acc = (odd) * 2^(30 + shift - tz(M0))
                    const int64_t accmax = std::llabs((int64_t)o.bias[oc]) + maxdev * wabs;
                    const int need = 30 + o.shift[oc] - __builtin_ctz((unsigned)o.M0[oc]);
                    if (need < 40 && accmax >= (1ll << need)) tie_free = false;
                }
                int64_t b = (int64_t)o.bias[oc] - (int64_t)ti.zp * wsum;
                if (b < INT32_MIN || b > INT32_MAX) return ISR_ERR_UNSUPPORTED;
                bias[oc] = (int32_t)b;
                m0x2[oc] = (uint32_t)o.M0[oc] << 1;
                uint64_t rnd = 1ull << (31 + o.shift[oc]);
                rlo[oc] = (uint32_t)rnd; rhi[oc] = (uint32_t)(rnd >> 32); sh[oc] = (uint32_t)o.shift[oc];
                if (o.shift[oc] >= 2 && o.shift[oc] <= 22) {
                    m0s[oc] = o.M0[oc];
                    chi[oc] = (1 << (o.shift[oc] - 2)) + to.zp * (1 << (o.shift[oc] - 1));
                    shm1[oc] = o.shift[oc] - 1;
                }
            }
            const bool flat = !c4 && k == 1 && o.stride == 1 && o.pad == 0 && cin_p % 64 == 0;
            std::vector<uint32_t> ktab(Kp / 16, 0xFFFFFFFFu);
            std::vector<int32_t> ktoff(Kp / 16, 0);
            for (int j = 0; j < Kp / 16; ++j) {
                if (c4) {
                    int per_row = kwp / 4, ky = j / per_row, kx0 = (j % per_row) * 4;
                    if (ky < k) { ktab[j] = (uint32_t)ky | ((uint32_t)kx0 << 8); ktoff[j] = (ky * ti.W + kx0) * 4; }
                } else {
                    int k0 = j * 16, tap = k0 / cin_p, ic = k0 % cin_p;
                    if (tap < k * k) {
                        ktab[j] = (uint32_t)(tap / k) | ((uint32_t)(tap % k) << 8);
                        ktoff[j] = ((tap / k) * ti.W + (tap % k)) * cin_p + ic;
                    }
                }
            }
            ConvParams &c = d.conv;
            c.w = (const int8_t *)arena.put(w.data(), w.size());
            c.bias = (const int32_t *)arena.put(bias.data(), bias.size() * 4);
            c.m0x2 = (const uint32_t *)arena.put(m0x2.data(), m0x2.size() * 4);
            c.rnd_lo = (const uint32_t *)arena.put(rlo.data(), rlo.size() * 4);
            c.rnd_hi = (const uint32_t *)arena.put(rhi.data(), rhi.size() * 4);
            c.shift = (const uint32_t *)arena.put(sh.data(), sh.size() * 4);
            c.m0s = (const int32_t *)arena.put(m0s.data(), m0s.size() * 4);
            c.chi = (const int32_t *)arena.put(chi.data(), chi.size() * 4);
            c.shm1 = (const int32_t *)arena.put(shm1.data(), shm1.size() * 4);
            c.fast_requant = fast ? 1 : 0;
            c.tie_free = tie_free ? 1 : 0;
            const std::vector<int8_t> zfill(16, (int8_t)ti.zp);
            c.zpad = (const int8_t *)arena.put(zfill.data(), zfill.size());
            c.ktab = flat ? (const uint32_t *)~(uintptr_t)0 : (const uint32_t *)arena.put(ktab.data(), ktab.size() * 4);
            c.ktoff = flat ? (const int32_t *)~(uintptr_t)0 : (const int32_t *)arena.put(ktoff.data(), ktoff.size() * 4);
            c.H = ti.H; c.W = ti.W; c.Cin_p = cin_p; c.Ho = to.H; c.Wo = to.W; c.Cout_p = cout_p;
            c.k = k; c.stride = o.stride; c.pad = o.pad; c.Kp = Kp; c.Mp = Mp; c.kb = kb;
            c.zp_in = ti.zp; c.zp_out = to.zp; c.relu = o.relu; c.c4 = c4 ? 1 : 0;
            int tm = conv_tile_m(cout_p);
            d.kclass = tm == 16 ? KC_CONV16 : tm == 32 ? KC_CONV32 : tm == 64 ? KC_CONV64 : KC_CONV128;
            d.ops_per_sample = 2.0 * to.C * to.H * to.W * ti.C * k * k;
            d.bytes_per_sample = (double)ti.C * ti.H * ti.W + (double)to.C * to.H * to.W;
            break; }
        case OP_ADD: {
            AddParams &a = d.add;
            a.za = pm.tensors[o.a].zp; a.zb = pm.tensors[o.b].zp; a.zo = pm.tensors[o.out].zp;
            a.Ma = o.Ma; a.Mb = o.Mb; a.sh = o.sh; a.relu = o.relu;
            d.kclass = KC_ADD;
            d.bytes_per_sample = 3.0 * pm.tensors[o.out].C * pm.tensors[o.out].H * pm.tensors[o.out].W;
            break; }
        case OP_MAXPOOL: {
            const TensorDesc &ti = pm.tensors[o.a], &to = pm.tensors[o.out];
            PoolParams &p = d.pool;
            p.H = ti.H; p.W = ti.W; p.Cp = ti.Cp; p.Ho = to.H; p.Wo = to.W; p.k = o.k; p.stride = o.stride; p.pad = o.pad;
            d.kclass = KC_POOL;
            d.bytes_per_sample = (double)ti.C * ti.H * ti.W + (double)to.C * to.H * to.W;
            break; }
        case OP_GAP: {
            const TensorDesc &ti = pm.tensors[o.a], &to = pm.tensors[o.out];
            GapParams &g = d.gap;
            g.HW = ti.H * ti.W; g.Cp = ti.Cp; g.zp_in = ti.zp; g.zp_out = to.zp; g.M0 = o.Ma; g.sh = o.sh;
            d.kclass = KC_GAP;
            d.bytes_per_sample = (double)ti.C * ti.H * ti.W + (double)to.C;
            break; }
        case OP_FC: {
            const TensorDesc &ti = pm.tensors[o.a];
            const int hw = ti.H * ti.W, Kp = hw * ti.Cp, classes = pm.classes, classes_p = (classes + 3) & ~3;
            std::vector<int8_t> w((size_t)classes_p * Kp, 0);
            std::vector<int32_t> bias(classes, 0);
            for (int c = 0; c < classes; ++c) {
                int64_t wsum = 0;
                for (int ch = 0; ch < ti.C; ++ch)
                    for (int s = 0; s < hw; ++s) {
                        int8_t v = o.w[(size_t)c * ti.C * hw + (size_t)ch * hw + s];
                        const size_t k = (size_t)s * ti.Cp + ch;
                        w[((k >> 4) * classes_p + c) * 16 + (k & 15)] = v;
                        wsum += v;
                    }
                int64_t b = (int64_t)o.bias[c] - (int64_t)ti.zp * wsum;
                if (b < INT32_MIN || b > INT32_MAX) return ISR_ERR_UNSUPPORTED;
                bias[c] = (int32_t)b;
            }
            FcParams &f = d.fc;
            f.w = (const int8_t *)arena.put(w.data(), w.size());
            f.bias = (const int32_t *)arena.put(bias.data(), bias.size() * 4);
            f.Kp = Kp; f.classes = classes; f.classes_p = classes_p;
            d.kclass = KC_FC;
            d.ops_per_sample = 2.0 * classes * ti.C * hw;
            d.bytes_per_sample = (double)ti.C * hw;
            break; }
        }
        m->ops.push_back(d);
    }
    return ISR_OK;
}

template <typename T>
void rebase(const T *&p, const uint8_t *base) {
    if ((uintptr_t)p == ~(uintptr_t)0) { p = nullptr; return; }
    p = (const T *)(base + (uintptr_t)p);
}

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
    for (uint64_t done = 0; done < count;) {
        uint32_t cnt = (uint32_t)std::min<uint64_t>(m->chunk, count - done);
        if (bc) cnt = (uint32_t)std::min<uint64_t>(cnt, (uint64_t)bc->n_per_item * 65534);   // one grid row per item
        const bool timed = m->profile_every && (m->chunk_counter++ % m->profile_every) == 0;
        size_t ev = 0;
        std::vector<int> ev_class;
        auto mark = [&](int kclass) -> int {   // event before a launch (kclass >= 0) / after the last one
            if (!timed) return ISR_OK;
            if (ev == m->events.size()) {
                hipEvent_t e;
                HIP_TRY(hipEventCreate(&e));
                m->events.push_back(e);
            }
            HIP_TRY(hipEventRecord(m->events[ev++], m->stream));
            if (kclass >= 0) ev_class.push_back(kclass);
            return ISR_OK;
        };
        std::vector<std::pair<double, double>> ev_work;   // (ops, bytes) per timed launch
        int prc;
        NoiseParams np;
        np.x = x; np.table = table; np.out = (int8_t *)(ws + pl.toff[0]);
        np.C = pm.C; np.H = pm.H; np.W = pm.W;
        np.key0 = (uint32_t)seed; np.key1 = (uint32_t)(seed >> 32);
        np.image = image; np.phase = phase; np.sample_begin = begin + (uint32_t)done; np.count = cnt;
        np.items = nullptr; np.n_per_item = 0; np.item_first = 0; np.item_count = 0; np.slot_begin = 0;
        if (bc) {
            np.items = bc->items; np.n_per_item = bc->n_per_item; np.slot_begin = done;
            np.item_first = (uint32_t)(done / bc->n_per_item);
            np.item_count = (uint32_t)((done + cnt - 1) / bc->n_per_item) - np.item_first + 1;
        }
        if ((prc = mark(KC_NOISE)) != ISR_OK) return prc;
        ev_work.push_back({0.0, (double)cnt * pm.H * pm.W * 4});
        HIP_TRY(launch_noise(np, m->stream));
        if (stop_tensor != 0) {
            for (const DevOp &d : pl.ops) {
                if ((prc = mark(d.kclass)) != ISR_OK) return prc;
                ev_work.push_back({d.ops_per_sample * cnt, d.bytes_per_sample * cnt});
                switch (d.type) {
                case OP_CONV: {
                    if (d.stem_pool) {
                        const TensorDesc &to = pm.tensors[d.out];
                        StemPoolParams sp;
                        sp.in = (const int8_t *)(ws + pl.toff[d.a]);
                        sp.out = (int8_t *)(ws + pl.toff[d.out]);
                        sp.w = d.conv.w; sp.bias = d.conv.bias; sp.m0s = d.conv.m0s; sp.chi = d.conv.chi; sp.shm1 = d.conv.shm1;
                        sp.H = d.conv.H; sp.W = d.conv.W; sp.Ho = d.conv.Ho; sp.Wo = d.conv.Wo; sp.Hp = to.H; sp.Wp = to.W;
                        sp.zp_in = d.conv.zp_in; sp.zp_out = d.conv.zp_out; sp.relu = d.conv.relu; sp.tie_free = d.conv.tie_free; sp.B = (int32_t)cnt;
                        HIP_TRY(launch_stem_pool(sp, m->stream));
                        break;
                    }
                    if (d.stem16) {
                        const ConvParams &c = d.conv;
                        Stem16Params sp;
                        sp.in = (const int8_t *)(ws + pl.toff[d.a]);
                        sp.out = (int8_t *)(ws + pl.toff[d.out]);
                        sp.w = c.w; sp.bias = c.bias; sp.m0s = c.m0s; sp.chi = c.chi; sp.shm1 = c.shm1;
                        sp.H = c.H; sp.W = c.W; sp.B = (int32_t)cnt; sp.zp_in = c.zp_in;
                        sp.lo = c.relu ? c.zp_out : -128; sp.tie_free = c.tie_free;
                        HIP_TRY(launch_stem16(sp, m->stream));
                        break;
                    }
                    if (d.block) {
                        BlockParams bp{};
                        bp.in = (const int8_t *)(ws + pl.toff[d.a]);
                        bp.out = (int8_t *)(ws + pl.toff[d.out]);
                        bp.blocks = m->dblocks + d.chain_off;
                        bp.nblocks = (int32_t)d.chain.size();
                        bp.C = d.conv.Cout_p; bp.S = d.conv.H; bp.B = (int32_t)cnt;
                        bp.tie_free = d.conv.tie_free && d.conv2.tie_free && d.conv2.add_tie_free;
                        HIP_TRY(launch_basic_block(bp, m->stream));
                        break;
                    }
                    if (d.trans) {
                        const ConvParams &c1 = d.conv, &c2 = d.conv2, &cp = d.conv3;
                        TransParams tp{};
                        tp.in = (const int8_t *)(ws + pl.toff[d.a]);
                        tp.out = (int8_t *)(ws + pl.toff[d.out]);
                        tp.w1 = c1.w; tp.bias1 = c1.bias; tp.m0s1 = c1.m0s; tp.chi1 = c1.chi; tp.shm11 = c1.shm1;
                        tp.w2 = c2.w; tp.bias2 = c2.bias; tp.m0s2 = c2.m0s; tp.chi2 = c2.chi; tp.shm12 = c2.shm1;
                        tp.wp = cp.w; tp.biasp = cp.bias; tp.m0sp = cp.m0s; tp.chip = cp.chi; tp.shm1p = cp.shm1;
                        tp.C = c1.Cout_p; tp.S = c1.Ho; tp.B = (int32_t)cnt;
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
                        bp.in = (const int8_t *)(ws + pl.toff[d.a]);
                        bp.out = (int8_t *)(ws + pl.toff[d.out]);
                        bp.w1 = c1.w; bp.bias1 = c1.bias; bp.m0s1 = c1.m0s; bp.chi1 = c1.chi; bp.shm11 = c1.shm1;
                        bp.w2 = c2.w; bp.bias2 = c2.bias; bp.m0s2 = c2.m0s; bp.chi2 = c2.chi; bp.shm12 = c2.shm1;
                        bp.zpad = c1.zpad;
                        bp.Cin_p = c1.Cin_p; bp.H = c1.H; bp.W = c1.W; bp.B = (int32_t)cnt; bp.tail = d.bneck == 2;
                        bp.zp_t1 = c1.zp_out;
                        bp.lo1 = c1.relu ? c1.zp_out : -128;
                        bp.lo2 = c2.relu ? c2.zp_out : -128;
                        bp.tie_free = c1.tie_free && c2.tie_free;
                        if (bp.tail) {
                            bp.w3 = c3.w; bp.bias3 = c3.bias; bp.m0s3 = c3.m0s; bp.chi3 = c3.chi; bp.shm13 = c3.shm1;
                            bp.Cout_p = c3.Cout_p;
                            bp.lo3 = c3.relu ? c3.zp_out : -128;
                            bp.add_mul_self = c3.add_mul_self; bp.add_mul_res = c3.add_mul_res; bp.add_c0 = c3.add_c0;
                            bp.add_k = c3.add_k; bp.add_sh = c3.add_sh; bp.add_lo = c3.add_lo;
                            bp.tie_free = bp.tie_free && c3.tie_free && c3.add_tie_free;
                        }
                        HIP_TRY(launch_bottleneck(bp, m->stream));
                        break;
                    }
                    ConvParams c = d.conv;
                    c.in = (const int8_t *)(ws + pl.toff[d.a]);
                    c.out = (int8_t *)(ws + pl.toff[d.out]);
                    c.res = c.fuse_add == 1 ? (const int8_t *)(ws + pl.toff[d.b]) : nullptr;
                    c.in2 = c.fuse_add == 2 ? (const int8_t *)(ws + pl.toff[d.b]) : nullptr;
                    c.npix = (int32_t)(cnt * c.Ho * c.Wo);
                    c.force_tile = m->conv_tile;
                    HIP_TRY(launch_conv(c, m->stream));
                    break; }
                case OP_ADD: {
                    AddParams a = d.add;
                    const TensorDesc &t = pm.tensors[d.out];
                    a.a = (const int8_t *)(ws + pl.toff[d.a]);
                    a.b = (const int8_t *)(ws + pl.toff[d.b]);
                    a.out = (int8_t *)(ws + pl.toff[d.out]);
                    a.n16 = (int64_t)cnt * t.H * t.W * t.Cp / 16;
                    HIP_TRY(launch_add(a, m->stream));
                    break; }
                case OP_MAXPOOL: {
                    PoolParams p = d.pool;
                    p.in = (const int8_t *)(ws + pl.toff[d.a]);
                    p.out = (int8_t *)(ws + pl.toff[d.out]);
                    p.B = (int32_t)cnt;
                    HIP_TRY(launch_maxpool(p, m->stream));
                    break; }
                case OP_GAP: {
                    GapParams g = d.gap;
                    g.in = (const int8_t *)(ws + pl.toff[d.a]);
                    g.out = (int8_t *)(ws + pl.toff[d.out]);
                    g.B = (int32_t)cnt;
                    HIP_TRY(launch_gap(g, m->stream));
                    break; }
                case OP_FC: {
                    FcParams f = d.fc;
                    f.in = (const int8_t *)(ws + pl.toff[d.a]);
                    f.B = (int32_t)cnt;
                    f.logits = logits_host ? (int32_t *)(ws + pl.logits_off) : nullptr;
                    f.argmax = argmax_host ? (int32_t *)(ws + pl.argmax_off) : nullptr;
                    f.counts = dcounts;
                    if (bc) { f.n_per_item = bc->n_per_item; f.slot_begin = done; }
                    HIP_TRY(launch_fc(f, m->stream));
                    break; }
                }
                if (stop_tensor > 0 && d.out == stop_tensor) break;
            }
        }
        if (timed) {
            if ((prc = mark(-1)) != ISR_OK) return prc;
            HIP_TRY(hipStreamSynchronize(m->stream));
            for (size_t i = 0; i + 1 < ev; ++i) {
                float ms = 0.f;
                HIP_TRY(hipEventElapsedTime(&ms, m->events[i], m->events[i + 1]));
                isr_kernel_stat &st = m->stats[ev_class[i]];
                st.launches += 1;
                st.total_ms += ms;
                st.alg_ops += ev_work[i].first;
                st.alg_bytes += ev_work[i].second;
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
    rc = build_device_ops(m, arena);
    if (rc != ISR_OK) { delete m; return rc; }
    auto cleanup = [&](int code) { isr_free_model(m); return code; };
    hipError_t e = hipMalloc((void **)&m->dconst, arena.host.size());
    if (e == hipSuccess) e = hipMemcpy(m->dconst, arena.host.data(), arena.host.size(), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMalloc((void **)&m->dtables, sizeof(DeviceNoiseTable) * TABLE_SLOTS);
    if (e == hipSuccess) e = hipHostMalloc((void **)&m->htables, sizeof(DeviceNoiseTable) * TABLE_SLOTS, hipHostMallocDefault);
    if (e == hipSuccess) e = hipMalloc((void **)&m->dcounts, sizeof(uint32_t) * 2 * m->pm.classes);
    if (e == hipSuccess) e = hipHostMalloc((void **)&m->hcounts, sizeof(uint32_t) * 2 * m->pm.classes, hipHostMallocDefault);
    if (e != hipSuccess) { g_last_hip_error = (int)e; return cleanup(ISR_ERR_DEVICE); }
    for (DevOp &d : m->ops) {
        if (d.type == OP_CONV) {
            rebase(d.conv.w, m->dconst); rebase(d.conv.bias, m->dconst); rebase(d.conv.m0x2, m->dconst);
            rebase(d.conv.rnd_lo, m->dconst); rebase(d.conv.rnd_hi, m->dconst); rebase(d.conv.shift, m->dconst);
            rebase(d.conv.ktab, m->dconst); rebase(d.conv.ktoff, m->dconst); rebase(d.conv.zpad, m->dconst);
            rebase(d.conv.m0s, m->dconst); rebase(d.conv.chi, m->dconst); rebase(d.conv.shm1, m->dconst);
        } else if (d.type == OP_FC) {
            rebase(d.fc.w, m->dconst); rebase(d.fc.bias, m->dconst);
        }
    }
    m->plan[0].ops = m->ops;
    fuse_adds(m->pm, m->ops, m->plan[1].ops);
    fuse_stem_pool(m->pm, m->plan[1].ops);
    if (!m->plan[1].ops.empty()) {
        DevOp &f = m->plan[1].ops[0];
        const ConvParams &c = f.conv;
        if (f.type == OP_CONV && c.c4 && !c.fuse_add && !f.stem_pool && c.Kp == 64 &&
            stem16_supported(c.k, c.stride, c.pad, c.Cout_p, c.H, c.W, c.fast_requant))
            f.stem16 = 1;
    }
    fuse_basic_blocks(m->pm, m->plan[1].ops);
    chain_basic_blocks(m->pm, m->plan[1].ops);
    fuse_trans_blocks(m->pm, m->plan[1].ops);
    fuse_bottlenecks(m->pm, m->plan[1].ops);
    {   // descriptors of the identity-block chains, in device memory
        std::vector<BlockDesc> descs;
        for (DevOp &d : m->plan[1].ops) {
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
    m->use_fused = enable ? 1 : 0;
    return ISR_OK;
}

int isr_discrete_quantile(uint32_t sigma, double p_lower, int32_t *t_out, uint64_t *radius_sq_out) {
    if (sigma < 1 || sigma > 1024 || !(p_lower >= 0.0 && p_lower <= 1.0)) return ISR_ERR_ARG;
    std::vector<uint64_t> T;
    uint32_t R = 0;
    if (!build_noise_table(sigma, T, R)) return ISR_ERR_ARG;
    // floor(2^64 p): exact for a double below 1 (53 significant bits, scaled by a power of two)
    const uint64_t u = p_lower >= 1.0 ? ~0ull : (uint64_t)std::ldexp(p_lower, 64);
    // thresholds ascend: the number of entries <= u by binary search
    const int64_t below = std::upper_bound(T.begin(), T.end(), u) - T.begin();
    const int64_t t = -(int64_t)R - 1 + below;
    if (t_out) *t_out = (int32_t)t;
    if (radius_sq_out) *radius_sq_out = t > 0 ? (uint64_t)(t * t) : 0;
    return ISR_OK;
}

int isr_noise_bank(uint32_t sigma, uint64_t seed, uint32_t bank_id, uint32_t first, uint32_t count, uint32_t d,
                   int16_t *out_device, void *hip_stream) {
    if (sigma < 1 || sigma > 1024 || !out_device || d == 0 || (d & 3) != 0) return ISR_ERR_ARG;
    if ((uint64_t)first + count > (1ull << 32)) return ISR_ERR_ARG;
    if (count == 0) return ISR_OK;
    std::vector<uint64_t> T;
    uint32_t R = 0;
    if (!build_noise_table(sigma, T, R)) return ISR_ERR_ARG;
    const size_t n = T.size();
    // device form: high words, low words, guide table (as 32-bit words so that one upload carries all)
    const size_t guide_words = (NOISE_GUIDE_SIZE + 2) / 2;
    std::vector<uint32_t> host(2 * n + guide_words, 0);
    for (size_t j = 0; j < n; ++j) { host[j] = (uint32_t)(T[j] >> 32); host[n + j] = (uint32_t)T[j]; }
    uint16_t *guide = (uint16_t *)(host.data() + 2 * n);
    size_t j = 0;
    for (uint32_t b = 0; b <= NOISE_GUIDE_SIZE; ++b) {
        const uint64_t start = (uint64_t)b << (32 - NOISE_GUIDE_BITS);
        while (j < n && (uint64_t)host[j] < start) ++j;
        guide[b] = (uint16_t)j;
    }
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
    if (!m || tile < 0 || tile > 4) return ISR_ERR_ARG;
    m->conv_tile = tile;
    return ISR_OK;
}

int isr_profile(isr_model *m, uint32_t every_chunks) {
    if (!m) return ISR_ERR_ARG;
    m->profile_every = every_chunks;
    m->chunk_counter = 0;
    for (int i = 0; i < KC_COUNT; ++i) {
        m->stats[i] = isr_kernel_stat{};
        std::strncpy(m->stats[i].name, KC_NAMES[i], sizeof(m->stats[i].name) - 1);
    }
    return ISR_OK;
}

int isr_profile_read(const isr_model *m, isr_kernel_stat *out_host, uint32_t cap, uint32_t *n_out) {
    if (!m || !n_out || (cap && !out_host)) return ISR_ERR_ARG;
    uint32_t n = 0;
    for (int i = 0; i < KC_COUNT; ++i)
        if (m->stats[i].launches) {
            if (n < cap) out_host[n] = m->stats[i];
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
    for (int i = 0; i < 2; ++i) {
        Plan pl;
        pl.ops = m->plan[i].ops;
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
    for (int i = 0; i < 2; ++i) plan_workspace(m->pm, chunk_samples, m->plan[i]);
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
    const Plan &pl = (m->use_fused && m->plan[1].has[tensor_id]) ? m->plan[1] : m->plan[0];
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
