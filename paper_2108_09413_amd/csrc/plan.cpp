// The planner: see plan.h.
#include "plan.h"

#include <algorithm>
#include <climits>
#include <cstdlib>
#include <cstring>

namespace isr {

namespace {

size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// MFMA 32x32 accumulator row r of lane half h, register i is 8*(i/4) + 4*h + i%4;
// weights of output channel 16*h + i go to that row so that a lane ends up
// holding 16 consecutive channels.
int mfma32_row_of_channel(int oc_local) {
    int h = oc_local >> 4, a = (oc_local & 15) >> 2, b = oc_local & 3;
    return 8 * a + 4 * h + b;
}

}  // namespace

// Sub-chunk schedule of a plan for chunks of B copies.  ISR_SEGMENTS="end:sub,end:sub,..." (op index
// after the segment's last op : copies per sub-chunk) overrides the built-in choice; for tuning.
void plan_segments(const ParsedModel &pm, uint32_t B, Plan &pl) {
    pl.segments.clear();
    (void)pm; (void)B;
    if (const char *env = std::getenv("ISR_SEGMENTS")) {
        const char *p = env;
        while (*p) {
            char *q = nullptr;
            const long end = std::strtol(p, &q, 10);
            if (q == p || *q != ':') break;
            p = q + 1;
            const long sub = std::strtol(p, &q, 10);
            if (q == p) break;
            p = *q == ',' ? q + 1 : q;
            if (end > 0 && sub > 0 && (pl.segments.empty() || (size_t)end > pl.segments.back().end))
                pl.segments.push_back({(size_t)end, (uint32_t)sub});
        }
    }
}

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
    // A segment runs its ops sub-chunk by sub-chunk, so every tensor it touches is live for the
    // whole segment: outputs are placed when the segment starts, inputs released when it ends.
    // An op outside the segments is a segment of its own.
    size_t seg = 0;
    for (int i = 0; i < (int)pl.ops.size();) {
        while (seg < pl.segments.size() && pl.segments[seg].end <= (size_t)i) ++seg;
        const int end = seg < pl.segments.size() ? (int)std::min(pl.segments[seg].end, pl.ops.size()) : i + 1;
        for (int j = i; j < end; ++j) {
            const DevOp &o = pl.ops[j];
            if (o.type != OP_FC) { pl.toff[o.out] = alloc(tbytes(o.out)); pl.has[o.out] = 1; }
            if (o.out2 >= 0) { pl.toff[o.out2] = alloc(tbytes(o.out2)); pl.has[o.out2] = 1; }
        }
        for (int j = i; j < end; ++j) {
            const DevOp &o = pl.ops[j];
            for (int t : {o.a, o.b})
                if (t >= 0 && last_use[t] == j && !(t == o.b && o.a == o.b)) release(pl.toff[t], tbytes(t));
        }
        i = end;
    }
    pl.logits_off = round_up(top, 256);
    pl.argmax_off = pl.logits_off + round_up((size_t)B * pm.classes * 4, 256);
    pl.bytes = pl.argmax_off + round_up((size_t)B * 4, 256);
}

namespace {

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
                        merged.conv.wfrag2 = rc.wfrag;
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

// Folds conv1x1 (-> 64 or 128 channels) -> conv3x3 of a bottleneck block into one kernel, and with
// them the closing conv1x1 + residual add when the residual is the block input (with 128 middle
// channels only whole blocks are folded).
// Runs on the list in which the adds are already folded into their convolutions.
void fuse_bottlenecks(const ParsedModel &pm, std::vector<DevOp> &ops, bool wide) {
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
        const int cm = c1.Cout_p;
        if (cm != 64 && !(cm == 128 && wide)) continue;
        if (c1.k != 1 || c1.stride != 1 || c1.pad != 0 || c1.Kp != c1.Cin_p) continue;
        if (c2.k != 3 || c2.stride != 1 || c2.pad != 1 || c2.Cin_p != cm || c2.Cout_p != cm || c2.Kp != 9 * cm) continue;
        if (b.a != a.out || uses[a.out] != 1) continue;
        // the closing 1x1 convolution + residual add with the block input, if the list goes on with it
        const DevOp *c = i + 2 < ops.size() ? &ops[i + 2] : nullptr;
        bool tail = false;
        if (c) {
            const ConvParams &c3 = c->conv;
            tail = plain(*c) && c3.fuse_add == 1 && c3.k == 1 && c3.stride == 1 && c3.pad == 0 && c3.Cin_p == cm && c3.Kp == cm &&
                   c->a == b.out && c->b == a.a && uses[b.out] == 1;
        }
        if (cm == 64) {
            if (!bottleneck_supported(c1.Cin_p, 64, 0, 0)) continue;
            tail = tail && bottleneck_supported(c1.Cin_p, 64, c->conv.Cout_p, 1);
        } else {
            // 128 middle channels: the whole block or nothing
            if (!tail || !bottleneck128_supported(c1.Cin_p, 128, c->conv.Cout_p)) continue;
        }
        const DevOp cc = tail ? *c : DevOp{};
        a.bneck = 1;
        a.conv2 = c2;
        a.ops_per_sample += b.ops_per_sample;
        a.bytes_per_sample = (double)pm.tensors[a.a].C * c1.H * c1.W + (double)pm.tensors[b.out].C * c1.H * c1.W;
        a.out = b.out;
        if (tail) {
            a.bneck = cm == 64 ? 2 : 3;
            a.conv3 = cc.conv;
            a.ops_per_sample += cc.ops_per_sample;
            a.bytes_per_sample = 2.0 * pm.tensors[a.a].C * c1.H * c1.W;
            a.out = cc.out;
        }
        ops.erase(ops.begin() + i + 1, ops.begin() + i + (tail ? 3 : 2));
        // First block of a stage: the head is followed by the closing 1x1 convolution whose residual is a
        // projection 1x1 convolution of the block input (already folded into one dual-convolution op): when the
        // block input has 64 stored channels the whole block runs in the bottleneck kernel.
        if (a.bneck == 1 && i + 1 < ops.size()) {
            const DevOp &m = ops[i + 1];
            const ConvParams &c3 = m.conv;
            if (m.type == OP_CONV && !m.stem_pool && !m.stem16 && !m.block && !m.trans && !m.bneck && c3.fuse_add == 2 &&
                c3.k == 1 && c3.stride == 1 && c3.pad == 0 && c3.Cin_p == 64 && c3.Kp == 64 && c3.Cin2_p == 64 && c3.fast_requant &&
                ((m.a == a.out && m.b == a.a) || (m.a == a.a && m.b == a.out)) && uses[a.out] == 1 && c1.Cin_p == 64 &&
                bottleneck_supported(64, 64, c3.Cout_p, 2)) {
                a.bneck = 4;
                a.proj_is_main = m.a == a.a;   // which of the dual op's two convolutions reads the block input
                a.conv3 = c3;
                a.ops_per_sample += m.ops_per_sample;
                a.bytes_per_sample = (double)pm.tensors[a.a].C * c1.H * c1.W + (double)pm.tensors[m.out].C * c1.H * c1.W;
                a.out = m.out;
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

}  // namespace

size_t ConstArena::put(const void *src, size_t n) {
    size_t off = round_up(host.size(), 256);
    host.resize(off + round_up(n, 16), 0);
    if (src) std::memcpy(host.data() + off, src, n);
    return off;
}

// Builds device descriptors; pointers into the constant arena are stored as
// offsets first and rebased after the upload.
int build_device_ops(const ParsedModel &pm, std::vector<DevOp> &ops, ConstArena &arena) {
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
            // fragment-major copies for the kernel that runs an expanding 1x1 + add and the next reducing 1x1 together
            // (expand_reduce.hip): one 1 KB block per MFMA operand fragment, 64 lanes x 16 bytes in lane order
            c.wfrag = (const int8_t *)~(uintptr_t)0;
            if (!c4 && k == 1 && o.pad == 0 && fast && perm && Kp == cin_p &&
                (((cin_p == 128 || cin_p == 256) && cout_p == 512) || (cin_p == 256 && cout_p == 1024))) {
                // 32x32x32 fragments [32-row block][K sub-step of 32]: lane l = row l & 31 (stored MFMA row order), K bytes 16 (l >> 5) ..
                std::vector<int8_t> f((size_t)cout_p * Kp);
                for (int blk = 0; blk < cout_p / 32; ++blk)
                    for (int ks = 0; ks < Kp / 32; ++ks)
                        for (int l = 0; l < 64; ++l)
                            std::memcpy(&f[(((size_t)blk * (Kp / 32) + ks) * 64 + l) * 16],
                                        &w[(size_t)(32 * blk + (l & 31)) * Kp + ks * 32 + 16 * (l >> 5)], 16);
                c.wfrag = (const int8_t *)arena.put(f.data(), f.size());
            } else if (flat && fast && perm && Kp == cin_p && ((cin_p == 512 && (cout_p == 128 || cout_p == 256)) || (cin_p == 1024 && cout_p == 256))) {
                // 16x16x64 fragments [16-channel block][K step of 64]: lane l = channel l & 15 of the block, K bytes 16 (l >> 4) ..
                std::vector<int8_t> f((size_t)cout_p * Kp);
                for (int mb = 0; mb < cout_p / 16; ++mb)
                    for (int ks = 0; ks < Kp / 64; ++ks)
                        for (int l = 0; l < 64; ++l) {
                            const int oc = 16 * mb + (l & 15), row = (oc & ~31) + mfma32_row_of_channel(oc & 31);
                            std::memcpy(&f[(((size_t)mb * (Kp / 64) + ks) * 64 + l) * 16], &w[(size_t)row * Kp + ks * 64 + 16 * (l >> 4)], 16);
                        }
                c.wfrag = (const int8_t *)arena.put(f.data(), f.size());
            }
            c.ktab = flat ? (const uint32_t *)~(uintptr_t)0 : (const uint32_t *)arena.put(ktab.data(), ktab.size() * 4);
            c.ktoff = flat ? (const int32_t *)~(uintptr_t)0 : (const int32_t *)arena.put(ktoff.data(), ktoff.size() * 4);
            c.H = ti.H; c.W = ti.W; c.Cin_p = cin_p; c.Ho = to.H; c.Wo = to.W; c.Cout_p = cout_p;
            c.k = k; c.stride = o.stride; c.pad = o.pad; c.Kp = Kp; c.Mp = Mp; c.kb = kb;
            c.zp_in = ti.zp; c.zp_out = to.zp; c.relu = o.relu; c.c4 = c4 ? 1 : 0;
            d.ops_per_sample = 2.0 * to.C * to.H * to.W * ti.C * k * k;
            d.bytes_per_sample = (double)ti.C * ti.H * ti.W + (double)to.C * to.H * to.W;
            break; }
        case OP_ADD: {
            AddParams &a = d.add;
            a.za = pm.tensors[o.a].zp; a.zb = pm.tensors[o.b].zp; a.zo = pm.tensors[o.out].zp;
            a.Ma = o.Ma; a.Mb = o.Mb; a.sh = o.sh; a.relu = o.relu;
            d.bytes_per_sample = 3.0 * pm.tensors[o.out].C * pm.tensors[o.out].H * pm.tensors[o.out].W;
            break; }
        case OP_MAXPOOL: {
            const TensorDesc &ti = pm.tensors[o.a], &to = pm.tensors[o.out];
            PoolParams &p = d.pool;
            p.H = ti.H; p.W = ti.W; p.Cp = ti.Cp; p.Ho = to.H; p.Wo = to.W; p.k = o.k; p.stride = o.stride; p.pad = o.pad;
            d.bytes_per_sample = (double)ti.C * ti.H * ti.W + (double)to.C * to.H * to.W;
            break; }
        case OP_GAP: {
            const TensorDesc &ti = pm.tensors[o.a], &to = pm.tensors[o.out];
            GapParams &g = d.gap;
            g.HW = ti.H * ti.W; g.Cp = ti.Cp; g.zp_in = ti.zp; g.zp_out = to.zp; g.M0 = o.Ma; g.sh = o.sh;
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
            d.ops_per_sample = 2.0 * classes * ti.C * hw;
            d.bytes_per_sample = (double)ti.C * hw;
            break; }
        }
        ops.push_back(d);
    }
    return ISR_OK;
}


namespace {

template <typename T>
void rebase(const T *&p, const uint8_t *base) {
    if ((uintptr_t)p == ~(uintptr_t)0) { p = nullptr; return; }
    p = (const T *)(base + (uintptr_t)p);
}

}  // namespace

void rebase_device_ops(std::vector<DevOp> &ops, const uint8_t *base) {
    for (DevOp &d : ops) {
        if (d.type == OP_CONV) {
            rebase(d.conv.w, base); rebase(d.conv.bias, base); rebase(d.conv.m0x2, base);
            rebase(d.conv.rnd_lo, base); rebase(d.conv.rnd_hi, base); rebase(d.conv.shift, base);
            rebase(d.conv.ktab, base); rebase(d.conv.ktoff, base); rebase(d.conv.zpad, base);
            rebase(d.conv.m0s, base); rebase(d.conv.chi, base); rebase(d.conv.shm1, base); rebase(d.conv.wfrag, base);
        } else if (d.type == OP_FC) {
            rebase(d.fc.w, base); rebase(d.fc.bias, base);
        }
    }
}

namespace {

// Folds an expanding 1x1 convolution + residual add (the end of a bottleneck block) and the reducing 1x1
// convolution that reads the sum (the start of the next block) into one kernel: the sum is still written (the
// next block's add reads it), but not read back by a second kernel.
void fuse_expand_reduce(const ParsedModel &pm, std::vector<DevOp> &ops) {
    auto plain = [](const DevOp &d) {
        return d.type == OP_CONV && !d.stem_pool && !d.stem16 && !d.block && !d.trans && !d.bneck && !d.xr;
    };
    for (size_t i = 0; i + 1 < ops.size(); ++i) {
        DevOp &a = ops[i];
        const DevOp &b = ops[i + 1];
        if (!plain(a) || !plain(b) || b.a != a.out || !expand_reduce_supported(a.conv, b.conv)) continue;
        const TensorDesc &ty = pm.tensors[a.out];
        a.xr = 1;
        a.conv2 = b.conv;
        a.out2 = b.out;
        a.ops_per_sample += b.ops_per_sample;
        a.bytes_per_sample += b.bytes_per_sample - (double)ty.C * ty.H * ty.W;   // the sum is not read back
        ops.erase(ops.begin() + i + 1);
    }
}

}  // namespace

void build_fused_plan(const ParsedModel &pm, const std::vector<DevOp> &plain, std::vector<DevOp> &fused, bool wide_bottlenecks) {
    fuse_adds(pm, plain, fused);
    fuse_stem_pool(pm, fused);
    if (!fused.empty()) {
        DevOp &f = fused[0];
        const ConvParams &c = f.conv;
        if (f.type == OP_CONV && c.c4 && !c.fuse_add && !f.stem_pool && c.Kp == 64 &&
            stem16_supported(c.k, c.stride, c.pad, c.Cout_p, c.H, c.W, c.fast_requant))
            f.stem16 = 1;
    }
    // the fused first layer draws its own noisy input when it is the only reader of the input tensor
    if (!fused.empty() && fused[0].stem_pool && fused[0].a == 0) {
        int readers = 0;
        for (const DevOp &d : fused) readers += (d.a == 0) + (d.b == 0);
        if (readers == 1) fused[0].noise_fused = 1;
    }
    fuse_basic_blocks(pm, fused);
    chain_basic_blocks(pm, fused);
    fuse_trans_blocks(pm, fused);
    fuse_bottlenecks(pm, fused, wide_bottlenecks);
    fuse_expand_reduce(pm, fused);
}

}  // namespace isr
