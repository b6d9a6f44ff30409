// ISRM model blob parser and validator (host only).
#include <cstring>

#include "isr_internal.h"

namespace isr {

namespace {

struct Reader {
    const uint8_t *p, *end;
    bool ok = true;
    int32_t i32() {
        if (end - p < 4) { ok = false; return 0; }
        int32_t v;
        std::memcpy(&v, p, 4);
        p += 4;
        return v;
    }
    const uint8_t *bytes(size_t n) {
        if ((size_t)(end - p) < n) { ok = false; return nullptr; }
        const uint8_t *q = p;
        p += n;
        return q;
    }
};

bool shape_ok(const TensorDesc &t) {
    return t.C >= 1 && t.C <= 65536 && t.H >= 1 && t.H <= 4096 && t.W >= 1 && t.W <= 4096 &&
           t.zp >= -128 && t.zp <= 127;
}

int out_dim(int in, int k, int stride, int pad) { return (in + 2 * pad - k) / stride + 1; }

}  // namespace

int parse_model(const void *blob, size_t bytes, ParsedModel &m, std::string &why) {
    auto fail = [&](int code, const char *msg) { why = msg; return code; };
    if (!blob || bytes < 32) return fail(ISR_ERR_FORMAT, "blob shorter than the header");
    Reader r{(const uint8_t *)blob, (const uint8_t *)blob + bytes};
    if (r.i32() != 0x4D525349) return fail(ISR_ERR_FORMAT, "bad magic");
    if (r.i32() != 1) return fail(ISR_ERR_FORMAT, "unknown version");
    m.C = r.i32(); m.H = r.i32(); m.W = r.i32(); m.classes = r.i32();
    int32_t nt = r.i32(), nops = r.i32();
    if (nt < 2 || nt > 100000 || nops < 1 || nops > 100000) return fail(ISR_ERR_FORMAT, "tensor/op count out of range");
    if (m.classes < 1) return fail(ISR_ERR_FORMAT, "no classes");
    m.tensors.resize(nt);
    for (auto &t : m.tensors) {
        t.C = r.i32(); t.H = r.i32(); t.W = r.i32(); t.zp = r.i32();
        t.Cp = 0;
        if (!r.ok) return fail(ISR_ERR_FORMAT, "truncated tensor table");
        if (!shape_ok(t)) return fail(ISR_ERR_FORMAT, "tensor shape or zero-point out of range");
    }
    const TensorDesc &in = m.tensors[0];
    if (in.C != m.C || in.H != m.H || in.W != m.W || in.zp != 0)
        return fail(ISR_ERR_FORMAT, "tensor 0 must be the input with zero-point 0");
    std::vector<char> defined(nt, 0);
    defined[0] = 1;
    auto tensor_ok = [&](int id, bool must_exist) {
        return id >= 0 && id < nt && (must_exist ? defined[id] : !defined[id]);
    };
    m.ops.resize(nops);
    bool have_logits = false;
    for (int oi = 0; oi < nops; ++oi) {
        HostOp &o = m.ops[oi];
        int32_t type = r.i32(), len = r.i32();
        if (!r.ok || len < 0 || (len & 3)) return fail(ISR_ERR_FORMAT, "bad op header");
        const uint8_t *pay = r.bytes((size_t)len);
        if (!pay) return fail(ISR_ERR_FORMAT, "truncated op payload");
        if (have_logits) return fail(ISR_ERR_FORMAT, "ops after the FC layer");
        Reader q{pay, pay + len};
        o.type = (OpType)type;
        switch (type) {
        case OP_CONV: {
            o.a = q.i32(); o.out = q.i32(); o.k = q.i32(); o.stride = q.i32(); o.pad = q.i32(); o.relu = q.i32();
            if (!q.ok || !tensor_ok(o.a, true) || !tensor_ok(o.out, false)) return fail(ISR_ERR_FORMAT, "conv: bad tensor ids");
            const TensorDesc &ti = m.tensors[o.a], &to = m.tensors[o.out];
            if (o.k < 1 || o.k > 15 || o.stride < 1 || o.stride > 8 || o.pad < 0 || o.pad >= o.k || (o.relu & ~1))
                return fail(ISR_ERR_FORMAT, "conv: bad geometry");
            if (ti.H + 2 * o.pad < o.k || ti.W + 2 * o.pad < o.k ||
                to.H != out_dim(ti.H, o.k, o.stride, o.pad) || to.W != out_dim(ti.W, o.k, o.stride, o.pad))
                return fail(ISR_ERR_FORMAT, "conv: output shape mismatch");
            size_t nw = (size_t)to.C * ti.C * o.k * o.k;
            const uint8_t *w = q.bytes((nw + 3) & ~(size_t)3);
            const uint8_t *bias = q.bytes((size_t)to.C * 4), *m0 = q.bytes((size_t)to.C * 4), *sh = q.bytes((size_t)to.C * 4);
            if (!q.ok || q.p != q.end) return fail(ISR_ERR_FORMAT, "conv: payload size mismatch");
            o.w.assign((const int8_t *)w, (const int8_t *)w + nw);
            o.bias.resize(to.C); o.M0.resize(to.C); o.shift.resize(to.C);
            std::memcpy(o.bias.data(), bias, (size_t)to.C * 4);
            std::memcpy(o.M0.data(), m0, (size_t)to.C * 4);
            std::memcpy(o.shift.data(), sh, (size_t)to.C * 4);
            int64_t maxbias = 0;
            for (int c = 0; c < to.C; ++c) {
                if (o.M0[c] < (1 << 30)) return fail(ISR_ERR_FORMAT, "conv: M0 outside [2^30, 2^31)");
                if (o.shift[c] < 0 || o.shift[c] > 31) return fail(ISR_ERR_FORMAT, "conv: shift outside [0, 31]");
                int64_t ab = o.bias[c] < 0 ? -(int64_t)o.bias[c] : o.bias[c];
                if (ab > maxbias) maxbias = ab;
            }
            for (int8_t v : o.w) if (v == -128) return fail(ISR_ERR_FORMAT, "conv: weight -128 not allowed");
            if ((int64_t)ti.C * o.k * o.k * 255 * 127 + maxbias >= (1ll << 31))
                return fail(ISR_ERR_FORMAT, "conv: accumulator may overflow 32 bits");
            if (o.relu && to.zp > 127) return fail(ISR_ERR_FORMAT, "conv: bad output zero-point");
            break; }
        case OP_ADD: {
            o.a = q.i32(); o.b = q.i32(); o.out = q.i32(); o.Ma = q.i32(); o.Mb = q.i32(); o.sh = q.i32(); o.relu = q.i32();
            if (!q.ok || q.p != q.end) return fail(ISR_ERR_FORMAT, "add: payload size mismatch");
            if (!tensor_ok(o.a, true) || !tensor_ok(o.b, true) || !tensor_ok(o.out, false)) return fail(ISR_ERR_FORMAT, "add: bad tensor ids");
            const TensorDesc &ta = m.tensors[o.a], &tb = m.tensors[o.b], &to = m.tensors[o.out];
            if (ta.C != tb.C || ta.H != tb.H || ta.W != tb.W || ta.C != to.C || ta.H != to.H || ta.W != to.W)
                return fail(ISR_ERR_FORMAT, "add: shape mismatch");
            if (o.sh < 0 || o.sh > 40 || (o.relu & ~1)) return fail(ISR_ERR_FORMAT, "add: bad shift");
            break; }
        case OP_MAXPOOL: {
            o.a = q.i32(); o.out = q.i32(); o.k = q.i32(); o.stride = q.i32(); o.pad = q.i32();
            if (!q.ok || q.p != q.end) return fail(ISR_ERR_FORMAT, "maxpool: payload size mismatch");
            if (!tensor_ok(o.a, true) || !tensor_ok(o.out, false)) return fail(ISR_ERR_FORMAT, "maxpool: bad tensor ids");
            const TensorDesc &ti = m.tensors[o.a], &to = m.tensors[o.out];
            if (o.k < 1 || o.k > 15 || o.stride < 1 || o.stride > 8 || o.pad < 0 || o.pad >= o.k)
                return fail(ISR_ERR_FORMAT, "maxpool: bad geometry");
            if (to.C != ti.C || to.zp != ti.zp || ti.H + 2 * o.pad < o.k || ti.W + 2 * o.pad < o.k ||
                to.H != out_dim(ti.H, o.k, o.stride, o.pad) || to.W != out_dim(ti.W, o.k, o.stride, o.pad))
                return fail(ISR_ERR_FORMAT, "maxpool: output shape mismatch");
            break; }
        case OP_GAP: {
            o.a = q.i32(); o.out = q.i32(); o.Ma = q.i32(); o.sh = q.i32();
            if (!q.ok || q.p != q.end) return fail(ISR_ERR_FORMAT, "gap: payload size mismatch");
            if (!tensor_ok(o.a, true) || !tensor_ok(o.out, false)) return fail(ISR_ERR_FORMAT, "gap: bad tensor ids");
            const TensorDesc &ti = m.tensors[o.a], &to = m.tensors[o.out];
            if (to.C != ti.C || to.H != 1 || to.W != 1) return fail(ISR_ERR_FORMAT, "gap: output shape mismatch");
            if (o.Ma < (1 << 30) || o.sh < 0 || o.sh > 31) return fail(ISR_ERR_FORMAT, "gap: bad multiplier");
            if ((int64_t)ti.H * ti.W * 255 >= (1ll << 31)) return fail(ISR_ERR_FORMAT, "gap: sum may overflow");
            break; }
        case OP_FC: {
            o.a = q.i32(); o.out = q.i32();
            if (!q.ok || !tensor_ok(o.a, true) || !tensor_ok(o.out, false)) return fail(ISR_ERR_FORMAT, "fc: bad tensor ids");
            const TensorDesc &ti = m.tensors[o.a], &to = m.tensors[o.out];
            if (to.C != m.classes || to.H != 1 || to.W != 1) return fail(ISR_ERR_FORMAT, "fc: output must be the logits");
            size_t cin = (size_t)ti.C * ti.H * ti.W, nw = cin * to.C;
            const uint8_t *w = q.bytes((nw + 3) & ~(size_t)3), *bias = q.bytes((size_t)to.C * 4);
            if (!q.ok || q.p != q.end) return fail(ISR_ERR_FORMAT, "fc: payload size mismatch");
            o.w.assign((const int8_t *)w, (const int8_t *)w + nw);
            o.bias.resize(to.C);
            std::memcpy(o.bias.data(), bias, (size_t)to.C * 4);
            int64_t maxbias = 0;
            for (int32_t b : o.bias) { int64_t ab = b < 0 ? -(int64_t)b : b; if (ab > maxbias) maxbias = ab; }
            for (int8_t v : o.w) if (v == -128) return fail(ISR_ERR_FORMAT, "fc: weight -128 not allowed");
            if ((int64_t)cin * 255 * 127 + maxbias >= (1ll << 31)) return fail(ISR_ERR_FORMAT, "fc: accumulator may overflow");
            have_logits = true;
            break; }
        default: return fail(ISR_ERR_FORMAT, "unknown op type");
        }
        defined[o.out] = 1;
    }
    if (r.p != r.end) return fail(ISR_ERR_FORMAT, "trailing bytes");
    if (!have_logits || m.ops.back().type != OP_FC) return fail(ISR_ERR_FORMAT, "the last op must be the FC layer");
    // what the kernels cover
    if (m.C > 3) return fail(ISR_ERR_UNSUPPORTED, "more than 3 input channels");
    if (m.W % 4 != 0) return fail(ISR_ERR_UNSUPPORTED, "input width must be a multiple of 4");
    if (m.classes > 1024) return fail(ISR_ERR_UNSUPPORTED, "more than 1024 classes");
    for (auto &t : m.tensors) t.Cp = (t.C + 15) & ~15;
    m.tensors[0].Cp = 4;
    for (const HostOp &o : m.ops) {
        if (o.type == OP_CONV) {
            const TensorDesc &ti = m.tensors[o.a];
            if (o.a == 0 && o.k > 8) return fail(ISR_ERR_UNSUPPORTED, "first-layer kernel wider than 8");
            int64_t kp = o.a == 0 ? (int64_t)o.k * ((o.k + 3) & ~3) * 4 : (int64_t)o.k * o.k * ti.Cp;
            if (kp > 8192) return fail(ISR_ERR_UNSUPPORTED, "convolution depth above 8192");
        } else if (o.a == 0 || o.b == 0) {
            return fail(ISR_ERR_UNSUPPORTED, "the input tensor must feed a convolution");
        }
    }
    return ISR_OK;
}

}  // namespace isr

extern "C" int isr_validate_model(const void *blob_host, size_t bytes) {
    isr::ParsedModel m;
    std::string why;
    return isr::parse_model(blob_host, bytes, m, why);
}
