// Host-only robustness check, built with -fsanitize=address,undefined by tests/test_host_sanitizers.py:
// the library's blob parser, planner, noise-table builder and statistics, and the oracle's parser and
// forward pass, on valid blobs and on systematically damaged ones (every truncation point of the
// front of the blob, every 32-bit word of it overwritten with edge values).  A damaged blob must
// be rejected with a format / unsupported status (library) or a null handle (oracle), or be accepted
// and then run cleanly -- never crash, never read or write out of bounds.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "isr_internal.h"
#include "plan.h"

extern "C" {
struct omodel;
omodel *isr_oracle_load(const void *blob, size_t bytes);
void isr_oracle_free(omodel *m);
void isr_oracle_info(const omodel *m, int32_t *C, int32_t *H, int32_t *W, int32_t *classes, int32_t *nt);
size_t isr_oracle_tensor_offset(const omodel *m, int32_t id);
int isr_oracle_forward(const omodel *m, const int8_t *a0, int8_t *acts, int32_t *logits);
int isr_oracle_noise_table(uint32_t sigma, uint64_t *T, size_t cap, uint32_t *R);
void isr_oracle_noisy_float(const uint8_t *x, uint32_t npix, float sigma, uint64_t seed, uint32_t image, uint32_t phase,
                            uint32_t sample, float *v);
void isr_oracle_noisy_quant(const uint8_t *x, uint32_t npix, float sigma, uint64_t seed, uint32_t image, uint32_t phase,
                            uint32_t sample, int8_t *a0);
int isr_oracle_forward_float(const omodel *m, const float *v, double *acts, double *logits);
}

// The planner asks the kernel files which shapes their kernels cover; those files are device code
// and are not part of this host build, so the questions are answered here (the same predicates,
// restated) -- what matters for this check is that the fusion passes run over the op list.
namespace isr {
int conv_tile_m(int cout_p) { return cout_p <= 16 ? 16 : (cout_p <= 32 ? 32 : (cout_p <= 64 ? 64 : 128)); }
int conv_k_step(int kreal, int cin_p, int cout_p, int fast) {
    return (fast && cin_p != 0 && cout_p >= 256 && kreal % 128 == 0 && kreal >= 1024) ? 128 : 64;
}
bool stem_pool_supported(int k, int stride, int pad, int cout_p, int H, int W, int fast, int pk, int ps, int pp) {
    return k == 7 && stride == 2 && pad == 3 && cout_p == 64 && fast && pk == 3 && ps == 2 && pp == 1 && W % 4 == 0 && W >= 8 && W <= 224 && H >= 1;
}
bool stem16_supported(int k, int stride, int pad, int cout_p, int H, int W, int fast) {
    return k == 3 && stride == 1 && pad == 1 && cout_p == 16 && fast && W % 16 == 0 && W >= 16 && W <= 64 && H >= 1 && H <= 64;
}
bool basic_block_supported(int c, int s) { return (c == 16 && s == 32) || (c == 32 && s == 16) || (c == 64 && s == 8); }
bool trans_block_supported(int c, int s) { return (c == 32 && s == 16) || (c == 64 && s == 8); }
bool bottleneck_supported(int cin_p, int cmid_p, int cout_p, int tail) {
    if (cin_p % 64 != 0 || cin_p < 64 || cin_p > 1024 || cmid_p != 64) return false;
    return !tail || (cout_p == cin_p && cout_p <= 256);
}
bool expand_reduce_supported(const ConvParams &e, const ConvParams &r) {
    if (e.fuse_add == 1 && e.Cin_p == 256)
        return e.k == 1 && e.stride == 1 && e.pad == 0 && e.Kp == 256 && e.Cout_p == 1024 && e.fast_requant && e.tie_free && !e.c4 && e.wfrag &&
               r.k == 1 && r.stride == 1 && r.pad == 0 && r.Cin_p == 1024 && r.Kp == 1024 && r.Cout_p == 256 && !r.fuse_add && r.fast_requant &&
               r.tie_free && !r.c4 && r.wfrag && e.Ho == r.H && e.Wo == r.W && r.Ho == r.H && r.Wo == r.W;
    bool expand = e.k == 1 && e.pad == 0 && e.Cout_p == 512 && e.fast_requant && e.tie_free && !e.c4 && e.wfrag;
    if (e.fuse_add == 1) expand = expand && e.stride == 1 && e.Cin_p == 128 && e.Kp == 128;
    else if (e.fuse_add == 2 && e.Cin_p == 256)
        expand = expand && (e.stride == 1 || e.stride == 2) && e.Kp == 256 && e.Cin2_p == 128 && e.tie_free2 && e.wfrag2 &&
                 (long)e.H * e.W * 256 < (1l << 31);
    else
        expand = expand && e.fuse_add == 2 && e.stride == 1 && e.Cin_p == 128 && e.Kp == 128 && e.Cin2_p == 256 && e.tie_free2 && e.wfrag2;
    const bool reduce = r.k == 1 && r.stride == 1 && r.pad == 0 && r.Cin_p == 512 && r.Kp == 512 &&
                        (r.Cout_p == 128 || (r.Cout_p == 256 && e.fuse_add == 1)) && !r.fuse_add && r.fast_requant && r.tie_free &&
                        !r.c4 && r.wfrag;
    return expand && reduce && e.Ho == r.H && e.Wo == r.W && r.Ho == r.H && r.Wo == r.W;
}
bool bottleneck128_supported(int cin_p, int cmid_p, int cout_p) {
    return cmid_p == 128 && cin_p % 64 == 0 && cin_p >= 64 && cin_p <= 2048 && cout_p == cin_p && cout_p % 32 == 0;
}
}  // namespace isr

using namespace isr;

static long g_accepted = 0, g_rejected = 0;

// The library side: parse; when accepted, build the descriptors, both fused plans and the workspace layout.
static int library_side(const std::vector<uint8_t> &blob) {
    ParsedModel pm;
    std::string why;
    const int rc = parse_model(blob.data(), blob.size(), pm, why);
    if (rc != ISR_OK && rc != ISR_ERR_FORMAT && rc != ISR_ERR_UNSUPPORTED) {
        std::printf("library parser returned status %d\n", rc);
        return 1;
    }
    if (rc != ISR_OK) { ++g_rejected; return isr_validate_model(blob.data(), blob.size()) == rc ? 0 : 1; }
    ++g_accepted;
    std::vector<DevOp> ops;
    ConstArena arena;
    arena.put(nullptr, 256);
    const int brc = build_device_ops(pm, ops, arena);
    if (brc != ISR_OK) return brc == ISR_ERR_UNSUPPORTED ? 0 : 1;
    rebase_device_ops(ops, arena.host.data());
    for (int wide = 0; wide < 2; ++wide) {
        Plan pl;
        build_fused_plan(pm, ops, pl.ops, wide != 0);
        for (uint32_t B : {1u, 7u}) {
            plan_segments(pm, B, pl);
            plan_workspace(pm, B, pl);
            if (pl.bytes == 0) return 1;
        }
    }
    Plan plain;
    plain.ops = ops;
    plan_workspace(pm, 3, plain);
    return 0;
}

// The oracle side: load; when accepted and small enough (a forward pass of a larger net takes a second
// under the sanitizers, and thousands of damaged copies are accepted), one forward pass on a constant input.
static int oracle_side(const std::vector<uint8_t> &blob) {
    omodel *m = isr_oracle_load(blob.data(), blob.size());
    if (!m) return 0;
    int32_t C, H, W, classes, nt;
    isr_oracle_info(m, &C, &H, &W, &classes, &nt);
    const size_t total = isr_oracle_tensor_offset(m, nt);
    static long accepted = 0;   // a forward pass for every eighth accepted blob keeps the sweep within a minute
    if (accepted++ % 8 == 0 && blob.size() < 100000 && total < (4u << 20) && (size_t)C * H * W < (1u << 16) && classes < 1000) {
        std::vector<int8_t> a0((size_t)C * H * W, 17), acts(total + 16);
        std::vector<int32_t> logits(classes);
        isr_oracle_forward(m, a0.data(), acts.data(), logits.data());
        if (accepted % 64 == 1) {   // and, less often, the two comparison systems: continuous noise, rounded input, float network
            std::vector<uint8_t> x((size_t)C * H * W, 200);
            std::vector<float> v(x.size());
            std::vector<double> facts(total + 16), flogits(classes);
            isr_oracle_noisy_float(x.data(), (uint32_t)x.size(), 255.0f, 7, 1, 1, 3, v.data());
            isr_oracle_noisy_quant(x.data(), (uint32_t)x.size(), 255.0f, 7, 1, 1, 3, a0.data());
            isr_oracle_forward(m, a0.data(), acts.data(), logits.data());
            isr_oracle_forward_float(m, v.data(), facts.data(), flogits.data());
        }
    }
    isr_oracle_free(m);
    return 0;
}

static int both(const std::vector<uint8_t> &blob) { return library_side(blob) | oracle_side(blob); }

static std::vector<uint8_t> read_file(const char *path) {
    std::vector<uint8_t> v;
    FILE *f = std::fopen(path, "rb");
    if (!f) return v;
    std::fseek(f, 0, SEEK_END);
    const long n = std::ftell(f);
    std::fseek(f, 0, SEEK_SET);
    v.resize((size_t)n);
    if (std::fread(v.data(), 1, v.size(), f) != v.size()) v.clear();
    std::fclose(f);
    return v;
}

int main(int argc, char **argv) {
    int bad = 0;
    for (int a = 1; a < argc; ++a) {
        const std::vector<uint8_t> blob = read_file(argv[a]);
        if (blob.size() < 64) { std::printf("cannot read %s\n", argv[a]); return 2; }
        const long before = g_accepted;
        bad |= both(blob);
        if (g_accepted != before + 1) { std::printf("%s: the undamaged blob was rejected\n", argv[a]); return 3; }
        // Small blobs get the dense sweep, large ones (hundreds of KB to copy and parse per variant) a sparse one.
        const bool dense = blob.size() < 100000;
        const size_t front = dense ? 2048 : 256;
        // truncations: every 4-byte boundary of the front, then a spread over the rest, then the last bytes
        for (size_t n = 0; n < blob.size(); n += (n < front ? 4 : blob.size() / (dense ? 97 : 23) + 4)) bad |= both(std::vector<uint8_t>(blob.begin(), blob.begin() + n));
        for (size_t cut = 1; cut <= 9 && cut < blob.size(); ++cut) bad |= both(std::vector<uint8_t>(blob.begin(), blob.end() - cut));
        // every 32-bit word of the front (header, tensor table, first op headers and fields) and a spread of later
        // words, overwritten with edge values and edge offsets
        const uint32_t edges[] = {0u, 1u, 0xFFFFFFFFu, 0x7FFFFFFFu, 0x80000000u, 0x00010000u, 0x40000000u, 65537u};
        for (size_t w = 0; w + 4 <= blob.size(); w += (w < front ? 4 : (blob.size() / (dense ? 211 : 31) + 4) & ~(size_t)3)) {
            uint32_t old;
            std::memcpy(&old, blob.data() + w, 4);
            for (uint32_t e : edges) {
                for (uint32_t val : {e, old + e, old ^ (e | 1u)}) {
                    if (val == old) continue;
                    std::vector<uint8_t> d = blob;
                    std::memcpy(d.data() + w, &val, 4);
                    bad |= both(d);
                }
            }
        }
        // appended bytes
        std::vector<uint8_t> longer = blob;
        longer.resize(blob.size() + 4, 0);
        bad |= both(longer);
    }
    // noise tables over the whole domain and outside it; statistics on edge tallies
    for (uint32_t sigma : {0u, 1u, 2u, 3u, 31u, 32u, 255u, 256u, 1023u, 1024u, 1025u, 0xFFFFFFFFu}) {
        std::vector<uint64_t> T;
        uint32_t R = 0;
        const bool ok = build_noise_table(sigma, T, R);
        if (ok != (sigma >= 1 && sigma <= 1024)) { std::printf("noise table domain: sigma %u\n", sigma); bad = 1; }
        DeviceNoiseTable dt;
        if (build_device_table(sigma, dt) != ok) bad = 1;
        std::vector<uint32_t> words;
        uint32_t n = 0;
        if (build_bank_table(sigma, words, n, R) != ok) bad = 1;
        std::vector<uint64_t> To(2 * 16384);
        uint32_t Ro = 0;
        const int orc = isr_oracle_noise_table(sigma, To.data(), To.size(), &Ro);
        if ((orc == 0) != ok) { std::printf("oracle noise table domain: sigma %u\n", sigma); bad = 1; }
        if (ok && (Ro != R || std::memcmp(To.data(), T.data(), T.size() * 8) != 0)) { std::printf("tables differ at sigma %u\n", sigma); bad = 1; }
    }
    for (uint32_t n : {1u, 2u, 100u, 100000u, 0xFFFFFFFFu})
        for (uint32_t k : {0u, 1u, n / 2, n - 1, n}) {
            double p = -1.0, z = 0.0;
            if (isr_cp_lower(k, n, 0.001, &p) != ISR_OK || !(p >= 0.0 && p <= 1.0)) { std::printf("cp_lower(%u, %u)\n", k, n); bad = 1; }
            if (p > 0.0 && p < 1.0 && isr_normal_quantile(p, &z) != ISR_OK) bad = 1;
            int32_t t = 0;
            uint64_t t2 = 0;
            if (isr_discrete_quantile(64, p, &t, &t2) != ISR_OK) bad = 1;
            double pv = -1.0;
            if (isr_binom_pvalue(k > n - k ? k : n - k, k > n - k ? n - k : k, &pv) != ISR_OK || !(pv >= 0.0 && pv <= 1.0)) bad = 1;
        }
    const uint32_t c0[3] = {5, 90, 5}, c1[3] = {10, 980, 10};
    isr_result res;
    if (isr_decide_certify(c0, c1, 3, 64.0, 1000, 0.001, &res) != ISR_OK || res.cls != 1 || res.radius_int <= 0) bad = 1;
    if (isr_decide_certify(nullptr, c1, 3, 64.0, 1000, 0.001, &res) != ISR_ERR_ARG) bad = 1;
    if (isr_decide_predict(c1, 3, 0.001, &res) != ISR_OK || res.cls != 1) bad = 1;
    std::printf("blobs accepted %ld, rejected %ld, status %d\n", g_accepted, g_rejected, bad);
    return bad;
}
