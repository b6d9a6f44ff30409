// Inverse-CDF threshold table of the discrete Gaussian N_Z(0, sigma^2)
// (Def. 3.3 with location 0), integer arithmetic only, and the compact form
// of it the device sampler reads.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <map>
#include <memory>
#include <mutex>
#include <vector>

#include "isr.h"
#include "isr_internal.h"

namespace isr {

typedef unsigned __int128 u128;

static inline uint64_t mul_q62(uint64_t a, uint64_t b) { return (uint64_t)(((u128)a * b) >> 62); }

// Thresholds T[i] = floor(2^64 * P[delta <= i - R]), i in [0, 2R).
// Unnormalised masses exp(-k^2 / (2 sigma^2)) are carried in Q62 fixed point:
// e1 = exp(-1/D), D = 2 sigma^2, from its alternating power series, then
// mass(k+1) = mass(k) * ratio(k), ratio(k+1) = ratio(k) * e1^2.  Masses are
// truncated by 10 bits so that their total fits 64 bits; R is the last k whose
// truncated mass is non-zero.
bool build_noise_table(uint32_t sigma, std::vector<uint64_t> &T, uint32_t &R) {
    if (sigma < 1 || sigma > 1024) return false;
    const uint64_t one = 1ull << 62;
    const uint64_t D = 2ull * sigma * sigma;
    uint64_t e1 = one, term = one;
    for (uint64_t j = 1; (term /= D * j) != 0; ++j) e1 = (j & 1) ? e1 - term : e1 + term;
    const uint64_t e2 = mul_q62(e1, e1);
    std::vector<uint64_t> mass;   // mass[k] for k >= 0, already truncated
    uint64_t cur = one, ratio = e1;
    while ((cur >> 10) != 0) {
        mass.push_back(cur >> 10);
        cur = mul_q62(cur, ratio);
        ratio = mul_q62(ratio, e2);
    }
    R = (uint32_t)mass.size() - 1;
    u128 total = mass[0];
    for (uint32_t k = 1; k <= R; ++k) total += 2 * (u128)mass[k];
    if (total >> 64) return false;
    T.assign(2 * (size_t)R, 0);
    u128 below = 0;  // sum of masses of all values <= current one
    for (uint32_t i = 0; i < 2 * R; ++i) {
        uint32_t dist = i < R ? R - i : i - R;
        below += mass[dist];
        T[i] = (uint64_t)((below << 64) / total);
    }
    return true;
}

// The table of a sigma is a pure function of sigma: built once per process and shared
// (the certification decision looks its quantile up in it on every call).
std::shared_ptr<const NoiseTable> cached_noise_table(uint32_t sigma) {
    static std::mutex mu;
    static std::map<uint32_t, std::shared_ptr<const NoiseTable>> cache;
    std::lock_guard<std::mutex> lock(mu);
    auto it = cache.find(sigma);
    if (it != cache.end()) return it->second;
    auto t = std::make_shared<NoiseTable>();
    if (!build_noise_table(sigma, t->T, t->R)) return nullptr;
    if (cache.size() >= 64) cache.clear();   // bounds the memory held (at most 147 KB per sigma)
    cache[sigma] = t;
    return t;
}

// Device form.  Pixels lie in [0, 255], so after saturation only
// clamp(delta, -255, 255) matters: keep the (at most 510) thresholds between
// -255 and 255, split into high/low words, plus a guide table on the top
// GUIDE_BITS bits of the high word: guide[b] = #{j : hi[j] < (b << (32-GUIDE_BITS))}.
bool build_device_table(uint32_t sigma, DeviceNoiseTable &out) {
    const auto tab = cached_noise_table(sigma);
    if (!tab) return false;
    const std::vector<uint64_t> &T = tab->T;
    const uint32_t R = tab->R;
    uint32_t reach = R < 255 ? R : 255;
    uint32_t first = R - reach;
    uint32_t n = 2 * reach;
    out.n = n;
    out.dmin = -(int32_t)reach;
    for (uint32_t j = 0; j < NOISE_TABLE_MAX; ++j) {
        uint64_t t = j < n ? T[first + j] : ~0ull;
        out.hi[j] = (uint32_t)(t >> 32);
        out.lo[j] = (uint32_t)t;
    }
    uint32_t j = 0;
    for (uint32_t b = 0; b <= NOISE_GUIDE_SIZE; ++b) {
        uint64_t start = (uint64_t)b << (32 - NOISE_GUIDE_BITS);
        while (j < n && (uint64_t)out.hi[j] < start) ++j;
        out.guide[b] = (uint16_t)j;
    }
    return true;
}

// Form read by the stored-noise generator, as 32-bit words so that one upload carries all:
// n high words, n low words, then the guide table (NOISE_GUIDE_SIZE + 2 entries of 16 bits) on
// the top bits of the high word over all n = 2R thresholds.
bool build_bank_table(uint32_t sigma, std::vector<uint32_t> &words, uint32_t &n_out, uint32_t &R_out) {
    const auto tab = cached_noise_table(sigma);
    if (!tab) return false;
    const std::vector<uint64_t> &T = tab->T;
    const size_t n = T.size();
    const size_t guide_words = (NOISE_GUIDE_SIZE + 2) / 2;
    words.assign(2 * n + guide_words, 0);
    for (size_t j = 0; j < n; ++j) { words[j] = (uint32_t)(T[j] >> 32); words[n + j] = (uint32_t)T[j]; }
    uint16_t *guide = (uint16_t *)(words.data() + 2 * n);
    size_t j = 0;
    for (uint32_t b = 0; b <= NOISE_GUIDE_SIZE; ++b) {
        const uint64_t start = (uint64_t)b << (32 - NOISE_GUIDE_BITS);
        while (j < n && (uint64_t)words[j] < start) ++j;
        guide[b] = (uint16_t)j;
    }
    n_out = (uint32_t)n;
    R_out = tab->R;
    return true;
}

}  // namespace isr

extern "C" int isr_noise_table(uint32_t sigma, uint64_t *T_host, size_t cap, uint32_t *R_out) {
    if (!R_out || (cap && !T_host)) return ISR_ERR_ARG;
    const auto tab = isr::cached_noise_table(sigma);
    if (!tab) return ISR_ERR_ARG;
    *R_out = tab->R;
    for (size_t i = 0; i < cap && i < tab->T.size(); ++i) T_host[i] = tab->T[i];
    return ISR_OK;
}

// Inverse cdf of the discrete law by lookup in the same table (Thm 3.2, proof steps 2 and 3).
extern "C" int isr_discrete_quantile(uint32_t sigma, double p_lower, int32_t *t_out, uint64_t *radius_sq_out) {
    if (sigma < 1 || sigma > 1024 || !(p_lower >= 0.0 && p_lower <= 1.0)) return ISR_ERR_ARG;
    const auto tab = isr::cached_noise_table(sigma);
    if (!tab) return ISR_ERR_ARG;
    // floor(2^64 p): exact for a double below 1 (53 significant bits, scaled by a power of two)
    const uint64_t u = p_lower >= 1.0 ? ~0ull : (uint64_t)std::ldexp(p_lower, 64);
    // thresholds ascend: the number of entries <= u by binary search
    const int64_t below = std::upper_bound(tab->T.begin(), tab->T.end(), u) - tab->T.begin();
    const int64_t t = -(int64_t)tab->R - 1 + below;
    if (t_out) *t_out = (int32_t)t;
    if (radius_sq_out) *radius_sq_out = t > 0 ? (uint64_t)(t * t) : 0;
    return ISR_OK;
}

