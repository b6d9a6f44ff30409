// Stored-noise generator without any device allocation: the variant of isr_noise_bank for
// callers that must not allocate (code under HIP graph capture, tight serving loops, harnesses
// that forbid hipMalloc).  The sampler's table -- the one piece of device memory isr_noise_bank
// allocates and frees per call -- lives in a file-scope device array instead.
#include <mutex>
#include <vector>

#include "isr_internal.h"

namespace {

// Room for the table of every sigma up to about 420 grid units (8 bytes per threshold, 2R = about
// 18 sigma thresholds, plus the 8200-byte guide table).  Every GPU the library runs on holds its
// own copy of this array until the process ends.
constexpr size_t SCRATCH_BYTES = 64 * 1024;
static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

// In host code the array's name is only a stand-in: the device address of each GPU's copy is
// asked for once per device, with that device current, and kept here.
constexpr int MAX_DEVICES = 64;
void *g_scratch_ptr[MAX_DEVICES] = {};
std::mutex g_scratch_mu;

hipError_t scratch_address(void **out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace

extern "C" size_t isr_noise_bank_static_capacity(void) { return SCRATCH_BYTES; }

extern "C" int isr_noise_bank_static(uint32_t sigma, uint64_t seed, uint32_t bank_id, uint32_t first, uint32_t count,
                                     uint32_t d, int16_t *out_device, void *hip_stream) {
    using namespace isr;
    if (sigma < 1 || sigma > 1024 || !out_device || d == 0 || (d & 3) != 0) return ISR_ERR_ARG;
    if ((uint64_t)first + count > (1ull << 32)) return ISR_ERR_ARG;
    if (count == 0) return ISR_OK;
    std::vector<uint32_t> host;   // host memory only
    uint32_t n = 0, R = 0;
    if (!build_bank_table(sigma, host, n, R)) return ISR_ERR_ARG;
    if (host.size() * 4 > SCRATCH_BYTES) return ISR_ERR_WORKSPACE;   // this sigma's table does not fit the fixed array
    void *ptr = nullptr;
    hipError_t e = scratch_address(&ptr);
    hipStream_t st = (hipStream_t)hip_stream;
    // every call on this GPU writes the same array: the whole table of this sigma replaces what
    // the last call left (the kernel reads n entries and the guide, nothing beyond)
    if (e == hipSuccess) e = hipMemcpyAsync(ptr, host.data(), host.size() * 4, hipMemcpyHostToDevice, st);
    if (e == hipSuccess) {
        uint32_t *dev = (uint32_t *)ptr;
        NoiseBankParams p;
        p.thi = dev; p.tlo = dev + n; p.guide = (const uint16_t *)(dev + 2 * n);
        p.n = (int32_t)n; p.R = (int32_t)R; p.out = out_device; p.d = d;
        p.key0 = (uint32_t)seed; p.key1 = (uint32_t)(seed >> 32); p.bank = bank_id; p.first = first; p.count = count;
        e = launch_noise_bank(p, st);
    }
    if (e == hipSuccess) e = hipStreamSynchronize(st);   // the host staging vector dies with this call
    if (e != hipSuccess) { set_last_device_error((int)e); return ISR_ERR_DEVICE; }
    return ISR_OK;
}
