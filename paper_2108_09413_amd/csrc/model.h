// The model object behind the C ABI's opaque handle, shared by the files that implement entry points.
#ifndef ISR_MODEL_H
#define ISR_MODEL_H

#include <map>
#include <string>
#include <vector>

#include "isr_internal.h"
#include "plan.h"

namespace isr {
constexpr int TABLE_SLOTS = 8;
struct FloatNet;   // float_api.cpp: the float network of the FloatRS-fp comparison system, built on first use
void free_float_net(FloatNet *net);
}  // namespace isr

using isr::Plan; using isr::DevOp; using isr::ParsedModel; using isr::DeviceNoiseTable; using isr::BlockDesc; using isr::NoiseItem;
using isr::TABLE_SLOTS;

struct isr_model {
    ParsedModel pm;
    std::vector<DevOp> ops;             // one descriptor per op of the blob
    Plan plan[3];                       // [0] op by op, [1] with the fusions that pay, [2] with every fusion the kernels cover
    int use_fused = 1;
    int conv_tile = 0;                  // forced conv output tile (0 = automatic)
    uint8_t *dconst = nullptr;          // weights and per-channel tables
    DeviceNoiseTable *dtables = nullptr;  // TABLE_SLOTS entries
    DeviceNoiseTable *htables = nullptr;  // pinned staging, TABLE_SLOTS entries
    uint32_t table_sigma[TABLE_SLOTS] = {0};
    int table_next = 0;
    uint32_t *dcounts = nullptr;        // 2 * classes
    uint32_t *hcounts = nullptr;        // pinned, 2 * classes
    BlockDesc *dblocks = nullptr;       // descriptors of the identity-block chains of plan[1] and plan[2]
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
    std::map<std::string, isr_kernel_stat> stats;   // per kernel instance (name as a profiler prints it)
    // floating-point comparison systems
    float quant_sigma = -1.f;           // >= 0 while a FloatRS-quant call runs: the noise stage draws continuous Gaussian noise and rounds it
    isr::FloatNet *fnet = nullptr;
};

namespace isr {
// The integer path's Monte-Carlo loop with the input stage of FloatRS-quant (api.cpp): noisy copies are
// clamp(round(x + sigma z)) with continuous z instead of discrete-Gaussian draws; everything after is the int8 network.
int run_quant_range(isr_model *m, const uint8_t *x, float sigma, uint64_t seed, uint32_t image, uint32_t phase,
                    uint32_t begin, uint64_t count, int32_t *logits_host, int32_t *argmax_host, uint32_t *dcounts,
                    int stop_tensor);
}  // namespace isr

#endif
