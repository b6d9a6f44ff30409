// The planner: device descriptors of the model's ops, the fusions the kernels cover, and the
// placement of every tensor of a chunk in the workspace.
#ifndef ISR_PLAN_H
#define ISR_PLAN_H

#include <utility>
#include <vector>

#include "isr_internal.h"

namespace isr {

struct DevOp {
    OpType type;
    int a = -1, b = -1, out = -1;
    double ops_per_sample = 0.0, bytes_per_sample = 0.0;   // algorithmic, for the timing report
    ConvParams conv{};
    int stem_pool = 0;                  // conv fused with the max pooling after it (out = the pooled tensor)
    int noise_fused = 0;                // the kernel of this (first) op draws the noisy input itself: no noise launch, tensor 0 never stored
    int stem16 = 0;                     // first 3x3 convolution into 16 channels: the LDS-resident kernel
    int block = 0;                      // identity residual block: this conv, conv2 and the add in one kernel
    std::vector<std::pair<ConvParams, ConvParams>> chain;   // block != 0: the blocks of the chain this op runs (each feeds the next)
    size_t chain_off = 0;               // first BlockDesc of the chain in the model's device array
    int trans = 0;                      // down-sampling block: this conv (3x3/2), conv2 (3x3) and conv3 (1x1/2 + add) in one kernel
    int bneck = 0;                      // 1: this 1x1 conv and the 3x3 conv2 in one kernel; 2: plus conv3 (1x1 + residual add); 3: as 2 with 128 middle channels; 4: as 2 with the residual computed by a projection 1x1 convolution of the block input (conv3 carries it as its second convolution)
    int xr = 0;                         // this expanding 1x1 + residual add and the reducing 1x1 that reads its sum (conv2, output out2) in one kernel
    int out2 = -1;                      // second output tensor of the op (xr != 0)
    int proj_is_main = 0;               // bneck == 4: conv3's first convolution is the projection of the block input, its second the closing 1x1
    ConvParams conv2{};
    ConvParams conv3{};
    AddParams add{};
    PoolParams pool{};
    GapParams gap{};
    FcParams fc{};
};

// A run of consecutive ops that is executed sub-chunk by sub-chunk: ops [previous end, end) of the
// plan on `sub` copies at a time.  Ops after the last segment run on the whole chunk.
struct Segment {
    size_t end;
    uint32_t sub;
};

// An executable op list plus where each tensor lives in the workspace.
struct Plan {
    std::vector<DevOp> ops;
    std::vector<Segment> segments;      // empty: every op runs on the whole chunk
    std::vector<size_t> toff;           // per tensor offset inside the workspace
    std::vector<char> has;              // tensor is produced by this plan
    size_t logits_off = 0, argmax_off = 0, bytes = 0;
};

// Host image of the constant arena (weights, per-channel tables); descriptors hold offsets into it
// until rebase_device_ops turns them into device pointers.
struct ConstArena {
    std::vector<uint8_t> host;
    size_t put(const void *src, size_t n);
};

// One descriptor per op of the blob, weights re-laid for the kernels into `arena`.  ISR_OK or ISR_ERR_UNSUPPORTED.
int build_device_ops(const ParsedModel &pm, std::vector<DevOp> &ops, ConstArena &arena);
// Arena offsets -> pointers into the uploaded arena at `base`.
void rebase_device_ops(std::vector<DevOp> &ops, const uint8_t *base);
// The op list with the fusions the kernels cover applied (from the rebased op-by-op list).
// wide_bottlenecks: also fold identity bottleneck blocks with 128 middle channels into one kernel
// (correct, but at present slower than their three separate kernels: off in the default plan).
void build_fused_plan(const ParsedModel &pm, const std::vector<DevOp> &plain, std::vector<DevOp> &fused, bool wide_bottlenecks);
// Chooses the sub-chunk segments of a plan for chunks of B samples (before plan_workspace).
void plan_segments(const ParsedModel &pm, uint32_t B, Plan &pl);
// Offsets of every tensor of a chunk of B samples in the workspace.
void plan_workspace(const ParsedModel &pm, uint32_t B, Plan &pl);

}  // namespace isr

#endif
