// Several independent reduce-scatter + Adam updates and unshards in one grid.
#pragma once

#include "reduce_kernels.h"
#include "unshard_kernels.h"

namespace {

// ---------------------------------------------------------------------------
// Batches of independent operations in one grid: up to kBatchOps fused
// reduce-scatter + Adam operations and up to kBatchOps unshards of other units
// (cast + gather of fp32 shards to bf16, or the plain gather of 16-bit shards).
// One launch floor for the whole batch, and the ramp and drain of the members
// overlap.  Workgroups [0, r_end[n_reduce-1]) serve the reduce operations in
// order, the rest the unshards.
// ---------------------------------------------------------------------------
constexpr int kBatchOps = 6;          // measured on MI355X: 3 -> 4 -> 6 members gain 0.9 % and 1.3 %, more gain nothing
// The members' rank pointers share one pool, so that a grid can hold twelve
// 8-rank members as well as one 64-rank update next to one 64-rank unshard.
constexpr int kBatchPtrs = 376;

struct BatchReduceOp {
    RsArgs a;
    int32_t ptr0;      // first of the member's a.W rank pointers (padded to whole wide batches) in the pool
    int32_t pad_;
};
struct BatchUnshardOp {
    int64_t S;
    uint16_t* out;
    int32_t tiles;
    int32_t lp;        // 1: the shards are 16-bit already (Sec. 4.4 hand-off): plain gather
    int32_t ptr0;      // first of the member's shard pointers in the pool
    int32_t pad_;
};
struct BatchArgs {
    int32_t n_reduce, n_unshard;
    uint32_t r_end[kBatchOps];     // exclusive end of each reduce operation's workgroup range
    uint32_t u_end[kBatchOps];     // same for the unshards, counted from the end of the reduce ranges
    BatchReduceOp r[kBatchOps];
    BatchUnshardOp u[kBatchOps];
    const void* ptrs[kBatchPtrs];
};
static_assert(sizeof(BatchArgs) <= 4096, "kernel arguments are limited to 4 KiB");

template <int GT, int PRE>
__global__ __launch_bounds__(kBlock) void batch_kernel(BatchArgs b)
{
    uint32_t bid = blockIdx.x;
    const uint32_t n_red_blocks = b.n_reduce > 0 ? b.r_end[b.n_reduce - 1] : 0u;
    if (bid < n_red_blocks) {
        int32_t i = 0;
        uint32_t start = 0;
        while (bid >= b.r_end[i]) { start = b.r_end[i]; ++i; }     // uniform, at most kBatchOps - 1 steps
        reduce_body<GT, PRE, true, false, kBlock, true>(b.ptrs + b.r[i].ptr0, b.r[i].a, bid - start);
    } else {
        bid -= n_red_blocks;
        int32_t i = 0;
        uint32_t start = 0;
        while (bid >= b.u_end[i]) { start = b.u_end[i]; ++i; }
        if (b.u[i].lp)   // uniform
            gather_lp_body(b.ptrs + b.u[i].ptr0, b.u[i].S, b.u[i].out, b.u[i].tiles, bid - start);
        else
            unshard_lp_body<kBF16>(b.ptrs + b.u[i].ptr0, b.u[i].S, b.u[i].out, b.u[i].tiles, bid - start);
    }
}

}  // namespace
