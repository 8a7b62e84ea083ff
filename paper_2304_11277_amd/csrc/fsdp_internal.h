// Internal declarations shared by the host planner and the kernel launchers of
// libfsdp_flat.  Not part of the public ABI.
#pragma once

#include <cstdint>
#include <vector>

#include "fsdp_flat.h"

// Host-side FlatParameter layout (Sec. 3.2.1).  Immutable after init.
struct fsdp_layout {
    int32_t num_params = 0;
    int32_t world_size = 0;
    int64_t N = 0;     // unpadded numel
    int64_t S = 0;     // shard numel, ceil(N / W)
    int64_t P = 0;     // padded numel, S * W
    int64_t pad = 0;   // P - N
    int32_t reduce_walk = FSDP_WALK_AUTO;   // tuning hint of fsdp_layout_init_ex
    std::vector<int64_t> off;    // [p + 1] exclusive prefix sum of numels
    std::vector<int64_t> numel;  // [p]
};

namespace fsdp {
void set_last_hip_error(int e);
}
