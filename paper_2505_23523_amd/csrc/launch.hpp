// Interface between the C ABI layer and the HIP translation unit.
#pragma once
#include "plan.hpp"

namespace sar {

struct LaunchShape {
    int total_blocks;  // workgroups per round, spread over the round's ops
    int unroll;        // 16-byte vectors in flight per thread (1, 2, 4, 8)
    int nontemporal;   // 0 plain, 1 nt stores, 2 nt loads + stores
};

// Enqueue every round of schedule `which` on the stream, one launch per round.
int run_schedule(const sar_plan* plan, int which, void* const* rank_bufs, void* hip_stream,
                 const LaunchShape& shape);

// Compute units of the current device.
int device_compute_units(int* out);

}  // namespace sar
