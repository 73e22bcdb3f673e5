// Interface between the C ABI layer and the HIP translation unit.
#pragma once
#include "plan.hpp"

namespace sar {

// Non-temporal hint bits: four per op kind, at bit 4 * kind
// (kind = SAR_COPY 0, SAR_REDUCE 1, SAR_REDUCE_EXCHANGE 2).
enum NtBits : uint32_t {
    NT_LOAD_SRC = 1u,   // the load of src[chunk]
    NT_LOAD_DST = 2u,   // the load of dst[chunk] (reducing ops)
    NT_STORE_DST = 4u,  // the store to dst[chunk]
    NT_STORE_SRC = 8u,  // the store back to src[chunk] (exchange only)
};

// The hint sets the kernels are compiled for.
constexpr uint32_t kHintsNone = 0;
constexpr uint32_t kHintsPrecondition = NT_LOAD_SRC << 4;
constexpr uint32_t kHintsCompletion = NT_STORE_DST | ((NT_LOAD_DST | NT_STORE_DST) << 8);
constexpr uint32_t kHintsCompletionHuge = kHintsCompletion | NT_LOAD_SRC;
constexpr uint32_t kHintsRing = NT_LOAD_SRC | (NT_LOAD_SRC << 4);
// Rank buffers larger than the memory-side cache: a round stores more than the cache holds, so
// nothing a reducing hop touches is still cached when the next round wants it.
constexpr uint32_t kHintsReduceAll = (NT_LOAD_SRC | NT_LOAD_DST | NT_STORE_DST) << 4;
constexpr uint32_t kHintsPreconditionHuge = kHintsReduceAll;
constexpr uint32_t kHintsRingHuge = NT_LOAD_SRC | kHintsReduceAll;
constexpr uint32_t kHintsRingHugest = kHintsRingHuge | NT_STORE_DST;   // from 2 GiB per rank

struct LaunchShape {
    int total_blocks;   // bound on workgroups per round, spread over its ops; 0 = one per tile
    int unroll;         // 16-byte vectors in flight per thread (1, 2, 4)
    uint32_t hints;     // one of the kHints* sets
    int fused_unroll;   // vectors per thread in the single-launch kernel (1, 2, 4)
    int fused_wgs_per_cu;  // cap on resident workgroups per compute unit there (0: none, 2..6)
    bool reverse_ops;   // dispatch a round's ops last to first (they are independent)
};

// Enqueue every round of schedule `which` on the stream, one launch per round.
int run_schedule(const sar_plan* plan, int which, void* const* rank_bufs, void* hip_stream,
                 const LaunchShape& shape);

// The same schedule in one launch (or a few, split by chunk index): each
// workgroup runs all rounds' ops on its own tile.  Only for plans can_fuse accepts.
bool can_fuse(const sar_plan* plan, int which);
int run_schedule_fused(const sar_plan* plan, int which, void* const* rank_bufs, void* hip_stream,
                       const LaunchShape& shape);

// Make work enqueued on the stream from here on wait for the event.
int stream_wait_event(void* hip_stream, void* hip_event);

// Enqueue a kernel that idles for about `nanoseconds` of wall-clock time.
int enqueue_delay(uint64_t nanoseconds, void* hip_stream);

// Compute units of the current device.
int device_compute_units(int* out);

}  // namespace sar
