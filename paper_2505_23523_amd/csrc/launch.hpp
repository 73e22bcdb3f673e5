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

// The hint sets the kernels are compiled for.  Which one a call takes depends on how the rank
// buffer size s compares with the memory-side cache: a round touches about 2s bytes (it reads up
// to n-1 chunks and writes as many).
constexpr uint32_t kHintsNone = 0;
constexpr uint32_t kHintsReduceAll = (NT_LOAD_SRC | NT_LOAD_DST | NT_STORE_DST) << 4;
// Completion.  The straggler forwards nothing before the tail rounds, so an exchange always
// hints the load of and the store to the straggler's copy.  Copies: left alone while several
// rounds fit the cache (this round's destination is a later round's source); then the stores
// are hinted and the sources, which their holders send again next round, stay cached; from
// three quarters of the cache per rank on nothing survives a round and the loads are hinted too.
constexpr uint32_t kHintsCompletion = (NT_LOAD_DST | NT_STORE_DST) << 8;
constexpr uint32_t kHintsCompletionStores = kHintsCompletion | NT_STORE_DST;
constexpr uint32_t kHintsCompletionAll = kHintsCompletionStores | NT_LOAD_SRC;
// Precondition: a ring hop's source chunk is never read again; with buffers larger than the
// cache nothing a reducing hop touches is still cached when the next round wants it.
constexpr uint32_t kHintsPrecondition = NT_LOAD_SRC << 4;
constexpr uint32_t kHintsPreconditionHuge = kHintsReduceAll;
// Ring: the same for its reducing half; in the all-gather half the source is dead after the hop
// and the destination is forwarded next round, so the copy's load is hinted and its store is not
// (from 2 GiB per rank on the store as well).
constexpr uint32_t kHintsRing = NT_LOAD_SRC | (NT_LOAD_SRC << 4);
constexpr uint32_t kHintsRingHuge = NT_LOAD_SRC | kHintsReduceAll;
constexpr uint32_t kHintsRingHugest = kHintsRingHuge | NT_STORE_DST;

struct LaunchShape {
    int total_blocks;   // bound on workgroups per round, spread over its ops; 0 = one per tile
    int unroll;         // 16-byte vectors in flight per thread (1, 2, 4)
    uint32_t hints;     // one of the kHints* sets
    bool fused_nt_loads;   // single-launch kernel: non-temporal hint on its loads ...
    bool fused_nt_stores;  // ... and on its stores
    bool fused_nt_other_load;  // straight-line completion kernel: hint on the load of the exchange's second
                               // operand (the straggler's input; the first is the precondition's fresh sum)
    int fused_unroll;   // vectors per thread in the single-launch kernel (1, 2, 4)
    int fused_wgs_per_cu;  // cap on resident workgroups per compute unit there (0: none, 2..6)
    bool fused_batch_chains;  // single-launch kernel: issue a reduce chain's operand loads four at a time
    bool fused_sum_to_all;  // single launch of a schedule whose chunks are one exchange + copies to all other
                            // ranks (the completion): the straight-line kernel instead of the op-list one
    bool fused_chain;   // single launch of a schedule made of reduce chains of one shape (sar_sched::chain_ring):
                        // the kernel that takes the ring and a start position per chunk index instead of op lists
    bool fused_split;   // run each chunk's producing ops in the op-list kernel and its trailing copies as a
                        // segment-ordered broadcast launch (only for schedules can_split accepts)
    bool reverse_ops;   // dispatch a round's ops last to first (they are independent)
    bool merge_copies;  // one launch per round, a round's copies of the same value read once (up to 32 ranks)
};

// Enqueue every round of schedule `which` on the stream, one launch per round.  With
// rank_bufs == nullptr nothing is enqueued; *launches (if given) receives the launch count either way.
int run_schedule(const sar_plan* plan, int which, void* const* rank_bufs, void* hip_stream,
                 const LaunchShape& shape, int* launches = nullptr);

// The same schedule in one launch (or a few, split by chunk index): each
// workgroup runs all rounds' ops on its own tile.  Only for plans can_fuse accepts.
// (chain: with the reduce-chain kernel where the schedule has that shape, which needs no op lists)
bool can_fuse(const sar_plan* plan, int which, bool chain = false);
bool can_split(const sar_plan* plan, int which, bool chain = false);   // ... and the split with a broadcast launch is possible
// launches the single-launch form takes (0: cannot): as a split; with the kernel written for the
// schedule's shape (straight-line completion, reduce chains) instead of the op-list kernel
int fused_launches(const sar_plan* plan, int which, bool split = false, bool direct = false);
int split_groups(const sar_plan* plan, int which);   // exchange-and-broadcast pairs of a split run
int run_schedule_fused(const sar_plan* plan, int which, void* const* rank_bufs, void* hip_stream,
                       const LaunchShape& shape);

// Make work enqueued on the stream from here on wait for the event.
int stream_wait_event(void* hip_stream, void* hip_event);

// Enqueue a kernel that idles for about `nanoseconds` of wall-clock time.
int enqueue_delay(uint64_t nanoseconds, void* hip_stream);

// Compute units of the current device.
int device_compute_units(int* out);

}  // namespace sar
