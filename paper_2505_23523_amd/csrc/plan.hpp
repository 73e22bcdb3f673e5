// Internal layout of a plan: host memory only.
#pragma once
#include <atomic>
#include <cstddef>
#include <cstdint>
#include <vector>

#include "stragglar.h"

// One op of a chunk index's list.  `forward`: the source cell holds the value the
// previous op on this chunk index left in the executing thread's registers.
// `dead`: nothing can observe the op's store to dst - no later op of the schedule
// reads that cell from memory before a later op overwrites it (or, for the
// precondition, the cell is one of those its postcondition leaves unspecified).
// `chained`: a reducing op that takes its source from registers and whose destination cell
// none of the three ops before it writes - its operand load may be issued together with
// theirs, ahead of their arithmetic and stores (the additions still happen in list order).
struct sar_chunk_op {
    uint8_t src, dst, kind;
    uint8_t forward : 1, dead : 1, chained : 1;
};

// One op of a round after the copies that hand on the same value have been merged.  Within a
// round several ranks may send the same fully reduced chunk (Sec. 3.1: every holder of the oldest
// active chunk sends it); their copies hold identical bits, so a COPY group reads the chunk from
// ONE holder and stores it to every destination in `dst_mask` (bit = physical rank).  Reducing
// ops stay as they are, with one destination bit.  Built for plans of up to 32 ranks.
struct sar_group_op {
    uint8_t kind, src, chunk;
    uint32_t dst_mask;
};

struct sar_sched {
    int parts = 0;                // number of chunks
    size_t chunk_elems = 0;       // elements per chunk (the last may be shorter)
    std::vector<std::vector<sar_op>> rounds;
    // The ops of each chunk index in round order (what the single-launch kernel consumes).
    std::vector<std::vector<sar_chunk_op>> by_chunk;
    // Per round, the ops with same-value copies merged (empty above 32 ranks).
    std::vector<std::vector<sar_group_op>> grouped;
    // Split of every chunk index's list into the ops that produce the chunk's final value and the
    // trailing copies that only hand it on (Alg. 1: after its straggler pairing a chunk is only
    // ever copied).  Present (non-empty `cut`) when every list ends in such copies, the op before
    // them leaves the value in memory, and the copies reach every rank except one or two (the
    // same number for every chunk index).  cut[c]: ops [0, cut[c]) produce, the rest hand on.
    // route[c]: holder | excluded0 << 8 | excluded1 << 16 - the rank whose cell holds the value
    // after the producing ops, and the ranks (ascending; twice the same if there is one) that
    // the copies do not write.  dests: ranks written per chunk index.
    std::vector<uint16_t> cut;
    std::vector<uint32_t> route;
    int dests = 0;
    // Reduce chains of one shape (a ring ReduceScatter: Sec. 3.1's precondition, App. E's ring):
    // every chunk index starts with adds that walk `chain_ring.size()` ranks in the cyclic order
    // `chain_ring`, chunk index c from position chain_start[c] - the first op loads two cells,
    // every later one takes its source from registers - and only the last rank's store can be
    // observed.  After the chain comes nothing (chain_to_all false) or copies that hand the sum
    // on to all other ranks of the ring (true).  chain_ring is empty for schedules of any other shape.
    std::vector<uint8_t> chain_ring;
    std::vector<uint16_t> chain_start;
    bool chain_to_all = false;
    // The split's simplest case, the completion's: every chunk index is one exchange between two
    // ranks followed by copies of the sum to all n-2 others (route: the exchange's two ranks).
    bool sum_to_all = false;
};

struct sar_plan {
    int n = 0;
    int log2n = 0;
    int straggler = 0;
    int dtype = 0;
    size_t count = 0;
    size_t elem_bytes = 0;
    sar_sched sched[SAR_NUM_SCHEDULES];   // indexed by sar_schedule
    // Per schedule, how the cost model orders the three launch forms for plans of more than 32
    // ranks: bit 0 = one launch beats one launch per round, bit 1 = the split form beats one launch
    // per round, bit 2 = the split form beats the one launch; -1 = not priced yet (filled in by
    // the first call that needs it; every thread would store the same value).
    // [1]: the same with the reduce-chain kernel in place of the op-list kernel.
    mutable std::atomic<int> form_order[SAR_NUM_SCHEDULES][2];
    // Launch options of this plan, indexed by sar_tunable; SAR_OPTION_INHERIT = the process-wide value.
    std::atomic<long> option[SAR_NUM_TUNABLES];
    sar_plan() {
        for (auto& pair : form_order)
            for (std::atomic<int>& v : pair) v.store(-1, std::memory_order_relaxed);
        for (std::atomic<long>& v : option) v.store(SAR_OPTION_INHERIT, std::memory_order_relaxed);
    }
};

namespace sar {
// Fills every field of *p; returns a sar_status.
int build_plan(int n, int straggler, size_t count, int dtype, sar_plan* p);
inline size_t dtype_bytes(int dtype) { return dtype == SAR_BF16 ? 2 : 4; }
}  // namespace sar
