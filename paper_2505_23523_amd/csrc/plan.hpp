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

struct sar_sched {
    int parts = 0;                // number of chunks
    size_t chunk_elems = 0;       // elements per chunk (the last may be shorter)
    std::vector<std::vector<sar_op>> rounds;
    // The ops of each chunk index in round order (what the single-launch kernel consumes).
    std::vector<std::vector<sar_chunk_op>> by_chunk;
};

struct sar_plan {
    int n = 0;
    int log2n = 0;
    int straggler = 0;
    int dtype = 0;
    size_t count = 0;
    size_t elem_bytes = 0;
    sar_sched sched[SAR_NUM_SCHEDULES];   // indexed by sar_schedule
    // Per schedule, whether the cost model prefers the single launch: -1 = not priced yet
    // (filled in by the first call that needs it; every thread would store the same value).
    mutable std::atomic<int> single_launch_pays[SAR_NUM_SCHEDULES];
    sar_plan() {
        for (std::atomic<int>& v : single_launch_pays) v.store(-1, std::memory_order_relaxed);
    }
};

namespace sar {
// Fills every field of *p; returns a sar_status.
int build_plan(int n, int straggler, size_t count, int dtype, sar_plan* p);
inline size_t dtype_bytes(int dtype) { return dtype == SAR_BF16 ? 2 : 4; }
}  // namespace sar
