// The C ABI: argument checks and marshalling only.
#include <algorithm>
#include <atomic>
#include <cstdint>
#include <new>

#include "launch.hpp"
#include "plan.hpp"
#include "stragglar.h"

namespace {

// Process-wide defaults of the launch options, indexed by sar_tunable.
std::atomic<long> g_tune[SAR_NUM_TUNABLES] = {{0}, {-1}, {-1}, {-1}, {-1}, {-1}, {0}, {-1}, {-1}};

bool valid_schedule(int which) { return which >= 0 && which < SAR_NUM_SCHEDULES; }

bool valid_tune_value(int key, long value) {
    switch (key) {
        case SAR_TUNE_BLOCKS_PER_CU: return value >= 0 && value <= 65536;
        case SAR_TUNE_UNROLL:
        case SAR_TUNE_FUSED_UNROLL: return value == -1 || value == 1 || value == 2 || value == 4;
        case SAR_TUNE_NONTEMPORAL:
        case SAR_TUNE_FUSE_ROUNDS:
        case SAR_TUNE_FUSED_SPLIT:
        case SAR_TUNE_FUSED_DIRECT: return value >= -1 && value <= 1;
        case SAR_TUNE_FUSED_WGS_PER_CU: return value == -1 || value == 0 || (value >= 2 && value <= 6);
        case SAR_TUNE_MERGE_COPIES: return value == 0 || value == 1;
        default: return false;
    }
}

// The value of a launch option for calls with this plan: the plan's own if it has one.
long tune(const sar_plan* plan, int key) {
    const long own = plan->option[key].load(std::memory_order_relaxed);
    return own != SAR_OPTION_INHERIT ? own : g_tune[key].load(std::memory_order_relaxed);
}

// Null, misaligned or overlapping rank buffers.  Overlap: sort the start addresses, then every
// buffer must end before the next one starts.
int check_buffers(const sar_plan* plan, void* const* rank_bufs) {
    if (!plan || !rank_bufs) return SAR_EINVAL;
    const uintptr_t bytes = plan->count * plan->elem_bytes;
    uintptr_t at[SAR_MAX_RANKS];
    for (int i = 0; i < plan->n; ++i) {
        at[i] = reinterpret_cast<uintptr_t>(rank_bufs[i]);
        if (at[i] == 0 || (at[i] & 15u) != 0) return SAR_EINVAL;
    }
    std::sort(at, at + plan->n);
    for (int i = 1; i < plan->n; ++i)
        if (at[i] - at[i - 1] < bytes) return SAR_EINVAL;
    return SAR_OK;
}

constexpr size_t kMiB = size_t(1) << 20;
constexpr size_t kMemorySideCache = 256 * kMiB;   // Infinity Cache of the MI355X

// Whether running a schedule's trailing copies as broadcast launches of their own is the faster
// single-launch form (measured; SAR_TUNE_FUSED_SPLIT = -1 follows this).  Only where the producing
// ops are a short pass - the completion's one exchange per chunk; a ring's reduce chains followed
// by a broadcast launch are slower than its one launch.  A workgroup storing its tile to all n
// ranks makes HBM take n write streams at once, which costs more the more ranks there are; the
// split pays one more rank buffer of traffic and a launch or more to get the one-stream rate
// back.  Completion, split against one launch, ms (f32, the benchmark's protocol):
//   32 ranks  16 MiB 0.112 / 0.114   64 MiB 0.38 / 0.43   256 MiB 1.57 / 1.74   512 MiB 3.58 / 3.63
//   24 ranks  32 MiB 0.161 / 0.175   64 MiB 0.30 / 0.32   256 MiB 1.18 / 1.31
//   20 ranks  64 MiB 0.257 / 0.266  256 MiB 0.99 / 1.11
//   16 ranks  64 MiB 0.21 / 0.20    128 MiB 0.40 / 0.38   192 MiB 0.59 / 0.63   256 MiB 0.80 / 0.84
//             512 MiB 1.90 / 1.80     1 GiB 3.85 / 3.54
//   12 ranks 256 MiB 0.62 / 0.62;  8 ranks: the one launch at every size (256 MiB 0.46 / 0.41)
// and everything that fits the memory-side cache twice over is better off in one launch (32
// ranks, 8 MiB: 61 / 45 us).  Above 32 ranks the op lists of all chunk indices no longer fit one
// launch's arguments, and the split form - an exchange launch and a broadcast launch per group
// instead of 4 to 255 launches - wins at every size (64 ranks, 1 MiB per rank: 0.025 vs 0.154 ms;
// 64 MiB: 0.71 vs 0.90; 256 MiB: 2.97 vs 3.38; 256 ranks, 64 MiB: 3.5 vs 11 ms, and 6.3 ms round
// by round).
int form_order(const sar_plan* plan, int which);
bool takes_split(const sar_plan* plan, int which);
bool takes_chain(const sar_plan* plan, int which);

bool split_pays(const sar_plan* plan, int which) {
    // other schedules (a ring: reduce chains, then the all-gather as broadcast launches): only above
    // 32 ranks, where the one launch becomes many, and by the cost model below
    // - and not where the reduce-chain kernel runs: its one launch beats its split at every size
    // (ring, 64 ranks x 64 MiB: 1.57 vs 1.82 ms; 256 ranks x 4 MiB: 0.46 vs 0.87 ms)
    if (!plan->sched[which].sum_to_all) return plan->n > 32 && !takes_chain(plan, which) && (form_order(plan, which) & 4) != 0;
    if (plan->n > 32) return true;
    const size_t per_rank = plan->count * plan->elem_bytes;
    if (per_rank > kMemorySideCache) return false;
    if (plan->n > 16) return per_rank * size_t(plan->n) >= 2 * kMemorySideCache;
    return plan->n == 16 && 4 * per_rank >= 3 * kMemorySideCache;
}

// Launch shape and cache hints for one call: the plan's options or the process-wide knobs where
// they are set, the measured defaults otherwise.
sar::LaunchShape choose_shape(const sar_plan* plan, int which, int compute_units) {
    sar::LaunchShape shape;
    shape.total_blocks = int(tune(plan, SAR_TUNE_BLOCKS_PER_CU)) * compute_units;

    // Non-temporal hints pay off once the ranks' buffers together no longer fit the memory-side
    // cache; below that everything is re-read from it anyway.  A round touches about twice a rank
    // buffer; the sets differ in what can still be cached at that size (launch.hpp).  The
    // thresholds are measured ones (random data; all-zero buffers run faster and rank the sets
    // differently).
    const size_t per_rank = plan->count * plan->elem_bytes;
    const long nt = tune(plan, SAR_TUNE_NONTEMPORAL);
    const bool streaming = nt >= 0 ? nt != 0 : per_rank * size_t(plan->n) > kMemorySideCache;
    const bool huge = per_rank > kMemorySideCache;   // one round's stores alone exceed the cache
    shape.hints = sar::kHintsNone;
    // Single launch: every load is the first and only read of its cell, every store final.  Both
    // are hinted, except the completion's loads: they fetch what the precondition stored last.
    shape.fused_nt_stores = streaming;
    shape.fused_nt_loads = streaming && which != SAR_SCHED_COMPLETION && which != SAR_SCHED_BCAST_COMPLETION;
    // The straight-line completion kernel loads the on-time rank's sum plainly (part of it is
    // still cached) and, from three quarters of the cache per rank on, the straggler's input with
    // the hint: that was written before the precondition ran and is dead after this read (8 ranks,
    // 192 / 224 / 256 MiB per rank: 0.311 -> 0.303, 0.381 -> 0.365, 0.416 -> 0.403 ms; 128 and
    // 160 MiB: 3 % slower, 16 ranks of 64 MiB: 14 % slower - there it is still cached).
    shape.fused_nt_other_load = streaming && 4 * per_rank >= 3 * kMemorySideCache;
    // What the precondition stores - each on-time rank's own chunk, one rank buffer's worth in all -
    // is what the completion loads first.  While that fits the memory-side cache it is stored without
    // the hint: time moves from the completion, the critical path once the straggler has arrived
    // (Sec. 3), into the phase its delay hides (8 ranks, 256 MiB: precondition 0.335 -> 0.357 ms,
    // completion 0.409 -> 0.393 ms; 192 MiB: +4 % / -4 %; 96 MiB: both 1.5 % faster; 16 ranks x 64
    // MiB: +3.7 % / -3.6 %).  Not where the completion runs split (its exchange launch does not
    // gain: 32 ranks +4.5 % / -0.5 %) nor beyond one cache size per rank (2.4 GB: +15 % / +1 %).
    if (which == SAR_SCHED_PRECONDITION && per_rank <= kMemorySideCache && !takes_split(plan, SAR_SCHED_COMPLETION))
        shape.fused_nt_stores = false;
    if (streaming) {
        if (which == SAR_SCHED_PRECONDITION || which == SAR_SCHED_RHD)
            shape.hints = huge ? sar::kHintsPreconditionHuge
                               : 2 * per_rank < kMemorySideCache ? sar::kHintsNone : sar::kHintsPrecondition;
        else if (which == SAR_SCHED_RING || which == SAR_SCHED_BCAST_PRECONDITION)
            shape.hints = !huge ? sar::kHintsRing
                                : per_rank >= 2048 * kMiB ? sar::kHintsRingHugest : sar::kHintsRingHuge;
        else
            shape.hints = 4 * per_rank <= kMemorySideCache       ? sar::kHintsCompletion
                          : 4 * per_rank < 3 * kMemorySideCache ? sar::kHintsCompletionStores
                                                                : sar::kHintsCompletionAll;
    }
    // Two vectors in flight per thread pay off as long as part of a round stays cached: up to one
    // cache size per rank for the reducing schedules, three quarters of it for the completion.
    const bool reducing = which != SAR_SCHED_COMPLETION && which != SAR_SCHED_BCAST_COMPLETION;
    const long unroll = tune(plan, SAR_TUNE_UNROLL);
    shape.unroll = unroll > 0 ? int(unroll)
                   : (reducing ? !huge : 4 * per_rank < 3 * kMemorySideCache) ? 2 : 1;
    // With buffers of a GiB and more, issuing a round's exchange after its copies leaves the
    // exchanged chunk - the next round's first source - the most recently written data.
    shape.reverse_ops = streaming && which == SAR_SCHED_COMPLETION && per_rank >= 1024 * kMiB;
    shape.merge_copies = tune(plan, SAR_TUNE_MERGE_COPIES) != 0;

    // Shape of the single launch (measured, random data).  HBM does better with fewer wavefronts
    // interleaving their streams than full occupancy gives.  The completion (2 loads, then n
    // stores per tile): full occupancy with 2 vectors per thread while everything fits the
    // memory-side cache, then 2 workgroups per compute unit (3 with 1 vector for buffers larger
    // than the cache).  The schedules built on reduce chains can send a chain's operand loads
    // out four at a time; that pays where latency rules - cache-resident sizes (4 workgroups, 2
    // vectors) and 32 ranks or more (3 workgroups for the precondition, 2 for ring and
    // both-phases-in-one) - and costs a few percent in between, where the chain stays serial:
    // precondition (n-1 loads, 1 store) 4 workgroups with 2 vectors, the others 6 with 1.
    const bool completion = which == SAR_SCHED_COMPLETION || which == SAR_SCHED_BCAST_COMPLETION;
    const bool loads_only = which == SAR_SCHED_PRECONDITION;
    const long fu = tune(plan, SAR_TUNE_FUSED_UNROLL), wgs = tune(plan, SAR_TUNE_FUSED_WGS_PER_CU);
    int auto_unroll, auto_wgs;
    shape.fused_batch_chains = !streaming || plan->n >= 32;
    if (completion) {
        auto_unroll = streaming && huge ? 1 : 2;
        auto_wgs = !streaming ? 0 : huge ? 3 : 2;
    } else if (!streaming) {
        auto_unroll = 2;
        auto_wgs = 4;
    } else if (shape.fused_batch_chains) {
        auto_unroll = 1;
        auto_wgs = loads_only ? 3 : 2;
    } else {
        auto_unroll = loads_only ? 2 : 1;
        auto_wgs = loads_only ? 4 : 6;
    }
    shape.fused_split = takes_split(plan, which);
    // The straight-line kernel for the completion's shape: faster than the op-list kernel up to one
    // cache size per rank (256 MiB per rank, 8 ranks: 0.420 vs 0.430 ms, each at its best shape -
    // here 1 vector and 3 workgroups per compute unit; 96 MiB: 0.147 vs 0.150 ms), slower beyond
    // (512 MiB: 0.882 vs 0.874 ms), where the automatic choice leaves it to the op-list kernel.
    const long direct = tune(plan, SAR_TUNE_FUSED_DIRECT);
    shape.fused_sum_to_all = plan->n <= 32 && plan->sched[which].sum_to_all && (direct >= 0 ? direct != 0 : !huge);
    shape.fused_chain = takes_chain(plan, which);
    if (shape.fused_chain && streaming) {
        // 1 vector; 4-byte elements 3 workgroups per compute unit (2 when the sum goes to every
        // rank), bf16 twice as many (16 ranks x 64 MiB bf16, precondition: +42 % with 3, +0.7 % with 6)
        auto_unroll = 1;
        auto_wgs = (plan->sched[which].chain_to_all ? 2 : 3) * (plan->elem_bytes == 4 ? 1 : 2);
    }
    if (shape.fused_sum_to_all && streaming) {
        auto_unroll = 1;
        auto_wgs = 3;
    }
    if (shape.fused_split && plan->sched[which].sum_to_all) {
        // what is left for the op-list kernel: a short pass of loads and one or two plain stores
        // (a split ring keeps its reduce chains there, and with them the shape of a chain schedule)
        auto_unroll = 2;
        auto_wgs = 4;
    } else if (shape.fused_split) {
        auto_unroll = shape.fused_batch_chains ? 1 : 2;      // the precondition's: loads and one store
        auto_wgs = !streaming ? 4 : shape.fused_batch_chains ? 3 : 4;
    }
    shape.fused_unroll = fu > 0 ? int(fu) : auto_unroll;
    shape.fused_wgs_per_cu = wgs >= 0 ? int(wgs) : auto_wgs;
    return shape;
}

// One launch per round is the schedule as the paper runs it (SAR_TUNE_FUSE_ROUNDS = 0).  The
// single-launch forms compute the same bits with fewer launches and less HBM traffic, so the
// automatic choice takes one wherever it is faster.  With the op-list kernel that stops being so
// with many ranks: a chunk index's op list gets long (n to 2n dependent steps per workgroup) and
// a launch's arguments hold few of them, so a call becomes many launches of few workgroups, each
// as long as its chain; the split form keeps only the producing half of every list and hands
// the rest to broadcast launches; the reduce-chain kernel needs no lists at all.  The three
// forms are priced with a small model fitted to measurements (40 to 256 ranks, 1 to 64 MiB per
// rank): a launch costs at least 3.7 us, HBM delivers about 6 TB/s to one launch per round,
// 5.5 TB/s to the single-launch kernels and 6.5 TB/s to a broadcast launch, and a step of a
// chain takes 0.3 us when it loads (operand loads go out four at a time) and 0.17 us when it
// only stores.  Ring with the op-list kernel, 64 ranks x 4 MiB, per round / one / split: model
// 0.47 / 0.76 / 0.30 ms, measured 0.49 / 0.80 / 0.37; 128 ranks x 16 MiB: measured 2.35 / 8.2 /
// 2.69, and the model keeps one launch per round there too.
int form_order(const sar_plan* plan, int which) {
    const bool chain = takes_chain(plan, which);
    const int known = plan->form_order[which][chain].load(std::memory_order_relaxed);
    if (known >= 0) return known;

    const sar_sched& sched = plan->sched[which];
    int order = 0;
    if (sar::can_fuse(plan, which, chain)) {
        const bool can_split = sar::can_split(plan, which, chain);
        double per_round_bytes = 0, one_bytes = 0, producing_bytes = 0, broadcast_bytes = 0;   // in chunks
        double one_chain_us = 0, producing_chain_us = 0;
        for (const auto& ops : sched.rounds)
            for (const sar_op& op : ops) per_round_bytes += op.op == SAR_COPY ? 2 : op.op == SAR_REDUCE ? 3 : 4;
        for (int c = 0; c < sched.parts; ++c) {
            const std::vector<sar_chunk_op>& ops = sched.by_chunk[c];
            const size_t cut = can_split ? size_t(sched.cut[c]) : ops.size();
            double us = 5.0, us_at_cut = 5.0;
            for (size_t k = 0; k < ops.size(); ++k) {
                const sar_chunk_op& op = ops[k];
                const int loads = (op.forward ? 0 : 1) + (op.kind != SAR_COPY ? 1 : 0);
                const int moved = loads + (op.dead ? 0 : 1) + (op.kind == SAR_REDUCE_EXCHANGE ? 1 : 0);
                one_bytes += moved;
                us += loads ? 0.3 : 0.17;
                if (k < cut) {
                    producing_bytes += moved;
                    us_at_cut = us;
                }
            }
            if (us > one_chain_us) one_chain_us = us;
            if (us_at_cut > producing_chain_us) producing_chain_us = us_at_cut;
            broadcast_bytes += 1 + sched.dests;
        }
        const double chunk_bytes = double(sched.chunk_elems) * double(plan->elem_bytes);
        auto at_least = [](double a, double b) { return a > b ? a : b; };
        const double rounds = double(sched.rounds.size());
        const double per_round_us = rounds * at_least(per_round_bytes * chunk_bytes / rounds / 6.0e6, 3.7);
        const double one_launches = double(sar::fused_launches(plan, which, false, chain));
        const double one_us = one_launches * at_least(one_bytes * chunk_bytes / one_launches / 5.5e6, one_chain_us);
        if (one_us < per_round_us) order |= 1;
        if (can_split) {
            const double groups = double(sar::split_groups(plan, which));
            const double producing_launches = double(sar::fused_launches(plan, which, true, chain)) - groups;
            const double split_us = producing_launches * at_least(producing_bytes * chunk_bytes / producing_launches / 5.5e6, producing_chain_us) +
                                    groups * at_least(broadcast_bytes * chunk_bytes / groups / 6.5e6, 3.7);
            if (split_us < per_round_us) order |= 2;
            if (split_us < one_us) order |= 4;
        }
    }
    plan->form_order[which][chain].store(order, std::memory_order_relaxed);
    return order;
}

// The reduce-chain kernel in place of the op-list kernel, for schedules of that shape
// (SAR_TUNE_FUSED_DIRECT).  Automatic: above 32 ranks, where op lists no longer fit one launch.
// Up to 32 ranks the two kernels are within 2 % of each other (each at its best shape), except for
// a ring AllReduce of 4-byte elements among 16 to 28 ranks, which the chain kernel runs 2 to 6 %
// faster (16 ranks x 64 MiB: 0.355 vs 0.379 ms; 20 and 28 ranks: -3 %, -2 %; bf16: no gain), and
// for the bf16 precondition on rank buffers beyond one cache size, where it is level to 5 %
// ahead (8 ranks x 2.48 GB: 3.08 vs 3.24 ms on three boxes; 384 MiB -4 %, 512 MiB and 1 GiB level).
bool takes_chain(const sar_plan* plan, int which) {
    const sar_sched& sched = plan->sched[which];
    if (sched.chain_ring.empty()) return false;
    const long direct = tune(plan, SAR_TUNE_FUSED_DIRECT);
    if (direct >= 0) return direct != 0;
    if (plan->n > 32) return true;
    if (sched.chain_to_all) return plan->n >= 16 && plan->n < 32 && plan->elem_bytes == 4;
    return plan->elem_bytes == 2 && plan->count * plan->elem_bytes > kMemorySideCache;
}

bool takes_split(const sar_plan* plan, int which) {
    const long split = tune(plan, SAR_TUNE_FUSED_SPLIT);
    return sar::can_split(plan, which, takes_chain(plan, which)) && (split >= 0 ? split != 0 : split_pays(plan, which));
}

bool use_single_launch(const sar_plan* plan, int which) {
    const long fuse = tune(plan, SAR_TUNE_FUSE_ROUNDS);
    if (fuse == 0 || !sar::can_fuse(plan, which, takes_chain(plan, which))) return false;
    if (fuse > 0 || plan->n <= 32) return true;   // one or two launches: always faster
    const bool split = takes_split(plan, which);
    if (split && plan->sched[which].sum_to_all) return true;     // measured (split_pays)
    return (form_order(plan, which) & (split ? 2 : 1)) != 0;
}

int run(const sar_plan* plan, int which, void* const* rank_bufs, void* stream) {
    const int st = check_buffers(plan, rank_bufs);
    if (st != SAR_OK) return st;
    int cus = 0;
    const int rc = sar::device_compute_units(&cus);
    if (rc != SAR_OK) return rc;
    const sar::LaunchShape shape = choose_shape(plan, which, cus);
    if (use_single_launch(plan, which)) return sar::run_schedule_fused(plan, which, rank_bufs, stream, shape);
    return sar::run_schedule(plan, which, rank_bufs, stream, shape);
}

}  // namespace

extern "C" {

int stragglar_plan(int n, int straggler_rank, size_t count, int dtype, sar_plan** out) {
    if (!out) return SAR_EINVAL;
    *out = nullptr;
    sar_plan* p = new (std::nothrow) sar_plan;
    if (!p) return SAR_ENOMEM;
    const int st = sar::build_plan(n, straggler_rank, count, dtype, p);
    if (st != SAR_OK) {
        delete p;
        return st;
    }
    *out = p;
    return SAR_OK;
}

void stragglar_plan_destroy(sar_plan* plan) { delete plan; }

int stragglar_plan_num_rounds(const sar_plan* plan, int which) {
    if (!plan || !valid_schedule(which)) return -1;
    return int(plan->sched[which].rounds.size());
}

int stragglar_plan_num_chunks(const sar_plan* plan, int which) {
    if (!plan || !valid_schedule(which)) return -1;
    return plan->sched[which].parts;
}

int stragglar_plan_round(const sar_plan* plan, int which, int round, const sar_op** ops, int* nops) {
    if (!plan || !valid_schedule(which) || !ops || !nops) return SAR_EINVAL;
    const auto& rounds = plan->sched[which].rounds;
    if (round < 0 || size_t(round) >= rounds.size()) return SAR_EINVAL;
    *ops = rounds[round].data();
    *nops = int(rounds[round].size());
    return SAR_OK;
}

int stragglar_plan_chunk(const sar_plan* plan, int which, int chunk, size_t* elem_offset, size_t* elem_len) {
    if (!plan || !valid_schedule(which) || !elem_offset || !elem_len) return SAR_EINVAL;
    const sar_sched& s = plan->sched[which];
    if (chunk < 0 || chunk >= s.parts) return SAR_EINVAL;
    const size_t lo = size_t(chunk) * s.chunk_elems;
    const size_t left = plan->count - lo;
    *elem_offset = lo;
    *elem_len = left < s.chunk_elems ? left : s.chunk_elems;
    return SAR_OK;
}

int stragglar_plan_launch_form(const sar_plan* plan, int which, sar_launch_form* out) {
    if (!plan || !valid_schedule(which) || !out) return SAR_EINVAL;
    const sar_sched& sched = plan->sched[which];
    auto chunk_bytes = [&](int chunk) -> unsigned long long {
        const size_t lo = size_t(chunk) * sched.chunk_elems;
        const size_t left = plan->count - lo;
        return (unsigned long long)((left < sched.chunk_elems ? left : sched.chunk_elems) * plan->elem_bytes);
    };
    *out = sar_launch_form{0, 0, 0, 0};
    const sar::LaunchShape shape = choose_shape(plan, which, 0);
    if (use_single_launch(plan, which)) {
        out->form = shape.fused_split ? 3 : 2;
        out->launches = sar::fused_launches(plan, which, shape.fused_split, shape.fused_sum_to_all || shape.fused_chain);
        for (int c = 0; c < sched.parts; ++c) {
            const std::vector<sar_chunk_op>& ops = sched.by_chunk[c];
            const size_t run = shape.fused_split ? size_t(sched.cut[c]) : ops.size();
            for (size_t k = 0; k < run; ++k) {
                const sar_chunk_op& op = ops[k];
                const int loads = (op.forward ? 0 : 1) + (op.kind != SAR_COPY ? 1 : 0);
                const int stores = (op.dead ? 0 : 1) + (op.kind == SAR_REDUCE_EXCHANGE ? 1 : 0);
                out->bytes_loaded += loads * chunk_bytes(c);
                out->bytes_stored += stores * chunk_bytes(c);
            }
            if (shape.fused_split) {   // the broadcast fetches the value once and stores it to every destination
                out->bytes_loaded += chunk_bytes(c);
                out->bytes_stored += sched.dests * chunk_bytes(c);
            }
        }
        return SAR_OK;
    }
    if (shape.merge_copies && !sched.grouped.empty()) {
        out->form = 1;
        for (const auto& groups : sched.grouped)
            for (const sar_group_op& g : groups) {
                out->bytes_loaded += (g.kind == SAR_COPY ? 1 : 2) * chunk_bytes(g.chunk);
                out->bytes_stored += (g.kind == SAR_REDUCE_EXCHANGE ? 2 : __builtin_popcount(g.dst_mask)) * chunk_bytes(g.chunk);
            }
    } else {
        for (const auto& ops : sched.rounds)
            for (const sar_op& op : ops) {
                out->bytes_loaded += (op.op == SAR_COPY ? 1 : 2) * chunk_bytes(op.chunk);
                out->bytes_stored += (op.op == SAR_REDUCE_EXCHANGE ? 2 : 1) * chunk_bytes(op.chunk);
            }
    }
    return sar::run_schedule(plan, which, nullptr, nullptr, shape, &out->launches);
}

int stragglar_allreduce(const sar_plan* plan, void* const* rank_bufs, void* hip_stream, void* straggler_ready) {
    // Nothing to wait for between the phases: one launch can take every tile through both - unless
    // the completion on its own would take the split form, whose rank-by-rank stores beat the
    // one launch's n-stream stores by more than the second launch costs (32 ranks, 64 MiB each:
    // 0.355 + 0.365 ms for the two calls against 0.775 ms).
    const bool split_completion = plan && tune(plan, SAR_TUNE_FUSED_SPLIT) != 0 && tune(plan, SAR_TUNE_FUSE_ROUNDS) != 0 &&
                                  sar::can_split(plan, SAR_SCHED_COMPLETION) && split_pays(plan, SAR_SCHED_COMPLETION);
    if (plan && !straggler_ready && !split_completion && use_single_launch(plan, SAR_SCHED_ALLREDUCE))
        return run(plan, SAR_SCHED_ALLREDUCE, rank_bufs, hip_stream);
    int st = run(plan, SAR_SCHED_PRECONDITION, rank_bufs, hip_stream);
    if (st != SAR_OK) return st;
    if (straggler_ready) {
        st = sar::stream_wait_event(hip_stream, straggler_ready);
        if (st != SAR_OK) return st;
    }
    return run(plan, SAR_SCHED_COMPLETION, rank_bufs, hip_stream);
}

int stragglar_phase1_reducescatter(const sar_plan* plan, void* const* rank_bufs, void* hip_stream) {
    return run(plan, SAR_SCHED_PRECONDITION, rank_bufs, hip_stream);
}

int stragglar_phase2_complete(const sar_plan* plan, void* const* rank_bufs, void* hip_stream) {
    return run(plan, SAR_SCHED_COMPLETION, rank_bufs, hip_stream);
}

int ring_allreduce(const sar_plan* plan, void* const* rank_bufs, void* hip_stream) {
    return run(plan, SAR_SCHED_RING, rank_bufs, hip_stream);
}

int rhd_allreduce(const sar_plan* plan, void* const* rank_bufs, void* hip_stream) {
    if (plan && plan->log2n < 0) return SAR_EUNSUPPORTED;   // recursive halving needs a power of two
    return run(plan, SAR_SCHED_RHD, rank_bufs, hip_stream);
}

int broadcast_phase1_allreduce(const sar_plan* plan, void* const* rank_bufs, void* hip_stream) {
    return run(plan, SAR_SCHED_BCAST_PRECONDITION, rank_bufs, hip_stream);
}

int broadcast_phase2_complete(const sar_plan* plan, void* const* rank_bufs, void* hip_stream) {
    return run(plan, SAR_SCHED_BCAST_COMPLETION, rank_bufs, hip_stream);
}

int stragglar_delay(unsigned long long nanoseconds, void* hip_stream) {
    if (nanoseconds > 1000000000ull) return SAR_EINVAL;
    return sar::enqueue_delay(nanoseconds, hip_stream);
}

int stragglar_tune_set(int key, long value) {
    if (!valid_tune_value(key, value)) return SAR_EINVAL;
    g_tune[key].store(value);
    return SAR_OK;
}

long stragglar_tune_get(int key) {   // -1 doubles as the 'automatic' value of several keys
    if (key < 0 || key >= SAR_NUM_TUNABLES) return -1;
    return g_tune[key].load();
}

int stragglar_plan_option_set(sar_plan* plan, int key, long value) {
    if (!plan || key < 0 || key >= SAR_NUM_TUNABLES) return SAR_EINVAL;
    if (value != SAR_OPTION_INHERIT && !valid_tune_value(key, value)) return SAR_EINVAL;
    plan->option[key].store(value);
    return SAR_OK;
}

long stragglar_plan_option_get(const sar_plan* plan, int key) {
    if (!plan || key < 0 || key >= SAR_NUM_TUNABLES) return -1;
    return tune(plan, key);
}

const char* stragglar_strerror(int status) {
    switch (status) {
        case SAR_OK: return "ok";
        case SAR_EINVAL: return "invalid argument";
        case SAR_EUNSUPPORTED: return "unsupported rank count (an even number from 2 to 256 is required)";
        case SAR_ENOMEM: return "out of host memory";
        case SAR_EDEVICE: return "HIP device error";
        default: return "unknown status";
    }
}

}  // extern "C"
