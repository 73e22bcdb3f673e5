// Host-only check of the per-chunk op lists the single-launch kernel consumes.
//
// For every schedule of a plan, two simulations on symbolic 64-bit cell values
// (wrapping add as the reduction): (A) the rounds one after the other, every op
// loading and storing; (B) each chunk index's list by itself, taking `forward`
// sources from a register and dropping `dead` stores.  B must leave every cell
// as A does - except after the precondition, where only the cell each chunk's
// last op writes is defined and the others must be either A's value or
// untouched - and must make exactly the loads and stores the byte model states:
//   completion (n+2), precondition n, ring and both phases in one 2n chunk passes per chunk index.
// (C) the rounds with a round's copies of one value merged into one multi-destination op must
// equal A after every round, with the loads the merged byte model states.
// (D) where the planner describes a schedule as reduce chains around one ring of ranks (the
// precondition, the ring AllReduce), that description must reproduce A.
#include <cstdint>
#include <cstdio>
#include <vector>

#include "plan.hpp"

namespace {

uint64_t mix(uint64_t x) {
    x += 0x9E3779B97F4A7C15ull;
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    return x ^ (x >> 31);
}

int check_plan(int n, int straggler) {
    sar_plan plan;
    if (sar::build_plan(n, straggler, size_t(n) * n * 64, SAR_I32, &plan) != SAR_OK) {
        std::printf("n=%d: plan failed\n", n);
        return 1;
    }
    const bool pow2 = plan.log2n >= 0;
    for (int which = 0; which < SAR_NUM_SCHEDULES; ++which) {
        if (which == SAR_SCHED_RHD && !pow2) continue;
        const sar_sched& sc = plan.sched[which];
        const int parts = sc.parts;
        std::vector<uint64_t> init(size_t(n) * parts);
        for (size_t i = 0; i < init.size(); ++i) init[i] = mix(i * 131 + which);
        auto cell = [&](int rank, int chunk) { return size_t(rank) * parts + chunk; };

        std::vector<uint64_t> a = init;
        for (const auto& ops : sc.rounds) {
            std::vector<uint64_t> next = a;   // a round's ops read the state before the round
            for (const sar_op& op : ops) {
                const uint64_t s = a[cell(op.src, op.chunk)], d = a[cell(op.dst, op.chunk)];
                const uint64_t v = op.op == SAR_COPY ? s : s + d;
                next[cell(op.dst, op.chunk)] = v;
                if (op.op == SAR_REDUCE_EXCHANGE) next[cell(op.src, op.chunk)] = v;
            }
            a = next;
        }

        std::vector<uint64_t> b = init;
        std::vector<char> defined(init.size(), which == SAR_SCHED_PRECONDITION ? 0 : 1);
        size_t loads = 0, stores = 0;
        for (int c = 0; c < parts; ++c) {
            uint64_t reg = 0;
            const auto& ops = sc.by_chunk[c];
            for (size_t k = 0; k < ops.size();) {
                // as the kernel does: up to four consecutive `chained` reductions load their
                // operands first, then add and store in list order
                size_t run = 0;
                uint64_t operand[4];
                while (run < 4 && k + run < ops.size() && ops[k + run].chained) {
                    operand[run] = b[cell(ops[k + run].dst, c)];
                    ++run;
                }
                if (run) {
                    for (size_t i = 0; i < run; ++i) {
                        const sar_chunk_op& op = ops[k + i];
                        if (op.kind != SAR_REDUCE || !op.forward) { std::printf("bad chain flag\n"); return 1; }
                        reg += operand[i]; ++loads;
                        if (!op.dead) { b[cell(op.dst, c)] = reg; ++stores; }
                        if (k + i + 1 == ops.size()) defined[cell(op.dst, c)] = 1;
                    }
                    k += run;
                    continue;
                }
                const sar_chunk_op& op = ops[k];
                if (!op.forward) { reg = b[cell(op.src, c)]; ++loads; }
                if (op.kind != SAR_COPY) { reg += b[cell(op.dst, c)]; ++loads; }
                if (!op.dead) { b[cell(op.dst, c)] = reg; ++stores; }
                if (op.kind == SAR_REDUCE_EXCHANGE) { b[cell(op.src, c)] = reg; ++stores; }
                if (k + 1 == ops.size()) defined[cell(op.dst, c)] = 1;
                ++k;
            }
        }
        for (size_t i = 0; i < init.size(); ++i) {
            const bool ok = defined[i] ? b[i] == a[i] : (b[i] == a[i] || b[i] == init[i]);
            if (!ok) {
                std::printf("n=%d straggler=%d schedule %d: cell %zu differs\n", n, straggler, which, i);
                return 1;
            }
        }
        // (C) the rounds with same-value copies merged (up to 32 ranks): a COPY group loads its
        // one source and stores to every destination of its mask.  After EVERY round the cells
        // must equal A's, and the loads must be those of the byte model: one per distinct value
        // copied in a round, two per reducing op.  For Alg. 1 (power-of-two n) the copies' loads
        // sum to D = 5, 20, 59, 154 chunks at n = 4, 8, 16, 32; the stores are unchanged (n per chunk).
        if (n <= 32) {
            if (sc.grouped.size() != sc.rounds.size()) { std::printf("n=%d schedule %d: no merged rounds\n", n, which); return 1; }
            std::vector<uint64_t> ref = init, got = init;
            size_t gloads = 0, gstores = 0, copy_loads = 0, plain_stores = 0;
            for (size_t r = 0; r < sc.rounds.size(); ++r) {
                std::vector<uint64_t> next = ref;
                for (const sar_op& op : sc.rounds[r]) {
                    const uint64_t sv = ref[cell(op.src, op.chunk)], dv = ref[cell(op.dst, op.chunk)];
                    const uint64_t v = op.op == SAR_COPY ? sv : sv + dv;
                    next[cell(op.dst, op.chunk)] = v;
                    if (op.op == SAR_REDUCE_EXCHANGE) next[cell(op.src, op.chunk)] = v;
                    plain_stores += op.op == SAR_REDUCE_EXCHANGE ? 2 : 1;
                }
                ref = next;
                std::vector<uint64_t> gnext = got;
                for (const sar_group_op& g : sc.grouped[r]) {
                    if (g.dst_mask == 0) { std::printf("empty group\n"); return 1; }
                    const uint64_t sv = got[cell(g.src, g.chunk)];
                    ++gloads;
                    if (g.kind == SAR_COPY) {
                        ++copy_loads;
                        for (int d = 0; d < n; ++d)
                            if (g.dst_mask >> d & 1u) { gnext[cell(d, g.chunk)] = sv; ++gstores; }
                        if (n < 32 && (g.dst_mask >> n)) { std::printf("destination beyond n\n"); return 1; }
                    } else {
                        if (g.dst_mask & (g.dst_mask - 1)) { std::printf("reducing op with several destinations\n"); return 1; }
                        const int d = __builtin_ctz(g.dst_mask);
                        const uint64_t v = sv + got[cell(d, g.chunk)];
                        ++gloads;
                        gnext[cell(d, g.chunk)] = v; ++gstores;
                        if (g.kind == SAR_REDUCE_EXCHANGE) { gnext[cell(g.src, g.chunk)] = v; ++gstores; }
                    }
                }
                got = gnext;
                if (got != ref) { std::printf("n=%d straggler=%d schedule %d: merged round %zu differs\n", n, straggler, which, r); return 1; }
            }
            if (gstores != plain_stores) { std::printf("n=%d schedule %d: merged rounds store %zu, plain %zu\n", n, which, gstores, plain_stores); return 1; }
            if (which == SAR_SCHED_COMPLETION && pow2 && n >= 4) {
                const size_t D = n == 4 ? 5 : n == 8 ? 20 : n == 16 ? 59 : 154;
                if (copy_loads != D || gloads != D + 2 * size_t(n - 1)) {
                    std::printf("n=%d completion: %zu copy loads (expected %zu), %zu loads\n", n, copy_loads, D, gloads);
                    return 1;
                }
            }
        } else if (!sc.grouped.empty()) {
            std::printf("n=%d: merged rounds above 32 ranks\n", n);
            return 1;
        }
        // (D) the reduce-chain description: walking the ring from each chunk index's start position,
        // adding as it goes and storing to the last rank (or to every rank of the ring), gives A's cells
        const bool chain_expected = (which == SAR_SCHED_PRECONDITION && n > 2) || which == SAR_SCHED_RING;
        if (chain_expected && sc.chain_ring.empty()) {
            std::printf("n=%d schedule %d: chain shape not recognised\n", n, which);
            return 1;
        }
        if (!sc.chain_ring.empty()) {
            const size_t m = sc.chain_ring.size();
            if (sc.chain_start.size() != size_t(parts) || (chain_expected && sc.chain_to_all != (which == SAR_SCHED_RING))) {
                std::printf("n=%d schedule %d: chain description incomplete\n", n, which);
                return 1;
            }
            for (int c = 0; c < parts; ++c) {
                size_t pos = sc.chain_start[c];
                uint64_t sum = init[cell(sc.chain_ring[pos], c)];
                for (size_t k = 1; k < m; ++k) {
                    pos = (pos + 1) % m;
                    sum += init[cell(sc.chain_ring[pos], c)];
                }
                for (int r = 0; r < n; ++r) {
                    bool in_ring = false;
                    for (uint8_t member : sc.chain_ring) in_ring = in_ring || member == r;
                    const bool written = sc.chain_to_all ? in_ring : r == sc.chain_ring[pos];
                    if (written && a[cell(r, c)] != sum) {
                        std::printf("n=%d schedule %d chunk %d rank %d: the chain walk gives another value\n", n, which, c, r);
                        return 1;
                    }
                }
            }
        }
        size_t want = 0;
        if (which == SAR_SCHED_COMPLETION) want = size_t(n + 2) * parts;
        if (which == SAR_SCHED_PRECONDITION) want = n > 2 ? size_t(n) * parts : 0;
        if (which == SAR_SCHED_RING) want = size_t(2) * n * parts;
        if (which == SAR_SCHED_ALLREDUCE) want = size_t(2) * n * parts;
        if (want && loads + stores != want) {
            std::printf("n=%d schedule %d: %zu chunk passes, expected %zu\n", n, which, loads + stores, want);
            return 1;
        }
    }
    return 0;
}

}  // namespace

int main() {
    int plans = 0;
    for (int n = 2; n <= 64; n += 2)
        for (int straggler : {0, n / 2, n - 1}) {
            if (check_plan(n, straggler)) return 1;
            ++plans;
        }
    for (int n : {96, 128, 254, 256}) {
        if (check_plan(n, 1)) return 1;
        ++plans;
    }
    std::printf("%d plans ok\n", plans);
    return 0;
}
