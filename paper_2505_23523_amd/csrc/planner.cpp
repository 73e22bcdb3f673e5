// Host-side schedule planner: the completion rounds of Alg. 1 (power-of-two n)
// and of App. D (other even n), the ring ReduceScatter used as the precondition
// of Sec. 3.1, and the baselines of App. E (ring, recursive halving/doubling,
// Broadcast).  Pure integer work, no GPU.
//
// Alg. 1 - state kept per on-time rank g (paper ranks 0..n-2; the straggler is n-1):
//   active[g]  index of the one active chunk g currently holds (-1: none yet).
// "Active" is Sec. 3.1's definition: reduced with the straggler, not yet on all
// ranks.  The proofs of App. C guarantee one active chunk per on-time rank from
// round log n on, which is why a flat array is enough here.
//
// Choices where Alg. 1 leaves freedom (any valid matching yields the same
// buffers; these make the output deterministic):
//   ramp rounds    senders by (chunk, rank) ascending meet the free ranks
//                  above 2(log n - 1) in ascending order;
//   window ranks   one in Q takes the lowest free P rank outside the window; one
//                  in P takes the free out-of-window Q rank with the oldest
//                  chunk (ties: lowest rank);
//   the rest       remaining P and Q ascending, pairwise;
//   tail rounds    the straggler joins Q as a sender of c_{n-2}; nothing is
//                  sent to it.
#include <algorithm>
#include <new>

#include "matching.hpp"
#include "plan.hpp"

namespace {

int ilog2_exact(int n) {
    int l = 0;
    while ((1 << l) < n) ++l;
    return (1 << l) == n ? l : -1;
}

// chunk length in elements, or 0 if some chunk would be empty
size_t chunk_len(size_t count, int parts, size_t elem_bytes) {
    const size_t quantum = 16 / elem_bytes;
    size_t per = (count + parts - 1) / parts;
    per = (per + quantum - 1) / quantum * quantum;
    if (per * static_cast<size_t>(parts - 1) >= count) return 0;
    return per;
}

struct Relabel {
    int n, straggler;
    int32_t operator()(int logical) const {
        if (logical == n - 1) return straggler;
        return logical + (logical >= straggler ? 1 : 0);
    }
};

void emit(std::vector<sar_op>& ops, const Relabel& phys, int src, int dst, int chunk, int kind) {
    ops.push_back(sar_op{phys(src), phys(dst), chunk, kind});
}

// Alg. 1.
void build_completion(int n, int L, const Relabel& phys, sar_sched& out) {
    const int sigma = n - 1;
    const int nrounds = n + L - 2;
    std::vector<int> active(n, -1);
    std::vector<char> taken(n);
    std::vector<int> P, Q;
    std::vector<std::pair<int, int>> gained;  // (rank, chunk) received this round

    out.rounds.assign(nrounds, {});
    for (int r = 0; r < nrounds; ++r) {
        std::vector<sar_op>& ops = out.rounds[r];
        std::fill(taken.begin(), taken.end(), 0);
        gained.clear();

        if (r < n - 1) {  // straggler pairing: c_r becomes fully reduced on r and sigma
            emit(ops, phys, r, sigma, r, SAR_REDUCE_EXCHANGE);
            taken[r] = taken[sigma] = 1;
        }

        if (r > 0 && r < L) {
            // ramp: c_{r-1} goes to rank r-1+log n; every other holder feeds a free high rank
            emit(ops, phys, r - 1, r - 1 + L, r - 1, SAR_COPY);
            gained.emplace_back(r - 1 + L, r - 1);
            taken[r - 1] = taken[r - 1 + L] = 1;
            int next_free = 2 * (L - 1) + 1;
            for (int c = 0; c < r; ++c) {
                for (int h = 0; h < n - 1; ++h) {
                    if (active[h] != c || taken[h]) continue;
                    while (next_free < n - 1 && (active[next_free] >= 0 || taken[next_free])) ++next_free;
                    // Lemma 1 guarantees a free receiver
                    emit(ops, phys, h, next_free, c, SAR_COPY);
                    gained.emplace_back(next_free, c);
                    taken[h] = taken[next_free] = 1;
                }
            }
        } else if (r >= L) {
            const int oldest = r - L;
            const int win_lo = r + 1, win_hi = std::min(r + L, n - 2);
            auto in_window = [&](int g) { return g >= win_lo && g <= win_hi; };
            auto chunk_of = [&](int g) { return g == sigma ? n - 2 : active[g]; };
            auto pair_up = [&](int p, int q) {
                if (q != sigma) emit(ops, phys, p, q, oldest, SAR_COPY);
                emit(ops, phys, q, p, chunk_of(q), SAR_COPY);
                gained.emplace_back(p, chunk_of(q));
                taken[p] = taken[q] = 1;
            };
            // window ranks first, ascending
            for (int g = win_lo; g <= win_hi; ++g) {
                if (taken[g]) continue;
                if (active[g] == oldest) {  // g in P_r: needs an old enough chunk from outside
                    int best = -1;
                    for (int q = 0; q < n - 1; ++q) {
                        if (taken[q] || in_window(q) || active[q] == oldest) continue;
                        if (best < 0 || active[q] < active[best]) best = q;
                    }
                    if (best >= 0) pair_up(g, best);   // always found for the n this is built for
                } else {                    // g in Q_r: any free P rank outside the window
                    for (int p = 0; p < n - 1; ++p) {
                        if (taken[p] || in_window(p) || active[p] != oldest) continue;
                        pair_up(p, g);
                        break;
                    }
                }
            }
            // everyone else: ascending P with ascending Q (sigma, when eligible, is last)
            P.clear();
            Q.clear();
            for (int g = 0; g < n - 1; ++g) {
                if (taken[g]) continue;
                (active[g] == oldest ? P : Q).push_back(g);
            }
            if (r >= n - 1) Q.push_back(sigma);
            for (size_t i = 0; i < P.size() && i < Q.size(); ++i) pair_up(P[i], Q[i]);
        }

        // bookkeeping for the next round
        if (r >= L)
            for (int g = 0; g < n - 1; ++g)
                if (active[g] == r - L) active[g] = -1;
        if (r < n - 1) active[r] = r;
        for (auto& gc : gained) active[gc.first] = gc.second;
    }
}

// Completion for an even n that is not a power of two (App. D).  Ranks can hold
// several chunks that others lack, so each round is a maximum-weight matching on
// the free ranks: an edge weighs 2 if both ends hold a reduced chunk the other
// lacks, 1 if only one does.  The straggler pairings (rank r with the straggler
// in round r) stay as in Alg. 1; once the straggler has met every rank it joins
// the graph as a pure sender.
//
// What the paper leaves open, and what is done here:
//   which chunk an edge carries   the newest one the sender holds and the receiver lacks;
//   which maximum matching        the one that also maximises a small bonus - rarer
//                                 chunks and needier receivers first: a transfer
//                                 of chunk c to rank d scores (n - holders of c)
//                                 + (reduced chunks d still lacks) - scaled so
//                                 it can never outweigh an edge;
//   the matching algorithm        up to 20 ranks the exact recursion over subsets,
//                                 whose choice among equally heavy matchings is
//                                 fixed; above, the blossom algorithm.
struct ChunkSet {                 // chunks 0..254
    uint64_t w[4] = {0, 0, 0, 0};
    void add(int c) { w[c >> 6] |= uint64_t(1) << (c & 63); }
    bool has(int c) const { return (w[c >> 6] >> (c & 63)) & 1u; }
    bool operator==(const ChunkSet& o) const { return w[0] == o.w[0] && w[1] == o.w[1] && w[2] == o.w[2] && w[3] == o.w[3]; }
    // highest chunk in *this and not in o, or -1
    int newest_missing_in(const ChunkSet& o) const {
        for (int k = 3; k >= 0; --k) {
            const uint64_t d = w[k] & ~o.w[k];
            if (d) return k * 64 + 63 - __builtin_clzll(d);
        }
        return -1;
    }
};

void build_completion_matching(int n, const Relabel& phys, sar_sched& out) {
    const int sigma = n - 1;
    const int nchunks = n - 1;
    ChunkSet all;
    for (int c = 0; c < nchunks; ++c) all.add(c);
    constexpr int64_t kEdge = int64_t(1) << 20;   // bonuses of one matching stay far below this

    std::vector<ChunkSet> full(n);                // reduced chunks each rank holds
    std::vector<int> holders(nchunks), lacks(n), verts, mate;
    std::vector<int> carry;                       // carry[a * k + b]: chunk verts[a] would send verts[b], or -1
    std::vector<int64_t> weight;

    for (int r = 0;; ++r) {
        std::vector<sar_op> ops;
        std::vector<char> busy(n, 0);
        if (r < n - 1) {
            emit(ops, phys, r, sigma, r, SAR_REDUCE_EXCHANGE);
            busy[r] = busy[sigma] = 1;
        }
        // chunks 0 .. r-1 are reduced by now: who holds them, who lacks how many
        const int reduced = std::min(r, nchunks);
        std::fill(holders.begin(), holders.end(), 0);
        std::fill(lacks.begin(), lacks.end(), 0);
        for (int g = 0; g < n; ++g)
            for (int c = 0; c < reduced; ++c) {
                const bool h = full[g].has(c);
                holders[c] += h;
                lacks[g] += !h;
            }
        verts.clear();
        for (int g = 0; g < n; ++g)
            if (!busy[g]) verts.push_back(g);
        const int k = int(verts.size());

        carry.assign(size_t(k) * k, -1);
        weight.assign(size_t(k) * k, 0);
        for (int a = 0; a < k; ++a)
            for (int b = 0; b < k; ++b)
                if (a != b) carry[size_t(a) * k + b] = full[verts[a]].newest_missing_in(full[verts[b]]);
        auto bonus = [&](int chunk, int dst) -> int64_t {
            return chunk < 0 ? 0 : (n - holders[chunk]) + lacks[dst];
        };
        for (int a = 0; a < k; ++a)
            for (int b = a + 1; b < k; ++b) {
                const int ab = carry[size_t(a) * k + b], ba = carry[size_t(b) * k + a];
                const int edges = (ab >= 0) + (ba >= 0);
                if (!edges) continue;
                const int64_t w = edges * kEdge + bonus(ab, verts[b]) + bonus(ba, verts[a]);
                weight[size_t(a) * k + b] = weight[size_t(b) * k + a] = w;
            }

        if (k <= sar::kMaxSubsetVertices)
            sar::max_weight_matching_subsets(k, weight, mate);
        else
            sar::max_weight_matching_blossom(k, weight, mate);

        std::vector<std::pair<int, int>> gained;
        for (int a = 0; a < k; ++a) {
            const int b = mate[a];
            if (b < a) continue;                  // unmatched (-1) or already emitted
            const int ab = carry[size_t(a) * k + b], ba = carry[size_t(b) * k + a];
            if (ab >= 0) {
                emit(ops, phys, verts[a], verts[b], ab, SAR_COPY);
                gained.emplace_back(verts[b], ab);
            }
            if (ba >= 0) {
                emit(ops, phys, verts[b], verts[a], ba, SAR_COPY);
                gained.emplace_back(verts[a], ba);
            }
        }
        if (r < n - 1) {
            full[r].add(r);
            full[sigma].add(r);
        }
        for (auto& gc : gained) full[gc.first].add(gc.second);
        out.rounds.push_back(std::move(ops));

        bool done = r >= n - 2;
        for (int g = 0; g < n && done; ++g) done = full[g] == all;
        if (done) break;
    }
}

void build_ring_reduce_scatter(int m, const Relabel* phys, sar_sched& out) {
    for (int t = 0; t + 1 < m; ++t) {
        std::vector<sar_op> ops;
        for (int i = 0; i < m; ++i) {
            const int dst = (i + 1) % m;
            const int chunk = ((i - t - 1) % m + m) % m;
            ops.push_back(sar_op{phys ? (*phys)(i) : i, phys ? (*phys)(dst) : dst, chunk, SAR_REDUCE});
        }
        out.rounds.push_back(std::move(ops));
    }
}

void build_ring_all_gather(int m, sar_sched& out) {
    for (int t = 0; t + 1 < m; ++t) {
        std::vector<sar_op> ops;
        for (int i = 0; i < m; ++i)
            ops.push_back(sar_op{i, (i + 1) % m, ((i - t) % m + m) % m, SAR_COPY});
        out.rounds.push_back(std::move(ops));
    }
}

// Recursive halving / doubling (App. E, "Butterfly") on n chunks.  Halving step k
// pairs rank i with i ^ (n >> (k+1)); of the n >> k chunks rank i is still
// responsible for (those sharing its top k index bits) it keeps the half that
// also shares bit k and sends the other half, which the partner adds to its own.
// After log n steps rank i holds the reduced chunk i; the doubling steps mirror
// the halving steps in reverse and copy the owned blocks back out.
void build_rhd(int n, int L, sar_sched& out) {
    for (int k = 0; k < L; ++k) {
        const int d = n >> (k + 1);
        std::vector<sar_op> ops;
        for (int i = 0; i < n; ++i) {
            const int p = i ^ d;
            const int base = p & ~(d - 1);      // block of d chunks the partner keeps
            for (int c = base; c < base + d; ++c) ops.push_back(sar_op{i, p, c, SAR_REDUCE});
        }
        out.rounds.push_back(std::move(ops));
    }
    for (int k = L - 1; k >= 0; --k) {
        const int d = n >> (k + 1);
        std::vector<sar_op> ops;
        for (int i = 0; i < n; ++i) {
            const int p = i ^ d;
            const int base = i & ~(d - 1);      // block of d chunks rank i owns by now
            for (int c = base; c < base + d; ++c) ops.push_back(sar_op{i, p, c, SAR_COPY});
        }
        out.rounds.push_back(std::move(ops));
    }
}

// The straggler-aware Broadcast baseline (App. E).  Precondition: an AllReduce
// among the n-1 on-time ranks (ring reduce-scatter, then ring all-gather), done
// while the straggler is late.  Completion: the straggler swaps its whole buffer
// with on-time rank 0 (both end fully reduced), then the holders double every
// round - each sends the whole buffer to the lowest rank that lacks it - log n
// rounds of s bytes in all.
void build_broadcast_precondition(int m, const Relabel& phys, sar_sched& out) {
    build_ring_reduce_scatter(m, &phys, out);
    for (int t = 0; t + 1 < m; ++t) {
        std::vector<sar_op> ops;
        for (int i = 0; i < m; ++i)
            ops.push_back(sar_op{phys(i), phys((i + 1) % m), ((i - t) % m + m) % m, SAR_COPY});
        out.rounds.push_back(std::move(ops));
    }
}

void build_broadcast_completion(int n, const Relabel& phys, sar_sched& out) {
    const int sigma = n - 1;
    std::vector<sar_op> ops;
    for (int c = 0; c < n - 1; ++c) ops.push_back(sar_op{phys(0), phys(sigma), c, SAR_REDUCE_EXCHANGE});
    out.rounds.push_back(std::move(ops));
    std::vector<int> holders{0, sigma};
    std::vector<char> has(n, 0);
    has[0] = has[sigma] = 1;
    while (int(holders.size()) < n) {
        ops.clear();
        std::vector<int> senders = holders;
        std::sort(senders.begin(), senders.end());
        int next = 0;
        for (int h : senders) {
            while (next < n && has[next]) ++next;
            if (next >= n) break;
            for (int c = 0; c < n - 1; ++c) ops.push_back(sar_op{phys(h), phys(next), c, SAR_COPY});
            has[next] = 1;
            holders.push_back(next);
        }
        out.rounds.push_back(ops);
    }
}

// Set simulation of a completion schedule (logical ranks): every COPY moves a
// reduced chunk its sender holds to a rank that lacks it, every rank ends with all
// chunks.  A generator bug must not reach a GPU as a silently wrong AllReduce.
bool completion_is_valid(int n, const Relabel& phys, const sar_sched& sched) {
    std::vector<int> logical(n);
    for (int l = 0; l < n; ++l) logical[phys(l)] = l;
    std::vector<std::vector<char>> has(n, std::vector<char>(n - 1, 0));
    for (const std::vector<sar_op>& ops : sched.rounds) {
        std::vector<std::pair<int, int>> gained;
        for (const sar_op& op : ops) {
            const int s = logical[op.src], d = logical[op.dst];
            if (op.op == SAR_COPY) {
                if (!has[s][op.chunk] || has[d][op.chunk]) return false;
                gained.emplace_back(d, op.chunk);
            } else if (op.op == SAR_REDUCE_EXCHANGE) {
                if (d != n - 1 || s != op.chunk || has[s][op.chunk] || has[d][op.chunk]) return false;
                gained.emplace_back(s, op.chunk);
                gained.emplace_back(d, op.chunk);
            } else {
                return false;
            }
        }
        for (auto& gc : gained) has[gc.first][gc.second] = 1;
    }
    for (int g = 0; g < n; ++g)
        for (int c = 0; c < n - 1; ++c)
            if (!has[g][c]) return false;
    return true;
}

// Per chunk index, the ops in round order.  An op is marked `forward` when its
// source cell holds the value the previous op on this chunk index left in the
// executing thread's registers: `same[chunk]` is the set of ranks whose cell
// equals that value.  A COPY adds its destination (and, if it had to load,
// restarts the set from its source); a reducing op produces a new value.
void index_by_chunk(int n, sar_sched& sched) {
    sched.by_chunk.assign(sched.parts, {});
    std::vector<std::vector<char>> same(sched.parts, std::vector<char>(n, 0));
    for (const std::vector<sar_op>& ops : sched.rounds) {
        for (const sar_op& op : ops) {
            std::vector<char>& held = same[op.chunk];
            const bool forward = held[op.src] != 0;
            if (op.op == SAR_COPY) {
                if (!forward) {
                    std::fill(held.begin(), held.end(), 0);
                    held[op.src] = 1;
                }
                held[op.dst] = 1;
            } else {
                std::fill(held.begin(), held.end(), 0);
                held[op.dst] = 1;
                if (op.op == SAR_REDUCE_EXCHANGE) held[op.src] = 1;
            }
            sched.by_chunk[op.chunk].push_back(
                sar_chunk_op{uint8_t(op.src), uint8_t(op.dst), uint8_t(op.op), uint8_t(forward), 0, 0});
        }
    }
}

// Marks the stores the single-launch kernel may drop.  Walking on from an op's
// store to cell (dst, chunk): a later op that loads the cell (as a source it does
// not take from registers, or as the destination operand of a reducing op) needs
// it; a later op that overwrites the cell first makes it dead.  A store nothing
// follows is the cell's final content and stays - except in the precondition,
// whose postcondition defines, per chunk index, only the cell its last op writes
// (Sec. 3.1: rank g ends with the partially reduced c_g; the other chunks of the
// on-time ranks are scratch that the completion overwrites without reading).
// Both stores of an exchange always stay.
void mark_dead_stores(sar_sched& sched, bool only_last_store_defined) {
    for (std::vector<sar_chunk_op>& ops : sched.by_chunk) {
        for (size_t k = 0; k < ops.size(); ++k) {
            if (ops[k].kind == SAR_REDUCE_EXCHANGE) continue;
            const uint8_t cell = ops[k].dst;
            bool dead = only_last_store_defined && k + 1 < ops.size();
            for (size_t j = k + 1; j < ops.size(); ++j) {
                const sar_chunk_op& later = ops[j];
                const bool loads = (later.src == cell && !later.forward) ||
                                   (later.kind != SAR_COPY && later.dst == cell);
                const bool overwrites = later.dst == cell ||
                                        (later.kind == SAR_REDUCE_EXCHANGE && later.src == cell);
                if (loads) {
                    dead = false;
                    break;
                }
                if (overwrites) {
                    dead = true;
                    break;
                }
            }
            ops[k].dead = dead;
        }
        // reduce chains (a ring's hops): which operand loads may be hoisted over the ops before
        for (size_t k = 0; k < ops.size(); ++k) {
            bool chained = ops[k].kind == SAR_REDUCE && ops[k].forward;
            for (size_t j = k >= 3 ? k - 3 : 0; j < k && chained; ++j) {
                const bool writes_dst = !ops[j].dead && ops[j].dst == ops[k].dst;
                const bool writes_src = ops[j].kind == SAR_REDUCE_EXCHANGE && ops[j].src == ops[k].dst;
                if (writes_dst || writes_src) chained = false;
            }
            ops[k].chained = chained;
        }
    }
}

// Merges, per round, the copies that hand on the same value (see sar_group_op).  "Same value" is
// established by following every cell's content symbolically: each cell (rank, chunk) starts
// with a value of its own, a reducing op gives its destination (an exchange: both ends) a new
// one, a copy hands its source's on.  Copies of one chunk index whose sources hold the same
// value form one group, read from the first of those sources.  No op of a round reads a cell
// another op of the round writes, so the values at the start of the round decide.
void group_same_value_copies(int n, sar_sched& sched) {
    sched.grouped.clear();
    if (n > 32) return;
    std::vector<int> value(size_t(n) * sched.parts);
    for (size_t i = 0; i < value.size(); ++i) value[i] = int(i);
    int fresh = int(value.size());
    struct Key { int chunk, value; size_t group; };
    for (const std::vector<sar_op>& ops : sched.rounds) {
        std::vector<sar_group_op> groups;
        std::vector<Key> keys;
        for (const sar_op& op : ops) {
            const uint32_t bit = uint32_t(1) << op.dst;
            if (op.op == SAR_COPY) {
                const int v = value[size_t(op.src) * sched.parts + op.chunk];
                size_t g = groups.size();
                for (const Key& k : keys)
                    if (k.chunk == op.chunk && k.value == v) g = k.group;
                if (g == groups.size()) {
                    keys.push_back(Key{op.chunk, v, g});
                    groups.push_back(sar_group_op{uint8_t(SAR_COPY), uint8_t(op.src), uint8_t(op.chunk), 0});
                }
                groups[g].dst_mask |= bit;
            } else {
                groups.push_back(sar_group_op{uint8_t(op.op), uint8_t(op.src), uint8_t(op.chunk), bit});
            }
        }
        for (const sar_op& op : ops) {   // values after the round (sources are read as of its start)
            int& dst = value[size_t(op.dst) * sched.parts + op.chunk];
            int& src = value[size_t(op.src) * sched.parts + op.chunk];
            if (op.op == SAR_COPY) {
                dst = src;
            } else {
                dst = fresh++;
                if (op.op == SAR_REDUCE_EXCHANGE) src = dst;
            }
        }
        sched.grouped.push_back(std::move(groups));
    }
}

// Finds the split described at sar_sched::cut (leaves it empty if the schedule has none).
void split_off_trailing_copies(int n, sar_sched& sched) {
    sched.cut.clear();
    sched.route.clear();
    sched.dests = 0;
    sched.sum_to_all = false;
    std::vector<uint16_t> cut;
    std::vector<uint32_t> route;
    int dests = -1;
    for (const std::vector<sar_chunk_op>& ops : sched.by_chunk) {
        size_t k = ops.size();
        while (k > 0 && ops[k - 1].kind == SAR_COPY && ops[k - 1].forward) --k;
        if (k == 0 || k == ops.size()) return;           // nothing produces the value / nothing hands it on
        const sar_chunk_op& last = ops[k - 1];
        if (last.dead) return;                            // the value never reaches memory
        std::vector<char> written(n, 0);
        for (size_t j = k; j < ops.size(); ++j) written[ops[j].dst] = 1;
        if (written[last.dst]) return;
        int excluded[2], nex = 0;
        for (int r = 0; r < n; ++r)
            if (!written[r]) {
                if (nex == 2) return;
                excluded[nex++] = r;
            }
        if (nex == 1) excluded[1] = excluded[0];
        if (dests >= 0 && dests != n - nex) return;
        dests = n - nex;
        cut.push_back(uint16_t(k));
        route.push_back(uint32_t(last.dst) | uint32_t(excluded[0]) << 8 | uint32_t(excluded[1]) << 16);
    }
    if (dests <= 0) return;
    sched.cut = std::move(cut);
    sched.route = std::move(route);
    sched.dests = dests;
    sched.sum_to_all = dests == n - 2;
    for (size_t c = 0; c < sched.by_chunk.size() && sched.sum_to_all; ++c) {
        const sar_chunk_op& first = sched.by_chunk[c][0];
        if (sched.cut[c] != 1 || first.kind != SAR_REDUCE_EXCHANGE || first.forward) sched.sum_to_all = false;
    }
}

// Recognises schedules whose chunk indices all start with a reduce chain around one ring of ranks
// (sar_sched::chain_ring), followed by nothing or by copies of the sum to every other rank of the ring.
void find_reduce_chains(int n, sar_sched& sched) {
    sched.chain_ring.clear();
    sched.chain_start.clear();
    sched.chain_to_all = false;
    std::vector<uint8_t> ring;
    std::vector<uint16_t> start;
    std::vector<int> where;       // position of a rank in the ring, -1 if it is not part of it
    int to_all = -1;
    for (const std::vector<sar_chunk_op>& ops : sched.by_chunk) {
        size_t k = 0;
        std::vector<uint8_t> walk;
        while (k < ops.size() && ops[k].kind == SAR_REDUCE && (k == 0 ? !ops[k].forward : ops[k].forward && ops[k].src == ops[k - 1].dst)) {
            if (k == 0) walk.push_back(ops[k].src);
            walk.push_back(ops[k].dst);
            ++k;
        }
        if (k == 0) return;
        for (size_t j = 0; j < k; ++j)
            if (bool(ops[j].dead) != (j + 1 < k)) return;         // exactly the last store is observable
        // what follows: nothing, or forwarded copies to each of the other n - 1 ranks once
        std::vector<char> written(n, 0);
        for (size_t j = k; j < ops.size(); ++j) {
            if (ops[j].kind != SAR_COPY || !ops[j].forward || ops[j].dead || written[ops[j].dst] || ops[j].dst == walk.back()) return;   // once each
            written[ops[j].dst] = 1;
        }
        const int tail = ops.size() == k ? 0 : 1;
        if (to_all >= 0 && to_all != tail) return;
        to_all = tail;
        if (ring.empty()) {
            ring = walk;
            where.assign(n, -1);
            for (size_t j = 0; j < ring.size(); ++j) {
                if (where[ring[j]] >= 0) return;                   // a rank twice
                where[ring[j]] = int(j);
            }
        }
        if (tail) {                                                // ... to exactly the ring's other members
            if (ops.size() - k != ring.size() - 1) return;
            for (size_t j = k; j < ops.size(); ++j)
                if (where[ops[j].dst] < 0) return;
        }
        if (walk.size() != ring.size() || where[walk[0]] < 0) return;
        const size_t s0 = size_t(where[walk[0]]);
        for (size_t j = 0; j < walk.size(); ++j)
            if (walk[j] != ring[(s0 + j) % ring.size()]) return;
        start.push_back(uint16_t(s0));
    }
    if (ring.size() < 2) return;
    sched.chain_ring = std::move(ring);
    sched.chain_start = std::move(start);
    sched.chain_to_all = to_all == 1;
}

}  // namespace

int sar::build_plan(int n, int straggler, size_t count, int dtype, sar_plan* p) {
    if (n < 2 || n > SAR_MAX_RANKS) return n >= 2 ? SAR_EUNSUPPORTED : SAR_EINVAL;
    const int L = ilog2_exact(n);
    // odd n is undefined in the paper; even non-powers of two use App. D's generator
    if (L < 0 && n % 2 != 0) return SAR_EUNSUPPORTED;
    if (straggler < 0 || straggler >= n || count == 0) return SAR_EINVAL;
    if (dtype != SAR_I32 && dtype != SAR_F32 && dtype != SAR_BF16) return SAR_EINVAL;

    const size_t eb = dtype_bytes(dtype);
    if (count > SIZE_MAX / eb / 2) return SAR_EINVAL;
    const size_t per_sar = chunk_len(count, n - 1, eb);
    const size_t per_ring = chunk_len(count, n, eb);
    if (per_sar == 0 || per_ring == 0) return SAR_EINVAL;

    try {
        p->n = n;
        p->log2n = L;
        p->straggler = straggler;
        p->dtype = dtype;
        p->count = count;
        p->elem_bytes = eb;
        const Relabel phys{n, straggler};

        sar_sched& pre = p->sched[SAR_SCHED_PRECONDITION];
        pre.parts = n - 1;
        pre.chunk_elems = per_sar;
        build_ring_reduce_scatter(n - 1, &phys, pre);

        sar_sched& comp = p->sched[SAR_SCHED_COMPLETION];
        comp.parts = n - 1;
        comp.chunk_elems = per_sar;
        if (L >= 0)
            build_completion(n, L, phys, comp);
        else
            build_completion_matching(n, phys, comp);
        if (!completion_is_valid(n, phys, comp)) return SAR_EUNSUPPORTED;

        sar_sched& ring = p->sched[SAR_SCHED_RING];
        ring.parts = n;
        ring.chunk_elems = per_ring;
        build_ring_reduce_scatter(n, nullptr, ring);
        build_ring_all_gather(n, ring);

        sar_sched& rhd = p->sched[SAR_SCHED_RHD];
        rhd.parts = n;
        rhd.chunk_elems = per_ring;
        if (L >= 0) build_rhd(n, L, rhd);   // halving needs a power of two: no rounds otherwise

        sar_sched& bpre = p->sched[SAR_SCHED_BCAST_PRECONDITION];
        bpre.parts = n - 1;
        bpre.chunk_elems = per_sar;
        build_broadcast_precondition(n - 1, phys, bpre);

        sar_sched& bcomp = p->sched[SAR_SCHED_BCAST_COMPLETION];
        bcomp.parts = n - 1;
        bcomp.chunk_elems = per_sar;
        build_broadcast_completion(n, phys, bcomp);

        // both phases back to back, for a call that has no straggler delay to wait for
        sar_sched& both = p->sched[SAR_SCHED_ALLREDUCE];
        both.parts = n - 1;
        both.chunk_elems = per_sar;
        both.rounds = pre.rounds;
        both.rounds.insert(both.rounds.end(), comp.rounds.begin(), comp.rounds.end());

        for (int which = 0; which < SAR_NUM_SCHEDULES; ++which) {
            index_by_chunk(n, p->sched[which]);
            mark_dead_stores(p->sched[which], which == SAR_SCHED_PRECONDITION);
            group_same_value_copies(n, p->sched[which]);
            split_off_trailing_copies(n, p->sched[which]);
            find_reduce_chains(n, p->sched[which]);
        }
    } catch (const std::bad_alloc&) {
        return SAR_ENOMEM;
    }
    return SAR_OK;
}
