"""Schedules of the StragglAR AllReduce, written out from the paper.

TEST INFRASTRUCTURE (see the package docstring): plain Python, no blocking,
no sharing with the HIP library's planner.

A schedule is a list of rounds; a round is a list of ops
``(src, dst, chunk, kind)`` over *physical* rank ids:

* ``COPY``             dst[chunk]  = src[chunk]
* ``REDUCE``           dst[chunk]  = rnd(dst[chunk] + src[chunk])
* ``REDUCE_EXCHANGE``  t = rnd(src[chunk] + dst[chunk]); both ranks store t
  (``src`` is the on-time rank, ``dst`` the straggler).

Notation follows Sec. 3.1 / Alg. 1: n ranks, L = log2 n, the straggler is
logical rank sigma = n-1, the buffer is cut into n-1 chunks c_0..c_{n-2},
``A`` maps an active chunk to the set of on-time ranks holding it.

Readings taken where the paper leaves a choice (all value-neutral; any valid
matching gives the same buffers):

* rounds are r = 0 .. n+L-3, i.e. n+L-2 of them (Thm. 1; Alg. 1 "Output");
* ramp rounds (0 < r < L): senders ordered by (chunk, rank), free receivers
  g > 2(L-1) ascending, zipped; ranks L..2L-2 stay reserved for the
  "r-1 -> r-1+L" rule;
* steady rounds: a window rank in Q takes the lowest free P rank outside the
  window; a window rank in P takes the free out-of-window Q rank with the
  oldest (smallest index) active chunk, ties to the lowest rank; then the
  remaining P and Q are zipped in ascending order;
* tail rounds (r >= n-1): sigma joins Q holding c_{n-2}; nothing is sent
  *to* sigma (it already holds every reduced chunk);
* a straggler at physical rank s: on-time ranks keep their order and become
  logical 0..n-2, s becomes logical n-1.
"""

from . import COPY, REDUCE, REDUCE_EXCHANGE


class Unsupported(ValueError):
    """n is not a power of two >= 2 (odd n is undefined in the paper, even
    non-powers of two need the matching-based generator of App. D)."""


def log2_exact(n):
    if n < 2:
        raise ValueError("n must be >= 2")
    if n & (n - 1):
        raise Unsupported("n must be a power of two")
    return n.bit_length() - 1


def chunk_layout(count, parts, elem_bytes, align_bytes=16):
    """Cut ``count`` elements into ``parts`` chunks (Sec. 3.1: equal chunks of
    s/(n-1); App. E: s/n for ring).  Chunk length is ceil(count/parts) rounded
    up to ``align_bytes`` so every chunk starts aligned; the last chunk takes
    what is left.  Returns [(offset, length)] in elements; ValueError if a
    chunk would be empty."""
    if count <= 0 or parts <= 0:
        raise ValueError("count and parts must be positive")
    per = -(-count // parts)
    q = max(1, align_bytes // elem_bytes)
    per = -(-per // q) * q
    out = []
    for k in range(parts):
        lo = k * per
        hi = min(lo + per, count)
        if hi <= lo:
            raise ValueError("count too small: chunk %d would be empty" % k)
        out.append((lo, hi - lo))
    return out


def to_physical(logical, n, straggler):
    """Order-preserving relabel (Sec. 3.1, "by symmetry")."""
    if logical == n - 1:
        return straggler
    return logical + (1 if logical >= straggler else 0)


# --------------------------------------------------------------------------
# Precondition: ReduceScatter among the n-1 on-time ranks (Sec. 3.1).
# The paper calls a library ReduceScatter; a ring over m = n-1 ranks has the
# beta-cost (n-2)/(n-1) s that Sec. 3.2 quotes for it.
# --------------------------------------------------------------------------
def rs_precondition_logical(n):
    if n < 2:
        raise ValueError("n must be >= 2")
    m = n - 1
    rounds = []
    for t in range(m - 1):
        ops = []
        for i in range(m):
            ops.append((i, (i + 1) % m, (i - t - 1) % m, REDUCE))
        rounds.append(ops)
    return rounds


# --------------------------------------------------------------------------
# Completion: Alg. 1.
# --------------------------------------------------------------------------
def completion_logical(n, trace=None, window_rule=True):
    """Rounds of Alg. 1 over logical ranks.  If ``trace`` is a list, a
    snapshot (r, A-before-round, P_r, Q_r) is appended per round so tests can
    check Lemma 1 and invariant I(r).  ``window_rule=False`` skips the
    critical-window step; it exists only so a test can show that the checks
    notice its absence."""
    L = log2_exact(n)
    sigma = n - 1
    last = n - 2                      # index of the final chunk c_{n-2}
    A = {}                            # active chunk -> set of on-time holders
    act = {}                          # on-time rank -> its one active chunk
    schedule = []

    for r in range(n + L - 2):
        ops = []
        busy = set()
        received = []                 # (rank, chunk) learnt this round
        A_before = {c: set(h) for c, h in A.items()}

        if r < n - 1:                 # straggler pairing
            ops.append((r, sigma, r, REDUCE_EXCHANGE))
            busy.update((r, sigma))

        P_r, Q_r = [], []
        if 0 < r < L:                 # ramp ("Phase 1" of Sec. 3.1)
            ops.append((r - 1, r - 1 + L, r - 1, COPY))
            received.append((r - 1 + L, r - 1))
            busy.update((r - 1, r - 1 + L))
            senders = sorted((c, h) for c, hs in A.items() for h in hs
                             if h not in busy)
            free = [g for g in range(2 * (L - 1) + 1, n - 1)
                    if g not in act and g not in busy]
            assert len(free) >= len(senders), "Lemma 1 violated"
            for (c, h), g in zip(senders, free):
                ops.append((h, g, c, COPY))
                received.append((g, c))
        elif r >= L:                  # steady / tail ("Phase 2" + Remark 1)
            oldest = r - L
            assert min(A) == oldest
            P = sorted(h for h in A[oldest] if h not in busy)
            Q = sorted(h for c, hs in A.items() if c != oldest
                       for h in hs if h not in busy)
            q_chunk = {h: act[h] for h in Q}
            if r >= n - 1:            # sigma may now help, sending c_{n-2}
                Q.append(sigma)
                q_chunk[sigma] = last
            P_r, Q_r = list(P), list(Q)
            window = range(r + 1, min(r + L, n - 2) + 1) if window_rule else range(0)
            in_window = set(window)
            pairs = []
            freeP, freeQ = list(P), list(Q)
            for g in window:
                if g in freeQ:
                    cand = [p for p in freeP if p not in in_window]
                    p = min(cand)
                    pairs.append((p, g))
                    freeP.remove(p)
                    freeQ.remove(g)
                elif g in freeP:
                    cand = [q for q in freeQ if q not in in_window]
                    q = min(cand, key=lambda h: (q_chunk[h], h))
                    assert q_chunk[q] <= g - L, "window rule infeasible"
                    pairs.append((g, q))
                    freeP.remove(g)
                    freeQ.remove(q)
            assert len(freeP) == len(freeQ)
            pairs.extend(zip(sorted(freeP), sorted(freeQ)))
            for p, q in pairs:
                if q != sigma:
                    ops.append((p, q, oldest, COPY))
                ops.append((q, p, q_chunk[q], COPY))
                received.append((p, q_chunk[q]))

        schedule.append(ops)
        if trace is not None:
            trace.append((r, A_before, P_r, Q_r))

        # update A (end of the Alg. 1 loop body)
        if r >= L:
            for h in A.pop(r - L):
                act.pop(h, None)
        if r < n - 1:
            A[r] = {r}
            act[r] = r
        for g, c in received:
            A[c].add(g)
            act[g] = c
    return schedule


def rs_precondition_rounds(n, straggler):
    if not 0 <= straggler < n:
        raise ValueError("straggler out of range")
    return [[(to_physical(s, n, straggler), to_physical(d, n, straggler), c, k)
             for s, d, c, k in ops] for ops in rs_precondition_logical(n)]


def completion_rounds(n, straggler):
    if not 0 <= straggler < n:
        raise ValueError("straggler out of range")
    return [[(to_physical(s, n, straggler), to_physical(d, n, straggler), c, k)
             for s, d, c, k in ops] for ops in completion_logical(n)]


# --------------------------------------------------------------------------
# Ring AllReduce baseline (App. E): n chunks of s/n, 2(n-1) rounds.
# --------------------------------------------------------------------------
def ring_allreduce_rounds(n):
    if n < 2:
        raise ValueError("n must be >= 2")
    rounds = []
    for t in range(n - 1):            # ReduceScatter half
        rounds.append([(i, (i + 1) % n, (i - t - 1) % n, REDUCE)
                       for i in range(n)])
    for t in range(n - 1):            # AllGather half
        rounds.append([(i, (i + 1) % n, (i - t) % n, COPY)
                       for i in range(n)])
    return rounds


# --------------------------------------------------------------------------
# Recursive halving / doubling baseline (App. E): n chunks of s/n, 2 log n
# rounds.  Rank i starts responsible for all n chunks; in halving step k it
# meets the rank whose index differs in bit (log n - 1 - k), keeps the half of
# its chunks whose index has its own value of that bit, and hands over the rest
# for the partner to add.  The doubling steps undo this in reverse order with
# plain copies.
# --------------------------------------------------------------------------
def rhd_allreduce_rounds(n):
    L = log2_exact(n)
    owned = {i: set(range(n)) for i in range(n)}
    rounds = []
    for k in range(L):
        bit = L - 1 - k
        ops = []
        nxt = {}
        for i in range(n):
            partner = i ^ (1 << bit)
            keep = {c for c in owned[i] if (c >> bit) & 1 == (i >> bit) & 1}
            for c in sorted(owned[i] - keep):
                ops.append((i, partner, c, REDUCE))
            nxt[i] = keep
        owned = nxt
        rounds.append(ops)
    for k in reversed(range(L)):
        bit = L - 1 - k
        ops = []
        nxt = {i: set(owned[i]) for i in range(n)}
        for i in range(n):
            partner = i ^ (1 << bit)
            for c in sorted(owned[i]):
                ops.append((i, partner, c, COPY))
            nxt[partner] |= owned[i]
        owned = nxt
        rounds.append(ops)
    assert all(owned[i] == set(range(n)) for i in range(n))
    return rounds


# --------------------------------------------------------------------------
# Broadcast baseline (App. E), straggler-aware.  While the straggler is late
# the n-1 on-time ranks AllReduce among themselves (ring: the reduce-scatter
# above, then n-2 all-gather steps).  When it arrives it swaps its whole buffer
# with one on-time rank (logical rank 0 here) - both then hold the full sum -
# and every round each holder passes the whole buffer to a rank without it.
# log n rounds of s bytes after arrival.
# --------------------------------------------------------------------------
def broadcast_precondition_logical(n):
    m = n - 1
    rounds = rs_precondition_logical(n)
    for t in range(m - 1):
        rounds.append([(i, (i + 1) % m, (i - t) % m, COPY) for i in range(m)])
    return rounds


def broadcast_completion_logical(n):
    if n < 2:
        raise ValueError("n must be >= 2")
    sigma = n - 1
    chunks = range(n - 1)
    rounds = [[(0, sigma, c, REDUCE_EXCHANGE) for c in chunks]]
    have = [0, sigma]
    while len(have) < n:
        lacking = [g for g in range(n) if g not in have]
        ops = []
        for h, g in zip(sorted(have), lacking):
            ops += [(h, g, c, COPY) for c in chunks]
            have = have + [g]
        rounds.append(ops)
    return rounds


def _relabel(rounds, n, straggler):
    if not 0 <= straggler < n:
        raise ValueError("straggler out of range")
    return [[(to_physical(s, n, straggler), to_physical(d, n, straggler), c, k)
             for s, d, c, k in ops] for ops in rounds]


def broadcast_precondition_rounds(n, straggler):
    return _relabel(broadcast_precondition_logical(n), n, straggler)


def broadcast_completion_rounds(n, straggler):
    return _relabel(broadcast_completion_logical(n), n, straggler)


# --------------------------------------------------------------------------
# Completion for even n that is not a power of two (App. D).  Each round is a
# maximum-weight matching: weight 2 when both ranks hold a reduced chunk the
# other lacks, 1 when only one does.  The pairings with the straggler stay as
# in Alg. 1 (rank r in round r); afterwards the straggler only sends.
#
# The paper fixes neither the chunk an edge carries, nor which maximum matching
# to take, nor the matching algorithm.  Readings (they decide the round count,
# not the values): an edge carries the newest chunk the sender has and the
# receiver lacks; among maximum-weight matchings the one with the largest bonus
# wins, where a transfer of chunk c to rank d scores (n - holders of c) + (number
# of reduced chunks d still lacks); the matching is found exactly, by recursion
# over subsets of the free ranks - the lowest free rank stays unmatched or pairs
# with a higher one, options tried in that order, first best kept.
# --------------------------------------------------------------------------
def completion_matching_logical(n):
    if n < 2 or n % 2:
        raise Unsupported("n must be even")
    import functools
    sigma = n - 1
    EDGE = 1 << 20
    full = [set() for _ in range(n)]
    schedule = []
    r = 0
    while True:
        ops = []
        busy = set()
        if r < n - 1:
            ops.append((r, sigma, r, REDUCE_EXCHANGE))
            busy = {r, sigma}
        reduced = range(min(r, n - 1))         # chunks 0 .. r-1 are reduced by now
        holders = {c: sum(1 for g in range(n) if c in full[g]) for c in reduced}
        lacks = [sum(1 for c in reduced if c not in full[g]) for g in range(n)]
        verts = [g for g in range(n) if g not in busy]

        def carry(a, b):
            offer = full[a] - full[b]
            return max(offer) if offer else None

        def bonus(c, dst):
            return 0 if c is None else (n - holders[c]) + lacks[dst]

        weight = {}
        for i, u in enumerate(verts):
            for j in range(i + 1, len(verts)):
                v = verts[j]
                cu, cv = carry(u, v), carry(v, u)
                edges = (cu is not None) + (cv is not None)
                if edges:
                    weight[(i, j)] = edges * EDGE + bonus(cu, v) + bonus(cv, u)

        @functools.lru_cache(maxsize=None)
        def best(mask):
            if mask == 0:
                return 0, ()
            i = (mask & -mask).bit_length() - 1
            rest = mask & (mask - 1)
            top = best(rest)
            m = rest
            while m:
                j = (m & -m).bit_length() - 1
                m &= m - 1
                w = weight.get((i, j))
                if w:
                    sub = best(rest & ~(1 << j))
                    if w + sub[0] > top[0]:
                        top = (w + sub[0], ((i, j),) + sub[1])
            return top

        gained = []
        for i, j in best((1 << len(verts)) - 1)[1]:
            u, v = verts[i], verts[j]
            for a, b in ((u, v), (v, u)):
                c = carry(a, b)
                if c is not None:
                    ops.append((a, b, c, COPY))
                    gained.append((b, c))
        if r < n - 1:
            gained += [(r, r), (sigma, r)]
        for g, c in gained:
            full[g].add(c)
        schedule.append(ops)
        if r >= n - 2 and all(len(f) == n - 1 for f in full):
            return schedule
        r += 1


def completion_rounds_any(n, straggler):
    """Completion for any supported n: Alg. 1 for powers of two, App. D otherwise."""
    if n & (n - 1) == 0:
        return completion_rounds(n, straggler)
    return _relabel(completion_matching_logical(n), n, straggler)
