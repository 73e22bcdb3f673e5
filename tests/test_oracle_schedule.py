"""Pins of the oracle's schedules against the paper (no GPU)."""

import os
import time
from fractions import Fraction

import pytest

from oracle import COPY, REDUCE, REDUCE_EXCHANGE
from oracle import schedule as S
from sched_checks import check_round_hazards, ilog2, simulate_completion

POW2 = [2, 4, 8, 16, 32, 64, 128, 256]
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "table1_costs.txt")


def golden_costs():
    rows = {}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, rounds, beta, _ = [f.strip() for f in line.split("|")]
        rows[name] = (rounds, beta)
    return rows


def evaluate(expr, n):
    return eval(expr, {"__builtins__": {}}, {"n": Fraction(n), "L": Fraction(ilog2(n))})


# ---- Thm. 1 / Table 1 -------------------------------------------------------
@pytest.mark.parametrize("n", POW2)
def test_round_counts_match_table1(n):
    g = golden_costs()
    assert len(S.completion_logical(n)) == evaluate(g["stragglar_completion"][0], n)
    assert len(S.ring_allreduce_rounds(n)) == evaluate(g["ring_allreduce"][0], n)
    assert len(S.rs_precondition_logical(n)) == evaluate(g["rs_precondition"][0], n)


def test_round_counts_literal():
    # Thm. 1 evaluated by hand
    for n, want in [(2, 1), (4, 4), (8, 9), (16, 18), (32, 35), (256, 262)]:
        assert len(S.completion_logical(n)) == want
        assert want >= n - 1          # Sec. 3.1: at least n-1 rounds are needed


@pytest.mark.parametrize("n", POW2)
def test_beta_cost_one_chunk_per_rank_per_round(n):
    """Serialized bytes per rank = rounds x one chunk (Sec. 3, cost model):
    no rank sends more than one chunk in a round, and some rank is busy in
    every round, so the beta coefficient is rounds / parts."""
    g = golden_costs()
    for name, rounds, parts in [
        ("stragglar_completion", S.completion_logical(n), n - 1),
        ("ring_allreduce", S.ring_allreduce_rounds(n), n),
        ("rs_precondition", S.rs_precondition_logical(n), n - 1),
    ]:
        for ops in rounds:
            senders = [s for s, d, c, k in ops] + [d for s, d, c, k in ops if k == REDUCE_EXCHANGE]
            assert len(senders) == len(set(senders)) and senders
        assert Fraction(len(rounds), parts) == evaluate(g[name][1], n)


@pytest.mark.parametrize("n", POW2[:6])
def test_rhd_and_broadcast_costs(n):
    """Rounds and serialized bytes per rank of the other baselines (Table 1, App. E).  A rank
    may send several chunks to its one partner in a round; the round costs the largest such
    message."""
    g = golden_costs()
    for name, rounds, parts in [
        ("rhd_allreduce", S.rhd_allreduce_rounds(n), n),
        ("broadcast_completion", S.broadcast_completion_logical(n), n - 1),
        ("broadcast_precondition", S.broadcast_precondition_logical(n), n - 1),
    ]:
        assert len(rounds) == evaluate(g[name][0], n), name
        beta = Fraction(0)
        for ops in rounds:
            sent, partner = {}, {}
            for s_, d, c, k in ops:
                pairs = [(s_, d)] + ([(d, s_)] if k == REDUCE_EXCHANGE else [])
                for a, b in pairs:
                    sent[a] = sent.get(a, 0) + 1
                    assert partner.setdefault(a, b) == b        # one peer per rank per round
            beta += Fraction(max(sent.values()), parts)
        assert beta == evaluate(g[name][1], n), name
        check_round_hazards(rounds)


@pytest.mark.parametrize("n", POW2[:6])
def test_rhd_and_broadcast_structure(n):
    # RHD: every chunk of every rank ends as the sum of all n contributions, each once
    contrib = [[{g} for _ in range(n)] for g in range(n)]
    for ops in S.rhd_allreduce_rounds(n):
        snap = [[set(x) for x in row] for row in contrib]
        for s_, d, c, k in ops:
            if k == REDUCE:
                assert not (snap[s_][c] & snap[d][c])
                contrib[d][c] = snap[s_][c] | snap[d][c]
            else:
                assert k == COPY and snap[s_][c] == set(range(n))
                contrib[d][c] = set(snap[s_][c])
    assert all(contrib[g][c] == set(range(n)) for g in range(n) for c in range(n))
    # Broadcast: precondition leaves every on-time rank with the on-time sum, straggler alone
    m, sigma = n - 1, n - 1
    contrib = [[{g} for _ in range(m)] for g in range(n)]
    for ops in S.broadcast_precondition_logical(n) + S.broadcast_completion_logical(n):
        snap = [[set(x) for x in row] for row in contrib]
        for s_, d, c, k in ops:
            if k == COPY:
                contrib[d][c] = set(snap[s_][c])
            else:
                assert not (snap[s_][c] & snap[d][c])
                contrib[d][c] = snap[s_][c] | snap[d][c]
                if k == REDUCE_EXCHANGE:
                    assert {s_, d} == {0, sigma}
                    contrib[s_][c] = set(contrib[d][c])
    assert all(contrib[g][c] == set(range(n)) for g in range(n) for c in range(m))
    mid = [[{g} for _ in range(m)] for g in range(n)]
    for ops in S.broadcast_precondition_logical(n):
        snap = [[set(x) for x in row] for row in mid]
        for s_, d, c, k in ops:
            assert sigma not in (s_, d)
            mid[d][c] = set(snap[s_][c]) if k == COPY else snap[s_][c] | snap[d][c]
    assert all(mid[g][c] == set(range(m)) for g in range(m) for c in range(m))


def test_limits_of_beta_cost():
    g = golden_costs()
    big = 1 << 20
    assert abs(float(evaluate(g["ring_allreduce"][1], big)) - 2.0) < 1e-4
    assert abs(float(evaluate(g["stragglar_completion"][1], big)) - 1.0) < 1e-4


# ---- structure of Alg. 1 ----------------------------------------------------
@pytest.mark.parametrize("n", POW2)
def test_completion_set_simulation(n):
    rounds = S.completion_logical(n)
    simulate_completion(n, rounds)
    check_round_hazards(rounds)


@pytest.mark.parametrize("n", [4, 8, 16, 32, 64, 128, 256])
def test_lemma1_and_invariant(n):
    L = ilog2(n)
    trace = []
    S.completion_logical(n, trace=trace)
    for r, A, P, Q in trace:
        holders = [h for hs in A.values() for h in hs]
        assert len(holders) == len(set(holders))           # pairwise disjoint
        if r == L:                                          # Lemma 1
            assert sorted(A) == list(range(L))
            for j in range(L):
                assert len(A[j]) == 2 ** (L - 1 - j)
            assert sorted(holders) == list(range(n - 1))
            assert L in A[0]                                # rank log n got c_0 (base case)
        if r >= L:                                          # invariant I(r)
            live = [j for j in range(r - L, r) if j <= n - 2]
            assert sorted(A) == live
            for j in live:
                want = 2 ** (r - j - 1)
                if j == n - 2:                              # Remark 1: c_{n-2} starts on two
                    want = 2 * want - 1                     # ranks; sigma is not listed in A
                assert len(A[j]) == want, (n, r, j)
            if r <= n - 2:
                assert r in A[r - L]                        # rank r in P_r
                assert len(P) == n // 2 - 1 and r not in P  # r itself is with sigma
                assert len(Q) == n // 2 - 1
            else:
                assert len(P) == n // 2 and len(Q) == n // 2 and (n - 1) in Q


def test_remark1_sigma_share_of_last_chunk():
    # the want-adjustment above, spelled out for n = 8: before round 8 the last
    # chunk c_6 sits on 4 ranks, one of them sigma, so 3 on-time holders
    trace = []
    S.completion_logical(8, trace=trace)
    A = trace[8][1]
    assert len(A[6]) == 3


@pytest.mark.parametrize("n", POW2)
def test_lemma2_propagation_deadlines(n):
    L = ilog2(n)
    after = simulate_completion(n, S.completion_logical(n))
    for c in range(n - 1):
        assert c in after[c][c] and c in after[c][n - 1]    # reduced in round c on rank c and sigma
        if c > 0:
            assert all(c not in after[c - 1][g] for g in range(n))
        due = c + L if c < n - 2 else c + L - 1             # Lemma 2 / Remark 1
        assert all(c in after[due][g] for g in range(n))
        if due > c:
            assert not all(c in after[due - 1][g] for g in range(n))


def test_ramp_rule_rank0_to_rank_logn():
    for n in [4, 8, 16, 32, 64]:
        L = ilog2(n)
        assert (0, L, 0, COPY) in S.completion_logical(n)[1]
        for r in range(1, L):
            assert (r - 1, r - 1 + L, r - 1, COPY) in S.completion_logical(n)[r]


def test_fig3b_ranks_3_and_5_not_matched_in_round_4():
    ops = S.completion_logical(8)[4]
    pairs = {frozenset((s, d)) for s, d, c, k in ops}
    assert frozenset((3, 5)) not in pairs
    # and the reason: 5 is in the critical window, 3 holds the newest chunk c_3
    assert any(s == 3 and c == 3 for s, d, c, k in ops)


def test_window_rule_is_exercised():
    """With the critical-window step removed the schedule breaks for n >= 8
    (n = 4 has too few ranks for it to matter)."""
    simulate_completion(4, S.completion_logical(4, window_rule=False))
    for n in [8, 16, 32]:
        with pytest.raises((AssertionError, KeyError, ValueError)):
            rounds = S.completion_logical(n, window_rule=False)
            simulate_completion(n, rounds)
            trace = []
            S.completion_logical(n, trace=trace, window_rule=False)
            for r, A, P, Q in trace:
                if ilog2(n) <= r <= n - 2:
                    assert r in A[r - ilog2(n)]


def test_schedule_fixture_is_current():
    """Regression guard on the tie-breaks (the fixture is written by
    tests/golden/make_schedule_fixture.py from the oracle; it is not a paper value)."""
    import importlib.util
    path = os.path.join(os.path.dirname(__file__), "golden", "make_schedule_fixture.py")
    spec = importlib.util.spec_from_file_location("make_schedule_fixture", path)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    stored = open(os.path.join(os.path.dirname(__file__), "golden", "completion_schedules.txt")).read()
    assert stored == mod.render()
    # the n = 4 rounds, spelled out: 4 rounds, 3 exchanges, 6 copies
    rows = [l.split() for l in stored.splitlines() if l.startswith("4 ")]
    assert len(rows) == 9 and sum(r[5] == "EXCHANGE" for r in rows) == 3
    assert ["4", "1", "0", "2", "0", "COPY"] in rows       # rank 0 -> rank log n in round 1


def test_generation_time_n256():
    t0 = time.perf_counter()
    S.completion_logical(256)
    assert time.perf_counter() - t0 < 1.04   # Sec. 4, "Schedule generator"


EVEN_NOT_POW2 = [6, 10, 12, 14]


@pytest.mark.parametrize("n", EVEN_NOT_POW2)
def test_matching_generator_validity_and_cost(n):
    """App. D: no bound is proven; the paper reports about n + 2 log n - 2 rounds and a beta
    cost still below the baselines'.  Structure rules are those of Sec. 3.1."""
    rounds = S.completion_matching_logical(n)
    simulate_completion(n, rounds, power_of_two=False)
    check_round_hazards(rounds)
    L_up = (n - 1).bit_length()
    assert n - 1 <= len(rounds) <= n + 2 * L_up - 2
    assert Fraction(len(rounds), n - 1) < Fraction(2 * (n - 1), n)      # cheaper than ring / RHD (Table 1)
    for r, ops in enumerate(rounds):                                     # straggler pairings as in Alg. 1
        assert ((r, n - 1, r, REDUCE_EXCHANGE) in ops) == (r < n - 1)
    # regression guard on the tie-breaks (derived, not a paper value)
    assert len(rounds) == {6: 7, 10: 12, 12: 15, 14: 17}[n]


@pytest.mark.parametrize("n", [6, 10])
def test_matching_generator_rounds_are_maximum_weight(n):
    """Every round's matching attains the maximum of App. D's weights (2 if both ranks can
    give the other a chunk it lacks, 1 if one can), checked by enumerating all matchings."""
    rounds = S.completion_matching_logical(n)
    sigma = n - 1
    full = [set() for _ in range(n)]

    def all_matchings(vs):
        if len(vs) < 2:
            yield []
            return
        a, rest = vs[0], vs[1:]
        yield from all_matchings(rest)
        for i, b in enumerate(rest):
            for m in all_matchings(rest[:i] + rest[i + 1:]):
                yield [(a, b)] + m

    def w(a, b):
        return (1 if full[a] - full[b] else 0) + (1 if full[b] - full[a] else 0)

    for r, ops in enumerate(rounds):
        free = [g for g in range(n) if not (r < n - 1 and g in (r, sigma))]
        best = max(sum(w(a, b) for a, b in m) for m in all_matchings(free))
        copies = [(s_, d, c) for s_, d, c, k in ops if k == COPY]
        got = len(copies)                       # each unit of weight is one chunk transfer
        assert got == best, (n, r, got, best)
        for s_, d, c in copies:
            assert c in full[s_] and c not in full[d]
        for s_, d, c in copies:
            full[d].add(c)
        if r < n - 1:
            full[r].add(r)
            full[sigma].add(r)


def test_unsupported_n():
    for n in [3, 5, 6, 12, 100]:
        with pytest.raises(S.Unsupported):
            S.completion_logical(n)
    for n in [3, 7, 9]:
        with pytest.raises(S.Unsupported):
            S.completion_matching_logical(n)
    for n in [0, 1, -4]:
        with pytest.raises(ValueError):
            S.completion_logical(n)


# ---- relabelling, precondition, ring ---------------------------------------
@pytest.mark.parametrize("n", [2, 4, 8, 16])
def test_physical_relabel(n):
    for sg in range(n):
        phys = [S.to_physical(l, n, sg) for l in range(n)]
        assert sorted(phys) == list(range(n)) and phys[n - 1] == sg
        assert phys[:n - 1] == sorted(phys[:n - 1])
        rounds = S.completion_rounds(n, sg)
        inv = {p: l for l, p in enumerate(phys)}
        back = [[(inv[s], inv[d], c, k) for s, d, c, k in ops] for ops in rounds]
        assert back == S.completion_logical(n)
        for ops in S.rs_precondition_rounds(n, sg):
            assert all(s != sg and d != sg for s, d, c, k in ops)


@pytest.mark.parametrize("n", POW2[:6])
def test_rs_precondition_structure(n):
    m = n - 1
    rounds = S.rs_precondition_logical(n)
    check_round_hazards(rounds)
    # contributions[rank][chunk] = set of ranks summed into that cell
    contrib = [[{g} for _ in range(m)] for g in range(m)]
    for ops in rounds:
        assert len(ops) == m
        snap = [[set(s) for s in row] for row in contrib]
        for s, d, c, k in ops:
            assert k == REDUCE
            assert not (snap[s][c] & snap[d][c])            # nothing counted twice
            contrib[d][c] = snap[s][c] | snap[d][c]
    for g in range(m):
        assert contrib[g][g] == set(range(m))               # rank g owns reduced c_g


@pytest.mark.parametrize("n", [2, 3, 4, 7, 8, 16])
def test_ring_structure(n):
    rounds = S.ring_allreduce_rounds(n)
    assert len(rounds) == 2 * (n - 1)
    check_round_hazards(rounds)
    contrib = [[{g} for _ in range(n)] for g in range(n)]
    for ops in rounds:
        snap = [[set(s) for s in row] for row in contrib]
        for s, d, c, k in ops:
            if k == REDUCE:
                assert not (snap[s][c] & snap[d][c])
                contrib[d][c] = snap[s][c] | snap[d][c]
            else:
                assert snap[s][c] == set(range(n))
                contrib[d][c] = set(snap[s][c])
    assert all(contrib[g][c] == set(range(n)) for g in range(n) for c in range(n))


def test_chunk_layout():
    # fp32, 16-byte alignment: chunk length is a multiple of 4 elements
    lay = S.chunk_layout(4096, 3, 4)
    assert lay == [(0, 1368), (1368, 1368), (2736, 1360)]
    lay = S.chunk_layout(64 << 20, 7, 4)
    assert lay[0] == (0, 9586984) and sum(l for _, l in lay) == 64 << 20
    assert all(o % 4 == 0 for o, _ in lay)
    lay = S.chunk_layout(8 * 2048 * 3072, 7, 2)
    assert lay[0][1] == 7190240 and all(o % 8 == 0 for o, _ in lay)
    assert S.chunk_layout(1_240_000_000, 7, 2)[0][1] == 177142864
    assert S.chunk_layout(16 << 20, 15, 4)[0][1] == 1118484
    assert S.chunk_layout(16 << 20, 31, 4)[0][1] == 541204
    with pytest.raises(ValueError):
        S.chunk_layout(7, 7, 4)            # chunk 1 would start past the end
    with pytest.raises(ValueError):
        S.chunk_layout(0, 3, 4)
    assert S.chunk_layout(7, 7, 4, align_bytes=4) == [(i, 1) for i in range(7)]
