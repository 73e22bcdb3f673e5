"""Checks of a completion schedule against what Sec. 3.1, Alg. 1 and the
proofs of App. C fix.  Works on any list of rounds of (src, dst, chunk, kind)
over LOGICAL ranks (straggler = n-1), whoever produced it."""

COPY, REDUCE, REDUCE_EXCHANGE = 0, 1, 2


def ilog2(n):
    return n.bit_length() - 1


def simulate_completion(n, rounds, power_of_two=True):
    """Set simulation.  Returns per-round snapshots of `full[rank]` (the set of
    fully reduced chunks each rank holds AFTER that round).  Asserts every
    structural rule on the way.  ``power_of_two=False`` drops the one rule that
    only Alg. 1 has (Remark 1: the straggler forwards nothing but c_{n-2})."""
    L = ilog2(n)
    sigma = n - 1
    full = [set() for _ in range(n)]
    after = []
    n_rx = n_copy = 0
    for r, ops in enumerate(rounds):
        sends, recvs = {}, {}
        new = []
        for src, dst, c, kind in ops:
            assert 0 <= src < n and 0 <= dst < n and src != dst
            assert 0 <= c < n - 1
            if kind == REDUCE_EXCHANGE:
                # Alg. 1: rank r <-> sigma exchange c_r, only while r < n-1
                assert (src, dst, c) == (r, sigma, r) and r < n - 1
                for a, b in ((src, dst), (dst, src)):
                    assert a not in sends and a not in recvs
                    sends[a] = b
                    recvs[a] = b
                assert c not in full[src] and c not in full[dst]
                new += [(src, c), (dst, c)]
                n_rx += 1
            elif kind == COPY:
                assert c in full[src], "round %d: rank %d sends c%d before holding it" % (r, src, c)
                assert c not in full[dst], "round %d: rank %d already holds c%d" % (r, dst, c)
                assert src not in sends, "round %d: rank %d sends twice" % (r, src)
                assert dst not in recvs, "round %d: rank %d receives twice" % (r, dst)
                sends[src] = dst
                recvs[dst] = src
                new.append((dst, c))
                n_copy += 1
                if src == sigma:      # sigma sends only once it has met every rank ...
                    assert r >= n - 1
                    if power_of_two:  # ... and then (Remark 1) only c_{n-2}
                        assert c == n - 2
                assert dst != sigma   # sigma gets its data from the pairings only
            else:
                raise AssertionError("op kind %r not allowed in completion" % kind)
        # one matching per rank per round (Sec. 3.1): whoever a rank sends to
        # is also the only rank it may receive from
        for a, b in sends.items():
            if a in recvs:
                assert recvs[a] == b, "round %d: rank %d talks to two peers" % (r, a)
        for rank, c in new:
            full[rank].add(c)
        after.append([set(s) for s in full])
    assert n_rx == n - 1
    assert n_copy == (n - 1) * (n - 2)
    for rank in range(n):
        assert full[rank] == set(range(n - 1)), "rank %d misses chunks" % rank
    return after


def check_round_hazards(rounds):
    """Within a round no op may read or write a (rank, chunk) cell another op
    writes: the ranks' buffers live in one address space here."""
    for r, ops in enumerate(rounds):
        writer = {}
        for i, (src, dst, c, kind) in enumerate(ops):
            cells = [(dst, c)] if kind != REDUCE_EXCHANGE else [(src, c), (dst, c)]
            for cell in cells:
                assert cell not in writer, "round %d: ops %d,%d write the same cell" % (r, writer[cell], i)
                writer[cell] = i
        for i, (src, dst, c, kind) in enumerate(ops):
            reads = [(src, c)] if kind == COPY else [(src, c), (dst, c)]
            for cell in reads:
                assert writer.get(cell, i) == i, "round %d: op %d writes what op %d reads" % (r, writer[cell], i)
