"""Pins of the oracle's arithmetic: brute-force sums, fold order, tolerance,
bf16 rounding against a library conversion (no GPU)."""

import numpy as np
import pytest
import torch

from oracle import bf16 as B
from oracle import reference as R
from oracle import replay as P
from oracle import schedule as S
import synth_inputs as W

EB = {"i32": 4, "f32": 4, "bf16": 2}
TOL = {"f32": 1e-5, "bf16": 2.0 ** -7}      # x n, relative to sum_i |x_i|


def stragglar_o1(inputs, straggler, dtype, align_bytes=16, stop_after_rs=False):
    n = len(inputs)
    bufs = [x.copy() for x in inputs]
    chunks = S.chunk_layout(len(inputs[0]), n - 1, EB[dtype], align_bytes)
    P.replay(S.rs_precondition_rounds(n, straggler), chunks, bufs, dtype)
    if not stop_after_rs:
        P.replay(S.completion_rounds(n, straggler), chunks, bufs, dtype)
    return bufs, chunks


def ring_o1(inputs, dtype, align_bytes=16):
    n = len(inputs)
    bufs = [x.copy() for x in inputs]
    chunks = S.chunk_layout(len(inputs[0]), n, EB[dtype], align_bytes)
    P.replay(S.ring_allreduce_rounds(n), chunks, bufs, dtype)
    return bufs


def rand_inputs(n, count, dtype, seed, dist=None):
    if dist is None:
        dist = ("uniform_int", -1000, 1000) if dtype == "i32" else ("normal", 1.0)
    w = W.Workload("t", n, 0, count, dtype, dist, seed)
    return w.host_all()


# ---- exact sums, brute force on tiny cases ---------------------------------
@pytest.mark.parametrize("n", [2, 4, 8])
def test_bruteforce_exact_small(n):
    m = n - 1
    tried = 0
    for count in range(n, 6 * m + 4):
        try:                     # some counts leave the last chunk empty: not a valid input
            S.chunk_layout(count, m, 4, 4), S.chunk_layout(count, n, 4, 4)
        except ValueError:
            continue
        tried += 1
        xs = rand_inputs(n, count, "i32", seed=count)
        want = [sum(int(x[e]) for x in xs) for e in range(count)]   # plain Python
        for sg in range(n):
            bufs, _ = stragglar_o1(xs, sg, "i32", align_bytes=4)
            for b in bufs:
                assert b.tolist() == want
        for b in ring_o1(xs, "i32", align_bytes=4):
            assert b.tolist() == want
        # small integers stored as floats: every order is exact
        xf = [x.astype(np.float32) for x in xs]
        for b in stragglar_o1(xf, n - 1, "f32", align_bytes=4)[0]:
            assert b.tolist() == [float(v) for v in want]
    assert tried >= 5


@pytest.mark.parametrize("n", [2, 4, 8, 16, 32])
def test_each_contribution_exactly_once(n):
    """Rank i contributes 2^i: any omission or double count changes the bits
    (mod 2^32 for n = 32)."""
    count = 16 * (n - 1) * n + 3
    xs = [np.full(count, (1 << i) & 0xFFFFFFFF, dtype=np.uint32).view(np.int32) for i in range(n)]
    want = np.uint32((1 << n) - 1 & 0xFFFFFFFF)
    for sg in range(n):
        bufs, _ = stragglar_o1(xs, sg, "i32")
        for b in bufs:
            assert (b.view(np.uint32) == want).all()
    for b in ring_o1(xs, "i32"):
        assert (b.view(np.uint32) == want).all()


def test_int32_wraps():
    xs = [np.full(64, 2**31 - 1, np.int32), np.full(64, 1, np.int32)]
    bufs, _ = stragglar_o1(xs, 1, "i32")
    assert (bufs[0] == -2**31).all() and (bufs[1] == -2**31).all()


def test_cfg1_all_definitions_agree():
    w = W.cfg1()
    xs = w.host_all()
    assert all(np.abs(x).max() <= 8 and (x == np.round(x)).all() for x in xs)
    exact = R.allreduce_exact_int(xs)
    bufs, chunks = stragglar_o1(xs, w.straggler, "f32")
    assert chunks == [(0, 1368), (1368, 1368), (2736, 1360)]
    fold = R.stragglar_fold(xs, w.straggler, "f32", elem_bytes=4)
    f64 = R.allreduce_f64(xs, "f32")
    for b in bufs + ring_o1(xs, "f32"):
        assert (b.astype(np.int64) == exact).all()
        assert (b == fold).all() and (b.astype(np.float64) == f64).all()


# ---- precondition postcondition (Sec. 3.1) ---------------------------------
@pytest.mark.parametrize("n", [2, 4, 8, 16])
def test_precondition_leaves_partial_sums(n):
    xs = rand_inputs(n, 40 * (n - 1) * n + 5, "i32", seed=n)
    for sg in range(n):
        bufs, chunks = stragglar_o1(xs, sg, "i32", stop_after_rs=True)
        assert (bufs[sg] == xs[sg]).all()                       # straggler untouched
        part = R.allreduce_exact_int([x for i, x in enumerate(xs) if i != sg])
        for g in range(n - 1):
            lo, ln = chunks[g]
            assert (bufs[S.to_physical(g, n, sg)][lo:lo + ln] == part[lo:lo + ln]).all()


# ---- floating-point order ----------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n", [2, 4, 8, 16])
def test_replay_equals_fold_bitexact(n, dtype):
    count = 1000 * (n - 1) + 13
    xs = rand_inputs(n, count, dtype, seed=100 + n)
    for sg in sorted({0, n // 2, n - 1}):
        bufs, chunks = stragglar_o1(xs, sg, dtype)
        fold = R.stragglar_fold(xs, sg, dtype, chunks=chunks)
        for b in bufs:
            assert (b.view(np.uint8) == fold.view(np.uint8)).all()
    rf = R.ring_fold(xs, dtype, elem_bytes=EB[dtype])
    for b in ring_o1(xs, dtype):
        assert (b.view(np.uint8) == rf.view(np.uint8)).all()


@pytest.mark.parametrize("dtype", ["i32", "f32", "bf16"])
@pytest.mark.parametrize("n", [2, 4, 8, 16])
def test_precondition_fold_is_the_replayed_partial(n, dtype):
    """The precondition's closed form per chunk: the replay of the ring ReduceScatter leaves
    exactly these bits in the owner's chunk (Sec. 3.1 precondition); for integers it is the
    exact sum over the on-time ranks; and the straggler's one add on top of it is the final
    value."""
    count = 700 * (n - 1) + 9
    xs = rand_inputs(n, count, dtype, seed=300 + n)
    for sg in sorted({0, n // 2, n - 1}):
        bufs, chunks = stragglar_o1(xs, sg, dtype, stop_after_rs=True)
        for c, (lo, ln) in enumerate(chunks):
            cols = [x[lo:lo + ln] for x in xs]
            part = R.precondition_fold_chunk(cols, c, sg, dtype)
            owner = bufs[S.to_physical(c, n, sg)][lo:lo + ln]
            assert (owner.view(np.uint8) == part.view(np.uint8)).all()
            if dtype == "i32":
                exact = R.allreduce_exact_int([col for i, col in enumerate(cols) if i != sg])
                assert (part.astype(np.int64) == exact).all()
            full = R.stragglar_fold_chunk(cols, c, sg, dtype)
            assert (full.view(np.uint8) == P.add(part, cols[sg], dtype).view(np.uint8)).all()


def run_rounds(rounds, parts, inputs, dtype, align_bytes=16):
    bufs = [x.copy() for x in inputs]
    chunks = S.chunk_layout(len(inputs[0]), parts, EB[dtype], align_bytes)
    P.replay(rounds, chunks, bufs, dtype)
    return bufs


@pytest.mark.parametrize("dtype", ["i32", "f32", "bf16"])
@pytest.mark.parametrize("n", [2, 4, 8, 16])
def test_rhd_and_broadcast_values(n, dtype):
    count = 600 * (n - 1) * 2 + 13
    xs = rand_inputs(n, count, dtype, seed=200 + n)
    rhd = run_rounds(S.rhd_allreduce_rounds(n), n, xs, dtype)
    tree = R.rhd_fold(xs, dtype, elem_bytes=EB[dtype])
    for b in rhd:
        assert (b.view(np.uint8) == tree.view(np.uint8)).all()
    for sg in sorted({0, n - 1}):
        mid = run_rounds(S.broadcast_precondition_rounds(n, sg), n - 1, xs, dtype)
        assert (mid[sg] == xs[sg]).all()
        chunks = S.chunk_layout(count, n - 1, EB[dtype])
        out = [b.copy() for b in mid]
        P.replay(S.broadcast_completion_rounds(n, sg), chunks, out, dtype)
        # same additions in the same order as StragglAR: identical bits
        want = R.stragglar_fold(xs, sg, dtype, chunks=chunks)
        for b in out:
            assert (b.view(np.uint8) == want.view(np.uint8)).all()
    if dtype == "i32":
        exact = (R.allreduce_exact_int(xs) & 0xFFFFFFFF).astype(np.uint32).view(np.int32)
        assert (rhd[0] == exact).all()
    else:
        ref = R.allreduce_f64(xs, dtype)
        bound = TOL[dtype] * n * R.abs_sum_f64(xs, dtype)
        assert (np.abs(R.to_f64(rhd[0], dtype) - ref) <= bound).all()


def test_rhd_small_bruteforce():
    for n in (2, 4, 8):
        xs = rand_inputs(n, 8 * n + 3, "i32", seed=n)
        want = [sum(int(x[e]) for x in xs) for e in range(len(xs[0]))]
        for b in run_rounds(S.rhd_allreduce_rounds(n), n, xs, "i32", align_bytes=4):
            assert b.tolist() == want


@pytest.mark.parametrize("dtype", ["i32", "f32", "bf16"])
@pytest.mark.parametrize("n", [6, 10, 12])
def test_even_non_power_of_two_values(n, dtype):
    """App. D schedules: different rounds, same additions - the fold of the ring precondition
    plus the straggler, so the closed form still gives the bits."""
    count = 500 * (n - 1) * n + 11
    xs = rand_inputs(n, count, dtype, seed=300 + n)
    for sg in sorted({0, n // 2, n - 1}):
        chunks = S.chunk_layout(count, n - 1, EB[dtype])
        bufs = [x.copy() for x in xs]
        P.replay(S.rs_precondition_rounds(n, sg), chunks, bufs, dtype)
        P.replay(S.completion_rounds_any(n, sg), chunks, bufs, dtype)
        want = R.stragglar_fold(xs, sg, dtype, chunks=chunks)
        for b in bufs:
            assert (b.view(np.uint8) == want.view(np.uint8)).all()
    if dtype == "i32":
        exact = (R.allreduce_exact_int(xs) & 0xFFFFFFFF).astype(np.uint32).view(np.int32)
        assert (bufs[0] == exact).all()


def test_fold_order_is_visible():
    """The fold is not the sorted-order sum: with N(0,1) data a different
    association changes some bits, so 'replay == fold' really pins the order."""
    n, count = 8, 7 * 4096
    xs = rand_inputs(n, count, "f32", seed=7)
    fold = R.stragglar_fold(xs, 0, "f32", elem_bytes=4)
    naive = xs[0].copy()
    for x in xs[1:]:
        naive = naive + x
    assert (fold != naive).any()
    ring = R.ring_fold(xs, "f32", elem_bytes=4)
    assert (fold != ring).any()          # allowed to differ; both within tolerance


def test_n2_is_one_add():
    xs = rand_inputs(2, 1001, "f32", seed=1)
    for sg in (0, 1):
        bufs, _ = stragglar_o1(xs, sg, "f32")
        assert (bufs[0] == xs[0] + xs[1]).all() and (bufs[1] == bufs[0]).all()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n", [4, 8, 16, 32])
def test_within_tolerance_of_f64(n, dtype):
    xs = rand_inputs(n, 2000 * (n - 1) + 7, dtype, seed=n)
    ref = R.allreduce_f64(xs, dtype)
    bound = TOL[dtype] * n * R.abs_sum_f64(xs, dtype)
    for out in (stragglar_o1(xs, n // 2, dtype)[0][0], ring_o1(xs, dtype)[0]):
        assert (np.abs(R.to_f64(out, dtype) - ref) <= bound).all()


def test_tolerance_catches_a_dropped_rank():
    n = 8
    xs = rand_inputs(n, 7000, "f32", seed=3)
    ref = R.allreduce_f64(xs, "f32")
    bound = TOL["f32"] * n * R.abs_sum_f64(xs, "f32")
    wrong = R.allreduce_f64(xs[:-1], "f32")
    assert (np.abs(wrong - ref) > bound).mean() > 0.99


# ---- bf16 ---------------------------------------------------------------------
def test_bf16_narrowing_matches_library_conversion():
    hi = np.arange(1 << 16, dtype=np.uint32) << 16
    rng = np.random.Generator(np.random.Philox(key=[9, 9]))
    lows = np.concatenate([
        np.array([0, 1, 2, 0x7FFE, 0x7FFF, 0x8000, 0x8001, 0x8002, 0xFFFE, 0xFFFF], np.uint32),
        rng.integers(0, 1 << 16, size=40, dtype=np.uint32)])
    bits = (hi[:, None] | lows[None, :]).ravel()
    x = bits.view(np.float32)
    got = B.f32_to_bf16(x)
    want = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    finite_or_inf = ~np.isnan(x)
    assert (got[finite_or_inf] == want[finite_or_inf]).all()
    assert np.isnan(B.bf16_to_f32(got[~finite_or_inf])).all()     # NaN stays NaN
    # ties go to even
    assert B.f32_to_bf16(np.array([0x3F808000], np.uint32).view(np.float32))[0] == 0x3F80
    assert B.f32_to_bf16(np.array([0x3F818000], np.uint32).view(np.float32))[0] == 0x3F82
    # carry into the exponent, and overflow to infinity
    assert B.f32_to_bf16(np.array([0x3FFFFFFF], np.uint32).view(np.float32))[0] == 0x4000
    assert B.f32_to_bf16(np.array([0x7F7FFFFF], np.uint32).view(np.float32))[0] == 0x7F80


def test_bf16_widening_and_add_match_library():
    u = np.arange(1 << 16, dtype=np.uint16)
    t = torch.from_numpy(u.view(np.int16).copy()).view(torch.bfloat16)
    f = B.bf16_to_f32(u)
    assert (f.view(np.uint32) == t.float().numpy().view(np.uint32)).all()
    rng = np.random.Generator(np.random.Philox(key=[5, 5]))
    a = rng.integers(0, 1 << 16, size=1 << 20, dtype=np.uint16)
    b = rng.integers(0, 1 << 16, size=1 << 20, dtype=np.uint16)
    ta = torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16)
    tb = torch.from_numpy(b.view(np.int16).copy()).view(torch.bfloat16)
    want = (ta.float() + tb.float()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = B.bf16_add(a, b)
    ok = ~np.isnan(B.bf16_to_f32(want))
    assert (got[ok] == want[ok]).all()
    assert np.isnan(B.bf16_to_f32(got[~ok])).all()


# ---- the input generator -----------------------------------------------------
def test_inputs_are_seeded_and_tiled_consistently():
    w = W.Workload("t", 4, 1, 5000, "bf16", ("normal", 1e-3), seed=11)
    a, b = w.host(2), w.host(2)
    assert (a == b).all() and a.dtype == np.uint16
    assert (w.host(1) != w.host(2)).any()
    old = W.TILE_THRESHOLD
    try:
        W.TILE_THRESHOLD = 1 << 10
        W_base = W._BASE_PERIOD
        W._BASE_PERIOD = 1501
        t = W.Workload("t", 4, 1, 5000, "f32", ("normal", 1.0), seed=11)
        assert t.tiled and len({t.period(r) for r in range(4)}) == 4
        full = t.host(3)
        idx = np.array([0, 1, 1400, 1500, 2999, 4999])
        assert (t.gather(3, idx) == full[idx]).all()
        for lo, ln in ((0, 5000), (1400, 200), (2999, 2001), (4999, 1), (1483, 1483)):
            assert (t.window(3, lo, ln) == full[lo:lo + ln]).all()
        assert (w.window(2, 100, 900) == w.host(2)[100:1000]).all()      # untiled: a plain slice
    finally:
        W.TILE_THRESHOLD = old
        W._BASE_PERIOD = W_base
    for dt, dist in (("f32", ("normal", 1.0)), ("i32", ("uniform_int", -1000, 1000)), ("bf16", ("normal", 1e-3))):
        h = W.Workload("t", 4, 1, 100000, dt, dist, seed=3)
        assert (h.head(2, 777) == h.host(2)[:777]).all()
    assert W.cfg3().tiled and not W.cfg2().tiled
    assert 0 <= W.cfg3().straggler < 8


def test_streamed_fold_equals_the_fold_in_one_piece(monkeypatch):
    """The window-by-window evaluation the GPU tests use for buffers too large to hold n of on
    the host gives the same bits as the oracle's fold over whole (tiled) buffers."""
    import gpu_util as G
    monkeypatch.setattr(G, "WINDOW", 1000)
    monkeypatch.setattr(G, "BLOCK", 300)
    monkeypatch.setattr(W, "TILE_THRESHOLD", 1 << 10)
    monkeypatch.setattr(W, "_BASE_PERIOD", 1501)
    for dt in ("bf16", "f32", "i32"):
        dist = ("uniform_int", -1000, 1000) if dt == "i32" else ("normal", 1.0)
        w = W.Workload("t", 8, 5, 7 * 2300 + 11, dt, dist, seed=9)
        assert w.tiled
        xs = w.host_all()
        bases = [w.base(r) for r in range(w.n)]
        chunks = S.chunk_layout(w.count, w.n - 1, EB[dt])
        mid, _ = stragglar_o1(xs, 5, dt, stop_after_rs=True)
        want = R.stragglar_fold(xs, 5, dt, elem_bytes=EB[dt])
        seen = 0
        for c, lo, final, partial in G.streamed_fold(w, "stragglar", bases):
            assert chunks[c][0] <= lo and lo + len(final) <= chunks[c][0] + chunks[c][1]
            assert (final.view(np.uint8) == want[lo:lo + len(final)].view(np.uint8)).all()
            owner = mid[S.to_physical(c, w.n, 5)][lo:lo + len(final)]
            assert (partial.view(np.uint8) == owner.view(np.uint8)).all()
            seen += len(final)
        assert seen == w.count
        rwant = R.ring_fold(xs, dt, elem_bytes=EB[dt])
        seen = 0
        for c, lo, final, _ in G.streamed_fold(w, "ring", bases):
            assert (final.view(np.uint8) == rwant[lo:lo + len(final)].view(np.uint8)).all()
            seen += len(final)
        assert seen == w.count
