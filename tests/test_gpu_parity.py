"""GPU parity: the HIP library, called through its C ABI, against the CPU
oracle on the same seeded inputs.  Bit-exact for int32 and for the
schedule-ordered fp32 / bf16 result; within 1e-5*n (fp32) / 2^-7*n (bf16),
relative to sum_i |x_i|, of the fp64 sum."""

import numpy as np
import pytest
import torch

import synth_inputs as W
from gpu_util import (EB, check_tolerance, gpu_call, gpu_ring, gpu_stragglar, oracle_ring,
                      oracle_rounds, oracle_stragglar, same_bits, streamed_compare, to_device, to_host)
from oracle import reference as R
from oracle import replay as P
from oracle import schedule as S

pytestmark = pytest.mark.gpu


def full_check(lib, w, stream=None, ring=True):
    xs = w.host_all()
    mid, out = gpu_stragglar(lib, xs, w.straggler, w.dtype, stream)
    omid, oout = oracle_stragglar(xs, w.straggler, w.dtype)
    check_precondition(lib, mid, omid, xs, w.straggler, w.dtype)
    for r in range(w.n):
        assert same_bits(out[r], oout[r]), "completion, rank %d" % r
    fold = R.stragglar_fold(xs, w.straggler, w.dtype, elem_bytes=EB[w.dtype])
    assert same_bits(out[0], fold)
    check_tolerance(out[0], xs, w.dtype)
    if ring:
        rout = gpu_ring(lib, xs, w.dtype, stream)
        oring = oracle_ring(xs, w.dtype)
        for r in range(w.n):
            assert same_bits(rout[r], oring[r]), "ring, rank %d" % r
        check_tolerance(rout[0], xs, w.dtype)


def full_check_chains_only(lib, w):
    """Precondition and ring against the oracle's replay, the completion against the schedule-free
    fold (rank counts whose completion schedule the oracle plans too slowly)."""
    xs = w.host_all()
    mid, out = gpu_stragglar(lib, xs, w.straggler, w.dtype)
    eb = EB[w.dtype]
    omid = [x.copy() for x in xs]
    P.replay(S.rs_precondition_rounds(w.n, w.straggler), S.chunk_layout(w.count, w.n - 1, eb), omid, w.dtype)
    check_precondition(lib, mid, omid, xs, w.straggler, w.dtype)
    fold = R.stragglar_fold(xs, w.straggler, w.dtype, elem_bytes=eb)
    assert all(same_bits(o, fold) for o in out)
    rout = gpu_ring(lib, xs, w.dtype)
    oring = oracle_ring(xs, w.dtype)
    for r in range(w.n):
        assert same_bits(rout[r], oring[r]), "ring, rank %d" % r


def check_precondition(lib, mid, omid, xs, straggler, dtype):
    """State after the precondition against the oracle's replay.  One launch per round leaves
    every cell as the replay does.  The single launch writes what the postcondition defines
    (Sec. 3.1: on-time rank g holds the partially reduced c_g; the straggler is untouched); any
    other chunk holds either the replay's partial sum or still its input."""
    n = len(xs)
    single = lib.tune_get("fuse_rounds") != 0     # the automatic mode may take either form
    assert same_bits(mid[straggler], xs[straggler])
    chunks = S.chunk_layout(len(xs[0]), n - 1, EB[dtype])
    for g in range(n - 1):
        r = S.to_physical(g, n, straggler)
        if not single:
            assert same_bits(mid[r], omid[r]), "precondition, rank %d" % r
            continue
        for c, (lo, ln) in enumerate(chunks):
            got, want = mid[r][lo:lo + ln], omid[r][lo:lo + ln]
            if c == g:
                assert same_bits(got, want), "precondition, rank %d own chunk" % r
            else:
                assert same_bits(got, want) or same_bits(got, xs[r][lo:lo + ln]), (r, c)


@pytest.fixture
def fused(lib):
    old = lib.tune_get("fuse_rounds")
    lib.tune_set("fuse_rounds", 1)
    yield lib
    lib.tune_set("fuse_rounds", old)


@pytest.fixture
def per_round(lib):
    old = lib.tune_get("fuse_rounds")
    lib.tune_set("fuse_rounds", 0)
    yield lib
    lib.tune_set("fuse_rounds", old)


def test_cfg1(lib):
    w = W.cfg1()
    full_check(lib, w)
    xs = w.host_all()
    _, out = gpu_stragglar(lib, xs, 0, "f32")
    exact = R.allreduce_exact_int(xs)
    assert all((o.astype(np.int64) == exact).all() for o in out)


@pytest.mark.parametrize("dtype", ["i32", "f32", "bf16"])
@pytest.mark.parametrize("n", [2, 4, 8, 16, 32])
def test_small_multi_tile_ragged(per_round, n, dtype):
    """Several tiles per chunk, a ragged vector tail and a ragged element tail."""
    count = (n - 1) * (3 * 4096 + 1000) + 13
    dist = ("uniform_int", -1000, 1000) if dtype == "i32" else ("normal", 1.0)
    for sg in sorted({0, n // 2, n - 1}):
        full_check(per_round, W.Workload("t", n, sg, count, dtype, dist, seed=n))


@pytest.mark.parametrize("n", [64, 256])
def test_many_ranks(per_round, n):
    lib = per_round
    count = 40 * n * n + 5
    full_check(lib, W.Workload("t", n, n // 3, count, "f32", ("normal", 1.0), seed=1))
    full_check(lib, W.Workload("t", n, 0, count, "bf16", ("normal", 1.0), seed=2), ring=False)


@pytest.mark.parametrize("fuse", [0, 1])
@pytest.mark.parametrize("dtype", ["i32", "f32", "bf16"])
def test_minimum_sizes(lib, dtype, fuse):
    q = 16 // EB[dtype]
    old = lib.tune_get("fuse_rounds")
    lib.tune_set("fuse_rounds", fuse)
    for n in (2, 4, 8):
        for count in (q * (n - 1) + 1, q * n, q * n + q - 1, 2 * q * n + 1):
            try:
                S.chunk_layout(count, n - 1, EB[dtype]), S.chunk_layout(count, n, EB[dtype])
            except ValueError:
                with pytest.raises(lib.StragglarError):
                    lib.stragglar_plan(n, 0, count, dtype)
                continue
            dist = ("uniform_int", -9, 9) if dtype == "i32" else ("normal", 1.0)
            full_check(lib, W.Workload("t", n, n - 1, count, dtype, dist, seed=count))
    lib.tune_set("fuse_rounds", old)


@pytest.mark.parametrize("unroll", [1, 2, 4])
@pytest.mark.parametrize("nt", [0, 1, -1])
def test_launch_shapes(lib, unroll, nt):
    old = {k: lib.tune_get(k) for k in ("unroll", "nontemporal", "blocks_per_cu", "fuse_rounds")}
    try:
        lib.tune_set("fuse_rounds", 0)
        lib.tune_set("unroll", unroll)
        lib.tune_set("nontemporal", nt)
        for bpc in (1, 3, 16):
            lib.tune_set("blocks_per_cu", bpc)
            full_check(lib, W.Workload("t", 8, 3, 7 * 300000 + 5, "bf16", ("normal", 1.0), seed=bpc))
    finally:
        for k, v in old.items():
            lib.tune_set(k, v)


@pytest.mark.parametrize("dtype", ["i32", "f32", "bf16"])
@pytest.mark.parametrize("n", [2, 4, 8, 16, 32])
def test_single_launch_mode(fused, n, dtype):
    """All rounds in one launch: same bits as the oracle's round-by-round replay."""
    count = (n - 1) * (3 * 4096 + 1000) + 13
    dist = ("uniform_int", -1000, 1000) if dtype == "i32" else ("normal", 1.0)
    for sg in sorted({0, n // 2, n - 1}):
        full_check(fused, W.Workload("t", n, sg, count, dtype, dist, seed=n))
    # launch shapes and hints; `direct`: the completion in the kernel written for its shape (1) or
    # in the general op-list kernel (0); the split form has a test of its own
    for nt, fu, wg, direct in ((0, 4, 0, 1), (1, 2, 2, 0), (0, 2, 6, 0), (1, 4, 3, 1), (1, 1, 4, 1), (0, 1, 0, 0)):
        fused.tune_set("nontemporal", nt)
        fused.tune_set("fused_unroll", fu)
        fused.tune_set("fused_wgs_per_cu", wg)
        fused.tune_set("fused_direct", direct)
        fused.tune_set("fused_split", 0)
        full_check(fused, W.Workload("t", n, 1, 40 * n * n + 5, dtype, dist, seed=3))
        full_check(fused, W.Workload("t", n, 0, (n - 1) * 2600 + 3, dtype, dist, seed=4), ring=False)
    fused.tune_set("nontemporal", -1)
    fused.tune_set("fused_unroll", -1)
    fused.tune_set("fused_wgs_per_cu", -1)
    fused.tune_set("fused_direct", -1)
    fused.tune_set("fused_split", -1)


@pytest.fixture
def merged(lib):
    """One launch per round with a round's copies of the same value read once."""
    old = {k: lib.tune_get(k) for k in ("fuse_rounds", "merge_copies")}
    lib.tune_set("fuse_rounds", 0)
    lib.tune_set("merge_copies", 1)
    yield lib
    for k, v in old.items():
        lib.tune_set(k, v)


@pytest.mark.parametrize("dtype", ["i32", "f32", "bf16"])
@pytest.mark.parametrize("n", [2, 4, 6, 8, 12, 16, 20, 32])
def test_merged_copies_mode(merged, n, dtype):
    """Round by round, but the copies of one value within a round are one multi-destination op
    (one holder read, k stores): same bits as the oracle's op-by-op replay, for StragglAR, the
    ring and the other baselines (the Broadcast baseline's doubling rounds are all such copies)."""
    lib = merged
    count = (n - 1) * (3 * 4096 + 1000) + 13
    dist = ("uniform_int", -1000, 1000) if dtype == "i32" else ("normal", 1.0)
    for sg in sorted({0, n // 2, n - 1}):
        w = W.Workload("t", n, sg, count, dtype, dist, seed=n)
        assert lib.stragglar_plan(n, sg, count, dtype).launch_form(lib.COMPLETION)["form"] == "per_round_merged_copies"
        if n <= 14 or n & (n - 1) == 0:
            full_check(lib, w)
        else:           # the oracle's App. D generator is too slow here: the schedule-free fold
            xs = w.host_all()
            _, out = gpu_stragglar(lib, xs, sg, dtype)
            fold = R.stragglar_fold(xs, sg, dtype, elem_bytes=EB[dtype])
            assert all(same_bits(o, fold) for o in out)
    baselines_check(lib, W.Workload("t", n, n - 1, n * (n - 1) * 300 + 13, dtype, dist, seed=n + 1))
    for unroll, nt, bpc in ((1, 1, 0), (4, 0, 3), (2, 1, 16)):
        old = {k: lib.tune_get(k) for k in ("unroll", "nontemporal", "blocks_per_cu")}
        try:
            lib.tune_set("unroll", unroll)
            lib.tune_set("nontemporal", nt)
            lib.tune_set("blocks_per_cu", bpc)
            full_check(lib, W.Workload("t", n, 1 % n, (n - 1) * 2600 + 3, dtype, dist, seed=4), ring=False)
        finally:
            for k, v in old.items():
                lib.tune_set(k, v)


@pytest.fixture
def split(lib):
    """Single-launch mode with every chunk's trailing copies run as a broadcast launch of their own."""
    old = {k: lib.tune_get(k) for k in ("fuse_rounds", "fused_split")}
    lib.tune_set("fuse_rounds", 1)
    lib.tune_set("fused_split", 1)
    yield lib
    for k, v in old.items():
        lib.tune_set(k, v)


@pytest.mark.parametrize("dtype", ["i32", "f32", "bf16"])
@pytest.mark.parametrize("n", [2, 4, 6, 8, 12, 16, 20, 32, 64])
def test_single_launch_split_mode(split, n, dtype):
    """The producing ops of every chunk in the op-list kernel, its trailing copies as a segment-
    ordered broadcast launch: same bits as the oracle's replay for StragglAR (both phases, also as
    one call), the ring and the other baselines; several tiles per chunk, more than one segment,
    a ragged vector tail and a ragged element tail."""
    lib = split
    dist = ("uniform_int", -1000, 1000) if dtype == "i32" else ("normal", 1.0)
    count = (n - 1) * (19 * 4096 + 1000) // (1 if n <= 16 else 4) + 13
    for sg in sorted({0, n // 2, n - 1}):
        w = W.Workload("t", n, sg, count, dtype, dist, seed=n)
        plan = lib.stragglar_plan(n, sg, count, dtype)
        if n > 2:
            assert plan.launch_form(lib.COMPLETION)["form"] == "single_launch_split"
            assert plan.launch_form(lib.COMPLETION)["launches"] == 2
        if n <= 14 or n & (n - 1) == 0:
            full_check(lib, w)
        xs = w.host_all()
        fold = R.stragglar_fold(xs, sg, dtype, elem_bytes=EB[dtype])
        dev = [to_device(x, dtype) for x in xs]
        lib.stragglar_allreduce(plan, dev)                    # both phases as one schedule, split as well
        torch.cuda.synchronize()
        for r in range(n):
            assert same_bits(to_host(dev[r], dtype), fold), (sg, r)
    baselines_check(lib, W.Workload("t", n, n - 1, n * (n - 1) * 300 + 13, dtype, dist, seed=n + 1))
    # tiny: chunks of n vectors, the last one a single element
    full_check(lib, W.Workload("t", n, 0, (16 // EB[dtype]) * n * (n - 1) + 1, dtype, dist, seed=5))


def test_merged_copies_many_ranks_falls_back(merged):
    """Above 32 ranks the merged form is not built: the call runs the rounds as written."""
    w = W.Workload("t", 64, 7, 40 * 64 * 64 + 5, "f32", ("normal", 1.0), seed=1)
    assert merged.stragglar_plan(64, 7, w.count, "f32").launch_form(merged.COMPLETION)["form"] == "per_round"
    full_check(merged, w, ring=False)


def test_plan_options_two_plans_two_forms_concurrently(lib):
    """Launch options belong to a plan: two plans of one shape, one set to run round by round and
    one as a single launch, called from two host threads at once on their own streams, each take
    their own form and both give the oracle's bits."""
    import threading
    w = W.Workload("t", 8, 3, 7 * 120000 + 5, "bf16", ("normal", 1.0), seed=91)
    xs = w.host_all()
    _, want = oracle_stragglar(xs, 3, "bf16")
    plans, bufs, streams, errors = [], [], [], []
    for form in (0, 1):
        p = lib.stragglar_plan(8, 3, w.count, "bf16")
        p.option_set("fuse_rounds", form)
        plans.append(p)
        bufs.append([to_device(x, "bf16") for x in xs])
        streams.append(torch.cuda.Stream())
    assert plans[0].launch_form(lib.COMPLETION)["form"] == "per_round"
    assert plans[1].launch_form(lib.COMPLETION)["form"] == "single_launch"
    pristine = [to_device(x, "bf16") for x in xs]
    torch.cuda.synchronize()

    def worker(i):
        try:
            with torch.cuda.stream(streams[i]):
                for _ in range(20):
                    for d, p0 in zip(bufs[i], pristine):
                        d.copy_(p0, non_blocking=True)
                    lib.stragglar_phase1_reducescatter(plans[i], bufs[i], streams[i])
                    lib.stragglar_phase2_complete(plans[i], bufs[i], streams[i])
            streams[i].synchronize()
        except Exception as e:
            errors.append(e)

    threads = [threading.Thread(target=worker, args=(i,)) for i in (0, 1)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for i in (0, 1):
        for r in range(8):
            assert same_bits(to_host(bufs[i][r], "bf16"), want[r]), (i, r)


@pytest.mark.parametrize("n", [64, 128, 256])
def test_single_launch_many_ranks(fused, n):
    """Above 32 ranks the precondition and the ring run as reduce chains described by their ring
    (one launch at any rank count); with the op-list kernel instead (fused_direct 0) a call uses
    the wide argument layout and takes several launches, and the 256-rank ring exceeds one launch
    per chunk index and runs round by round."""
    w = W.Workload("t", n, 5, 20 * n * n + 5, "f32", ("normal", 1.0), seed=1)
    plan = fused.stragglar_plan(n, 5, w.count, "f32")
    assert plan.launch_form(fused.PRECONDITION) == dict(plan.launch_form(fused.PRECONDITION), form="single_launch", launches=1)
    assert plan.launch_form(fused.RING)["launches"] == 1
    full_check(fused, w)
    if n == 64:
        full_check(fused, W.Workload("t", n, 63, 20 * n * n + 3, "bf16", ("normal", 1.0), seed=2))
        baselines_check(fused, W.Workload("t", n, 0, 20 * n * n + 5, "i32", ("uniform_int", -99, 99), seed=3))
    if n != 128:
        old = fused.tune_get("fused_direct")
        fused.tune_set("fused_direct", 0)
        try:
            assert fused.stragglar_plan(n, 5, w.count, "f32").launch_form(fused.PRECONDITION)["launches"] > 1
            full_check(fused, w)
        finally:
            fused.tune_set("fused_direct", old)


@pytest.mark.parametrize("dtype", ["i32", "f32", "bf16"])
@pytest.mark.parametrize("n", [2, 6, 8, 12, 32, 34])
def test_reduce_chain_kernel(fused, n, dtype):
    """The precondition, the ring AllReduce and the Broadcast baseline's AllReduce among the
    on-time ranks in the kernel that walks a ring of ranks from a start position per chunk index
    (fused_direct 1), in one launch and - the ring - split into a chain launch and a broadcast
    launch: same bits as the oracle's replay; several tiles, ragged tails, tiny chunks."""
    lib = fused
    dist = ("uniform_int", -1000, 1000) if dtype == "i32" else ("normal", 1.0)
    old = {k: lib.tune_get(k) for k in ("fused_direct", "fused_split", "fused_unroll", "fused_wgs_per_cu", "nontemporal")}
    try:
        lib.tune_set("fused_direct", 1)
        for split, fu, wg, nt in ((0, -1, -1, -1), (1, 1, 3, 1), (0, 2, 0, 0), (1, 2, 2, -1)):
            lib.tune_set("fused_split", split)
            lib.tune_set("fused_unroll", fu)
            lib.tune_set("fused_wgs_per_cu", wg)
            lib.tune_set("nontemporal", nt)
            count = (n - 1) * (5 * 4096 + 1000) // (1 if n <= 16 else 4) + 13
            plan = lib.stragglar_plan(n, n // 2, count, dtype)
            if n > 2:
                assert plan.launch_form(lib.PRECONDITION)["launches"] == 1
            assert plan.launch_form(lib.RING)["launches"] == (2 if split else 1)
            for sg in sorted({0, n - 1}):
                w = W.Workload("t", n, sg, count, dtype, dist, seed=n + split)
                if n <= 14 or n & (n - 1) == 0:
                    full_check(lib, w)
                else:       # the oracle's App. D generator is too slow here: precondition and ring only
                    full_check_chains_only(lib, w)
            baselines_check(lib, W.Workload("t", n, n - 1, n * (n - 1) * 300 + 13, dtype, dist, seed=n + 1))
            if n <= 14 or n & (n - 1) == 0:     # tiny: chunks of n vectors, the last one a single element
                full_check(lib, W.Workload("t", n, 0, (16 // EB[dtype]) * n * (n - 1) + 1, dtype, dist, seed=5))
    finally:
        for k, v in old.items():
            lib.tune_set(k, v)


@pytest.mark.parametrize("dtype", ["i32", "f32", "bf16"])
@pytest.mark.parametrize("n", [2, 8, 32])
def test_per_round_mode_small(per_round, n, dtype):
    """Small buffers default to the single launch; the per-round path must agree too."""
    dist = ("uniform_int", -1000, 1000) if dtype == "i32" else ("normal", 1.0)
    full_check(per_round, W.Workload("t", n, n - 1, (n - 1) * 5000 + 7, dtype, dist, seed=n))


def baselines_check(lib, w):
    """Recursive halving/doubling and the Broadcast baseline against the oracle's replay."""
    xs = w.host_all()
    n, sg, dt = w.n, w.straggler, w.dtype
    if n & (n - 1) == 0:
        (rhd,) = gpu_call(lib, ["rhd_allreduce"], xs, sg, dt)
        want = oracle_rounds(S.rhd_allreduce_rounds(n), n, xs, dt)
        for r in range(n):
            assert same_bits(rhd[r], want[r]), "rhd, rank %d" % r
        assert same_bits(rhd[0], R.rhd_fold(xs, dt, elem_bytes=EB[dt]))
        check_tolerance(rhd[0], xs, dt)
    else:
        with pytest.raises(lib.StragglarError) as e:
            gpu_call(lib, ["rhd_allreduce"], xs, sg, dt)
        assert e.value.status == 2
    mid, out = gpu_call(lib, ["broadcast_phase1_allreduce", "broadcast_phase2_complete"], xs, sg, dt)
    wmid = oracle_rounds(S.broadcast_precondition_rounds(n, sg), n - 1, xs, dt)
    wout = oracle_rounds(S.broadcast_completion_rounds(n, sg), n - 1, wmid, dt)
    for r in range(n):
        assert same_bits(mid[r], wmid[r]), "broadcast phase 1, rank %d" % r
        assert same_bits(out[r], wout[r]), "broadcast phase 2, rank %d" % r
    assert same_bits(mid[sg], xs[sg])
    assert same_bits(out[0], R.stragglar_fold(xs, sg, dt, elem_bytes=EB[dt]))    # same bits as StragglAR


@pytest.mark.parametrize("fuse", [0, 1])
@pytest.mark.parametrize("dtype", ["i32", "f32", "bf16"])
@pytest.mark.parametrize("n", [2, 4, 8, 16, 32])
def test_rhd_and_broadcast_baselines(lib, n, dtype, fuse):
    old = lib.tune_get("fuse_rounds")
    lib.tune_set("fuse_rounds", fuse)
    try:
        dist = ("uniform_int", -1000, 1000) if dtype == "i32" else ("normal", 1.0)
        count = n * (n - 1) * 300 + 13
        for sg in sorted({0, n - 1}):
            baselines_check(lib, W.Workload("t", n, sg, count, dtype, dist, seed=n))
    finally:
        lib.tune_set("fuse_rounds", old)


@pytest.mark.parametrize("fuse", [0, 1])
@pytest.mark.parametrize("dtype", ["i32", "f32", "bf16"])
@pytest.mark.parametrize("n", [6, 10, 12, 20, 24, 40])
def test_even_non_power_of_two_ranks(lib, n, dtype, fuse):
    """App. D schedules (maximum-weight matching per round) on the same kernels."""
    old = lib.tune_get("fuse_rounds")
    lib.tune_set("fuse_rounds", fuse)
    try:
        dist = ("uniform_int", -1000, 1000) if dtype == "i32" else ("normal", 1.0)
        count = n * (n - 1) * 200 + 13
        for sg in sorted({0, n - 1}):
            w = W.Workload("t", n, sg, count, dtype, dist, seed=n)
            if n <= 14:
                full_check(lib, w)
                baselines_check(lib, w)
            else:       # the oracle's generator is too slow here: schedule-free references only
                xs = w.host_all()
                _, out = gpu_stragglar(lib, xs, sg, dtype)
                fold = R.stragglar_fold(xs, sg, dtype, elem_bytes=EB[dtype])
                assert all(same_bits(o, fold) for o in out)
                check_tolerance(out[0], xs, dtype)
    finally:
        lib.tune_set("fuse_rounds", old)


def test_baselines_many_ranks(lib):
    baselines_check(lib, W.Workload("t", 64, 9, 64 * 63 * 40 + 5, "f32", ("normal", 1.0), seed=6))


def test_special_values(lib):
    """Denormals are kept, infinities propagate, bf16 ties go to even."""
    n, count = 4, 3 * 4096
    rng = np.random.Generator(np.random.Philox(key=[1, 2]))
    xs = [(rng.integers(0, 1 << 23, count, dtype=np.uint32) | (rng.integers(0, 2, count, dtype=np.uint32) << 31))
          .view(np.float32).copy() for _ in range(n)]                        # all subnormal
    xs[1][::7] = np.float32(3e38)
    xs[2][::7] = np.float32(3e38)                                             # overflow to +inf
    xs[3][::11] = np.float32(1.0)
    mid, out = gpu_stragglar(lib, xs, 2, "f32")
    omid, oout = oracle_stragglar(xs, 2, "f32")
    assert all(same_bits(a, b) for a, b in zip(out, oout))
    assert np.isinf(out[0][::7]).all() and (np.abs(out[0][1:7]) < 1e-37).all() and (out[0][1:7] != 0).any()
    # bf16: 1.0 + 2^-8 is a tie in bf16 (8 significand bits): goes to even
    a = np.full(count, 0x3F80, np.uint16)          # 1.0
    b = np.full(count, 0x3B80, np.uint16)          # 2^-8
    c = np.full(count, 0x3F81, np.uint16)          # 1.0078125
    z = np.zeros(count, np.uint16)
    _, out = gpu_stragglar(lib, [a, z, z, b], 3, "bf16")
    assert (out[0] == 0x3F80).all()
    _, out = gpu_stragglar(lib, [c, z, z, b], 3, "bf16")
    assert (out[0] == 0x3F82).all()
    rnd = [rng.integers(0, 1 << 16, count, dtype=np.uint16) & np.uint16(0xFF7F) for _ in range(n)]
    for x in rnd:                                   # keep them finite: clear exponent 0xFF
        x[(x & 0x7F80) == 0x7F80] = 0
    _, out = gpu_stragglar(lib, rnd, 0, "bf16")
    _, oout = oracle_stragglar(rnd, 0, "bf16")
    nan = np.isnan(R.to_f64(oout[0], "bf16"))
    assert (out[0][~nan] == oout[0][~nan]).all() and np.isnan(R.to_f64(out[0], "bf16")[nan]).all()


def test_side_stream(lib):
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        full_check(lib, W.Workload("t", 8, 5, 7 * 200000 + 3, "f32", ("normal", 1.0), seed=8), stream=s)


def test_delay_kernel_holds_a_stream_and_overlaps(lib):
    """The straggler emulation of Sec. 4.1: a timed idle kernel on one stream while the
    precondition runs on another; both must finish, and the idle time must be about right."""
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    lib.stragglar_delay(1000)            # warm-up launch
    torch.cuda.synchronize()
    a.record()
    lib.stragglar_delay(3_000_000)
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b)
    assert 2.9 <= ms <= 10.0, ms       # never shorter than asked; the upper bound is generous
    # overlap: delay on a side stream, precondition on the main stream, completion after both
    w = W.Workload("t", 8, 7, 7 * 400000 + 5, "f32", ("normal", 1.0), seed=12)
    xs = w.host_all()
    dev = [to_device(x, "f32") for x in xs]
    plan = lib.stragglar_plan(8, 7, w.count, "f32")
    late = torch.cuda.Stream()
    main = torch.cuda.current_stream()
    torch.cuda.synchronize()
    arrived = torch.cuda.Event()
    lib.stragglar_delay(2_000_000, late)
    arrived.record(late)
    lib.stragglar_phase1_reducescatter(plan, dev, main)
    main.wait_event(arrived)
    lib.stragglar_phase2_complete(plan, dev, main)
    torch.cuda.synchronize()
    _, oout = oracle_stragglar(xs, 7, "f32")
    assert all(same_bits(to_host(d, "f32"), o) for d, o in zip(dev, oout))


@pytest.mark.parametrize("fuse", [0, 1, 2])
@pytest.mark.parametrize("one_call", [False, True])
def test_graph_capture_and_replay(lib, fuse, one_call):
    """The entry points only enqueue kernels on the caller's stream, so they can be recorded
    into a HIP graph; every replay must reproduce the eager result."""
    def enqueue(plan, work, stream):
        if one_call:
            lib.stragglar_allreduce(plan, work, stream)
        else:
            lib.stragglar_phase1_reducescatter(plan, work, stream)
            lib.stragglar_phase2_complete(plan, work, stream)

    old = lib.tune_get("fuse_rounds")
    old_split = lib.tune_get("fused_split")
    lib.tune_set("fuse_rounds", min(fuse, 1))
    lib.tune_set("fused_split", 1 if fuse == 2 else -1)       # 2: single launch with the broadcast split off
    try:
        w = W.Workload("t", 8, 2, 7 * 150000 + 9, "bf16", ("normal", 1.0), seed=21)
        xs = w.host_all()
        pristine = [to_device(x, "bf16") for x in xs]
        work = [torch.empty_like(t) for t in pristine]
        plan = lib.stragglar_plan(8, 2, w.count, "bf16")
        _, want = oracle_stragglar(xs, 2, "bf16")
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            for d, p in zip(work, pristine):           # warm-up outside the capture
                d.copy_(p)
            enqueue(plan, work, side)
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                for d, p in zip(work, pristine):
                    d.copy_(p)
                enqueue(plan, work, side)
        torch.cuda.synchronize()
        for rep in range(3):
            for d in work:
                d.zero_()                              # eager work between replays
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for r in range(8):
                assert same_bits(to_host(work[r], "bf16"), want[r]), (rep, r)
    finally:
        lib.tune_set("fuse_rounds", old)
        lib.tune_set("fused_split", old_split)


@pytest.mark.parametrize("fuse", [0, 1, 2, 3])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_buffers_with_different_16_byte_offsets(lib, dtype, fuse):
    """Rank buffers need only be 16-byte aligned, each at its own offset from a 128-byte line.
    fuse: 0 one launch per round, 1 single launch, 2 single launch with the broadcast split off,
    3 one launch per round with a round's same-value copies merged."""
    old = lib.tune_get("fuse_rounds")
    old_more = {k: lib.tune_get(k) for k in ("fused_split", "merge_copies")}
    lib.tune_set("fuse_rounds", 1 if fuse in (1, 2) else 0)
    lib.tune_set("fused_split", 1 if fuse == 2 else 0)
    lib.tune_set("merge_copies", 1 if fuse == 3 else 0)
    try:
        n, sg = 8, 6
        w = W.Workload("t", n, sg, 7 * 9000 + 5, dtype, ("normal", 1.0), seed=77)
        xs = w.host_all()
        eb = EB[dtype]
        tdt = torch.float32 if dtype == "f32" else torch.bfloat16
        pad = 256 // eb
        stride = -(-w.count // pad) * pad + pad                          # a multiple of 256 bytes
        arena = torch.zeros(n * stride, dtype=tdt, device="cuda:0")
        dev = []
        for r in range(n):
            lo = r * stride + (16 // eb) * ((3 * r + 1) % 8)              # offsets 16, 64, 112, 32, ...
            view = arena[lo:lo + w.count]
            assert view.data_ptr() % 16 == 0
            view.copy_(to_device(xs[r], dtype))
            dev.append(view)
        assert len({d.data_ptr() % 128 for d in dev}) > 4
        plan = lib.stragglar_plan(n, sg, w.count, dtype)
        lib.stragglar_phase1_reducescatter(plan, dev)
        lib.stragglar_phase2_complete(plan, dev)
        torch.cuda.synchronize()
        _, want = oracle_stragglar(xs, sg, dtype)
        for r in range(n):
            assert same_bits(to_host(dev[r], dtype), want[r]), r
        # nothing outside the views was touched
        mask = torch.ones_like(arena, dtype=torch.bool)
        for r, d in enumerate(dev):
            lo = (d.data_ptr() - arena.data_ptr()) // eb
            mask[lo:lo + w.count] = False
        assert float(arena[mask].float().abs().sum()) == 0.0
    finally:
        lib.tune_set("fuse_rounds", old)
        for k, v in old_more.items():
            lib.tune_set(k, v)


def test_plain_c_consumer(lib):
    """tests/c_abi_smoke.c: hipMalloc'ed buffers, the C ABI called from C, exact integer sums
    checked in C - no Python or PyTorch on the path.  Built beforehand with the library."""
    import os
    import subprocess
    exe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_abi_smoke")
    if not os.path.exists(exe):
        from paper_2505_23523_amd import build
        build.build_c_smoke()
    res = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "15 cases, 0 failed" in res.stdout


def test_two_streams_two_plans_concurrently(lib):
    """Plans are immutable and the library keeps no per-call state: two AllReduces of different
    shapes enqueued on two streams at once must both come out right."""
    wa = W.Workload("a", 8, 1, 7 * 250000 + 3, "f32", ("normal", 1.0), seed=31)
    wb = W.Workload("b", 16, 9, 15 * 70000 + 9, "bf16", ("normal", 1.0), seed=32)
    xa, xb = wa.host_all(), wb.host_all()
    da = [to_device(x, "f32") for x in xa]
    db = [to_device(x, "bf16") for x in xb]
    pa = lib.stragglar_plan(8, 1, wa.count, "f32")
    pb = lib.stragglar_plan(16, 9, wb.count, "bf16")
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    old = lib.tune_get("fuse_rounds")
    for fuse in (0, 1):
        lib.tune_set("fuse_rounds", fuse)
        for d, x in zip(da, xa):
            d.copy_(to_device(x, "f32"))
        for d, x in zip(db, xb):
            d.copy_(to_device(x, "bf16"))
        torch.cuda.synchronize()
        lib.stragglar_phase1_reducescatter(pa, da, sa)
        lib.stragglar_phase1_reducescatter(pb, db, sb)
        lib.stragglar_phase2_complete(pa, da, sa)
        lib.stragglar_phase2_complete(pb, db, sb)
        torch.cuda.synchronize()
        _, oa = oracle_stragglar(xa, 1, "f32")
        _, ob = oracle_stragglar(xb, 9, "bf16")
        assert all(same_bits(to_host(d, "f32"), o) for d, o in zip(da, oa))
        assert all(same_bits(to_host(d, "bf16"), o) for d, o in zip(db, ob))
    lib.tune_set("fuse_rounds", old)


def test_two_host_threads(lib):
    """Two host threads, each with its own plan, buffers and stream, call the library at the same
    time (ctypes releases the interpreter lock during a call); many rounds of calls, then both
    results are checked.  A 40-rank plan is among them, whose launch mode is priced on first use.
    The expected values replay the completion rounds the LIBRARY emitted (the oracle's own App. D
    generator is too slow at 40 ranks; any valid schedule gives the same values, and that these
    rounds are valid is what the host tests of the emitted schedules check)."""
    import threading
    cases = [W.Workload("a", 8, 5, 7 * 90000 + 3, "f32", ("normal", 1.0), seed=61),
             W.Workload("b", 40, 11, 39 * 2100 + 7, "bf16", ("normal", 1.0), seed=62)]
    state = []
    for w in cases:
        xs = w.host_all()
        state.append({"w": w, "xs": xs, "pristine": [to_device(x, w.dtype) for x in xs],
                      "plan": lib.stragglar_plan(w.n, w.straggler, w.count, w.dtype),
                      "stream": torch.cuda.Stream(), "error": None})
    for st in state:
        st["work"] = [torch.empty_like(t) for t in st["pristine"]]
    torch.cuda.synchronize()

    def worker(st):
        try:
            with torch.cuda.stream(st["stream"]):
                for _ in range(25):
                    for d, p in zip(st["work"], st["pristine"]):
                        d.copy_(p, non_blocking=True)
                    lib.stragglar_allreduce(st["plan"], st["work"], st["stream"])
                    for d, p in zip(st["work"], st["pristine"]):
                        d.copy_(p, non_blocking=True)
                    lib.stragglar_phase1_reducescatter(st["plan"], st["work"], st["stream"])
                    lib.stragglar_phase2_complete(st["plan"], st["work"], st["stream"])
            st["stream"].synchronize()
        except Exception as e:          # surfaced in the main thread below
            st["error"] = e

    threads = [threading.Thread(target=worker, args=(st,)) for st in state]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    for st in state:
        assert st["error"] is None, st["error"]
        w = st["w"]
        chunks = S.chunk_layout(w.count, w.n - 1, EB[w.dtype])
        bufs = [x.copy() for x in st["xs"]]
        from oracle import replay as P
        P.replay(S.rs_precondition_rounds(w.n, w.straggler), chunks, bufs, w.dtype)
        P.replay(st["plan"].rounds(lib.COMPLETION), chunks, bufs, w.dtype)   # 40 ranks: the emitted plan
        for r in range(w.n):
            assert same_bits(to_host(st["work"][r], w.dtype), bufs[r]), (w.name, r)


def test_allreduce_one_call_with_arrival_event(lib):
    """stragglar_allreduce: precondition at once, completion behind the straggler's event.  The
    straggler's buffer is written on the late stream AFTER an emulated delay, so a completion
    that did not wait for the event would add stale data."""
    w = W.Workload("t", 8, 4, 7 * 300000 + 1, "f32", ("normal", 1.0), seed=41)
    xs = w.host_all()
    _, want = oracle_stragglar(xs, 4, "f32")
    plan = lib.stragglar_plan(8, 4, w.count, "f32")
    late, main = torch.cuda.Stream(), torch.cuda.current_stream()
    fresh = to_device(xs[4], "f32")
    old = lib.tune_get("fuse_rounds")
    for fuse in (0, 1):
        lib.tune_set("fuse_rounds", fuse)
        dev = [to_device(x, "f32") for x in xs]
        dev[4].zero_()                                   # the straggler has not produced its data yet
        torch.cuda.synchronize()
        ready = torch.cuda.Event()
        lib.stragglar_delay(3_000_000, late)             # ... it is 3 ms late
        with torch.cuda.stream(late):
            dev[4].copy_(fresh, non_blocking=True)
        ready.record(late)
        lib.stragglar_allreduce(plan, dev, main, ready)
        torch.cuda.synchronize()
        assert all(same_bits(to_host(d, "f32"), o) for d, o in zip(dev, want)), fuse
        dev = [to_device(x, "f32") for x in xs]          # and without an event: back to back
        lib.stragglar_allreduce(plan, dev)
        torch.cuda.synchronize()
        assert all(same_bits(to_host(d, "f32"), o) for d, o in zip(dev, want)), fuse
    lib.tune_set("fuse_rounds", old)


def test_precondition_runs_while_the_straggler_is_late(lib):
    """Sec. 3 / Sec. 4.1: the precondition overlaps the straggler's delay, so a call that has to
    wait 6 ms for the straggler takes about 6 ms plus the completion, not plus both phases.  The
    late rank idles on a stream that is first shown to run beside the main stream (streams that
    share a hardware queue would run one after the other)."""
    main = torch.cuda.current_stream()
    late = None
    for _ in range(8):
        cand = torch.cuda.Stream()
        torch.cuda.synchronize()
        t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0.record(main)
        cand.wait_event(t0)
        lib.stragglar_delay(2_000_000, cand)
        lib.stragglar_delay(1_000, main)
        t1.record(main)
        torch.cuda.synchronize()
        if t0.elapsed_time(t1) < 1.0:
            late = cand
            break
    if late is None:
        pytest.skip("no second stream runs beside the main stream here")
    n, count = 8, 64 << 20                       # 256 MiB per rank: each phase takes a few tenths of a ms
    dev = [torch.zeros(count, dtype=torch.float32, device="cuda:0") for _ in range(n)]
    plan = lib.stragglar_plan(n, 0, count, "f32")
    plan.option_set("fuse_rounds", 0)

    def timed(fn):
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(main)
        fn()
        b.record(main)
        torch.cuda.synchronize()
        return a.elapsed_time(b)

    lib.stragglar_allreduce(plan, dev, main)     # warm-up
    p1 = min(timed(lambda: lib.stragglar_phase1_reducescatter(plan, dev, main)) for _ in range(3))
    p2 = min(timed(lambda: lib.stragglar_phase2_complete(plan, dev, main)) for _ in range(3))
    assert p1 > 0.3 and p2 > 0.3, (p1, p2)

    def delayed_call():
        start, arrived = torch.cuda.Event(), torch.cuda.Event()
        start.record(main)
        late.wait_event(start)
        lib.stragglar_delay(6_000_000, late)
        arrived.record(late)
        lib.stragglar_allreduce(plan, dev, main, arrived)

    total = min(timed(delayed_call) for _ in range(3))
    assert total >= 6.0 + 0.8 * p2, (total, p1, p2)          # the completion did wait for the straggler
    assert total <= 6.0 + p2 + 0.5 * p1, (total, p1, p2)      # ... and the precondition did not


@pytest.mark.parametrize("dtype", ["i32", "f32", "bf16"])
@pytest.mark.parametrize("n", [2, 4, 6, 8, 12, 16, 32, 64])
def test_allreduce_both_phases_in_one_launch(fused, n, dtype):
    """stragglar_allreduce without an arrival event in single-launch mode: every tile goes through
    the precondition's and the completion's ops in one launch; same bits as the oracle's replay
    of the two schedules."""
    count = (n - 1) * (2 * 4096 + 700) + 11
    dist = ("uniform_int", -1000, 1000) if dtype == "i32" else ("normal", 1.0)
    for sg in sorted({0, n // 2, n - 1}):
        w = W.Workload("t", n, sg, count, dtype, dist, seed=50 + n)
        xs = w.host_all()
        _, want = oracle_stragglar(xs, sg, dtype)
        dev = [to_device(x, dtype) for x in xs]
        plan = fused.stragglar_plan(n, sg, count, dtype)
        assert plan.num_rounds(fused.ALLREDUCE) == plan.num_rounds(fused.PRECONDITION) + plan.num_rounds(fused.COMPLETION)
        fused.stragglar_allreduce(plan, dev)
        torch.cuda.synchronize()
        for r in range(n):
            assert same_bits(to_host(dev[r], dtype), want[r]), (sg, r)


def test_allreduce_one_launch_cfg2(fused):
    w = W.cfg2()
    xs = w.host_all()
    fold = R.stragglar_fold(xs, w.straggler, "f32", elem_bytes=4)
    dev = [to_device(x, "f32") for x in xs]
    plan = fused.stragglar_plan(w.n, w.straggler, w.count, "f32")
    fused.stragglar_allreduce(plan, dev)
    torch.cuda.synchronize()
    want = torch.from_numpy(fold.view(np.int32)).to("cuda:0")
    for r in range(w.n):
        assert torch.equal(dev[r].view(torch.int32), want), r


@pytest.mark.parametrize("seed", range(32))
def test_seeded_random_cases(lib, seed):
    """Rank count, straggler, dtype, length and every launch option drawn from a seed: full
    comparison with the oracle's replay after both phases and for the ring."""
    rng = np.random.Generator(np.random.Philox(key=[77, seed]))
    n = int(rng.choice([2, 4, 6, 8, 10, 12, 14, 16, 18, 20, 32, 64]))     # the oracle's own generator is quick for these
    dtype = ["i32", "f32", "bf16"][int(rng.integers(0, 3))]
    sg = int(rng.integers(0, n))
    count = int(rng.integers(n * 8, 40000 + 3000 * n))
    options = {"fuse_rounds": int(rng.integers(-1, 2))}
    if seed >= 16:          # the first sixteen cases keep the draws they always had
        options.update(merge_copies=int(rng.integers(0, 2)), fused_split=int(rng.integers(-1, 2)),
                       fused_direct=int(rng.integers(-1, 2)), unroll=int(rng.choice([-1, 1, 2, 4])),
                       fused_unroll=int(rng.choice([-1, 1, 2, 4])), nontemporal=int(rng.integers(-1, 2)),
                       fused_wgs_per_cu=int(rng.choice([-1, 0, 2, 3, 4, 6])), blocks_per_cu=int(rng.choice([0, 0, 2, 7])))
    dist = ("uniform_int", -1000, 1000) if dtype == "i32" else ("normal", 1.0)
    old = {k: lib.tune_get(k) for k in options}
    for k, v in options.items():
        lib.tune_set(k, v)
    try:
        full_check(lib, W.Workload("t", n, sg, count, dtype, dist, seed=1000 + seed))
    finally:
        for k, v in old.items():
            lib.tune_set(k, v)


@pytest.mark.parametrize("seed", range(12))
def test_seeded_random_cases_many_ranks(lib, seed):
    """34 to 256 ranks (also even rank counts that are not powers of two), every single-launch
    option drawn from a seed: precondition and ring against the oracle's replay, the completion
    against the schedule-free fold."""
    rng = np.random.Generator(np.random.Philox(key=[78, seed]))
    n = int(rng.choice([34, 40, 48, 64, 66, 96, 128, 130, 256]))
    dtype = ["i32", "f32", "bf16"][int(rng.integers(0, 3))]
    sg = int(rng.integers(0, n))
    count = int(rng.integers(8 * n * n, 8 * n * n + 3000 * n))      # every chunk non-empty under the 16-byte rule
    options = {"fuse_rounds": int(rng.integers(-1, 2)), "fused_split": int(rng.integers(-1, 2)),
               "fused_direct": int(rng.integers(-1, 2)), "fused_unroll": int(rng.choice([-1, 1, 2, 4])),
               "nontemporal": int(rng.integers(-1, 2)), "fused_wgs_per_cu": int(rng.choice([-1, 0, 2, 3, 4, 6]))}
    dist = ("uniform_int", -1000, 1000) if dtype == "i32" else ("normal", 1.0)
    old = {k: lib.tune_get(k) for k in options}
    for k, v in options.items():
        lib.tune_set(k, v)
    try:
        full_check_chains_only(lib, W.Workload("t", n, sg, count, dtype, dist, seed=2000 + seed))
    finally:
        for k, v in old.items():
            lib.tune_set(k, v)


def test_int32_wraparound(lib):
    n, count = 8, 7 * 5000
    xs = [np.full(count, 2 ** 30, np.int32) for _ in range(n)]
    _, out = gpu_stragglar(lib, xs, 1, "i32")
    assert all((o == 0).all() for o in out)         # 8 * 2^30 = 2^33 = 0 mod 2^32


def test_device_errors_are_reported(lib):
    plan = lib.stragglar_plan(4, 0, 4096, "f32")
    t = [torch.zeros(4096, device="cuda:0") for _ in range(4)]
    with pytest.raises(ValueError):
        lib.stragglar_phase2_complete(plan, t[:3])
    with pytest.raises(lib.StragglarError):
        lib.stragglar_phase2_complete(plan, [t[0], t[1], t[2], t[2]])       # overlapping
    view = torch.zeros(4100, device="cuda:0")[1:4097]
    with pytest.raises(lib.StragglarError):
        lib.ring_allreduce(plan, [t[0], t[1], t[2], view])                  # misaligned


# ---- the benchmark configurations at full size --------------------------------
# "per_round" is the configuration bench.py's headline is timed in; "fused" the library default.
@pytest.mark.parametrize("dtype", ["f32", "i32"])
def test_cfg2_full_size(per_round, dtype):
    full_check(per_round, W.cfg2(dtype))


def test_cfg2_full_size_single_launch(fused):
    full_check(fused, W.cfg2("f32"))


def test_cfg2_full_size_merged_copies(merged):
    full_check(merged, W.cfg2("f32"), ring=False)


@pytest.mark.parametrize("fuse", [0, 1])
def test_cfg4_full_size(lib, fuse):
    old = lib.tune_get("fuse_rounds")
    lib.tune_set("fuse_rounds", fuse)
    try:
        full_check(lib, W.cfg4())
        baselines_check(lib, W.cfg4())
    finally:
        lib.tune_set("fuse_rounds", old)


@pytest.mark.parametrize("n", [16, 32])
def test_cfg5_all_stragglers(lib, n):
    """Every straggler rank; even ranks one launch per round (every other one of them with a
    round's same-value copies merged), odd ranks single launch."""
    base = W.cfg5(n, 0)
    xs = base.host_all()
    L = n.bit_length() - 1
    dev0 = [to_device(x, "f32") for x in xs]
    dev = [torch.empty_like(t) for t in dev0]
    old = lib.tune_get("fuse_rounds")
    for sg in range(n):
        lib.tune_set("fuse_rounds", sg % 2)
        plan = lib.stragglar_plan(n, sg, base.count, "f32")
        plan.option_set("merge_copies", 1 if sg % 4 == 2 else 0)      # every fourth: copies read once per round
        assert plan.num_rounds(lib.COMPLETION) == n + L - 2          # Thm. 1
        for d, s in zip(dev, dev0):
            d.copy_(s)
        lib.stragglar_phase1_reducescatter(plan, dev)
        lib.stragglar_phase2_complete(plan, dev)
        torch.cuda.synchronize()
        fold = R.stragglar_fold(xs, sg, "f32", elem_bytes=4)
        fold_dev = torch.from_numpy(fold).to("cuda:0")
        for r in range(n):
            assert torch.equal(dev[r].view(torch.int32), fold_dev.view(torch.int32)), (sg, r)
        if sg in (0, n - 1):
            _, oout = oracle_stragglar(xs, sg, "f32")
            assert same_bits(oout[0], fold) and same_bits(to_host(dev[sg], "f32"), oout[sg])
            check_tolerance(fold, xs, "f32")
    lib.tune_set("fuse_rounds", old)


@pytest.mark.parametrize("fuse", [0, 1])
def test_cfg3_full_size_sampled(lib, fuse):
    """1.24e9 bf16 per rank: the oracle's fold is evaluated on sampled windows
    (chunk heads and tails, tile borders, random interior) of every rank."""
    old = lib.tune_get("fuse_rounds")
    lib.tune_set("fuse_rounds", fuse)
    try:
        _cfg3_sampled(lib)
    finally:
        lib.tune_set("fuse_rounds", old)


def _cfg3_sampled(lib):
    sampled_check(lib, W.cfg3())


def run_both_modes(lib, w, bases, fn_names, keep_partials=False):
    """The entry points ``fn_names`` in sequence on fresh device copies of ``w``, once with one
    launch per round and once as a single launch.  Returns (all rank buffers of both runs, per run
    the on-time owners' chunks as they were after the first call)."""
    n, sg = w.n, w.straggler
    chunks = S.chunk_layout(w.count, n - 1, EB[w.dtype])
    plan = lib.stragglar_plan(n, sg, w.count, w.dtype)
    finals, partials = [], []
    old = lib.tune_get("fuse_rounds")
    try:
        for fuse in (0, 1):
            lib.tune_set("fuse_rounds", fuse)
            dev = [w.device(r, base=bases[r]) for r in range(n)]
            for k, name in enumerate(fn_names):
                getattr(lib, name)(plan, dev)
                if k == 0 and keep_partials:
                    torch.cuda.synchronize()
                    partials.append([dev[S.to_physical(g, n, sg)][lo:lo + ln].clone()
                                     for g, (lo, ln) in enumerate(chunks)])
            torch.cuda.synchronize()
            finals += dev
    finally:
        lib.tune_set("fuse_rounds", old)
    return finals, partials


@pytest.mark.parametrize("n,count,dtype", [(16, 48 * (1 << 20) + 4099, "f32"), (34, 76 * (1 << 20) + 77, "bf16")])
def test_split_completion_in_several_groups(lib, n, count, dtype):
    """Rank buffers large enough that the split completion runs as several exchange-and-broadcast
    pairs, each over a group of chunk indices (16 ranks: the exchange launch; 34 ranks - the
    matching-based schedule of App. D - the op-list kernel's producing pass): EVERY element of
    every rank buffer against the oracle's fold, streamed."""
    w = W.Workload("split-groups-n%d" % n, n, 3, count, dtype, ("normal", 1.0), seed=31)
    bases = [w.base(r) for r in range(n)]
    plan = lib.stragglar_plan(n, w.straggler, count, dtype)
    plan.option_set("fuse_rounds", 1)
    plan.option_set("fused_split", 1)
    form = plan.launch_form(lib.COMPLETION)
    assert form["form"] == "single_launch_split" and form["launches"] >= 4, form
    dev = [w.device(r, base=bases[r]) for r in range(n)]
    lib.stragglar_phase1_reducescatter(plan, dev)
    lib.stragglar_phase2_complete(plan, dev)
    torch.cuda.synchronize()
    assert streamed_compare(w, "stragglar", bases, dev) == count


def test_cfg3_full_size(lib):
    """The data-parallel gradient workload, 1.24e9 bf16 per rank, EVERY element: the oracle's fold
    is streamed over the whole buffer in windows and compared bit for bit with all 8 rank buffers
    of a round-by-round run and of a single-launch run, and its precondition partial with each
    on-time owner's chunk as the precondition left it.  (The fp64 tolerance is checked on the
    windows of the sampled test above.)"""
    w = W.cfg3()
    bases = [w.base(r) for r in range(w.n)]
    finals, partials = run_both_modes(lib, w, bases, ["stragglar_phase1_reducescatter", "stragglar_phase2_complete"],
                                      keep_partials=True)
    assert len(finals) == 2 * w.n and len(partials) == 2
    assert streamed_compare(w, "stragglar", bases, finals, partials) == 1_240_000_000


@pytest.mark.gpu
def test_largest_chunk_two_ranks(lib):
    """Two ranks of 64 GiB and a ragged tail each: the completion's single chunk has more 4 KiB
    tiles than one grid dimension holds (2^32 threads), so the per-round kernel strides and the
    single launch steps aside.  Windows straddle the point where the second stride begins."""
    count = (1 << 35) + 8 * 1000 + 5
    free, _ = torch.cuda.mem_get_info()
    if free < 2 * 2 * count + (4 << 30):
        pytest.skip("needs 130 GiB of free HBM")
    w = W.Workload("two-ranks-64GiB", 2, 1, count, "bf16", ("normal", 1.0), seed=21)
    wrap = ((1 << 24) - 1) * 256 * 8        # first element of the second stride (bf16, 8 per vector)
    sampled_check(lib, w, windows_per_chunk=24, extra_starts=(wrap - 2048, wrap - 4096, wrap, count - 4096 - 5))


def sampled_check(lib, w, windows_per_chunk=9, extra_starts=()):
    """Buffers too large for a full host replay: the oracle's fold on sampled 4096-element
    windows (each chunk's head, tail and middle plus random interior) of every rank, and the
    size-independent property that all ranks end with identical bits."""
    n, sg, dt = w.n, w.straggler, w.dtype
    eb = EB[dt]
    view = torch.int16 if dt == "bf16" else torch.int32
    bases = [w.base(r) for r in range(n)]
    dev = [w.device(r, base=bases[r]) for r in range(n)]
    plan = lib.stragglar_plan(n, sg, w.count, dt)
    lib.stragglar_phase1_reducescatter(plan, dev)
    lib.stragglar_phase2_complete(plan, dev)
    torch.cuda.synchronize()
    chunks = S.chunk_layout(w.count, n - 1, eb)
    rng = np.random.Generator(np.random.Philox(key=[33, 0]))
    for c, (lo, ln) in enumerate(chunks):
        starts = [lo, lo + ln - 4096, lo + ln // 2 - 2048] + \
                 [int(lo + v) for v in rng.integers(0, ln - 4096, size=windows_per_chunk - 3)] + \
                 [st for st in extra_starts if lo <= st and st + 4096 <= lo + ln]
        for st in starts:
            idx = np.arange(st, st + 4096)
            cols = [w.gather(r, idx, base=bases[r]) for r in range(n)]
            want = R.stragglar_fold_chunk(cols, c, sg, dt)
            want_dev = torch.from_numpy(want.view(np.int16 if dt == "bf16" else np.int32)).to("cuda:0")
            for r in range(n):
                got = dev[r][st:st + 4096].view(view)
                assert torch.equal(got, want_dev), (c, st, r)
            check_tolerance(want, cols, dt)
    for r in range(1, n):
        assert torch.equal(dev[0].view(view), dev[r].view(view))


@pytest.mark.parametrize("mib", [320, 2049])
def test_ring_large_buffers_full(lib, mib):
    """Ring baseline on rank buffers beyond the memory-side cache (other cache-hint sets than at
    the benchmark sizes), ragged tail included: the oracle's ring fold streamed over every element
    and compared with all ranks of a round-by-round and of a single-launch run."""
    w = W.cfg4(mib * (1 << 19) + 8 * 777 + 3)
    bases = [w.base(r) for r in range(w.n)]
    finals, _ = run_both_modes(lib, w, bases, ["ring_allreduce"])
    assert streamed_compare(w, "ring", bases, finals) == w.count


@pytest.mark.parametrize("mib", [1 << p for p in range(11)])
def test_cfg4_message_size_sweep(lib, mib):
    """1 MiB .. 1 GiB per rank in powers of two (the buffer sweep of Sec. 4.1), both launch modes,
    every element at every size: the oracle's fold streamed in windows (final value on all ranks,
    precondition partial on the owners)."""
    count = mib << 19
    assert count in W.cfg4_sweep_counts()
    w = W.cfg4(count)
    bases = [w.base(r) for r in range(w.n)]
    finals, partials = run_both_modes(lib, w, bases, ["stragglar_phase1_reducescatter", "stragglar_phase2_complete"],
                                      keep_partials=True)
    assert streamed_compare(w, "stragglar", bases, finals, partials) == count


def test_cfg4_hundred_calls(lib):
    """The tensor-parallel pattern: 100 AllReduces back to back on one stream, no host
    synchronisation in between; every call must give the bits of the first."""
    w = W.cfg4()
    pristine = [w.device(r) for r in range(w.n)]
    work = [torch.empty_like(t) for t in pristine]
    plan = lib.stragglar_plan(w.n, w.straggler, w.count, "bf16")
    first = None
    bad = torch.zeros((), dtype=torch.int64, device="cuda:0")
    for call in range(100):
        for d, p in zip(work, pristine):
            d.copy_(p, non_blocking=True)
        lib.stragglar_phase1_reducescatter(plan, work)
        lib.stragglar_phase2_complete(plan, work)
        if first is None:
            first = work[0].clone()
        else:
            for d in (work[0], work[w.n - 1], work[call % w.n]):
                bad += (d.view(torch.int16) != first.view(torch.int16)).sum()
    torch.cuda.synchronize()
    assert int(bad) == 0
    xs = w.host_all()
    assert same_bits(to_host(first, "bf16"), R.stragglar_fold(xs, w.straggler, "bf16", elem_bytes=2))
