"""Host-side checks of the C ABI: symbols, planner output, argument errors.
Nothing here launches a kernel (no GPU needed)."""

import ctypes
import os
import re
import time

import pytest

from oracle import schedule as S
from sched_checks import check_round_hazards, simulate_completion

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "stragglar.h")
POW2 = [2, 4, 8, 16, 32, 64, 128, 256]


def declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    names = re.findall(r"^\s*(?:const\s+)?(?:int|void|long|char\s*\*)\s*\*?\s*(\w+)\s*\(", text, flags=re.M)
    return sorted(set(names))


def test_library_exports_every_declared_symbol(lib):
    L = lib.load()
    names = declared_functions()
    assert len(names) >= 17 and "stragglar_allreduce" in names and "stragglar_delay" in names and "rhd_allreduce" in names and "stragglar_phase2_complete" in names and "ring_allreduce" in names
    for name in names:
        assert hasattr(L, name), name
    from paper_2505_23523_amd.binding import SYMBOLS
    assert sorted(SYMBOLS) == names


def test_loaded_library_is_the_one_built_from_these_sources(lib, monkeypatch):
    """The build leaves a digest of its sources beside the library; load() rebuilds when the tree's
    sources give another one (modification times do not survive every way a tree is copied)."""
    from paper_2505_23523_amd import binding, build
    lib.load()
    assert os.path.exists(build.STAMP)
    assert open(build.STAMP).read().strip() == build.source_digest()
    assert not binding._stale(binding.lib_path())
    monkeypatch.setattr(build, "source_digest", lambda: "0" * 64)
    assert binding._stale(binding.lib_path())


def test_binding_constants_match_the_header(lib):
    """Schedule ids, dtypes and tunable keys of the Python binding are the header's enumerators."""
    text = open(HEADER).read()
    enum = {m.group(1): int(m.group(2)) for m in re.finditer(r"\b(SAR_[A-Z0-9_]+)\s*=\s*(-?\d+)", text)}
    for name in ("PRECONDITION", "COMPLETION", "RING", "RHD", "BCAST_PRECONDITION", "BCAST_COMPLETION", "ALLREDUCE"):
        assert getattr(lib, name) == enum["SAR_SCHED_" + name], name
    assert int(re.search(r"#define SAR_NUM_SCHEDULES (\d+)", text).group(1)) == 1 + max(
        v for k, v in enum.items() if k.startswith("SAR_SCHED_"))
    assert lib.DTYPES == {"i32": enum["SAR_I32"], "f32": enum["SAR_F32"], "bf16": enum["SAR_BF16"]}
    from paper_2505_23523_amd.binding import TUNABLES
    assert TUNABLES == {k[len("SAR_TUNE_"):].lower(): v for k, v in enum.items() if k.startswith("SAR_TUNE_")}


def logical(rounds, n, sg):
    phys = [S.to_physical(l, n, sg) for l in range(n)]
    inv = {p: l for l, p in enumerate(phys)}
    return [[(inv[s], inv[d], c, k) for s, d, c, k in ops] for ops in rounds]


@pytest.mark.parametrize("n", POW2)
def test_library_planner_obeys_the_paper(lib, n):
    for sg in sorted({0, 1, n // 2, n - 1}):
        p = lib.stragglar_plan(n, sg, 1 << 20, "f32")
        comp = p.rounds(lib.COMPLETION)
        L = n.bit_length() - 1
        assert len(comp) == n + L - 2                                  # Thm. 1
        assert p.num_rounds(lib.PRECONDITION) == n - 2
        assert p.num_rounds(lib.RING) == 2 * (n - 1)                   # Table 1
        simulate_completion(n, logical(comp, n, sg))
        check_round_hazards(comp)
        check_round_hazards(p.rounds(lib.PRECONDITION))
        check_round_hazards(p.rounds(lib.RING))
        assert p.num_rounds(lib.RHD) == 2 * L                          # Table 1
        assert p.num_rounds(lib.BCAST_COMPLETION) == L                 # App. E, T_Bcast
        assert p.num_rounds(lib.BCAST_PRECONDITION) == 2 * (n - 2)
        for which in (lib.RHD, lib.BCAST_PRECONDITION, lib.BCAST_COMPLETION):
            check_round_hazards(p.rounds(which))
        for ops in p.rounds(lib.PRECONDITION):
            assert all(s != sg and d != sg for s, d, c, k in ops)
        assert p.rounds(lib.ALLREDUCE) == p.rounds(lib.PRECONDITION) + comp    # both phases back to back
        assert p.chunks(lib.ALLREDUCE) == p.chunks(lib.COMPLETION)


@pytest.mark.parametrize("n", POW2)
def test_library_planner_equals_oracle_twin(lib, n):
    """Two planners written separately under the same tie-breaks agree."""
    for sg in range(n) if n <= 16 else (0, 7, n - 1):
        for dtype, eb, count in (("f32", 4, 1 << 20), ("bf16", 2, (1 << 20) + 77)):
            p = lib.stragglar_plan(n, sg, count, dtype)
            assert p.rounds(lib.COMPLETION) == S.completion_rounds(n, sg)
            assert p.rounds(lib.PRECONDITION) == S.rs_precondition_rounds(n, sg)
            assert p.rounds(lib.RING) == S.ring_allreduce_rounds(n)
            assert p.rounds(lib.RHD) == S.rhd_allreduce_rounds(n)
            assert p.rounds(lib.BCAST_PRECONDITION) == S.broadcast_precondition_rounds(n, sg)
            assert p.rounds(lib.BCAST_COMPLETION) == S.broadcast_completion_rounds(n, sg)
            assert p.chunks(lib.RHD) == S.chunk_layout(count, n, eb)
            assert p.chunks(lib.BCAST_COMPLETION) == S.chunk_layout(count, n - 1, eb)
            assert p.chunks(lib.COMPLETION) == S.chunk_layout(count, n - 1, eb)
            assert p.chunks(lib.PRECONDITION) == S.chunk_layout(count, n - 1, eb)
            assert p.chunks(lib.RING) == S.chunk_layout(count, n, eb)
            p.close()


@pytest.mark.parametrize("n", [6, 10, 12, 14, 18, 20, 22, 24, 36, 48, 96, 254])
def test_library_planner_even_non_power_of_two(lib, n):
    """App. D: valid schedules, no more than the n + 2 log n - 2 rounds the paper reports,
    cheaper than ring; equal to the oracle's separately written generator where that one is
    fast enough.  Up to 20 ranks the matching is the exact subset recursion, above that the
    blossom algorithm."""
    L_up = (n - 1).bit_length()
    for sg in sorted({0, n // 2, n - 1}) if n < 200 else [3]:
        p = lib.stragglar_plan(n, sg, 1 << 24, "bf16")
        comp = p.rounds(lib.COMPLETION)
        simulate_completion(n, logical(comp, n, sg), power_of_two=False)
        for which in range(6):
            check_round_hazards(p.rounds(which))
        assert n - 1 <= len(comp) <= n + 2 * L_up - 2
        assert len(comp) * n < 2 * (n - 1) * (n - 1)                   # beta cost below ring's
        assert p.num_rounds(lib.PRECONDITION) == n - 2 and p.num_rounds(lib.RING) == 2 * (n - 1)
        assert p.num_rounds(lib.RHD) == 0                              # halving needs a power of two
        if n <= 14:
            assert comp == S.completion_rounds_any(n, sg)
        assert p.rounds(lib.PRECONDITION) == S.rs_precondition_rounds(n, sg)
        assert p.rounds(lib.RING) == S.ring_allreduce_rounds(n)
    L = lib.load()
    bufs = (ctypes.c_void_p * n)(*[0x10000000 * (i + 1) for i in range(n)])
    assert L.rhd_allreduce(p.handle, bufs, None) == 2


def test_matching_solvers_agree():
    """tests/matching_selftest.cpp: the blossom algorithm against the exact subset recursion
    (and that against brute force) on thousands of random graphs.  Host code only."""
    import subprocess
    import tempfile
    csrc = os.path.join(ROOT, "paper_2505_23523_amd", "csrc")
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "matching_selftest")
        subprocess.run(["g++", "-O2", "-std=c++17", "-I", csrc, "-o", exe,
                        os.path.join(ROOT, "tests", "matching_selftest.cpp"), os.path.join(csrc, "matching.cpp")],
                       check=True)
        res = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "graphs ok" in res.stdout


def test_chunk_lists_forwarding_and_dead_stores():
    """tests/chunk_lists_selftest.cpp: the per-chunk op lists of the single-launch kernel, with
    register forwarding and dropped stores, leave every defined cell as the round-by-round
    schedule does and make exactly the loads and stores of the byte model.  Host code only."""
    import subprocess
    import tempfile
    csrc = os.path.join(ROOT, "paper_2505_23523_amd", "csrc")
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "chunk_lists_selftest")
        subprocess.run(["g++", "-O2", "-std=c++17", "-I", csrc, "-I", os.path.join(ROOT, "include"), "-o", exe,
                        os.path.join(ROOT, "tests", "chunk_lists_selftest.cpp"),
                        os.path.join(csrc, "planner.cpp"), os.path.join(csrc, "matching.cpp")], check=True)
        res = subprocess.run([exe], capture_output=True, text=True, timeout=600)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "plans ok" in res.stdout


def test_launch_policy_under_host_sanitizers():
    """tests/launch_form_selftest.cpp: the library's host code (planner, launch policy, launch and
    byte counting) built with the address and undefined-behaviour sanitizers on the host side
    and driven through stragglar_plan_launch_form over a grid of rank counts, sizes, element
    types and options.  No GPU is touched (the device code is compiled but nothing is launched)."""
    import shutil
    import subprocess
    import tempfile
    from paper_2505_23523_amd import build
    hipcc = build.hipcc_path()
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("no hipcc")
    csrc = os.path.join(ROOT, "paper_2505_23523_amd", "csrc")
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "launch_form_selftest")
        cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-std=c++17", "-Wno-unused-command-line-argument",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all",
               "-I", os.path.join(ROOT, "include"), "-I", csrc, "-o", exe, os.path.join(ROOT, "tests", "launch_form_selftest.cpp")]
        cmd += [os.path.join(csrc, name) for name in build.SOURCES]
        res = subprocess.run(cmd, capture_output=True, text=True, cwd=tmp, timeout=900)
        assert res.returncode == 0, res.stderr[-2000:]
        res = subprocess.run([exe], capture_output=True, text=True, cwd=tmp, timeout=600)
    assert res.returncode == 0, res.stdout[-1000:] + res.stderr[-3000:]
    assert "launch forms ok" in res.stdout


def test_planner_speed_n256(lib):
    t0 = time.perf_counter()
    lib.stragglar_plan(256, 3, 1 << 24, "f32")
    assert time.perf_counter() - t0 < 1.04          # Sec. 4 "Schedule generator"


def test_plan_argument_errors(lib):
    def status(*a):
        with pytest.raises(lib.StragglarError) as e:
            lib.stragglar_plan(*a)
        return e.value.status
    assert status(7, 0, 1 << 20, "f32") == 2        # odd (Sec. 4 "Limitations")
    assert status(9, 0, 1 << 20, "f32") == 2
    assert status(512, 0, 1 << 20, "f32") == 2
    assert status(1, 0, 1 << 20, "f32") == 1
    assert status(0, 0, 1 << 20, "f32") == 1
    assert status(8, 8, 1 << 20, "f32") == 1
    assert status(8, -1, 1 << 20, "f32") == 1
    assert status(8, 0, 0, "f32") == 1
    assert status(8, 0, 7, "f32") == 1              # a chunk would be empty
    assert status(8, 0, 1 << 20, 3) == 1
    L = lib.load()
    assert L.stragglar_plan(8, 0, 1 << 20, 1, None) == 1
    assert L.stragglar_plan_num_rounds(None, 0) == -1
    p = lib.stragglar_plan(8, 0, 1 << 20, "f32")
    assert p.num_rounds(7) == -1 and p.num_chunks(-1) == -1
    assert p.num_rounds(6) == p.num_rounds(0) + p.num_rounds(1)     # both phases back to back
    with pytest.raises(lib.StragglarError):
        p.round(lib.COMPLETION, 9)
    with pytest.raises(lib.StragglarError):
        p.chunk(lib.COMPLETION, 7)
    assert p.chunk(lib.RING, 7)[0] == 7 * (1 << 17)


def test_run_argument_errors_without_gpu(lib):
    """Bad buffers are refused before anything is enqueued."""
    L = lib.load()
    p = lib.stragglar_plan(4, 0, 4096, "f32")
    for fn in (L.stragglar_phase1_reducescatter, L.stragglar_phase2_complete, L.ring_allreduce,
               L.rhd_allreduce, L.broadcast_phase1_allreduce, L.broadcast_phase2_complete):
        assert fn(p.handle, None, None) == 1
        assert fn(None, (ctypes.c_void_p * 4)(), None) == 1
        bufs = (ctypes.c_void_p * 4)(0x10000, 0x20000, 0, 0x40000)
        assert fn(p.handle, bufs, None) == 1                      # null pointer
        bufs = (ctypes.c_void_p * 4)(0x10000, 0x20008, 0x30000, 0x40000)
        assert fn(p.handle, bufs, None) == 1                      # misaligned
        bufs = (ctypes.c_void_p * 4)(0x10000, 0x13000, 0x30000, 0x40000)
        assert fn(p.handle, bufs, None) == 1                      # overlapping


def test_delay_argument_error(lib):
    assert lib.load().stragglar_delay(2_000_000_000, None) == 1      # more than a second


def test_no_device_is_an_error_not_a_crash(lib):
    """Without a GPU the execution entry points must come back with SAR_EDEVICE."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present: this would launch on made-up addresses")
    L = lib.load()
    p = lib.stragglar_plan(4, 0, 4096, "f32")
    bufs = (ctypes.c_void_p * 4)(0x10000000, 0x20000000, 0x30000000, 0x40000000)
    for fn in (L.stragglar_phase1_reducescatter, L.stragglar_phase2_complete, L.ring_allreduce,
               L.rhd_allreduce, L.broadcast_phase1_allreduce, L.broadcast_phase2_complete):
        assert fn(p.handle, bufs, None) == 4
    assert L.stragglar_allreduce(p.handle, bufs, None, None) == 4
    assert L.stragglar_delay(1000, None) == 4


def test_tunables(lib):
    for key, good, bad in (("blocks_per_cu", 4, -1), ("unroll", 4, 3), ("nontemporal", 1, 2), ("fuse_rounds", 1, 2), ("fused_unroll", 2, 3),
                           ("fused_wgs_per_cu", 3, 7), ("merge_copies", 1, 2), ("fused_split", 1, 2), ("fused_direct", 0, 2)):
        old = lib.tune_get(key)
        lib.tune_set(key, good)
        assert lib.tune_get(key) == good
        with pytest.raises(lib.StragglarError):
            lib.tune_set(key, bad)
        assert lib.tune_get(key) == good
        lib.tune_set(key, old)
    assert lib.load().stragglar_tune_get(99) == -1
    assert lib.load().stragglar_strerror(4) == b"HIP device error"


def test_plan_options_are_per_plan(lib):
    """A plan's launch options win over the process-wide tunables for that plan only, can be
    handed back, and are range-checked like the tunables."""
    a = lib.stragglar_plan(8, 0, 1 << 20, "f32")
    b = lib.stragglar_plan(8, 0, 1 << 20, "f32")
    old = lib.tune_get("fuse_rounds")
    try:
        lib.tune_set("fuse_rounds", 0)
        a.option_set("fuse_rounds", 1)
        assert a.option_get("fuse_rounds") == 1 and b.option_get("fuse_rounds") == 0
        assert a.launch_form(lib.COMPLETION)["form"] == "single_launch"
        assert b.launch_form(lib.COMPLETION)["form"] == "per_round"
        lib.tune_set("fuse_rounds", 1)
        a.option_set("fuse_rounds", 0)
        assert a.launch_form(lib.COMPLETION)["form"] == "per_round"
        assert b.launch_form(lib.COMPLETION)["form"] == "single_launch"
        a.option_set("fuse_rounds", lib.OPTION_INHERIT)
        assert a.option_get("fuse_rounds") == 1
        with pytest.raises(lib.StragglarError):
            a.option_set("fuse_rounds", 2)
        with pytest.raises(lib.StragglarError):
            a.option_set("unroll", 3)
        assert a.option_get("fuse_rounds") == 1
        L = lib.load()
        assert L.stragglar_plan_option_set(None, 3, 0) == 1 and L.stragglar_plan_option_set(a.handle, 99, 0) == 1
        assert L.stragglar_plan_option_get(None, 3) == -1 and L.stragglar_plan_option_get(a.handle, -1) == -1
        assert L.stragglar_plan_launch_form(a.handle, 1, None) == 1 and L.stragglar_plan_launch_form(None, 1, None) == 1
    finally:
        lib.tune_set("fuse_rounds", old)


def distinct_copies(rounds):
    """Chunks read when every round's copies of one chunk index are read once (the oracle's
    completion only ever copies fully reduced chunks, so same index = same value)."""
    return [c for ops in rounds for c in sorted({c for _, _, c, k in ops if k == 0})]


@pytest.mark.parametrize("n", [2, 4, 8, 16, 32])
def test_launch_form_counts_the_bytes_of_each_form(lib, n):
    """Bytes loaded / stored as the library reports them for the three ways a call can run,
    against counts made from the ORACLE's schedules and the byte model: one launch per round
    2ns for the completion (each copy 1 + 1, each pairing 2 + 2), 3(n-2)s for the precondition,
    5(n-1)s for the ring; copies of one chunk read once per round: (2(n-1) + D) chunk loads with
    D = 5, 20, 59, 154 for n = 4 ... 32; single launch (n+2)s / ns / 2ns."""
    count = 997 * n * (n - 1) + 5
    p = lib.stragglar_plan(n, n // 3, count, "bf16")
    sar_chunks = S.chunk_layout(count, n - 1, 2)
    ring_chunks = S.chunk_layout(count, n, 2)
    comp = S.completion_rounds(n, n // 3)
    pre = S.rs_precondition_rounds(n, n // 3)
    ring = S.ring_allreduce_rounds(n)

    def plain(rounds, chunks):
        ld = sum((1 if k == 0 else 2) * 2 * chunks[c][1] for ops in rounds for _, _, c, k in ops)
        st = sum((2 if k == 2 else 1) * 2 * chunks[c][1] for ops in rounds for _, _, c, k in ops)
        return ld, st

    p.option_set("fuse_rounds", 0)
    for which, rounds, chunks in ((lib.COMPLETION, comp, sar_chunks), (lib.PRECONDITION, pre, sar_chunks), (lib.RING, ring, ring_chunks)):
        f = p.launch_form(which)
        assert f["form"] == "per_round" and f["launches"] == len(rounds)
        assert (f["bytes_loaded"], f["bytes_stored"]) == plain(rounds, chunks)
    s = 2 * count
    f = p.launch_form(lib.COMPLETION)
    assert f["bytes_loaded"] == n * s and f["bytes_stored"] == n * s          # 2ns
    p.option_set("merge_copies", 1)
    f = p.launch_form(lib.COMPLETION)
    assert f["form"] == "per_round_merged_copies" and f["launches"] == len(comp)
    D = distinct_copies(comp)
    if n >= 4:
        assert len(D) == {4: 5, 8: 20, 16: 59, 32: 154}[n]
    want = sum(2 * sar_chunks[c][1] for c in D) + sum(2 * 2 * sar_chunks[c][1] for ops in comp for _, _, c, k in ops if k == 2)
    assert f["bytes_loaded"] == want and f["bytes_stored"] == n * s
    assert p.launch_form(lib.PRECONDITION)["bytes_loaded"] == plain(pre, sar_chunks)[0]   # nothing to merge
    p.option_set("fuse_rounds", 1)
    f = p.launch_form(lib.COMPLETION)
    assert f["form"] == "single_launch" and f["launches"] == 1
    assert (f["bytes_loaded"], f["bytes_stored"]) == (2 * s, n * s)
    f = p.launch_form(lib.PRECONDITION)
    assert (f["bytes_loaded"], f["bytes_stored"]) == ((n - 1) * s if n > 2 else 0, s if n > 2 else 0)
    f = p.launch_form(lib.RING)
    assert (f["bytes_loaded"], f["bytes_stored"]) == (n * s, n * s)
    assert f["launches"] == (2 if n == 32 else 1)


def test_launch_counts_of_the_split_and_chain_forms(lib):
    """Launches a call takes, as the library reports them (host logic only).  The split completion
    walks the chunk indices in groups of at most 100 MiB of holder cells, one producing launch
    and one broadcast launch per group, at any rank count; precondition and ring as reduce chains are one launch at any rank count,
    through op lists several; bytes do not depend on the grouping."""
    MiB = 1 << 18      # fp32 elements

    def form(n, count, which, **options):
        p = lib.stragglar_plan(n, 1, count, "f32")
        for k, v in options.items():
            p.option_set(k, v)
        return p.launch_form(which)

    # the automatic split: more than 16 ranks from 512 MiB in all, up to 256 MiB per rank
    assert form(32, 64 * MiB, lib.COMPLETION)["form"] == "single_launch_split"
    assert form(32, 64 * MiB, lib.COMPLETION)["launches"] == 2
    assert form(32, 256 * MiB, lib.COMPLETION)["launches"] == 6            # 3 groups
    assert form(32, 512 * MiB, lib.COMPLETION)["form"] == "single_launch"
    assert form(32, 8 * MiB, lib.COMPLETION)["form"] == "single_launch"
    assert form(16, 64 * MiB, lib.COMPLETION)["form"] == "single_launch"
    assert form(16, 192 * MiB, lib.COMPLETION) == dict(form(16, 192 * MiB, lib.COMPLETION), form="single_launch_split", launches=4)
    assert form(8, 256 * MiB, lib.COMPLETION)["form"] == "single_launch"
    assert form(64, 1 * MiB, lib.COMPLETION) == dict(form(64, 1 * MiB, lib.COMPLETION), form="single_launch_split", launches=2)
    assert form(256, 1 * MiB, lib.COMPLETION)["launches"] == 2
    one = form(16, 192 * MiB, lib.COMPLETION, fuse_rounds=1, fused_split=0)
    split = form(16, 192 * MiB, lib.COMPLETION, fuse_rounds=1, fused_split=1)
    s = 4 * 192 * MiB
    assert (one["bytes_loaded"], one["bytes_stored"]) == (2 * s, 16 * s)                  # (n+2)s
    assert (split["bytes_loaded"], split["bytes_stored"]) == (3 * s, 16 * s)              # (n+3)s
    # reduce chains
    for n in (64, 130, 256):
        assert form(n, n * n * 64, lib.PRECONDITION, fuse_rounds=1)["launches"] == 1
        assert form(n, n * n * 64, lib.RING, fuse_rounds=1)["launches"] == 1
        assert form(n, n * n * 64, lib.PRECONDITION, fuse_rounds=1, fused_direct=0)["launches"] > 1
    assert form(256, 256 * 256 * 64, lib.RING, fuse_rounds=1, fused_direct=0)["form"] == "per_round"   # 510 ops per chunk index
    assert form(16, 64 * MiB, lib.RING, fuse_rounds=1, fused_direct=1, fused_split=1)["launches"] == 2


@pytest.mark.parametrize("n", [12, 14, 20, 24, 40, 96, 130])
def test_app_d_rounds_are_maximum_weight_matchings_by_an_independent_solver(lib, n):
    """App. D beyond the sizes brute force reaches: for every round of the completion the LIBRARY
    emits, the graph of App. D is rebuilt from the ranks' holdings
    before the round - weight 2 if both ends hold a reduced chunk the other lacks, 1 if one does -
    and the number of chunks the round moves (one per unit of weight) must equal the weight of a
    maximum-weight matching as networkx computes it (an implementation of Edmonds' algorithm that
    shares nothing with the library's solvers)."""
    nx = pytest.importorskip("networkx")
    sg = n // 3
    p = lib.stragglar_plan(n, sg, n * n * 64, "f32")
    rounds = logical(p.rounds(lib.COMPLETION), n, sg)
    sigma = n - 1
    full = [set() for _ in range(n)]
    for r, ops in enumerate(rounds):
        copies = [(s_, d, c) for s_, d, c, k in ops if k == 0]
        free = [g for g in range(n) if not (r < n - 1 and g in (r, sigma))]
        G = nx.Graph()
        G.add_nodes_from(free)
        for i, a in enumerate(free):
            for b in free[i + 1:]:
                wt = (1 if full[a] - full[b] else 0) + (1 if full[b] - full[a] else 0)
                if wt:
                    G.add_edge(a, b, weight=wt)
        best = sum(G[a][b]["weight"] for a, b in nx.max_weight_matching(G))
        assert len(copies) == best, (n, r, len(copies), best)
        seen = set()
        for s_, d, c in copies:
            assert c in full[s_] and c not in full[d]
            assert (s_, 0) not in seen and (d, 1) not in seen      # one send and one receive per rank
            seen.add((s_, 0)), seen.add((d, 1))
        for s_, d, c in copies:
            full[d].add(c)
        if r < n - 1:
            assert [(s_, d, c) for s_, d, c, k in ops if k == 2] == [(r, sigma, r)]
            full[r].add(r)
            full[sigma].add(r)
    assert all(f == set(range(n - 1)) for f in full)
