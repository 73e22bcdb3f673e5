"""Host-side checks of bench.py (no GPU): the command-line contract, the workloads it names,
the traffic table it quotes and the CPU-baseline leg on a small workload."""

import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr and "--gpus 2" in res.stderr
    assert res.stdout.strip() == ""                      # no JSON line that could be mistaken for a result


def test_workloads_have_the_shapes_of_the_five_configurations():
    w = bench.workload_by_name("cfg1")
    assert (w.n, w.straggler, w.count, w.dtype) == (4, 0, 4096, "f32")
    w = bench.workload_by_name("cfg2")
    assert (w.n, w.straggler, w.count, w.dtype, w.bytes_per_rank) == (8, 0, 64 << 20, "f32", 256 << 20)
    assert bench.workload_by_name("cfg2-i32").dtype == "i32"
    w = bench.workload_by_name("cfg3")
    assert (w.n, w.count, w.dtype) == (8, 1_240_000_000, "bf16") and 0 <= w.straggler < 8
    w = bench.workload_by_name("cfg4")
    assert (w.n, w.straggler, w.count, w.dtype) == (8, 0, 8 * 2048 * 3072, "bf16")
    assert bench.workload_by_name("cfg4-%d" % (1 << 20)).bytes_per_rank == 1 << 20     # the message-size sweep
    for n in (16, 32):
        w = bench.workload_by_name("cfg5-%d" % n)
        assert (w.n, w.count, w.dtype) == (n, 16 << 20, "f32")
    w = bench.workload_by_name("delay-4GiB")
    assert (w.n, w.bytes_per_rank) == (8, 4 << 30)
    w = bench.workload_by_name("n24x96")
    assert (w.n, w.bytes_per_rank, w.dtype) == (24, 96 << 20, "f32")
    w = bench.workload_by_name("n12x64bf16")
    assert (w.n, w.bytes_per_rank, w.dtype) == (12, 64 << 20, "bf16")
    with pytest.raises(SystemExit):
        bench.workload_by_name("cfg9")


def test_traffic_table_matches_the_byte_model_for_the_headline():
    """roofline.traffic of the headline leg comes from profiles/l2_fabric_traffic.txt: the counters'
    figure for one launch of the per-round completion on cfg2 is the algorithmic 2ns / 9 within
    0.5 % (Sec. 3.1's rounds: n + log n - 2 = 9 launches)."""
    table = bench.measured_traffic()
    w = bench.workload_by_name("cfg2")
    per_launch = table[(w.name, "phase2", "per_round")]
    assert abs(per_launch / (2 * w.n * w.bytes_per_rank / 9) - 1) < 5e-3
    for key, value in table.items():
        assert key[1] in ("phase1", "phase2", "ring") and value > 0


def test_mean_and_standard_error():
    m, sem = bench.mean_sem([1.0, 2.0, 3.0, 4.0])
    assert m == 2.5 and abs(sem - (5.0 / 3 / 4) ** 0.5) < 1e-12
    assert bench.mean_sem([7.0]) == (7.0, 0.0)


def test_cpu_baseline_leg_on_a_small_workload():
    """The oracle-timing leg of the benchmark (the only part of bench.py that may touch oracle/):
    runs on the host alone, reports throughput in the metric's unit, the threads it used and
    what the sample was."""
    import synth_inputs as W
    w = W.Workload("tiny", 8, 0, 7 * 40000 + 3, "f32", ("normal", 1.0), seed=1)
    out = bench.cpu_baseline(w, target_seconds=0.2)
    assert out["kind"] == "oracle" and out["unit"] == "GB/s" and out["cores"] == 1
    assert out["value"] > 0 and "sample" in out and out["completion_s"] > 0
    assert out["all_cores"]["cores"] >= 1 and out["all_cores"]["value"] > 0
    json.dumps(out)
