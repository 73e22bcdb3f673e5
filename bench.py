#!/usr/bin/env python3
"""Benchmark of the StragglAR AllReduce hot path on one MI355X.

A *step* is one pass of the whole hot path over one batch of synthetic rank
buffers: the precondition ReduceScatter (phase 1), the completion rounds of
Alg. 1 (phase 2, the straggler's critical path) and the ring AllReduce
baseline, each timed with HIP events on the stream the kernels run on.  The
rank buffers are restored from a pristine device copy before each phase-1 and
each ring run, outside the event brackets (the kernels' cost does not depend
on the values; restoring keeps the values finite over many steps).

Headline `value`: algorithmic HBM bytes of the completion phase (2*n*s)
divided by its time, in GB/s, with inputs resident in HBM.

Prints ONE JSON line.
"""

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X published HBM3E peak

# HBM bytes per launch of the dominant kernel, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# runs of this script (scaled by a plain copy of known size in the same run); the figures and
# commands are in profiles/round_kernel_<phase>_cfg2.txt and profiles/fused_kernel_phase2_cfg2.txt.
# Only the profiled workload has one.
MEASURED_TRAFFIC = {
    ("cfg2-n8-f32-64Mi", "phase2"): 477.2e6,
    ("cfg2-n8-f32-64Mi", "phase2-single-launch"): 2684.5e6,
    ("cfg2-n8-f32-64Mi", "phase1-single-launch"): 2147.4e6,
    ("cfg2-n8-f32-64Mi", "ring-single-launch"): 4294.8e6,
    ("cfg2-n8-f32-64Mi", "phase1"): 805.3e6,
    ("cfg2-n8-f32-64Mi", "ring"): 671.1e6,
}


def alg_bytes(which, n, s):
    """Algorithmic HBM bytes of one pass (s = bytes per rank buffer):
    COPY reads 1 + writes 1 chunk, REDUCE reads 2 + writes 1, REDUCE_EXCHANGE
    reads 2 + writes 2.  Completion: (n-1)(n-2) copies + (n-1) exchanges of
    s/(n-1) -> 2ns.  Precondition: (n-1)(n-2) reduces -> 3(n-2)s.  Ring:
    n(n-1) reduces + n(n-1) copies of s/n -> 5(n-1)s."""
    return {"phase1": 3 * (n - 2) * s, "phase2": 2 * n * s, "ring": 5 * (n - 1) * s}[which]


def single_launch_bytes(which, n, s):
    """HBM bytes of the single-launch mode, where a value a workgroup produced stays in its
    registers for the following rounds and a store that a later round overwrites unread is
    dropped: per chunk index the completion reads 2 cells and writes n; a ring reduce-scatter
    over m ranks reads m cells and writes the last hop's only; the all-gather writes m-1."""
    return {"phase1": n * s, "phase2": (n + 2) * s, "ring": 2 * n * s}[which]


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def mean_sem(xs):
    m = sum(xs) / len(xs)
    if len(xs) < 2:
        return m, 0.0
    var = sum((x - m) ** 2 for x in xs) / (len(xs) - 1)
    return m, (var / len(xs)) ** 0.5


def workload_by_name(name):
    import synth_inputs as W
    if name == "cfg1":
        return W.cfg1()
    if name == "cfg2":
        return W.cfg2("f32")
    if name == "cfg2-i32":
        return W.cfg2("i32")
    if name == "cfg3":
        return W.cfg3()
    if name == "cfg4":
        return W.cfg4()
    if name.startswith("cfg4-"):          # cfg4-<bytes per rank>
        return W.cfg4(int(name.split("-")[1]) // 2)
    if name.startswith("cfg5-"):          # cfg5-<n>
        return W.cfg5(int(name.split("-")[1]), 0)
    raise SystemExit("unknown workload %r" % name)


def cpu_baseline(w, target_seconds=15.0):
    """The oracle's op-by-op replay (precondition + completion) timed on this host on a
    bounded sample of the workload: the first `m` elements of every rank buffer, m chosen from
    a short calibration run (the whole buffer if that takes less than the target).  Timed once
    on one thread - the oracle as it stands - and once with the same replay run by one thread
    per host core, each on its own slice of every chunk (ops are elementwise, so the slices
    are independent and the bits identical)."""
    from concurrent.futures import ThreadPoolExecutor
    from oracle import replay as P
    from oracle import schedule as S
    eb = 4 if w.dtype != "bf16" else 2
    pre = S.rs_precondition_rounds(w.n, w.straggler)
    comp = S.completion_rounds_any(w.n, w.straggler)

    def one(count, threads=1):
        xs = [w.head(r, count) for r in range(w.n)]
        chunks = S.chunk_layout(count, w.n - 1, eb)
        if threads == 1:
            parts = [chunks]
        else:
            parts = []
            for t in range(threads):
                sub = []
                for lo, ln in chunks:
                    a, b = ln * t // threads, ln * (t + 1) // threads
                    sub.append((lo + a, b - a))
                parts.append(sub)
        times = []
        with ThreadPoolExecutor(max_workers=threads) as pool:
            for rounds in (pre, comp):
                t0 = time.perf_counter()
                list(pool.map(lambda sub: P.replay(rounds, sub, xs, w.dtype), parts))
                times.append(time.perf_counter() - t0)
        return times[0], times[1]

    small = min(w.count, 1 << 20)
    p1, p2 = one(small)
    per_elem = (p1 + p2) / small
    count = int(min(w.count, max(small, target_seconds / max(per_elem, 1e-12))))
    count -= count % 64
    reps = [one(count) for _ in range(3)]
    p1, p2 = min(r[0] for r in reps), min(r[1] for r in reps)
    s = count * eb
    cores = min(os.cpu_count() or 1, 16)
    par = [one(count, cores) for _ in range(3)]
    q1, q2 = min(r[0] for r in par), min(r[1] for r in par)
    return {
        "value": alg_bytes("phase2", w.n, s) / p2 / 1e9,
        "unit": "GB/s",
        "cores": 1,
        "kind": "oracle",
        "sample": "first %d of %d elements of each of the %d rank buffers (%s); NumPy op-by-op replay, "
                  "one thread, best of 3; completion %.3f s, precondition %.3f s" % (count, w.count, w.n, w.name, p2, p1),
        "host_cpus": os.cpu_count(),
        "host_cpu_model": cpu_model(),
        "completion_s": p2,
        "precondition_s": p1,
        "all_cores": {"value": alg_bytes("phase2", w.n, s) / q2 / 1e9, "unit": "GB/s", "cores": cores,
                      "completion_s": q2, "precondition_s": q1,
                      "note": "same replay, one thread per core on disjoint slices of every chunk"},
    }


def other_baselines(torch, sar, plan, work, restore, n, s, steps, warmup):
    """The paper's other comparison algorithms on the same kernels (App. E), for context:
    recursive halving/doubling and the straggler-aware Broadcast (whose post-arrival part is
    log n rounds of the whole buffer)."""
    stream = torch.cuda.current_stream()
    L = n.bit_length() - 1
    legs = [("rhd", [sar.rhd_allreduce], 5 * (n - 1) * s),
            ("broadcast_phase1", [sar.broadcast_phase1_allreduce], 5 * (n - 2) * s),
            ("broadcast_phase2", [sar.broadcast_phase2_complete], 4 * s + 2 * (n - 2) * s)]
    res = {}
    rec = {name: [] for name, _, _ in legs}
    for it in range(warmup + steps):
        restore()
        for name, fns, _ in legs:
            if name == "broadcast_phase1":
                restore()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            for fn in fns:
                fn(plan, work, stream)
            b.record(stream)
            if it >= warmup:
                rec[name].append((a, b))
    torch.cuda.synchronize()
    for name, _, nbytes in legs:
        m, sem = mean_sem([a.elapsed_time(b) for a, b in rec[name]])
        res[name + "_ms"] = m
        res[name + "_ms_sem"] = sem
        res[name + "_GBps"] = nbytes / (m * 1e-3) / 1e9
    res["rounds"] = {"rhd": 2 * L, "broadcast_phase1": 2 * (n - 2), "broadcast_phase2": L}
    return res


def size_sweep(torch, sar, n, dtype, iters=20):
    """Message-size sweep in powers of two, 1 MiB .. 1 GiB per rank (Sec. 4.1 sweeps powers of
    two and reports algorithmic bandwidth = buffer bytes / time).  Buffers are zero-filled: the
    kernels' cost does not depend on the values.  Each size is timed with the library's default
    policy (single launch while the n buffers fit the memory-side cache) and with one launch per
    round forced."""
    import synth_inputs as W
    tdt = {"f32": torch.float32, "i32": torch.int32, "bf16": torch.bfloat16}[dtype]
    eb = W.ELEM_BYTES[dtype]
    stream = torch.cuda.current_stream()
    rows = []
    for p in range(20, 31):
        s = 1 << p
        count = s // eb
        bufs = [torch.zeros(count, dtype=tdt, device="cuda:0") for _ in range(n)]
        plan = sar.stragglar_plan(n, 0, count, dtype)
        row = {"bytes_per_rank": s}
        for mode, fuse in (("default", -1), ("per_round", 0)):
            sar.tune_set("fuse_rounds", fuse)
            for name, fn in (("phase1", sar.stragglar_phase1_reducescatter), ("phase2", sar.stragglar_phase2_complete),
                             ("ring", sar.ring_allreduce)):
                for _ in range(3):
                    fn(plan, bufs, stream)
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record(stream)
                for _ in range(iters):
                    fn(plan, bufs, stream)
                b.record(stream)
                torch.cuda.synchronize()
                ms = a.elapsed_time(b) / iters
                row["%s_%s_ms" % (mode, name)] = ms
                if name != "phase1":
                    row["%s_%s_algbw_GBps" % (mode, name)] = s / (ms * 1e-3) / 1e9
        rows.append(row)
        del bufs
    sar.tune_set("fuse_rounds", 0)
    return rows


def delay_sweep(torch, sar, plan, work, restore, stat, reps=5):
    """Total AllReduce time from the moment the on-time ranks call it, with the late rank
    emulated by an idle kernel on a second stream (Sec. 4.1, "Varying straggler delay").
    StragglAR: precondition starts at once, completion waits for the straggler.
    Ring: everything waits for the straggler."""
    main_s = torch.cuda.current_stream()
    late = torch.cuda.Stream()
    rows = []

    def total(d_ns, kind, fuse):
        sar.tune_set("fuse_rounds", fuse)
        ts = []
        for _ in range(reps):
            restore()
            torch.cuda.synchronize()
            t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            arrived = torch.cuda.Event()
            t0.record(main_s)
            late.wait_event(t0)
            sar.stragglar_delay(d_ns, late)
            arrived.record(late)
            if kind == "stragglar":      # precondition at once, completion behind the arrival event
                sar.stragglar_allreduce(plan, work, main_s, arrived)
            else:
                main_s.wait_event(arrived)
                sar.ring_allreduce(plan, work, main_s)
            t1.record(main_s)
            torch.cuda.synchronize()
            ts.append(t0.elapsed_time(t1))
        sar.tune_set("fuse_rounds", 0)
        return mean_sem(ts)[0]

    for fuse in (0, 1):                              # warm-up: stream creation, first launches
        total(0, "stragglar", fuse), total(0, "ring", fuse)
    for d_ms in (0.0, 0.1, 0.25, 0.5, 0.75, 1.0, 2.0, 5.0, 9.45):
        d_ns = int(d_ms * 1e6)
        rows.append({"delay_ms": d_ms, "stragglar_total_ms": total(d_ns, "stragglar", 0),
                     "ring_total_ms": total(d_ns, "ring", 0),
                     "single_launch_stragglar_total_ms": total(d_ns, "stragglar", 1),
                     "single_launch_ring_total_ms": total(d_ns, "ring", 1)})
    # the model of Sec. 4.1: StragglAR = max(delay, precondition) + completion, ring = delay + ring
    crit = stat["phase1"][0] + stat["phase2"][0] - stat["ring"][0]
    return {"rows": rows, "critical_delay_ms_from_phase_times": max(crit, 0.0),
            "note": "9.45 ms is the mean delay the paper observed; its critical delays (5.53 / 7.57 ms) are for "
                    "4 GiB buffers over NVLink - here time follows aggregate HBM bytes, so the break-even is near 0"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg2")
    ap.add_argument("--phases", default="all", choices=["all", "phase1", "phase2", "ring"],
                    help="'all' is the benchmark; a single phase is for profiling that kernel alone "
                         "(its input state is then arbitrary, which does not change its cost)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--size-sweep", action="store_true",
                    help="also time 1 MiB .. 1 GiB per rank in powers of two (the buffer sweep of Sec. 4.1)")
    ap.add_argument("--delay-sweep", action="store_true",
                    help="also time the whole AllReduce against an emulated straggler delay (Sec. 4.1): "
                         "precondition overlapped with the delay + completion, vs delay + ring")
    ap.add_argument("--blocks-per-cu", type=int)
    ap.add_argument("--unroll", type=int)
    ap.add_argument("--nontemporal", type=int)
    ap.add_argument("--fuse-rounds", type=int, help="0 one launch per round, 1 single launch, -1 automatic")
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the n ranks are emulated as n buffers in one "
              "GPU's HBM); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2505_23523_amd as sar
    sar.load()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    for key, val in (("blocks_per_cu", args.blocks_per_cu), ("unroll", args.unroll),
                     ("nontemporal", args.nontemporal), ("fuse_rounds", args.fuse_rounds)):
        if val is not None:
            sar.tune_set(key, val)

    if args.fuse_rounds is None:
        sar.tune_set("fuse_rounds", 0)     # headline: the schedule as rounds, one launch per round
    w = workload_by_name(args.workload)
    n, s = w.n, w.bytes_per_rank
    dev = torch.device("cuda:0")
    bases = [w.base(r) for r in range(n)]
    pristine = [w.device(r, dev, base=bases[r]) for r in range(n)]
    work = [torch.empty_like(t) for t in pristine]
    del bases
    plan = sar.stragglar_plan(n, w.straggler, w.count, w.dtype)
    stream = torch.cuda.current_stream()

    def restore():
        for d, p in zip(work, pristine):
            d.copy_(p, non_blocking=True)

    def ev():
        return torch.cuda.Event(enable_timing=True)

    phases = ["phase1", "phase2", "ring"] if args.phases == "all" else [args.phases]
    calls = {"phase1": sar.stragglar_phase1_reducescatter, "phase2": sar.stragglar_phase2_complete,
             "ring": sar.ring_allreduce}

    def step(record):
        if args.phases == "all":
            restore()
        for ph in phases:
            if ph == "ring" and args.phases == "all":
                restore()
            a, b = ev(), ev()
            a.record(stream)
            calls[ph](plan, work, stream)
            b.record(stream)
            if record is not None:
                record[ph].append((a, b))

    if args.phases != "all":
        restore()
    for _ in range(args.warmup):
        step(None)
    torch.cuda.synchronize()
    rec = {ph: [] for ph in phases}
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(rec)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    ms = {ph: [a.elapsed_time(b) for a, b in rec[ph]] for ph in phases}

    # the same pass in single-launch mode (reported beside the headline, never as it)
    single = None
    if args.phases == "all" and args.fuse_rounds is None:
        sar.tune_set("fuse_rounds", 1)
        for _ in range(args.warmup):
            step(None)
        torch.cuda.synchronize()
        rec1 = {ph: [] for ph in phases}
        for _ in range(args.steps):
            step(rec1)
        torch.cuda.synchronize()
        both = []                       # both phases as one call with no delay to wait for
        for i in range(args.warmup + args.steps):
            restore()
            a, b = ev(), ev()
            a.record(stream)
            sar.stragglar_allreduce(plan, work, stream)
            b.record(stream)
            if i >= args.warmup:
                both.append((a, b))
        torch.cuda.synchronize()
        sar.tune_set("fuse_rounds", 0)
        single = {"note": "all rounds of a call in one launch; a workgroup carries its tile of a chunk through "
                          "every round, so HBM sees only first reads and stores (bytes below), not 2ns"}
        for ph in phases:
            m1, sem1 = mean_sem([a.elapsed_time(b) for a, b in rec1[ph]])
            hb = single_launch_bytes(ph, n, s)
            single[ph + "_ms"] = m1
            single[ph + "_ms_sem"] = sem1
            single[ph + "_hbm_bytes"] = hb
            single[ph + "_hbm_GBps"] = hb / (m1 * 1e-3) / 1e9
            single[ph + "_frac_of_peak"] = hb / (m1 * 1e-3) / 1e9 / HBM_PEAK_GBS
        mb, semb = mean_sem([a.elapsed_time(b) for a, b in both])
        single["allreduce_no_delay_ms"] = mb          # stragglar_allreduce(event = NULL): one launch
        single["allreduce_no_delay_ms_sem"] = semb
        single["allreduce_no_delay_hbm_bytes"] = 2 * n * s
        single["allreduce_no_delay_hbm_GBps"] = 2 * n * s / (mb * 1e-3) / 1e9
    stat = {ph: mean_sem(ms[ph]) for ph in phases}
    main_ph = "phase2" if "phase2" in phases else phases[0]
    t_main = stat[main_ph][0]
    value = alg_bytes(main_ph, n, s) / (t_main * 1e-3) / 1e9
    which = {"phase1": sar.PRECONDITION, "phase2": sar.COMPLETION, "ring": sar.RING}
    rounds = {ph: plan.num_rounds(which[ph]) for ph in phases}

    out = {
        "metric": "post-arrival AllReduce (StragglAR completion rounds) HBM throughput, n=%d emulated ranks, 1 GPU" % n
                  if main_ph == "phase2" else "%s HBM throughput" % main_ph,
        "value": value,
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": sum(stat[ph][0] for ph in phases),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": w.name, "n_ranks": n, "straggler": w.straggler, "elements_per_rank": w.count,
                   "bytes_per_rank": s, "phases": args.phases,
                   "launch": {k: sar.tune_get(k) for k in ("blocks_per_cu", "unroll", "nontemporal", "fuse_rounds")}},
        "wall_ms_per_step_incl_restore": wall / args.steps * 1e3,
    }
    for ph in phases:
        out[ph + "_ms"] = stat[ph][0]
        out[ph + "_ms_sem"] = stat[ph][1]
        out[ph + "_GBps"] = alg_bytes(ph, n, s) / (stat[ph][0] * 1e-3) / 1e9
        out[ph + "_rounds"] = rounds[ph]
    if main_ph == "phase2":
        out["post_arrival_ms"] = t_main
        out["algbw_GBps"] = s / (t_main * 1e-3) / 1e9          # buffer bytes / time (Sec. 4.1)
    # alpha-beta view (Table 1): serialized bytes per rank, in units of s
    L = n.bit_length() - 1
    link = 450e9      # the paper's DGX H100 point-to-point bandwidth (Sec. 4.1), for scale only
    out["alpha_beta"] = {"completion_beta_s": (n + L - 2) / (n - 1), "ring_beta_s": 2 * (n - 1) / n,
                         "precondition_beta_s": (n - 2) / (n - 1),
                         "projected_ms_at_450GBps_links": {
                             "completion": (n + L - 2) / (n - 1) * s / link * 1e3,
                             "ring": 2 * (n - 1) / n * s / link * 1e3,
                             "precondition": (n - 2) / (n - 1) * s / link * 1e3},
                         "note": "per-link serialized bytes of the paper's model; the emulation's time follows "
                                 "the aggregate HBM bytes of all ranks instead"}
    fused_mode = sar.tune_get("fuse_rounds") > 0 or (sar.tune_get("fuse_rounds") < 0 and n <= 64)
    if fused_mode:
        # single-launch mode: priced against the bytes that mode has to move
        launches = 2 if (main_ph == "ring" and n == 32) else 1
        bytes_per_launch = single_launch_bytes(main_ph, n, s) / launches
        kernel = "fused_kernel (%s, %d launch%s per pass)" % (main_ph, launches, "" if launches == 1 else "es")
        traffic = MEASURED_TRAFFIC.get((w.name, main_ph + "-single-launch"))
    else:
        launches = rounds[main_ph]
        bytes_per_launch = alg_bytes(main_ph, n, s) / launches
        kernel = "round_kernel (%s, %d launches per pass)" % (main_ph, launches)
        traffic = MEASURED_TRAFFIC.get((w.name, main_ph))
    avg_launch_ms = t_main / launches
    out["roofline"] = {
        "bound": "hbm",
        "kernel": kernel,
        "achieved": bytes_per_launch / (avg_launch_ms * 1e-3) / 1e9,
        "peak": HBM_PEAK_GBS,
        "unit": "GB/s",
        "frac": bytes_per_launch / (avg_launch_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "traffic": traffic,
        "bytes_per_launch": bytes_per_launch,
        "avg_launch_ms": avg_launch_ms,
    }
    if single is not None:
        out["single_launch"] = single
    if args.phases == "all":
        out["other_baselines"] = other_baselines(torch, sar, plan, work, restore, n, s, args.steps, args.warmup)
    if args.size_sweep and args.phases == "all":
        out["size_sweep"] = size_sweep(torch, sar, n, w.dtype)
    if args.delay_sweep and args.phases == "all":
        out["delay_sweep"] = delay_sweep(torch, sar, plan, work, restore, stat)
    if not args.no_cpu_baseline and args.phases == "all":
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
