#!/usr/bin/env python3
"""Benchmark of the StragglAR AllReduce hot path on one MI355X.

A *step* is one pass of the whole hot path over one batch of synthetic rank
buffers: the precondition ReduceScatter (phase 1), the completion rounds of
Alg. 1 (phase 2, the straggler's critical path) and the ring AllReduce
baseline, each timed with HIP events on the stream the kernels run on.  The
rank buffers are restored from a pristine device copy before each phase-1 and
each ring run, outside the event brackets, so every timed call sees the memory
system in the state a fresh AllReduce would (timing does depend on it: passes
run back to back without the restore are 5-10 % faster at 64-96 MiB per rank).

Headline `value`: algorithmic HBM bytes of the completion phase (2*n*s, the
schedule executed round by round) divided by its time, in GB/s, with inputs
resident in HBM, on the headline workload (config 2).

Beside the headline the same line carries, for every other configuration
(`workloads`), for the message-size sweep (`size_sweep`) and for the emulated
straggler delay (`delay_sweep`, `delay_sweep_4GiB`), the times of the three ways
a call can run - one launch per round, one launch per round with a round's
same-value copies read once, all rounds in one launch - each priced against the
bytes THAT form has to move, as the library itself reports them
(stragglar_plan_launch_form).

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
PHASES = ("phase1", "phase2", "ring")
# the three forms a call can take, as plan options
FORMS = {"per_round": {"fuse_rounds": 0, "merge_copies": 0},
         "merged_copies": {"fuse_rounds": 0, "merge_copies": 1},
         "single_launch": {"fuse_rounds": 1, "merge_copies": 0}}


def alg_bytes(which, n, s):
    """Algorithmic HBM bytes of one pass executed round by round (s = bytes per rank buffer):
    COPY reads 1 + writes 1 chunk, REDUCE reads 2 + writes 1, REDUCE_EXCHANGE
    reads 2 + writes 2.  Completion: (n-1)(n-2) copies + (n-1) exchanges of
    s/(n-1) -> 2ns.  Precondition: (n-1)(n-2) reduces -> 3(n-2)s.  Ring:
    n(n-1) reduces + n(n-1) copies of s/n -> 5(n-1)s."""
    return {"phase1": 3 * (n - 2) * s, "phase2": 2 * n * s, "ring": 5 * (n - 1) * s}[which]


def measured_traffic():
    """Fabric-side traffic per launch from the committed rocprofv3 counter summaries
    (profiles/l2_fabric_traffic.txt: workload, phase, form, bytes per launch), if present."""
    table = {}
    try:
        with open(os.path.join(ROOT, "profiles", "l2_fabric_traffic.txt")) as f:
            for line in f:
                parts = line.split()
                if len(parts) >= 4 and not line.startswith("#"):
                    table[(parts[0], parts[1], parts[2])] = float(parts[3])
    except OSError:
        pass
    return table


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
    if name.startswith("n") and "x" in name:   # n<ranks>x<MiB per rank>[bf16]: fp32 (or bf16) N(0,1), straggler 0 (the audit's size grid)
        n, mib = name[1:].split("x")
        if mib.endswith("bf16"):
            return W.Workload("n%sx%sMiB-bf16" % (n, mib[:-4]), int(n), 0, int(mib[:-4]) << 19, "bf16", ("normal", 1.0), seed=7)
        return W.Workload("n%sx%sMiB-f32" % (n, mib), int(n), 0, int(mib) << 18, "f32", ("normal", 1.0), seed=7)
    if name == "delay-4GiB":              # Sec. 4.1 "Varying straggler delay": a 4 GiB buffer
        return W.Workload("delay-4GiB-n8-f32", 8, 0, 1 << 30, "f32", ("normal", 1.0), seed=6)
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


class Buffers:
    """The n rank buffers of a workload on the device: a pristine copy and the working set."""

    def __init__(self, torch, w, pristine=None):
        from concurrent.futures import ThreadPoolExecutor
        self.torch, self.w = torch, w
        if pristine is None:
            with ThreadPoolExecutor(max_workers=min(8, w.n)) as pool:       # the draws release the interpreter lock
                bases = list(pool.map(w.base, range(w.n)))
            pristine = [w.device(r, "cuda:0", base=bases[r]) for r in range(w.n)]
        self.pristine = pristine
        self.work = [torch.empty_like(t) for t in pristine]

    def restore(self):
        for d, p in zip(self.work, self.pristine):
            d.copy_(p, non_blocking=True)


def time_calls(torch, sar, bufs, plan, steps, warmup, phases=PHASES):
    """`steps` timed passes of [restore, phase 1, phase 2, restore, ring] after `warmup` untimed
    ones; HIP events on the stream the kernels run on bracket each call.  Returns
    {phase: (mean ms, sem)}."""
    stream = torch.cuda.current_stream()
    calls = {"phase1": sar.stragglar_phase1_reducescatter, "phase2": sar.stragglar_phase2_complete,
             "ring": sar.ring_allreduce}
    rec = {ph: [] for ph in phases}
    for it in range(warmup + steps):
        bufs.restore()
        for ph in phases:
            if ph == "ring" and len(phases) > 1:
                bufs.restore()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            calls[ph](plan, bufs.work, stream)
            b.record(stream)
            if it >= warmup:
                rec[ph].append((a, b))
    torch.cuda.synchronize()
    return {ph: mean_sem([a.elapsed_time(b) for a, b in rec[ph]]) for ph in phases}


def graph_replay_completion(torch, sar, bufs, plan, steps, warmup):
    """The completion call recorded once into a HIP graph and replayed: what remains of the
    launch gaps of a round-by-round call (n + log n - 2 launches) when the host is out of the
    loop.  Same protocol around it (restore, precondition, then the timed replay)."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    rec = []
    with torch.cuda.stream(side):
        bufs.restore()
        sar.stragglar_phase1_reducescatter(plan, bufs.work, side)
        sar.stragglar_phase2_complete(plan, bufs.work, side)          # first launches outside the capture
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            sar.stragglar_phase2_complete(plan, bufs.work, side)
        for it in range(warmup + steps):
            bufs.restore()
            sar.stragglar_phase1_reducescatter(plan, bufs.work, side)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(side)
            graph.replay()
            b.record(side)
            if it >= warmup:
                rec.append((a, b))
        side.synchronize()
    torch.cuda.current_stream().wait_stream(side)
    return mean_sem([a.elapsed_time(b) for a, b in rec])


def form_report(sar, plan, stat, phases=PHASES):
    """Per phase: time, launches and bytes of the form the plan's options select (the bytes are
    the library's own count for that form), bandwidth and fraction of the HBM peak."""
    which = {"phase1": sar.PRECONDITION, "phase2": sar.COMPLETION, "ring": sar.RING}
    out = {}
    for ph in phases:
        f = plan.launch_form(which[ph])
        nbytes = f["bytes_loaded"] + f["bytes_stored"]
        ms, sem = stat[ph]
        out[ph] = {"ms": ms, "ms_sem": sem, "form": f["form"], "launches": f["launches"], "bytes": nbytes,
                   "GBps": nbytes / (ms * 1e-3) / 1e9, "frac_of_peak": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
    return out


def plan_with(sar, w, options):
    plan = sar.stragglar_plan(w.n, w.straggler, w.count, w.dtype)
    for k, v in options.items():
        plan.option_set(k, v)
    return plan


def all_forms(torch, sar, bufs, steps, warmup):
    """The three forms, plus which one the library takes by itself."""
    w = bufs.w
    out = {}
    for name, options in FORMS.items():
        plan = plan_with(sar, w, options)
        out[name] = form_report(sar, plan, time_calls(torch, sar, bufs, plan, steps, warmup))
        if name == "per_round":
            m, sem = graph_replay_completion(torch, sar, bufs, plan, steps, warmup)
            out[name]["phase2"]["graph_replay_ms"] = m
            out[name]["phase2"]["graph_replay_ms_sem"] = sem
    auto = plan_with(sar, w, {"fuse_rounds": -1})
    out["library_default_form"] = {ph: auto.launch_form(wh)["form"] for ph, wh in
                                   (("phase1", sar.PRECONDITION), ("phase2", sar.COMPLETION), ("ring", sar.RING))}
    return out


def other_baselines(torch, sar, bufs, steps, warmup):
    """The paper's other comparison algorithms on the same kernels (App. E), for context:
    recursive halving/doubling and the straggler-aware Broadcast (whose post-arrival part is
    log n rounds of the whole buffer).  One launch per round."""
    w = bufs.w
    n, s = w.n, w.bytes_per_rank
    plan = plan_with(sar, w, FORMS["per_round"])
    stream = torch.cuda.current_stream()
    L = n.bit_length() - 1
    legs = [("rhd", sar.rhd_allreduce, sar.RHD), ("broadcast_phase1", sar.broadcast_phase1_allreduce, sar.BCAST_PRECONDITION),
            ("broadcast_phase2", sar.broadcast_phase2_complete, sar.BCAST_COMPLETION)]
    res = {}
    rec = {name: [] for name, _, _ in legs}
    for it in range(warmup + steps):
        bufs.restore()
        for name, fn, _ in legs:
            if name == "broadcast_phase1":
                bufs.restore()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            fn(plan, bufs.work, stream)
            b.record(stream)
            if it >= warmup:
                rec[name].append((a, b))
    torch.cuda.synchronize()
    for name, _, which in legs:
        m, sem = mean_sem([a.elapsed_time(b) for a, b in rec[name]])
        f = plan.launch_form(which)
        nbytes = f["bytes_loaded"] + f["bytes_stored"]
        res[name + "_ms"] = m
        res[name + "_ms_sem"] = sem
        res[name + "_bytes"] = nbytes
        res[name + "_GBps"] = nbytes / (m * 1e-3) / 1e9
    res["rounds"] = {"rhd": 2 * L, "broadcast_phase1": 2 * (n - 2), "broadcast_phase2": L}
    return res


def size_sweep(torch, sar, steps=20, warmup=3):
    """Message-size sweep in powers of two, 1 MiB .. 1 GiB per rank (Sec. 4.1 sweeps powers of
    two and reports algorithmic bandwidth = buffer bytes / time), n = 8, bf16, N(0,1) values:
    every size uses a prefix of the rank buffers of the 1 GiB workload.  The buffers are
    restored before every timed phase-1 and ring call, as in the headline legs."""
    import synth_inputs as W
    big = Buffers(torch, W.cfg4((1 << 30) // 2))
    rows = []
    for p in range(20, 31):
        s = 1 << p
        w = W.cfg4(s // 2)
        bufs = Buffers(torch, w, pristine=[t[:w.count] for t in big.pristine])
        row = {"bytes_per_rank": s}
        for name, options in FORMS.items():
            plan = plan_with(sar, w, options)
            rep = form_report(sar, plan, time_calls(torch, sar, bufs, plan, steps, warmup))
            row[name] = {ph: {"ms": rep[ph]["ms"], "frac_of_peak": rep[ph]["frac_of_peak"], "launches": rep[ph]["launches"]}
                         for ph in PHASES}
            row[name]["phase2_algbw_GBps"] = s / (rep["phase2"]["ms"] * 1e-3) / 1e9
            row[name]["ring_algbw_GBps"] = s / (rep["ring"]["ms"] * 1e-3) / 1e9
        row["library_default_form"] = plan_with(sar, w, {"fuse_rounds": -1}).launch_form(sar.COMPLETION)["form"]
        rows.append(row)
        del bufs
    return {"workload": "n=8 bf16 N(0,1), prefixes of the 1 GiB-per-rank buffers; restore before every phase-1 and ring call",
            "note": "with the n buffers inside the 256 MiB memory-side cache (up to 16-32 MiB per rank) a call can run "
                    "above the HBM peak: frac_of_peak is then a statement about the cache, not about HBM",
            "rows": rows}


def overlapping_stream(torch, sar):
    """A second stream whose kernels run beside the current stream's.  The runtime spreads streams
    over a few hardware queues, and two streams that share one run their kernels one after the
    other; which queue a new stream gets depends on how many were created before it.  Candidates
    are tried until a 2 ms idle kernel on one does not hold back a 1 us kernel on the current
    stream.  Returns (stream, whether it overlaps)."""
    main_s = torch.cuda.current_stream()
    tried = []
    for _ in range(8):
        tried.append(torch.cuda.Stream())
        torch.cuda.synchronize()
        t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0.record(main_s)
        tried[-1].wait_event(t0)
        sar.stragglar_delay(2_000_000, tried[-1])
        sar.stragglar_delay(1_000, main_s)
        t1.record(main_s)
        torch.cuda.synchronize()
        if t0.elapsed_time(t1) < 1.0:
            return tried[-1], True
    return tried[-1], False


def delay_sweep(torch, sar, bufs, delays_ms, reps=5):
    """Total AllReduce time from the moment the on-time ranks call it, with the late rank
    emulated by an idle kernel on a second stream (Sec. 4.1, "Varying straggler delay").
    StragglAR: precondition starts at once, completion waits for the straggler (one
    stragglar_allreduce call with the arrival event).  Ring: everything waits for the straggler."""
    w = bufs.w
    main_s = torch.cuda.current_stream()
    late, overlaps = overlapping_stream(torch, sar)
    plans = {name: plan_with(sar, w, FORMS[name]) for name in ("per_round", "single_launch")}

    def total(d_ns, kind, plan):
        ts = []
        for _ in range(reps):
            bufs.restore()
            torch.cuda.synchronize()
            t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            arrived = torch.cuda.Event()
            t0.record(main_s)
            late.wait_event(t0)
            sar.stragglar_delay(d_ns, late)
            arrived.record(late)
            if kind == "stragglar":      # precondition at once, completion behind the arrival event
                sar.stragglar_allreduce(plan, bufs.work, main_s, arrived)
            else:
                main_s.wait_event(arrived)
                sar.ring_allreduce(plan, bufs.work, main_s)
            t1.record(main_s)
            torch.cuda.synchronize()
            ts.append(t0.elapsed_time(t1))
        return mean_sem(ts)[0]

    for plan in plans.values():                        # warm-up: stream creation, first launches
        total(0, "stragglar", plan), total(0, "ring", plan)
    rows = []
    for d_ms in delays_ms:
        d_ns = int(d_ms * 1e6)
        row = {"delay_ms": d_ms}
        for name, plan in plans.items():
            row[name] = {"stragglar_total_ms": total(d_ns, "stragglar", plan), "ring_total_ms": total(d_ns, "ring", plan)}
        rows.append(row)

    def break_even(name):
        """Smallest swept delay from which StragglAR's total stays below the ring's."""
        ahead = [r[name]["stragglar_total_ms"] < r[name]["ring_total_ms"] for r in rows]
        for i in range(len(rows)):
            if all(ahead[i:]):
                return rows[i]["delay_ms"]
        return None

    return {"workload": w.name, "bytes_per_rank": w.bytes_per_rank, "rows": rows,
            "late_stream_runs_beside_the_main_stream": overlaps,
            "emulated_break_even_delay_ms": {name: break_even(name) for name in plans},
            "note": "the paper's critical delays (5.53 ms on H100, 7.57 ms on A100, 4 GiB buffers) are per-link NVLink "
                    "figures; here time follows the aggregate HBM bytes of all ranks (precondition + completion move "
                    "about as much as the ring), so the break-even delay is near 0 and StragglAR's lead approaches "
                    "the whole precondition time once the delay exceeds it"}


def policy_audit(torch, sar, names, steps, warmup):
    """The library's automatic launch shapes against a grid of explicit ones, per workload, form
    and phase, all timed with the benchmark's own protocol on this GPU.  Prints a table (this is
    what profiles/policy_audit.txt holds): automatic time, best time of the grid and its
    settings, and automatic / best."""
    grids = {
        "single_launch": [{"fuse_rounds": 1, "fused_unroll": u, "fused_wgs_per_cu": g, "fused_split": sp, "fused_direct": d}
                          for u in (1, 2) for g in (0, 2, 3, 4, 6) for sp in (0, 1) for d in (0, 1) if not (sp and (u, g) != (2, 2))],
        "per_round": [{"fuse_rounds": 0, "merge_copies": 0, "unroll": u, "nontemporal": nt} for u in (1, 2, 4) for nt in (-1, 0, 1)],
        "merged_copies": [{"fuse_rounds": 0, "merge_copies": 1, "unroll": u, "nontemporal": nt} for u in (1, 2, 4) for nt in (-1, 0, 1)],
    }
    print("launch-policy audit: automatic choice vs explicit settings (ms per call; %d timed passes after %d warm-up; "
          "restore before every phase-1 and ring call)" % (steps, warmup))
    worst = 1.0
    for name in names:
        w = workload_by_name(name)
        bufs = Buffers(torch, w)
        for form, grid in grids.items():
            auto = time_calls(torch, sar, bufs, plan_with(sar, w, FORMS[form]), steps, warmup)
            best = {ph: (auto[ph][0], "automatic") for ph in PHASES}
            for options in grid:
                stat = time_calls(torch, sar, bufs, plan_with(sar, w, options), steps, warmup)
                for ph in PHASES:
                    if stat[ph][0] < best[ph][0]:
                        best[ph] = (stat[ph][0], " ".join("%s=%d" % kv for kv in options.items() if kv[0] not in ("fuse_rounds", "merge_copies")))
            again = time_calls(torch, sar, bufs, plan_with(sar, w, FORMS[form]), steps, warmup)     # repeatability of the automatic leg
            for ph in PHASES:
                a = min(auto[ph][0], again[ph][0])
                ratio = a / best[ph][0]
                worst = max(worst, ratio)
                print("%-32s %-14s %-7s auto %8.4f (repeat %8.4f)  best %8.4f  auto/best %.3f  [%s]" % (
                    w.name, form, ph, auto[ph][0], again[ph][0], best[ph][0], ratio, best[ph][1]), flush=True)
        del bufs
        torch.cuda.empty_cache()
    print("largest auto/best: %.3f" % worst)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg2", help="the headline workload (cfg2 is the configuration the metric is quoted on)")
    ap.add_argument("--phases", default="all", choices=["all", "phase1", "phase2", "ring"],
                    help="'all' is the benchmark; a single phase is for profiling that kernel alone "
                         "(its input state is then arbitrary, and nothing but that phase is run)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--lean", action="store_true",
                    help="the headline leg only (all three phases of one form on one workload, the benchmark's own "
                         "protocol): what the rocprofv3 summaries in profiles/ are made with")
    ap.add_argument("--no-workloads", action="store_true", help="skip the other configurations (cfg3, cfg4, cfg5)")
    ap.add_argument("--no-sweeps", action="store_true", help="skip the message-size and straggler-delay sweeps")
    ap.add_argument("--policy-audit", action="store_true",
                    help="instead of the benchmark: time the automatic launch shapes against a grid of explicit ones on "
                         "every configuration and print the table")
    ap.add_argument("--audit-workloads", help="with --policy-audit: comma-separated workloads instead of the five configurations "
                                              "(cfg names, cfg4-<bytes per rank>, n<ranks>x<MiB per rank>)")
    ap.add_argument("--blocks-per-cu", type=int)
    ap.add_argument("--unroll", type=int)
    ap.add_argument("--nontemporal", type=int)
    ap.add_argument("--fuse-rounds", type=int, help="0 one launch per round, 1 single launch, -1 automatic")
    ap.add_argument("--merge-copies", type=int, help="1: a round's same-value copies are read once (with one launch per round)")
    ap.add_argument("--fused-unroll", type=int)
    ap.add_argument("--fused-wgs-per-cu", type=int)
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the n ranks are emulated as n buffers in one "
              "GPU's HBM); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2505_23523_amd as sar
    import synth_inputs as W
    sar.load()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    # explicit knobs become the process-wide defaults; the forms below are plan options and win over them
    explicit = {}
    for key, val in (("blocks_per_cu", args.blocks_per_cu), ("unroll", args.unroll), ("nontemporal", args.nontemporal),
                     ("fuse_rounds", args.fuse_rounds), ("merge_copies", args.merge_copies),
                     ("fused_unroll", args.fused_unroll), ("fused_wgs_per_cu", args.fused_wgs_per_cu)):
        if val is not None:
            sar.tune_set(key, val)
            explicit[key] = val

    if args.lean:
        args.no_cpu_baseline = args.no_workloads = args.no_sweeps = True
    if args.policy_audit:
        names = args.audit_workloads.split(",") if args.audit_workloads else ("cfg2", "cfg4", "cfg5-16", "cfg5-32", "cfg3")
        policy_audit(torch, sar, names, min(args.steps, 20), min(args.warmup, 3))
        return

    w = workload_by_name(args.workload)
    n, s = w.n, w.bytes_per_rank
    bufs = Buffers(torch, w)
    traffic = measured_traffic()

    # ---- headline leg: the schedule round by round unless a form was asked for explicitly ----
    head_options = {} if ("fuse_rounds" in explicit or "merge_copies" in explicit) else dict(FORMS["per_round"])
    plan = plan_with(sar, w, head_options)
    phases = PHASES if args.phases == "all" else (args.phases,)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    stat = time_calls(torch, sar, bufs, plan, args.steps, args.warmup, phases)
    wall = time.perf_counter() - t0
    rep = form_report(sar, plan, stat, phases)
    main_ph = "phase2" if "phase2" in phases else phases[0]
    t_main = stat[main_ph][0]
    form = rep[main_ph]["form"]
    # per-round headline: the byte model of the schedule as written (the library's count agrees up to chunk rounding)
    head_bytes = alg_bytes(main_ph, n, s) if form == "per_round" else rep[main_ph]["bytes"]
    value = head_bytes / (t_main * 1e-3) / 1e9
    launches = rep[main_ph]["launches"]

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
                   "bytes_per_rank": s, "phases": args.phases, "form": form,
                   "launch": {k: plan.option_get(k) for k in sar.binding.TUNABLES}},
        "wall_ms_per_step_incl_restore": wall / (args.steps + args.warmup) * 1e3,
    }
    for ph in phases:
        out[ph + "_ms"] = stat[ph][0]
        out[ph + "_ms_sem"] = stat[ph][1]
        out[ph + "_GBps"] = (alg_bytes(ph, n, s) if rep[ph]["form"] == "per_round" else rep[ph]["bytes"]) / (stat[ph][0] * 1e-3) / 1e9
        out[ph + "_rounds"] = plan.num_rounds({"phase1": sar.PRECONDITION, "phase2": sar.COMPLETION, "ring": sar.RING}[ph])
        out[ph + "_bytes_by_library_count"] = rep[ph]["bytes"]
        out[ph + "_launches"] = rep[ph]["launches"]
        out[ph + "_form"] = rep[ph]["form"]
    if main_ph == "phase2" and args.phases == "all" and not args.lean:
        m, sem = graph_replay_completion(torch, sar, bufs, plan, args.steps, args.warmup)
        out["phase2_graph_replay_ms"] = m          # the same call replayed from a HIP graph (context, never the headline)
        out["phase2_graph_replay_ms_sem"] = sem
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
    kernel = {"per_round": "round_kernel", "per_round_merged_copies": "group_kernel",
              "single_launch": "sum_to_all_kernel / fused_kernel", "single_launch_split": "exchange_kernel + broadcast_kernel"}[form]
    avg_launch_ms = t_main / launches
    out["roofline"] = {
        "bound": "hbm",
        "kernel": "%s (%s, %d launch%s per pass)" % (kernel, main_ph, launches, "" if launches == 1 else "es"),
        "achieved": head_bytes / launches / (avg_launch_ms * 1e-3) / 1e9,
        "peak": HBM_PEAK_GBS,
        "unit": "GB/s",
        "frac": head_bytes / launches / (avg_launch_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "traffic": traffic.get((w.name, main_ph, form)),
        "traffic_source": "profiles/l2_fabric_traffic.txt (rocprofv3 FETCH_SIZE / WRITE_SIZE of the same command; counted "
                          "between L2 and the fabric, so reads served by the memory-side cache are included)",
        "bytes_per_launch": head_bytes / launches,
        "avg_launch_ms": avg_launch_ms,
    }

    if args.phases == "all" and not args.lean:
        # the other forms on the headline workload (never the headline value)
        for name in ("single_launch", "merged_copies"):
            p2 = plan_with(sar, w, FORMS[name])
            out[name] = form_report(sar, p2, time_calls(torch, sar, bufs, p2, args.steps, args.warmup))
        both = []                       # both phases as one call with no delay to wait for
        p1 = plan_with(sar, w, FORMS["single_launch"])
        stream = torch.cuda.current_stream()
        for i in range(args.warmup + args.steps):
            bufs.restore()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            sar.stragglar_allreduce(p1, bufs.work, stream)
            b.record(stream)
            if i >= args.warmup:
                both.append((a, b))
        torch.cuda.synchronize()
        mb, semb = mean_sem([a.elapsed_time(b) for a, b in both])
        f = p1.launch_form(sar.ALLREDUCE)
        nb = f["bytes_loaded"] + f["bytes_stored"]
        out["single_launch"]["allreduce_no_delay"] = {"ms": mb, "ms_sem": semb, "bytes": nb, "launches": f["launches"],
                                                      "GBps": nb / (mb * 1e-3) / 1e9, "frac_of_peak": nb / (mb * 1e-3) / 1e9 / HBM_PEAK_GBS}
        out["library_default_form"] = {ph: plan_with(sar, w, {"fuse_rounds": -1}).launch_form(wh)["form"] for ph, wh in
                                       (("phase1", sar.PRECONDITION), ("phase2", sar.COMPLETION), ("ring", sar.RING))}
        out["other_baselines"] = other_baselines(torch, sar, bufs, args.steps, args.warmup)
        if not args.no_sweeps:
            out["delay_sweep"] = delay_sweep(torch, sar, bufs, (0.0, 0.1, 0.25, 0.5, 0.75, 1.0, 2.0, 5.0, 9.45))
    del bufs
    torch.cuda.empty_cache()

    if args.phases == "all" and not args.no_workloads:
        rows = []
        shared = {}
        for name in ("cfg3", "cfg4", "cfg5-32", "cfg5-16"):
            if name == args.workload:
                continue
            wk = workload_by_name(name)
            pristine = None
            if name == "cfg5-16" and "cfg5-32" in shared:      # same seed and per-rank streams: ranks 0..15 of the 32
                pristine = shared["cfg5-32"][:16]
            b = Buffers(torch, wk, pristine=pristine)
            if name == "cfg5-32":
                shared[name] = b.pristine
            row = {"workload": wk.name, "n_ranks": wk.n, "dtype": wk.dtype, "straggler": wk.straggler,
                   "bytes_per_rank": wk.bytes_per_rank, "steps": args.steps, "warmup": args.warmup}
            row.update(all_forms(torch, sar, b, args.steps, args.warmup))
            rows.append(row)
            del b
            torch.cuda.empty_cache()
        shared.clear()
        out["workloads"] = rows
    if args.phases == "all" and not args.no_sweeps:
        torch.cuda.empty_cache()
        out["size_sweep"] = size_sweep(torch, sar)
        torch.cuda.empty_cache()
        free, _ = torch.cuda.mem_get_info()
        if free > (80 << 30):
            big = Buffers(torch, workload_by_name("delay-4GiB"))
            out["delay_sweep_4GiB"] = delay_sweep(torch, sar, big, (0.0, 2.0, 4.0, 6.0, 8.0, 9.45, 12.0, 16.0, 24.0), reps=3)
            del big
            torch.cuda.empty_cache()
    if not args.no_cpu_baseline and args.phases == "all":
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
