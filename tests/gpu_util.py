"""Helpers for the GPU parity tests: move seeded inputs to the device, run the
library through its C ABI binding, bring results back as NumPy arrays."""

import numpy as np
import torch

from oracle import reference as R
from oracle import replay as P
from oracle import schedule as S

EB = {"i32": 4, "f32": 4, "bf16": 2}
TOL = {"f32": 1e-5, "bf16": 2.0 ** -7}      # x n, relative to sum_i |x_i|
DEV = "cuda:0"


def to_device(x, dtype):
    if dtype == "bf16":
        return torch.from_numpy(x.view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(x).to(DEV)


def to_host(t, dtype):
    if dtype == "bf16":
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def same_bits(a, b):
    return a.shape == b.shape and bool((a.view(np.uint8) == b.view(np.uint8)).all())


def oracle_stragglar(inputs, straggler, dtype):
    """O1: replay of the oracle's own schedules.  Returns (after precondition,
    after completion)."""
    n = len(inputs)
    chunks = S.chunk_layout(len(inputs[0]), n - 1, EB[dtype])
    bufs = [x.copy() for x in inputs]
    P.replay(S.rs_precondition_rounds(n, straggler), chunks, bufs, dtype)
    mid = [b.copy() for b in bufs]
    P.replay(S.completion_rounds_any(n, straggler), chunks, bufs, dtype)
    return mid, bufs


def oracle_ring(inputs, dtype):
    n = len(inputs)
    chunks = S.chunk_layout(len(inputs[0]), n, EB[dtype])
    bufs = [x.copy() for x in inputs]
    P.replay(S.ring_allreduce_rounds(n), chunks, bufs, dtype)
    return bufs


def check_tolerance(out, inputs, dtype):
    """|out - fp64 sum| <= tol * n * sum_i |x_i| per element."""
    if dtype == "i32":
        want = R.allreduce_exact_int(inputs)
        want = (want & 0xFFFFFFFF).astype(np.uint32).view(np.int32)
        assert (out == want).all()
        return
    n = len(inputs)
    ref = R.allreduce_f64(inputs, dtype)
    bound = TOL[dtype] * n * R.abs_sum_f64(inputs, dtype)
    err = np.abs(R.to_f64(out, dtype) - ref)
    assert (err <= bound).all(), "max excess %g" % float((err - bound).max())


def gpu_stragglar(lib, inputs, straggler, dtype, stream=None):
    """Run precondition then completion on the device; returns host copies
    (after precondition, after completion)."""
    n = len(inputs)
    dev = [to_device(x, dtype) for x in inputs]
    plan = lib.stragglar_plan(n, straggler, len(inputs[0]), dtype)
    lib.stragglar_phase1_reducescatter(plan, dev, stream)
    torch.cuda.synchronize()
    mid = [to_host(t, dtype) for t in dev]
    lib.stragglar_phase2_complete(plan, dev, stream)
    torch.cuda.synchronize()
    out = [to_host(t, dtype) for t in dev]
    return mid, out


def gpu_ring(lib, inputs, dtype, stream=None):
    n = len(inputs)
    dev = [to_device(x, dtype) for x in inputs]
    plan = lib.stragglar_plan(n, 0, len(inputs[0]), dtype)
    lib.ring_allreduce(plan, dev, stream)
    torch.cuda.synchronize()
    return [to_host(t, dtype) for t in dev]


def oracle_rounds(rounds, parts, inputs, dtype):
    chunks = S.chunk_layout(len(inputs[0]), parts, EB[dtype])
    bufs = [x.copy() for x in inputs]
    P.replay(rounds, chunks, bufs, dtype)
    return bufs


def gpu_call(lib, fns, inputs, straggler, dtype, stream=None):
    """Run the named entry points in sequence on fresh device copies; host copies after each."""
    n = len(inputs)
    dev = [to_device(x, dtype) for x in inputs]
    plan = lib.stragglar_plan(n, straggler, len(inputs[0]), dtype)
    outs = []
    for fn in fns:
        getattr(lib, fn)(plan, dev, stream)
        torch.cuda.synchronize()
        outs.append([to_host(t, dtype) for t in dev])
    return outs


# ---- buffers too large to hold n of on the host: the fold streamed in windows ------------
WINDOW = 1 << 24      # elements per upload and device comparison
BLOCK = 1 << 15       # elements per oracle call: its temporaries then stay in the host's caches


def streamed_fold(w, kind, bases):
    """The oracle's schedule-ordered result over the WHOLE buffer, window by window.

    kind "stragglar": yields (chunk, lo, final, partial) - ``final`` is what every rank holds in
    elements [lo, lo + len(final)) after precondition + completion, ``partial`` what the chunk's
    owner holds there after the precondition alone (``precondition_fold_chunk``; the final value
    is the straggler's one add on top of it, as in ``stragglar_fold_chunk``).  kind "ring":
    yields (chunk, lo, final, None) with ``ring_fold``.  A window never straddles a chunk border.
    The oracle functions are called as they stand, on blocks of BLOCK elements, on one host
    thread (measured: 30 ns per bf16 element at n = 8; threads only contend for the interpreter
    lock at this block size); the input columns come from ``Workload.window``.
    """
    n, sg, dt = w.n, w.straggler, w.dtype
    parts = n - 1 if kind == "stragglar" else n
    chunks = S.chunk_layout(w.count, parts, EB[dt])
    for c, (clo, cln) in enumerate(chunks):
        for lo in range(clo, clo + cln, WINDOW):
            ln = min(WINDOW, clo + cln - lo)
            cols = [w.window(r, lo, ln, base=bases[r]) for r in range(n)]
            final = np.empty(ln, dtype=cols[0].dtype)
            partial = np.empty(ln, dtype=cols[0].dtype) if kind == "stragglar" else None
            for a in range(0, ln, BLOCK):
                b = min(a + BLOCK, ln)
                sub = [col[a:b] for col in cols]
                if kind == "stragglar":
                    part = R.precondition_fold_chunk(sub, c, sg, dt)
                    partial[a:b] = part
                    final[a:b] = P.add(part, sub[sg], dt)
                else:
                    final[a:b] = R.ring_fold(sub, dt, chunks=[(0, 0)] * c + [(0, b - a)])   # the block as chunk c
            yield c, lo, final, partial


def _progress(line):
    """A long comparison says where it is (a quiet GPU job looks hung): on stdout when pytest does
    not capture it, and appended to the file the environment variable SAR_PROGRESS_LOG names."""
    import os
    print(line, flush=True)
    path = os.environ.get("SAR_PROGRESS_LOG")
    if path:
        with open(path, "a") as f:
            f.write(line + "\n")


def streamed_compare(w, kind, bases, finals, partials=()):
    """Every element of every tensor in ``finals`` (device tensors of w.count elements: the rank
    buffers after the call under test, of any number of runs) against the oracle's fold, bit for
    bit, and - kind "stragglar" - every element of the owners' chunks saved after the
    precondition: ``partials`` is a list (one entry per run) of lists of n-1 device tensors,
    entry g being chunk g of on-time rank g.  Returns the number of elements compared."""
    dt = w.dtype
    view = torch.int16 if dt == "bf16" else torch.int32
    npview = np.int16 if dt == "bf16" else np.int32
    chunks = S.chunk_layout(w.count, w.n - 1 if kind == "stragglar" else w.n, EB[dt])
    seen = 0
    for c, lo, final, partial in streamed_fold(w, kind, bases):
        ln = len(final)
        _progress("%s %s: chunk %d, elements %d..%d of %d" % (w.name, kind, c, lo, lo + ln, w.count))
        want = torch.from_numpy(final.view(npview)).to(DEV)
        bad = torch.zeros((), dtype=torch.int64, device=DEV)
        for t in finals:
            bad += (t[lo:lo + ln].view(view) != want).sum()
        if partials:
            wpart = torch.from_numpy(partial.view(npview)).to(DEV)
            off = lo - chunks[c][0]
            for run in partials:
                bad += (run[c][off:off + ln].view(view) != wpart).sum()
        assert int(bad) == 0, "%s: %d elements differ in chunk %d, window at %d" % (w.name, int(bad), c, lo)
        seen += ln
    assert seen == w.count
    return seen
