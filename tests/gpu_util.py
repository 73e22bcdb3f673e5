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
