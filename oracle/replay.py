"""Op-by-op replay of a schedule on host buffers.  TEST INFRASTRUCTURE.

``bufs`` is a list of n one-dimensional NumPy arrays (one per physical rank),
modified in place, exactly as the ranks' buffers are in Sec. 3.1: every op
touches one chunk of one or two ranks.  Ops are applied in list order, one at
a time; an exchange reads both operands before it writes either.

dtypes: ``"i32"`` (two's-complement wrap-around add), ``"f32"`` (one IEEE
round-to-nearest-even add per op), ``"bf16"`` (uint16 storage; widen, add in
fp32, round to nearest even, per op).
"""

import numpy as np

from . import COPY, REDUCE, REDUCE_EXCHANGE
from .bf16 import bf16_add

NP_DTYPE = {"i32": np.int32, "f32": np.float32, "bf16": np.uint16}
ELEM_BYTES = {"i32": 4, "f32": 4, "bf16": 2}


def add(a, b, dtype):
    """rnd(a + b) in the arithmetic of ``dtype``."""
    if dtype == "i32":
        return (a.view(np.uint32) + b.view(np.uint32)).view(np.int32)
    if dtype == "f32":
        return a + b
    if dtype == "bf16":
        return bf16_add(a, b)
    raise ValueError(dtype)


def replay(rounds, chunks, bufs, dtype):
    """Apply ``rounds`` (list of lists of (src, dst, chunk, kind)) to ``bufs``.
    ``chunks`` is [(offset, length)] in elements for that schedule's chunking."""
    want = NP_DTYPE[dtype]
    for b in bufs:
        if b.dtype != want or b.ndim != 1:
            raise ValueError("buffer dtype/shape does not match %s" % dtype)
    for ops in rounds:
        for src, dst, c, kind in ops:
            lo, ln = chunks[c]
            s = bufs[src][lo:lo + ln]
            d = bufs[dst][lo:lo + ln]
            if kind == COPY:
                d[:] = s
            elif kind == REDUCE:
                d[:] = add(d, s, dtype)
            elif kind == REDUCE_EXCHANGE:
                t = add(s, d, dtype)
                s[:] = t
                d[:] = t
            else:
                raise ValueError("unknown op kind %r" % (kind,))
    return bufs
