"""Schedule-free results.  TEST INFRASTRUCTURE.

* ``allreduce_f64``: the AllReduce postcondition of Sec. 3.1 - every rank
  ends with the elementwise sum over all n ranks - in float64.
* ``allreduce_exact_int``: the same sum in Python-width integers (int64),
  for integer-valued inputs where every order gives the same bits.
* ``stragglar_fold`` / ``ring_fold``: the floating-point result in the order
  the schedules add it, as a plain fold.  In the completion rounds every chunk
  is added to exactly once (its straggler pairing, Alg. 1) and otherwise only
  copied, so the result is fixed by the precondition's ring order:
  chunk c (owned by logical rank c) = (((x_{c+1} + x_{c+2}) + ...) + x_c),
  indices mod n-1 over the on-time ranks, then + x_sigma.  The ring AllReduce
  of App. E is the same fold over all n ranks and n chunks.
"""

import numpy as np

from .replay import add
from .schedule import chunk_layout, to_physical


def to_f64(x, dtype):
    if dtype == "bf16":
        from .bf16 import bf16_to_f32
        return bf16_to_f32(x).astype(np.float64)
    return np.asarray(x).astype(np.float64)


def allreduce_f64(inputs, dtype):
    acc = np.zeros(inputs[0].shape, dtype=np.float64)
    for x in inputs:
        acc += to_f64(x, dtype)
    return acc


def abs_sum_f64(inputs, dtype):
    acc = np.zeros(inputs[0].shape, dtype=np.float64)
    for x in inputs:
        acc += np.abs(to_f64(x, dtype))
    return acc


def allreduce_exact_int(inputs):
    acc = np.zeros(inputs[0].shape, dtype=np.int64)
    for x in inputs:
        acc += np.asarray(x).astype(np.int64)
    return acc


def stragglar_fold(inputs, straggler, dtype, chunks=None, elem_bytes=None,
                   align_bytes=16):
    """Value every rank holds after precondition + completion."""
    n = len(inputs)
    m = n - 1
    count = inputs[0].shape[0]
    if chunks is None:
        chunks = chunk_layout(count, m, elem_bytes, align_bytes)
    out = np.empty_like(inputs[0])
    for c, (lo, ln) in enumerate(chunks):
        sl = slice(lo, lo + ln)
        out[sl] = stragglar_fold_chunk([x[sl] for x in inputs], c, straggler, dtype)
    return out


def precondition_fold_chunk(cols, c, straggler, dtype):
    """What the precondition of Sec. 3.1 leaves in chunk ``c`` of its owner
    (logical rank c): the sum over the n-1 on-time ranks in ring order,
    (((x_{c+1} + x_{c+2}) + ...) + x_c), indices mod n-1.  ``cols[rank]`` are
    columns that all lie inside chunk ``c``."""
    n = len(cols)
    m = n - 1
    acc = cols[to_physical((c + 1) % m, n, straggler)].copy()
    for k in range(2, m + 1):
        acc = add(cols[to_physical((c + k) % m, n, straggler)], acc, dtype)
    return acc


def stragglar_fold_chunk(cols, c, straggler, dtype):
    """The fold for one chunk index ``c`` on columns ``cols[rank]`` that all
    lie inside that chunk (windows of buffers too large to hold n of): the
    precondition's partial sum plus the straggler's contribution, the one add
    the completion performs on the chunk (Alg. 1, straggler pairing)."""
    return add(precondition_fold_chunk(cols, c, straggler, dtype), cols[straggler], dtype)


def ring_fold(inputs, dtype, chunks=None, elem_bytes=None, align_bytes=16):
    """Value every rank holds after the ring AllReduce."""
    n = len(inputs)
    count = inputs[0].shape[0]
    if chunks is None:
        chunks = chunk_layout(count, n, elem_bytes, align_bytes)
    out = np.empty_like(inputs[0])
    for c, (lo, ln) in enumerate(chunks):
        sl = slice(lo, lo + ln)
        acc = inputs[(c + 1) % n][sl].copy()
        for k in range(2, n + 1):
            acc = add(inputs[(c + k) % n][sl], acc, dtype)
        out[sl] = acc
    return out


def rhd_fold(inputs, dtype, chunks=None, elem_bytes=None, align_bytes=16):
    """Value every rank holds after recursive halving/doubling (App. E): per
    chunk c a balanced tree - in step k the rank that keeps c adds the partial
    of the rank whose index differs in bit (log n - 1 - k).  V(i, 0) = x_i,
    V(i, k+1) = rnd(V(i, k) + V(i ^ bit, k)); the result is V(c, log n)."""
    n = len(inputs)
    L = n.bit_length() - 1
    count = inputs[0].shape[0]
    if chunks is None:
        chunks = chunk_layout(count, n, elem_bytes, align_bytes)
    out = np.empty_like(inputs[0])

    def partial(i, k, sl):
        if k == 0:
            return inputs[i][sl]
        bit = 1 << (L - k)            # the bit exchanged in step k-1
        return add(partial(i, k - 1, sl), partial(i ^ bit, k - 1, sl), dtype)

    for c, (lo, ln) in enumerate(chunks):
        sl = slice(lo, lo + ln)
        out[sl] = partial(c, L, sl)
    return out
