"""Seeded synthetic rank buffers shaped like the paper's AllReduce workloads.

This module only *draws inputs*: it holds none of the method's arithmetic and
is the one piece of code that both the tests' CPU oracle and the HIP path are
fed from.  AllReduce cost does not depend on the values, so the workloads of
Sec. 4 (data-parallel gradient buffers, tensor-parallel activations, the
power-of-two buffer sweep of Sec. 4.1) are represented by their shapes.

Every buffer is a one-dimensional host array:
  * "f32"  -> numpy.float32
  * "i32"  -> numpy.int32
  * "bf16" -> numpy.uint16 holding bfloat16 bit patterns (drawn in fp32 and
    narrowed with PyTorch's CPU round-to-nearest-even conversion).

Randomness is a counter-based Philox stream keyed by (seed, rank).

Buffers larger than ``TILE_THRESHOLD`` (2^26) elements are *tiled*: rank r draws a
base block of ``period(r)`` elements and repeats it, x_r[e] = base_r[e mod
period(r)].  The periods differ per rank (and are odd), so the alignment of
the ranks' blocks keeps shifting and element columns do not repeat for a very
long stretch.  This keeps host generation of the 1.24e9-element gradient
workload to seconds; ``gather`` evaluates any element without materialising
the buffer.
"""

import numpy as np

NP_DTYPE = {"i32": np.int32, "f32": np.float32, "bf16": np.uint16}
ELEM_BYTES = {"i32": 4, "f32": 4, "bf16": 2}

TILE_THRESHOLD = 1 << 26
_BASE_PERIOD = (1 << 24) - 1


class Workload:
    """n rank buffers of ``count`` elements of ``dtype``.

    dist: ("normal", std) | ("uniform_int", lo, hi)  (hi inclusive)
    """

    def __init__(self, name, n, straggler, count, dtype, dist, seed=0):
        self.name, self.n, self.straggler = name, n, straggler
        self.count, self.dtype, self.dist, self.seed = count, dtype, dist, seed

    @property
    def bytes_per_rank(self):
        return self.count * ELEM_BYTES[self.dtype]

    @property
    def tiled(self):
        return self.count > TILE_THRESHOLD

    def period(self, rank):
        """Length of rank's base block (== count when not tiled)."""
        if not self.tiled:
            return self.count
        return _BASE_PERIOD - 2 * (37 * rank + 5)

    # -- drawing -----------------------------------------------------------
    def _draw(self, rank, length):
        rng = np.random.Generator(np.random.Philox(key=[self.seed, rank]))
        kind = self.dist[0]
        if kind == "normal":
            x = rng.standard_normal(length, dtype=np.float32)
            x *= np.float32(self.dist[1])
        elif kind == "uniform_int":
            lo, hi = self.dist[1], self.dist[2]
            x = rng.integers(lo, hi + 1, size=length, dtype=np.int32)
        else:
            raise ValueError(kind)
        if self.dtype == "i32":
            return x.astype(np.int32)
        if self.dtype == "f32":
            return x.astype(np.float32)
        if self.dtype == "bf16":
            import torch
            t = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16)
            return t.view(torch.int16).numpy().view(np.uint16).copy()
        raise ValueError(self.dtype)

    def base(self, rank):
        return self._draw(rank, self.period(rank))

    def host(self, rank):
        """The full buffer of ``rank`` on the host."""
        b = self.base(rank)
        if not self.tiled:
            return b
        return np.resize(b, self.count)

    def head(self, rank, count):
        """The first ``count`` elements of rank's buffer (count <= period),
        drawn without generating the rest: the Philox stream fills arrays in
        order, so a shorter draw is a prefix of a longer one."""
        if count > self.period(rank):
            return self.host(rank)[:count]
        return self._draw(rank, count)

    def host_all(self):
        return [self.host(r) for r in range(self.n)]

    def gather(self, rank, idx, base=None):
        """x_rank[idx] for an index array, without the full buffer."""
        if base is None:
            base = self.base(rank)
        return base[np.asarray(idx, dtype=np.int64) % self.period(rank)]

    def window(self, rank, lo, length, base=None):
        """x_rank[lo : lo + length] as a contiguous array, without the full
        buffer (streamed comparisons of buffers too large to hold n of)."""
        if base is None:
            base = self.base(rank)
        p = self.period(rank)
        out = np.empty(length, dtype=base.dtype)
        pos, start = 0, lo % p
        while pos < length:
            take = min(p - start, length - pos)
            out[pos:pos + take] = base[start:start + take]
            pos += take
            start = 0
        return out

    # -- device (PyTorch is used for memory only) ---------------------------
    def device(self, rank, device="cuda:0", base=None):
        """The full buffer of ``rank`` as a flat torch tensor on ``device``
        (int32 / float32 / bfloat16)."""
        import torch
        if base is None:
            base = self.base(rank)
        if self.dtype == "bf16":
            t = torch.from_numpy(base.view(np.int16)).to(device).view(torch.bfloat16)
        else:
            t = torch.from_numpy(base).to(device)
        if not self.tiled:
            return t
        reps = -(-self.count // t.numel())
        out = torch.empty(self.count, dtype=t.dtype, device=device)
        p = t.numel()
        for k in range(reps):
            lo = k * p
            hi = min(lo + p, self.count)
            out[lo:hi] = t[:hi - lo]
        return out


def straggler_from_seed(seed, n):
    return int(np.random.Generator(np.random.Philox(key=[seed, 0xA11])).integers(0, n))


# The five configurations the benchmark and the parity tests are quoted on.
def cfg1():
    return Workload("cfg1-n4-f32-4096-smallint", 4, 0, 4096, "f32",
                    ("uniform_int", -8, 8), seed=0)


def cfg2(dtype="f32"):
    if dtype == "f32":
        return Workload("cfg2-n8-f32-64Mi", 8, 0, 64 << 20, "f32", ("normal", 1.0), seed=2)
    return Workload("cfg2-n8-i32-64Mi", 8, 0, 64 << 20, "i32",
                    ("uniform_int", -1000, 1000), seed=2)


def cfg3(seed=3):
    return Workload("cfg3-dp-grad-n8-bf16-1.24e9", 8, straggler_from_seed(seed, 8),
                    1_240_000_000, "bf16", ("normal", 1e-3), seed=seed)


def cfg4(count=8 * 2048 * 3072):
    return Workload("cfg4-tp-act-n8-bf16-%d" % count, 8, 0, count, "bf16",
                    ("normal", 1.0), seed=4)


def cfg4_sweep_counts():
    """1 MiB .. 1 GiB per rank in powers of two (bf16 elements)."""
    return [(1 << p) // 2 for p in range(20, 31)]


def cfg5(n, straggler):
    return Workload("cfg5-n%d-f32-16Mi-s%d" % (n, straggler), n, straggler,
                    16 << 20, "f32", ("normal", 1.0), seed=5)


def scaled(w, count, name=None):
    """Same recipe as ``w`` at a smaller element count (parity-test sizes)."""
    return Workload(name or (w.name + "@%d" % count), w.n, w.straggler, count,
                    w.dtype, w.dist, w.seed)
