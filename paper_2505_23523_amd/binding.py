"""ctypes binding of the C ABI declared in include/stragglar.h."""

import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

PRECONDITION, COMPLETION, RING, RHD, BCAST_PRECONDITION, BCAST_COMPLETION, ALLREDUCE = 0, 1, 2, 3, 4, 5, 6
DTYPES = {"i32": 0, "f32": 1, "bf16": 2}
TUNABLES = {"blocks_per_cu": 0, "unroll": 1, "nontemporal": 2, "fuse_rounds": 3, "fused_unroll": 4, "fused_wgs_per_cu": 5,
            "merge_copies": 6, "fused_split": 7, "fused_direct": 8}
OPTION_INHERIT = -1000
LAUNCH_FORMS = {0: "per_round", 1: "per_round_merged_copies", 2: "single_launch", 3: "single_launch_split"}

# every symbol include/stragglar.h declares
SYMBOLS = [
    "stragglar_plan", "stragglar_plan_destroy", "stragglar_plan_num_rounds",
    "stragglar_plan_num_chunks", "stragglar_plan_round", "stragglar_plan_chunk",
    "stragglar_phase1_reducescatter", "stragglar_phase2_complete", "ring_allreduce",
    "stragglar_tune_set", "stragglar_tune_get", "stragglar_strerror", "stragglar_delay",
    "rhd_allreduce", "broadcast_phase1_allreduce", "broadcast_phase2_complete", "stragglar_allreduce",
    "stragglar_plan_launch_form", "stragglar_plan_option_set", "stragglar_plan_option_get",
]


class StragglarError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        msg = load().stragglar_strerror(status).decode()
        super().__init__("%s: %s (status %d)" % (what, msg, status))


class _LaunchForm(ctypes.Structure):
    _fields_ = [("form", ctypes.c_int), ("launches", ctypes.c_int),
                ("bytes_loaded", ctypes.c_ulonglong), ("bytes_stored", ctypes.c_ulonglong)]


class _Op(ctypes.Structure):
    _fields_ = [("src", ctypes.c_int32), ("dst", ctypes.c_int32),
                ("chunk", ctypes.c_int32), ("op", ctypes.c_int32)]


def lib_path():
    return os.path.join(HERE, "libstragglar.so")


def _stale(path):
    """True if the library was built from other sources than those in the tree: by the digest the
    build leaves beside it, or - for a library built without one - by modification times."""
    from . import build as _build
    if os.path.exists(_build.STAMP):
        with open(_build.STAMP) as f:
            return f.read().strip() != _build.source_digest()
    built = os.path.getmtime(path)
    return any(os.path.getmtime(src) > built for src in _build.source_files() if os.path.exists(src))


def load():
    """Load the in-tree library, building it first if it is not there or was built from other
    sources than the tree holds (and a compiler is at hand); raises if that fails, or if the library lacks a symbol
    the header declares (there is no fallback path)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path) or _stale(path):
        from . import build as _build
        try:
            _build.build()
        except Exception:
            if not os.path.exists(path):
                raise
            raise RuntimeError("%s does not match its sources and rebuilding it failed; run "
                               "`python -m paper_2505_23523_amd.build`" % path)
    L = ctypes.CDLL(path)
    missing = [name for name in SYMBOLS if not hasattr(L, name)]
    if missing:
        raise RuntimeError("%s does not export %s: rebuild it" % (path, ", ".join(missing)))
    vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    L.stragglar_plan.argtypes = [ci, ci, sz, ci, ctypes.POINTER(vp)]
    L.stragglar_plan.restype = ci
    L.stragglar_plan_destroy.argtypes = [vp]
    L.stragglar_plan_destroy.restype = None
    L.stragglar_plan_num_rounds.argtypes = [vp, ci]
    L.stragglar_plan_num_rounds.restype = ci
    L.stragglar_plan_num_chunks.argtypes = [vp, ci]
    L.stragglar_plan_num_chunks.restype = ci
    L.stragglar_plan_round.argtypes = [vp, ci, ci, ctypes.POINTER(ctypes.POINTER(_Op)), ctypes.POINTER(ci)]
    L.stragglar_plan_round.restype = ci
    L.stragglar_plan_chunk.argtypes = [vp, ci, ci, ctypes.POINTER(sz), ctypes.POINTER(sz)]
    L.stragglar_plan_chunk.restype = ci
    for name in ("stragglar_phase1_reducescatter", "stragglar_phase2_complete", "ring_allreduce",
                 "rhd_allreduce", "broadcast_phase1_allreduce", "broadcast_phase2_complete"):
        fn = getattr(L, name)
        fn.argtypes = [vp, ctypes.POINTER(vp), vp]
        fn.restype = ci
    L.stragglar_allreduce.argtypes = [vp, ctypes.POINTER(vp), vp, vp]
    L.stragglar_allreduce.restype = ci
    L.stragglar_delay.argtypes = [ctypes.c_ulonglong, vp]
    L.stragglar_delay.restype = ci
    L.stragglar_tune_set.argtypes = [ci, ctypes.c_long]
    L.stragglar_tune_set.restype = ci
    L.stragglar_tune_get.argtypes = [ci]
    L.stragglar_tune_get.restype = ctypes.c_long
    L.stragglar_plan_launch_form.argtypes = [vp, ci, ctypes.POINTER(_LaunchForm)]
    L.stragglar_plan_launch_form.restype = ci
    L.stragglar_plan_option_set.argtypes = [vp, ci, ctypes.c_long]
    L.stragglar_plan_option_set.restype = ci
    L.stragglar_plan_option_get.argtypes = [vp, ci]
    L.stragglar_plan_option_get.restype = ctypes.c_long
    L.stragglar_strerror.argtypes = [ci]
    L.stragglar_strerror.restype = ctypes.c_char_p
    _LIB = L
    return L


class Plan:
    """Owner of a library plan (freed on garbage collection or ``close``)."""

    def __init__(self, handle, n, straggler, count, dtype):
        self._h = handle
        self.n, self.straggler, self.count, self.dtype = n, straggler, count, dtype

    def close(self):
        if self._h:
            load().stragglar_plan_destroy(self._h)
            self._h = None

    __del__ = close

    @property
    def handle(self):
        if not self._h:
            raise RuntimeError("plan is closed")
        return self._h

    def num_rounds(self, which):
        return load().stragglar_plan_num_rounds(self.handle, which)

    def num_chunks(self, which):
        return load().stragglar_plan_num_chunks(self.handle, which)

    def round(self, which, r):
        ops = ctypes.POINTER(_Op)()
        nops = ctypes.c_int()
        st = load().stragglar_plan_round(self.handle, which, r, ctypes.byref(ops), ctypes.byref(nops))
        if st:
            raise StragglarError(st, "stragglar_plan_round")
        return [(ops[i].src, ops[i].dst, ops[i].chunk, ops[i].op) for i in range(nops.value)]

    def rounds(self, which):
        return [self.round(which, r) for r in range(self.num_rounds(which))]

    def chunk(self, which, c):
        off, ln = ctypes.c_size_t(), ctypes.c_size_t()
        st = load().stragglar_plan_chunk(self.handle, which, c, ctypes.byref(off), ctypes.byref(ln))
        if st:
            raise StragglarError(st, "stragglar_plan_chunk")
        return off.value, ln.value

    def chunks(self, which):
        return [self.chunk(which, c) for c in range(self.num_chunks(which))]

    def launch_form(self, which):
        """How a call on schedule ``which`` would run now, and the bytes that form loads and stores."""
        out = _LaunchForm()
        st = load().stragglar_plan_launch_form(self.handle, which, ctypes.byref(out))
        if st:
            raise StragglarError(st, "stragglar_plan_launch_form")
        return {"form": LAUNCH_FORMS[out.form], "launches": out.launches,
                "bytes_loaded": out.bytes_loaded, "bytes_stored": out.bytes_stored}

    def option_set(self, key, value):
        st = load().stragglar_plan_option_set(self.handle, TUNABLES[key], int(value))
        if st:
            raise StragglarError(st, "stragglar_plan_option_set(%s=%r)" % (key, value))

    def option_get(self, key):
        return load().stragglar_plan_option_get(self.handle, TUNABLES[key])


def stragglar_plan(n, straggler_rank, count, dtype):
    """dtype: "i32" | "f32" | "bf16" (or the library's integer code)."""
    code = DTYPES.get(dtype, dtype)
    out = ctypes.c_void_p()
    st = load().stragglar_plan(int(n), int(straggler_rank), int(count), int(code), ctypes.byref(out))
    if st:
        raise StragglarError(st, "stragglar_plan(n=%r, straggler=%r, count=%r, dtype=%r)"
                             % (n, straggler_rank, count, dtype))
    return Plan(out.value, n, straggler_rank, count, dtype)


def _pointers(rank_bufs):
    """Device addresses from torch tensors (``data_ptr``) or plain ints."""
    arr = (ctypes.c_void_p * len(rank_bufs))()
    for i, b in enumerate(rank_bufs):
        arr[i] = b.data_ptr() if hasattr(b, "data_ptr") else int(b)
    return arr


def _stream(stream):
    if stream is None:
        return None
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _run(name, plan, rank_bufs, stream):
    if len(rank_bufs) != plan.n:
        raise ValueError("expected %d rank buffers, got %d" % (plan.n, len(rank_bufs)))
    st = getattr(load(), name)(plan.handle, _pointers(rank_bufs), _stream(stream))
    if st:
        raise StragglarError(st, name)


def stragglar_allreduce(plan, rank_bufs, stream=None, straggler_ready=None):
    """straggler_ready: a torch.cuda.Event (or raw hipEvent_t address) recorded when the
    straggler's buffer is final, or None."""
    if len(rank_bufs) != plan.n:
        raise ValueError("expected %d rank buffers, got %d" % (plan.n, len(rank_bufs)))
    ev = None
    if straggler_ready is not None:
        ev = ctypes.c_void_p(straggler_ready.cuda_event if hasattr(straggler_ready, "cuda_event")
                             else int(straggler_ready))
    st = load().stragglar_allreduce(plan.handle, _pointers(rank_bufs), _stream(stream), ev)
    if st:
        raise StragglarError(st, "stragglar_allreduce")


def stragglar_phase1_reducescatter(plan, rank_bufs, stream=None):
    _run("stragglar_phase1_reducescatter", plan, rank_bufs, stream)


def stragglar_phase2_complete(plan, rank_bufs, stream=None):
    _run("stragglar_phase2_complete", plan, rank_bufs, stream)


def ring_allreduce(plan, rank_bufs, stream=None):
    _run("ring_allreduce", plan, rank_bufs, stream)


def rhd_allreduce(plan, rank_bufs, stream=None):
    _run("rhd_allreduce", plan, rank_bufs, stream)


def broadcast_phase1_allreduce(plan, rank_bufs, stream=None):
    _run("broadcast_phase1_allreduce", plan, rank_bufs, stream)


def broadcast_phase2_complete(plan, rank_bufs, stream=None):
    _run("broadcast_phase2_complete", plan, rank_bufs, stream)


def stragglar_delay(nanoseconds, stream=None):
    st = load().stragglar_delay(int(nanoseconds), _stream(stream))
    if st:
        raise StragglarError(st, "stragglar_delay(%r)" % (nanoseconds,))


def tune_set(key, value):
    st = load().stragglar_tune_set(TUNABLES[key], int(value))
    if st:
        raise StragglarError(st, "stragglar_tune_set(%s=%r)" % (key, value))


def tune_get(key):
    return load().stragglar_tune_get(TUNABLES[key])
