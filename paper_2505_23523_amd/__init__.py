"""MI355X-native StragglAR AllReduce hot path (arXiv 2505.23523).

Thin ctypes binding over ``libstragglar.so`` (see ``include/stragglar.h``):
argument marshalling only - planning and every step of the data path run in
the library.  There is no fallback: if the library is missing or a call
fails, an exception is raised.
"""

from .binding import (  # noqa: F401
    ALLREDUCE, BCAST_COMPLETION, BCAST_PRECONDITION, COMPLETION, PRECONDITION, RHD, RING, DTYPES, OPTION_INHERIT, Plan,
    StragglarError, broadcast_phase1_allreduce, broadcast_phase2_complete, lib_path, load,
    rhd_allreduce, ring_allreduce, stragglar_phase1_reducescatter, stragglar_phase2_complete,
    stragglar_allreduce, stragglar_delay, stragglar_plan, tune_get, tune_set,
)
