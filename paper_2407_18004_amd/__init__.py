"""MI355X (gfx950) library for round-optimal broadcast schedules.

The product is the HIP shared library behind ``include/bcast.h``; this package
is its thin Python binding (argument marshalling only) plus the seeded
workload generators used by tests and the benchmark.  There is no CPU
fallback: without the built library every call raises.
"""
from .binding import (  # noqa: F401
    BCAST_OK, BCAST_EINVAL, BCAST_ENOMEM, BCAST_EHIP, BcastError, Verdict,
    library_path, load_library, exported_symbols,
    bcast_q, bcast_skips, bcast_schedules, bcast_schedules_digest, bcast_schedules_edgecheck, bcast_schedules_double,
    bcast_schedules_workspace, bcast_schedules_ws, bcast_schedules_digest_ws, bcast_schedules_digest_chunks, bcast_schedules_edgecheck_ws,
    bcast_baseblocks, bcast_schedules_doubling_workspace, bcast_schedules_doubling,
    bcast_schedules_batched, bcast_simulate_workspace, bcast_simulate, bcast_simulate_reduce, bcast_simulate_noalloc, bcast_strerror,
)
