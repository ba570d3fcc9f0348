"""CPU oracle for round-optimal broadcast schedules (arXiv 2407.18004).

TEST INFRASTRUCTURE ONLY.  A ctypes view of ``bcast_oracle.c``: plain
sequential C that follows the paper's Algorithms 1-6 step by step.  Only the
tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import
this package; the HIP library and its Python binding never do.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bcast_oracle.c")
_LIB = os.path.join(_HERE, "libbcast_oracle.so")

U64_MAX = (1 << 64) - 1


def build(force: bool = True) -> str:
    """Compile the oracle with gcc.  Returns the path of the shared object."""
    if force or not os.path.exists(_LIB):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
               "-Wall", "-Wextra", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True, cwd=_HERE)
    return _LIB


class RecvStats(ctypes.Structure):
    _fields_ = [("scans", ctypes.c_int64), ("calls", ctypes.c_int64),
                ("max_depth", ctypes.c_int64), ("anomalies", ctypes.c_int64)]


class Verdict(ctypes.Structure):
    _fields_ = [("flags", ctypes.c_uint32), ("rounds", ctypes.c_uint32),
                ("n_bad_recv_dup", ctypes.c_uint64),
                ("n_bad_send_unheld", ctypes.c_uint64),
                ("n_edge_mismatch", ctypes.c_uint64),
                ("n_incomplete_ranks", ctypes.c_uint64),
                ("first_bad", ctypes.c_uint64)]

    def as_dict(self) -> dict:
        return {name: int(getattr(self, name)) for name, _ in self._fields_}


_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB):
        build(force=True)
    lib = ctypes.CDLL(_LIB)
    i64, i32p = ctypes.c_int64, ctypes.POINTER(ctypes.c_int32)
    lib.orc_q.argtypes = [i64]
    lib.orc_skips.argtypes = [i64, ctypes.POINTER(ctypes.c_int64)]
    lib.orc_baseblock.argtypes = [i64, i64]
    lib.orc_recvschedule.argtypes = [i64, i64, i32p, ctypes.POINTER(RecvStats)]
    lib.orc_sendschedule_def.argtypes = [i64, i64, i32p]
    lib.orc_sendschedule.argtypes = [i64, i64, i32p, ctypes.POINTER(ctypes.c_int),
                                     ctypes.POINTER(ctypes.c_uint32)]
    lib.orc_schedules.argtypes = [i64, i64, i64, i64, i32p, i32p, i64,
                                  ctypes.c_int, ctypes.c_int]
    lib.orc_schedules_ranks.argtypes = [i64, i64, ctypes.POINTER(ctypes.c_uint32),
                                        i64, i32p, ctypes.c_int, ctypes.c_int]
    lib.orc_digest.argtypes = [i64, i64, i64, i64, ctypes.POINTER(ctypes.c_uint64),
                               ctypes.POINTER(ctypes.c_uint32), ctypes.c_int,
                               ctypes.c_int]
    lib.orc_digest_row.argtypes = [i64, i64, i64, i32p, i32p, ctypes.c_int,
                                   ctypes.c_int, ctypes.POINTER(ctypes.c_uint64),
                                   ctypes.POINTER(ctypes.c_uint32)]
    lib.orc_simulate.argtypes = [i64, i64, i64, i32p, ctypes.POINTER(Verdict)]
    lib.orc_simulate_reduce.argtypes = [i64, i64, i64, i32p, ctypes.POINTER(Verdict)]
    lib.orc_simulate_reduce.restype = ctypes.c_int
    for name in ("orc_q", "orc_skips", "orc_baseblock", "orc_recvschedule",
                 "orc_sendschedule_def", "orc_sendschedule", "orc_schedules",
                 "orc_schedules_ranks", "orc_digest", "orc_digest_row",
                 "orc_simulate"):
        getattr(lib, name).restype = ctypes.c_int
    u64p = ctypes.POINTER(ctypes.c_uint64)
    lib.orc_edgecheck.argtypes = [i64, i64, i64, i64, u64p, u64p, ctypes.c_int, ctypes.c_int]
    lib.orc_edgecheck.restype = ctypes.c_int
    lib.orc_edgecheck_table.argtypes = [i64, i32p, u64p, u64p]
    lib.orc_edgecheck_table.restype = ctypes.c_int
    lib.orc_sm64.argtypes = [ctypes.c_uint64]
    lib.orc_sm64.restype = ctypes.c_uint64
    _lib = lib
    return lib


def _i32p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _check(rc: int, what: str) -> int:
    if rc < 0:
        raise ValueError(f"oracle: {what} rejected its arguments (rc={rc})")
    return rc


def default_threads() -> int:
    return max(1, len(os.sched_getaffinity(0)))


def sm64(z: int) -> int:
    return int(_load().orc_sm64(z & U64_MAX))


def q_of(p: int) -> int:
    return _check(_load().orc_q(p), "orc_q")


def skips(p: int) -> list[int]:
    """Algorithm 2: [skip[0], ..., skip[q]] with skip[q] = p."""
    buf = (ctypes.c_int64 * 64)()
    q = _check(_load().orc_skips(p, buf), "orc_skips")
    return [int(buf[k]) for k in range(q + 1)]


def baseblock(p: int, r: int) -> int:
    """Algorithm 3."""
    return _check(_load().orc_baseblock(p, r), "orc_baseblock")


def recvschedule(p: int, r: int, with_stats: bool = False):
    """Algorithm 5 for root 0."""
    q = q_of(p)
    out = np.zeros(max(q, 1), dtype=np.int32)
    st = RecvStats()
    produced = _check(_load().orc_recvschedule(p, r, _i32p(out), ctypes.byref(st)),
                      "orc_recvschedule")
    out = out[:q]
    if with_stats:
        return out, {"scans": st.scans, "calls": st.calls, "max_depth": st.max_depth,
                     "anomalies": st.anomalies, "produced": produced}
    return out


def sendschedule_def(p: int, r: int) -> np.ndarray:
    """Send schedule by Condition 2 (definition)."""
    q = q_of(p)
    out = np.zeros(max(q, 1), dtype=np.int32)
    _check(_load().orc_sendschedule_def(p, r, _i32p(out)), "orc_sendschedule_def")
    return out[:q]


def sendschedule(p: int, r: int, with_violations: bool = False):
    """Algorithm 6 for root 0."""
    q = q_of(p)
    out = np.zeros(max(q, 1), dtype=np.int32)
    nv = ctypes.c_int(0)
    vm = ctypes.c_uint32(0)
    _check(_load().orc_sendschedule(p, r, _i32p(out), ctypes.byref(nv), ctypes.byref(vm)),
           "orc_sendschedule")
    if with_violations:
        return out[:q], int(nv.value), int(vm.value)
    return out[:q]


def schedules(p: int, root: int = 0, r_begin: int = 0, r_end: int | None = None,
              send_mode: int = 1, threads: int | None = None) -> np.ndarray:
    """int32 [r_end-r_begin][2q]: recv in columns 0..q-1, send in q..2q-1."""
    if r_end is None:
        r_end = p
    q = q_of(p)
    nrows = max(r_end - r_begin, 0)
    out = np.zeros((nrows, 2 * q), dtype=np.int32)
    if threads is None:
        threads = default_threads()
    if q == 0:
        _check(0 if (0 <= root < p and 0 <= r_begin <= r_end <= p) else -1, "orc_schedules")
        return out
    base = _i32p(out)
    send = ctypes.cast(ctypes.addressof(base.contents) + 4 * q,
                       ctypes.POINTER(ctypes.c_int32))
    _check(_load().orc_schedules(p, root, r_begin, r_end, base, send, 2 * q,
                                 send_mode, threads), "orc_schedules")
    return out


def schedules_ranks(p: int, root: int, ranks: np.ndarray, send_mode: int = 1,
                    threads: int | None = None) -> np.ndarray:
    """int32 [len(ranks)][2q] for the listed physical ranks."""
    q = q_of(p)
    ranks = np.ascontiguousarray(ranks, dtype=np.uint32)
    out = np.zeros((ranks.size, 2 * q), dtype=np.int32)
    if threads is None:
        threads = default_threads()
    _check(_load().orc_schedules_ranks(
        p, root, ranks.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)), ranks.size,
        _i32p(out) if out.size else None, send_mode, threads), "orc_schedules_ranks")
    return out


def digest(p: int, root: int, r_begin: int, r_end: int, send_mode: int = 1,
           threads: int | None = None) -> tuple[int, int]:
    """(64-bit digest, flags) over physical ranks [r_begin, r_end)."""
    dg = ctypes.c_uint64(0)
    fl = ctypes.c_uint32(0)
    if threads is None:
        threads = default_threads()
    _check(_load().orc_digest(p, root, r_begin, r_end, ctypes.byref(dg),
                              ctypes.byref(fl), send_mode, threads), "orc_digest")
    return int(dg.value), int(fl.value)


def digest_row(p: int, root: int, r: int, recv, send, viol_count: int = 0,
               produced: int | None = None) -> tuple[int, int]:
    """(hash, flags) of one given row."""
    q = q_of(p)
    recv = np.ascontiguousarray(recv, dtype=np.int32)
    send = np.ascontiguousarray(send, dtype=np.int32)
    assert recv.size == q and send.size == q
    if produced is None:
        produced = q
    h = ctypes.c_uint64(0)
    fl = ctypes.c_uint32(0)
    pad = np.zeros(1, dtype=np.int32)
    _check(_load().orc_digest_row(p, root, r, _i32p(recv if q else pad),
                                  _i32p(send if q else pad), viol_count, produced,
                                  ctypes.byref(h), ctypes.byref(fl)), "orc_digest_row")
    return int(h.value), int(fl.value)


def edgecheck(p: int, root: int, r_begin: int, r_end: int, send_mode: int = 1,
              threads: int | None = None) -> tuple[int, int]:
    """(xor_recv, xor_send) of the edge check over physical ranks [r_begin, r_end)."""
    xr, xs = ctypes.c_uint64(0), ctypes.c_uint64(0)
    if threads is None:
        threads = default_threads()
    _check(_load().orc_edgecheck(p, root, r_begin, r_end, ctypes.byref(xr), ctypes.byref(xs),
                                 send_mode, threads), "orc_edgecheck")
    return int(xr.value), int(xs.value)


def edgecheck_table(p: int, sched: np.ndarray) -> tuple[int, int]:
    """(xor_recv, xor_send) of a given table sched[p][2q]."""
    q = q_of(p)
    sched = np.ascontiguousarray(sched, dtype=np.int32)
    assert sched.shape == (p, 2 * q)
    xr, xs = ctypes.c_uint64(0), ctypes.c_uint64(0)
    pad = np.zeros(1, dtype=np.int32)
    _check(_load().orc_edgecheck_table(p, _i32p(sched if sched.size else pad), ctypes.byref(xr),
                                       ctypes.byref(xs)), "orc_edgecheck_table")
    return int(xr.value), int(xs.value)


def simulate_reduce(p: int, n: int, root: int = 0, sched: np.ndarray | None = None) -> dict:
    """The rounds of Algorithm 1 backwards (reduction to the root); verdict as a dict."""
    return simulate(p, n, root, sched, _fn="orc_simulate_reduce")


def simulate(p: int, n: int, root: int = 0, sched: np.ndarray | None = None,
             _fn: str = "orc_simulate") -> dict:
    """Algorithm 1 over possession marks; returns the verdict as a dict."""
    vd = Verdict()
    ptr = None
    if sched is not None:
        q = q_of(p)
        sched = np.ascontiguousarray(sched, dtype=np.int32)
        assert sched.shape == (p, 2 * q)
        ptr = _i32p(sched) if sched.size else None
    _check(getattr(_load(), _fn)(p, n, root, ptr, ctypes.byref(vd)), _fn)
    return vd.as_dict()
