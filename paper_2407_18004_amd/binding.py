"""ctypes binding of include/bcast.h: same names, marshalling only.

Device buffers are torch tensors (PyTorch supplies memory and streams, nothing
else); their addresses and the current stream's handle are passed to the C ABI
as plain integers.  Every step of the computation runs in the HIP kernels.
"""
from __future__ import annotations

import ctypes
import os
import re

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libbcast_mi355x.so")
_HEADER = os.path.join(os.path.dirname(_HERE), "include", "bcast.h")

BCAST_OK, BCAST_EINVAL, BCAST_ENOMEM, BCAST_EHIP = 0, -1, -2, -3


class BcastError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {bcast_strerror(code)} ({code})")


class Verdict(ctypes.Structure):
    """Mirror of struct bcast_verdict."""
    _fields_ = [("flags", ctypes.c_uint32), ("rounds", ctypes.c_uint32),
                ("n_bad_recv_dup", ctypes.c_uint64),
                ("n_bad_send_unheld", ctypes.c_uint64),
                ("n_edge_mismatch", ctypes.c_uint64),
                ("n_incomplete_ranks", ctypes.c_uint64),
                ("first_bad", ctypes.c_uint64)]

    def as_dict(self) -> dict:
        return {name: int(getattr(self, name)) for name, _ in self._fields_}


VERDICT_BYTES = ctypes.sizeof(Verdict)
_lib = None


def library_path() -> str:
    return _LIB_PATH


def exported_symbols() -> list[str]:
    """Names of the functions include/bcast.h declares."""
    with open(_HEADER) as fh:
        text = fh.read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bcast_[a-z_0-9]+)\s*\(", text)))


def load_library():
    """Loads the built library; raises if it is missing (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2407_18004_amd.build` "
            "(there is no CPU fallback)")
    try:  # share the HIP runtime PyTorch has loaded, if PyTorch is there
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(_LIB_PATH)
    vp, u32, u64, i64 = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_int64
    lib.bcast_q.argtypes = [u32]
    lib.bcast_skips.argtypes = [u32, ctypes.POINTER(u32), ctypes.POINTER(ctypes.c_int)]
    lib.bcast_schedules.argtypes = [u32, u32, u64, u64, vp, vp, i64, vp]
    lib.bcast_schedules_digest.argtypes = [u32, u32, u64, u64, vp, vp, vp]
    lib.bcast_schedules_edgecheck.argtypes = [u32, u32, u64, u64, vp, vp]
    lib.bcast_schedules_edgecheck.restype = ctypes.c_int
    lib.bcast_schedules_double.argtypes = [u32, vp, vp, vp]
    lib.bcast_schedules_double.restype = ctypes.c_int
    lib.bcast_schedules_batched.argtypes = [u32, vp, vp, vp, u32, vp, vp, u64, vp, vp]
    lib.bcast_simulate_workspace.argtypes = [u32, u32, u32]
    lib.bcast_simulate_workspace.restype = ctypes.c_size_t
    lib.bcast_simulate.argtypes = [u32, u32, ctypes.POINTER(u32), u32, vp, vp,
                                   ctypes.c_size_t, vp, vp]
    lib.bcast_simulate_reduce.argtypes = lib.bcast_simulate.argtypes
    lib.bcast_simulate_reduce.restype = ctypes.c_int
    lib.bcast_schedules_workspace.argtypes = [u32]
    lib.bcast_schedules_workspace.restype = ctypes.c_size_t
    lib.bcast_schedules_ws.argtypes = [u32, u32, u64, u64, vp, vp, i64, vp, ctypes.c_size_t, vp]
    lib.bcast_schedules_digest_ws.argtypes = [u32, u32, u64, u64, vp, vp, vp, ctypes.c_size_t, vp]
    lib.bcast_schedules_edgecheck_ws.argtypes = [u32, u32, u64, u64, vp, vp, ctypes.c_size_t, vp]
    lib.bcast_schedules_digest_chunks.argtypes = [u32, u32, u64, u64, u64, vp, vp, vp, ctypes.c_size_t, vp]
    lib.bcast_schedules_digest_chunks.restype = ctypes.c_int
    for name in ("bcast_schedules_ws", "bcast_schedules_digest_ws", "bcast_schedules_edgecheck_ws"):
        getattr(lib, name).restype = ctypes.c_int
    lib.bcast_baseblocks.argtypes = [u32, vp, vp]
    lib.bcast_baseblocks.restype = ctypes.c_int
    lib.bcast_schedules_doubling_workspace.argtypes = [u32]
    lib.bcast_schedules_doubling_workspace.restype = ctypes.c_size_t
    lib.bcast_schedules_doubling.argtypes = [u32, vp, vp, ctypes.c_size_t, vp]
    lib.bcast_schedules_doubling.restype = ctypes.c_int
    lib.bcast_simulate_noalloc.argtypes = [u32, u32, ctypes.POINTER(u32), u32, vp, vp, vp]
    lib.bcast_simulate_noalloc.restype = ctypes.c_int
    lib.bcast_strerror.argtypes = [ctypes.c_int]
    lib.bcast_strerror.restype = ctypes.c_char_p
    for name in ("bcast_q", "bcast_skips", "bcast_schedules", "bcast_schedules_digest",
                 "bcast_schedules_batched", "bcast_simulate"):
        getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def _stream_handle(stream) -> int:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return stream
    return int(stream.cuda_stream)


def _dev_ptr(t, dtype, what: str) -> int:
    import torch
    if t is None:
        return 0
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{what}: expected a contiguous device tensor of {dtype}")
    return int(t.data_ptr())


def _check(rc: int, what: str) -> None:
    if rc != BCAST_OK:
        raise BcastError(rc, what)


def bcast_strerror(code: int) -> str:
    return load_library().bcast_strerror(code).decode()


def bcast_q(p: int) -> int:
    rc = load_library().bcast_q(p)
    if rc < 0:
        raise BcastError(rc, "bcast_q")
    return rc


def bcast_skips(p: int) -> list[int]:
    """Algorithm 2: [skip[0], ..., skip[q]]."""
    buf = (ctypes.c_uint32 * 32)()
    q = ctypes.c_int(0)
    _check(load_library().bcast_skips(p, buf, ctypes.byref(q)), "bcast_skips")
    return [int(buf[k]) for k in range(q.value + 1)]


def bcast_schedules(p: int, root: int, r_begin: int, r_end: int, recv, send, ld: int,
                    stream=None, send_offset: int = 0) -> None:
    """recv/send: device int32 tensors.  If `send` is the same tensor as `recv`,
    the send rows start `send_offset` elements into it (the [ranks][2q] table is
    recv=send=table, ld=2q, send_offset=q)."""
    import torch
    rp = _dev_ptr(recv, torch.int32, "recv")
    sp = _dev_ptr(send, torch.int32, "send")
    if sp:
        sp += 4 * send_offset
    _check(load_library().bcast_schedules(p, root, r_begin, r_end, rp, sp, ld,
                                          _stream_handle(stream)), "bcast_schedules")


def bcast_schedules_workspace(p: int) -> int:
    return int(load_library().bcast_schedules_workspace(p))


def bcast_schedules_ws(p: int, root: int, r_begin: int, r_end: int, recv, send, ld: int,
                       workspace, stream=None, send_offset: int = 0) -> None:
    """bcast_schedules with a device workspace (uint8 tensor of bcast_schedules_workspace(p) bytes)."""
    import torch
    rp = _dev_ptr(recv, torch.int32, "recv")
    sp = _dev_ptr(send, torch.int32, "send")
    if sp:
        sp += 4 * send_offset
    _check(load_library().bcast_schedules_ws(
        p, root, r_begin, r_end, rp, sp, ld, _dev_ptr(workspace, torch.uint8, "workspace"),
        0 if workspace is None else workspace.numel(), _stream_handle(stream)), "bcast_schedules_ws")


def bcast_schedules_digest_ws(p: int, root: int, r_begin: int, r_end: int, digest, flags, workspace,
                              stream=None) -> None:
    import torch
    _check(load_library().bcast_schedules_digest_ws(
        p, root, r_begin, r_end, _dev_ptr(digest, torch.int64, "digest"),
        _dev_ptr(flags, torch.int32, "flags"), _dev_ptr(workspace, torch.uint8, "workspace"),
        0 if workspace is None else workspace.numel(), _stream_handle(stream)),
        "bcast_schedules_digest_ws")


def bcast_schedules_digest_chunks(p: int, root: int, r_begin: int, r_end: int, chunk_ranks: int, digests,
                                  flags, workspace=None, stream=None) -> None:
    """digests: device int64 tensor, flags: device int32 tensor, one element per chunk of chunk_ranks
    ranks; workspace: uint8 tensor of bcast_schedules_workspace(p) bytes, or None."""
    import torch
    _check(load_library().bcast_schedules_digest_chunks(
        p, root, r_begin, r_end, chunk_ranks, _dev_ptr(digests, torch.int64, "digests"),
        _dev_ptr(flags, torch.int32, "flags"), _dev_ptr(workspace, torch.uint8, "workspace"),
        0 if workspace is None else workspace.numel(), _stream_handle(stream)),
        "bcast_schedules_digest_chunks")


def bcast_schedules_edgecheck_ws(p: int, root: int, r_begin: int, r_end: int, xors, workspace,
                                 stream=None) -> None:
    import torch
    if xors is not None and xors.numel() < 2:
        raise TypeError("xors: two elements are written")
    _check(load_library().bcast_schedules_edgecheck_ws(
        p, root, r_begin, r_end, _dev_ptr(xors, torch.int64, "xors"),
        _dev_ptr(workspace, torch.uint8, "workspace"),
        0 if workspace is None else workspace.numel(), _stream_handle(stream)),
        "bcast_schedules_edgecheck_ws")


def bcast_schedules_digest(p: int, root: int, r_begin: int, r_end: int, digest, flags,
                           stream=None) -> None:
    """digest: device int64 tensor (1 element, read it as unsigned); flags: device int32 (1)."""
    import torch
    _check(load_library().bcast_schedules_digest(
        p, root, r_begin, r_end, _dev_ptr(digest, torch.int64, "digest"),
        _dev_ptr(flags, torch.int32, "flags"), _stream_handle(stream)),
        "bcast_schedules_digest")


def bcast_schedules_edgecheck(p: int, root: int, r_begin: int, r_end: int, xors,
                              stream=None) -> None:
    """xors: device int64 tensor of 2 elements (read them as unsigned)."""
    import torch
    if xors is not None and xors.numel() < 2:
        raise TypeError("xors: two elements are written")
    _check(load_library().bcast_schedules_edgecheck(
        p, root, r_begin, r_end, _dev_ptr(xors, torch.int64, "xors"), _stream_handle(stream)),
        "bcast_schedules_edgecheck")


def bcast_schedules_double(p: int, table_in, table_out, stream=None) -> None:
    """table_in: device int32 [p][2q] for root 0 (None for p = 1); table_out: device int32
    [2p][2(q+1)]."""
    import torch
    _check(load_library().bcast_schedules_double(
        p, _dev_ptr(table_in, torch.int32, "table_in"), _dev_ptr(table_out, torch.int32, "table_out"),
        _stream_handle(stream)), "bcast_schedules_double")


def bcast_schedules_batched(n_inst: int, p, root, ranks, m: int, row_off, out,
                            n_rejected=None, stream=None) -> None:
    """p, root, ranks: device int32 tensors holding uint32 bit patterns; row_off:
    device int64 (n_inst+1); out: device int32; n_rejected: device int32 (1) or None."""
    import torch
    _check(load_library().bcast_schedules_batched(
        n_inst, _dev_ptr(p, torch.int32, "p"), _dev_ptr(root, torch.int32, "root"),
        _dev_ptr(ranks, torch.int32, "ranks"), m, _dev_ptr(row_off, torch.int64, "row_off"),
        _dev_ptr(out, torch.int32, "out"), 0 if out is None else out.numel(),
        _dev_ptr(n_rejected, torch.int32, "n_rejected"), _stream_handle(stream)),
        "bcast_schedules_batched")


def bcast_baseblocks(p: int, out, stream=None) -> None:
    """out: device uint8 tensor of p elements; out[r] = baseblock of rank r (root 0)."""
    import torch
    if out is None or out.numel() < p:
        raise ValueError("out must hold p bytes")
    _check(load_library().bcast_baseblocks(p, _dev_ptr(out, torch.uint8, "out"), _stream_handle(stream)),
           "bcast_baseblocks")


def bcast_schedules_doubling_workspace(p: int) -> int:
    return int(load_library().bcast_schedules_doubling_workspace(p))


def bcast_schedules_doubling(p: int, out, workspace, stream=None) -> None:
    """out: device int32 tensor [p][2q]; workspace: device uint8 tensor."""
    import torch
    q = bcast_q(p)
    if out is not None and out.numel() < p * 2 * q:
        raise ValueError("out must hold p * 2q int32 elements")
    _check(load_library().bcast_schedules_doubling(
        p, _dev_ptr(out, torch.int32, "out"), _dev_ptr(workspace, torch.uint8, "workspace"),
        0 if workspace is None else workspace.numel(), _stream_handle(stream)), "bcast_schedules_doubling")


def bcast_simulate_workspace(p: int, n: int, n_roots: int) -> int:
    return int(load_library().bcast_simulate_workspace(p, n, n_roots))


def bcast_simulate_reduce(p: int, n: int, roots, sched, workspace, verdict, stream=None) -> None:
    """The reduction replay (rounds backwards); arguments as for bcast_simulate."""
    bcast_simulate(p, n, roots, sched, workspace, verdict, stream, _entry="bcast_simulate_reduce")


def bcast_simulate(p: int, n: int, roots, sched, workspace, verdict, stream=None,
                   _entry: str = "bcast_simulate") -> None:
    """roots: sequence of ints (host); sched: device int32 [n_roots][p][2q] or None;
    workspace: device uint8 tensor; verdict: device uint8 tensor of
    n_roots * sizeof(bcast_verdict) bytes."""
    import torch
    roots = list(roots)
    arr = (ctypes.c_uint32 * max(len(roots), 1))(*roots)
    _check(getattr(load_library(), _entry)(
        p, n, arr, len(roots), _dev_ptr(sched, torch.int32, "sched"),
        _dev_ptr(workspace, torch.uint8, "workspace"),
        0 if workspace is None else workspace.numel(),
        _dev_ptr(verdict, torch.uint8, "verdict"), _stream_handle(stream)), _entry)


def bcast_simulate_noalloc(p: int, n: int, roots, sched, verdict, stream=None) -> None:
    """bcast_simulate on the library's own scratch array (no workspace argument)."""
    import torch
    roots = list(roots)
    arr = (ctypes.c_uint32 * max(len(roots), 1))(*roots)
    _check(load_library().bcast_simulate_noalloc(
        p, n, arr, len(roots), _dev_ptr(sched, torch.int32, "sched"),
        _dev_ptr(verdict, torch.uint8, "verdict"), _stream_handle(stream)), "bcast_simulate_noalloc")


def verdicts_from_bytes(raw: bytes) -> list[dict]:
    """Decodes a host copy of the verdict buffer."""
    n = len(raw) // VERDICT_BYTES
    return [Verdict.from_buffer_copy(raw, i * VERDICT_BYTES).as_dict() for i in range(n)]
