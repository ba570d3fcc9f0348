"""Seeded synthetic inputs for the five workloads (numpy only).

This module serves both the HIP path and the CPU oracle and holds none of the
method's arithmetic: it only draws processor counts, roots and rank lists.
Randomness comes from a counter-based generator (the SplitMix64 finaliser on
(seed, stream, index)), so any element can be regenerated on its own.

The paper's own workload is "every rank of every p in a range" (its appendix on
overheads) and exhaustive checking of all schedules; the instances below are
that workload made concrete, plus random (p, root, rank) draws that cover the
whole domain up to p = 2^31 - 1.
"""
from __future__ import annotations

import numpy as np

_U64 = np.uint64


def _mix(z: np.ndarray) -> np.ndarray:
    """SplitMix64 finaliser on uint64 arrays (wrap-around arithmetic)."""
    with np.errstate(over="ignore"):
        z = (z + _U64(0x9E3779B97F4A7C15)).astype(np.uint64)
        z = ((z ^ (z >> _U64(30))) * _U64(0xBF58476D1CE4E5B9)).astype(np.uint64)
        z = ((z ^ (z >> _U64(27))) * _U64(0x94D049BB133111EB)).astype(np.uint64)
        return z ^ (z >> _U64(31))


def counter_random(seed: int, stream, index) -> np.ndarray:
    """uint64 values that depend only on (seed, stream, index); broadcasts."""
    stream = np.asarray(stream, dtype=np.uint64)
    index = np.asarray(index, dtype=np.uint64)
    with np.errstate(over="ignore"):
        key = _mix(_mix(np.asarray(seed, dtype=np.uint64)) ^ stream)
        return _mix(key + index)


# ---- workload 1: exhaustive small sweep ------------------------------------

SMALL_SWEEP_MAX_P = 4096


def small_sweep_blocks(q: int) -> int:
    """Number of blocks simulated for an instance with q rounds per phase."""
    return 2 * q + 3


# ---- workload 2: one materialised instance ---------------------------------

MATERIALISED_P = 1_000_003

# ---- workload 3: huge streamed instance ------------------------------------

STREAMED_P = 2**31 - 1
STREAMED_CHUNK = 2**26


def streamed_chunks(p: int = STREAMED_P, chunk: int = STREAMED_CHUNK):
    """[(r_begin, r_end)] covering [0, p) in chunks."""
    return [(a, min(a + chunk, p)) for a in range(0, p, chunk)]


def streamed_sample_ranks(count: int = 2**20, seed: int = 42, p: int = STREAMED_P) -> np.ndarray:
    """Seeded random subset of ranks (with repetition) of the huge instance."""
    return (counter_random(seed, 3, np.arange(count)) % _U64(p)).astype(np.uint32)


# ---- workload 4: batched random instances ----------------------------------

def batched_instances(n_inst: int = 65536, m: int = 4096, seed: int = 42,
                      first: int = 0, with_ranks: bool = True):
    """Instances first .. first+n_inst-1 of the batched workload.

    p is "log-uniform" made integer-exact: the bit length L is uniform in
    {2..31} and p uniform in [2^(L-1), 2^L), so 2 <= p < 2^31.  root and the m
    ranks are uniform in [0, p).  Returns (p, root, ranks[n_inst][m]) as uint32.
    """
    inst = np.arange(first, first + n_inst, dtype=np.uint64)
    L = (counter_random(seed, 10, inst) % _U64(30)) + _U64(2)
    lo = _U64(1) << (L - _U64(1))
    p = lo + counter_random(seed, 11, inst) % lo
    root = counter_random(seed, 12, inst) % p
    ranks = None
    if with_ranks:
        j = np.arange(m, dtype=np.uint64)[None, :]
        with np.errstate(over="ignore"):
            stream = (inst[:, None] << _U64(8)) + _U64(13)
        ranks = (counter_random(seed, stream, j) % p[:, None]).astype(np.uint32)
    return p.astype(np.uint32), root.astype(np.uint32), ranks


def batched_ranks_on_device(p: np.ndarray, m: int, seed: int, first: int, device):
    """The ranks of batched_instances(len(p), m, seed, first), generated on `device` with torch
    (int32 tensor [len(p)][m] holding the uint32 values): the same counter-based draws in
    64-bit wrap-around arithmetic, for workloads too large to draw on the host in reasonable time."""
    import torch

    def u64(x):                                    # a Python int as the int64 with the same bits
        x &= (1 << 64) - 1
        return x - (1 << 64) if x >= (1 << 63) else x

    def shr(z, k):                                 # logical shift right of int64 bit patterns
        return (z >> k) & ((1 << (64 - k)) - 1)

    def mix(z):
        z = z + u64(0x9E3779B97F4A7C15)
        z = (z ^ shr(z, 30)) * u64(0xBF58476D1CE4E5B9)
        z = (z ^ shr(z, 27)) * u64(0x94D049BB133111EB)
        return z ^ shr(z, 31)

    n_inst = len(p)
    inst = torch.arange(first, first + n_inst, dtype=torch.int64, device=device)
    stream = (inst << 8) + 13
    seed_mixed = u64(int(_mix(np.asarray(seed, dtype=np.uint64))))
    key = mix(stream ^ seed_mixed)[:, None]
    j = torch.arange(m, dtype=torch.int64, device=device)[None, :]
    z = mix(key + j)                               # uint64 draws as int64 bit patterns
    pt = torch.from_numpy(np.asarray(p, dtype=np.int64)).to(device)[:, None]
    hi, lo = shr(z, 32), z & 0xFFFFFFFF            # z mod p from its halves: p < 2^31, no overflow
    two32 = (1 << 32) % pt
    r = ((hi % pt) * two32 + lo % pt) % pt
    return r.to(torch.int32)


def q_of(p) -> np.ndarray:
    """ceil(log2 p) for arrays of processor counts (layout only, no schedule math)."""
    p = np.asarray(p, dtype=np.int64)
    q = np.zeros(p.shape, dtype=np.int64)
    for b in range(32):
        q = np.where((np.int64(1) << b) < p, b + 1, q)
    return q


def batched_row_offsets(p: np.ndarray, m: int) -> np.ndarray:
    """Prefix sums (int64, n_inst+1) of m * 2q(p[i]) int32 elements."""
    off = np.zeros(p.size + 1, dtype=np.int64)
    np.cumsum(q_of(p) * 2 * m, out=off[1:])
    return off


# ---- workload 5: broadcast simulation --------------------------------------

SIMULATION_P = 65_537
SIMULATION_N = 256
SIMULATION_ROOT = 12_345


def simulation_roots(count: int = 64, seed: int = 42, p: int = SIMULATION_P) -> list[int]:
    return [int(x) for x in counter_random(seed, 20, np.arange(count)) % _U64(p)]
