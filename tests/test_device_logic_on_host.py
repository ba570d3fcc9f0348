"""The HIP library's per-rank device functions, compiled for the CPU with a
small stand-in for the HIP header, against the oracle.  No GPU is involved:
this checks the state-machine form of the receive search, the send walk, the
32-bit arithmetic near p = 2^31 and the flag logic before anything is launched."""
import ctypes
import os
import subprocess

import numpy as np
import pytest

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))
SHIM_DIR = os.path.join(HERE, "host_shim")
SHIM_SO = os.path.join(SHIM_DIR, "libdevice_on_host.so")


@pytest.fixture(scope="module")
def shim():
    src = os.path.join(SHIM_DIR, "device_on_host.cpp")
    hdr = os.path.join(os.path.dirname(HERE), "paper_2407_18004_amd", "csrc", "bcast_device.hpp")
    newest = max(os.path.getmtime(src), os.path.getmtime(hdr))
    if not os.path.exists(SHIM_SO) or os.path.getmtime(SHIM_SO) < newest:
        subprocess.run(["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-I", SHIM_DIR,
                        "-Wall", "-o", SHIM_SO, src], check=True)
    lib = ctypes.CDLL(SHIM_SO)
    lib.shim_schedules_ranks.argtypes = [ctypes.c_uint32, ctypes.c_uint32, ctypes.c_void_p,
                                         ctypes.c_uint64, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                                         ctypes.c_void_p]
    lib.shim_digest_row.argtypes = [ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint32,
                                    ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    lib.shim_digest_row.restype = None
    lib.shim_edge_row.argtypes = [ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint32,
                                  ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    lib.shim_edge_row.restype = None
    lib.shim_schedules_tiles.argtypes = [ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint32,
                                         ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int, ctypes.c_int,
                                         ctypes.c_void_p, ctypes.c_void_p,
                                         ctypes.c_void_p, ctypes.c_void_p]
    lib.shim_last_replays.restype = ctypes.c_uint64
    lib.shim_last_from_table.restype = ctypes.c_uint64
    lib.shim_last_generic.restype = ctypes.c_uint64
    lib.shim_wave_operations.restype = ctypes.c_uint64
    lib.shim_wave_mismatches.restype = ctypes.c_uint64
    lib.shim_recv_two_ways.argtypes = [ctypes.c_uint32, ctypes.c_uint32, ctypes.c_void_p,
                                       ctypes.c_void_p, ctypes.c_void_p]
    lib.shim_recv_two_ways.restype = ctypes.c_uint32
    lib.shim_last_top_replays.restype = ctypes.c_uint64
    lib.shim_last_mid_replays.restype = ctypes.c_uint64
    return lib


def shim_rows(lib, p, root, ranks, flat=False):
    ranks = np.ascontiguousarray(ranks, dtype=np.uint32)
    q = oracle.q_of(p)
    rows = np.zeros((ranks.size, 2 * q), dtype=np.int32)
    flags = np.zeros(ranks.size, dtype=np.uint32)
    hashes = np.zeros(ranks.size, dtype=np.uint64)
    got_q = lib.shim_schedules_ranks(p, root, ranks.ctypes.data, ranks.size, int(flat),
                                     rows.ctypes.data if rows.size else None,
                                     flags.ctypes.data, hashes.ctypes.data)
    assert got_q == q
    return rows, flags, hashes


def shim_tiles(lib, p, root, r_begin, n, run_tiles=0, descending=True, use_table=False):
    """Rows, flags and hashes of n consecutive ranks, computed tile by tile by a wavefront of 64
    lanes on the CPU (runs of run_tiles tiles; 0 = one run), and the violations of Algorithm 6
    that were answered from a neighbour's row."""
    q = oracle.q_of(p)
    rows = np.zeros((n, 2 * q), dtype=np.int32)
    flags = np.zeros(n, dtype=np.uint32)
    hashes = np.zeros(n, dtype=np.uint64)
    borrowed = ctypes.c_uint64(0)
    lib.shim_schedules_tiles(p, root, r_begin, n, run_tiles, int(descending), int(use_table),
                             rows.ctypes.data if rows.size else None,
                             flags.ctypes.data, hashes.ctypes.data, ctypes.byref(borrowed))
    assert int(lib.shim_wave_mismatches()) == 0       # the lanes met at the same operations
    return rows, flags, hashes, int(borrowed.value)


def test_tiles_of_consecutive_ranks(shim):
    # violations filled in from a neighbour's row of the same 64-rank tile
    total_borrowed = 0
    for p in list(range(1, 600)) + [1025, 4097, 65537]:
        for root in {0, p // 2, p - 1}:
            rows, flags, _, borrowed = shim_tiles(shim, p, root, 0, p)
            assert np.array_equal(rows, oracle.schedules(p, root=root, send_mode=1)), (p, root)
            assert not flags.any()
            total_borrowed += borrowed
    assert total_borrowed > 10000
    for p, root, a, n in [(1000003, 17, 499000, 5000), (2**31 - 1, 99, 2**31 - 5000, 4999),
                          (3 * 2**28 + 5, 2**29, 2**29 - 1000, 3000), (65537, 65536, 65000, 537)]:
        rows, flags, _, borrowed = shim_tiles(shim, p, root, a, n)
        assert np.array_equal(rows, oracle.schedules(p, root=root, r_begin=a, r_end=a + n))
        assert not flags.any()


def test_all_ranks_small_p(shim):
    for p in range(1, 2049):
        rows, flags, hashes = shim_rows(shim, p, 0, np.arange(p))
        want = oracle.schedules(p, send_mode=1)
        assert np.array_equal(rows, want), p
        assert not flags.any(), p
        flat_rows, flat_flags, _ = shim_rows(shim, p, 0, np.arange(p), flat=True)    # the branch-free search
        assert np.array_equal(flat_rows, want) and not flat_flags.any(), p
        dg, fl = oracle.digest(p, 0, 0, p)
        assert int(np.bitwise_xor.reduce(hashes)) == dg and fl == 0


def test_roots_and_large_p(shim):
    for p in (1000003, 65537, 2**31 - 1, 2**31 - 2, 2**30 + 1, 2**20, 3 * 2**28 + 5):
        rng = np.random.default_rng(p + 1)
        root = int(rng.integers(0, p))
        ranks = np.unique(np.concatenate([
            rng.integers(0, p, size=6000), np.arange(0, 70), np.arange(p - 70, p),
            (root + np.arange(-3, 4)) % p])).astype(np.uint32)
        rows, flags, hashes = shim_rows(shim, p, root, ranks)
        want = oracle.schedules_ranks(p, root, ranks, send_mode=1)
        assert np.array_equal(rows, want), p
        assert not flags.any()
        flat_rows, flat_flags, _ = shim_rows(shim, p, root, ranks, flat=True)
        assert np.array_equal(flat_rows, want) and not flat_flags.any(), p
        for j in range(0, len(ranks), 97):
            h, fl = oracle.digest_row(p, root, int(ranks[j]), want[j, :want.shape[1] // 2],
                                      want[j, want.shape[1] // 2:])
            assert (h, fl) == (int(hashes[j]), 0)


def test_flags_on_planted_mistakes(shim):
    p, root = 1000, 17
    q = oracle.q_of(p)
    rng = np.random.default_rng(5)
    for r in rng.integers(0, p, size=60):
        r = int(r)
        row = oracle.schedules_ranks(p, root, np.array([r]))[0]
        for trial in range(12):
            bad = row.copy()
            pos = int(rng.integers(0, 2 * q))
            # values of the legal range, any byte, and the bytes that agree with the right value
            # in their low six bits (the quick test of a row knows a value by those)
            if trial % 4 == 0:
                bad[pos] = int(rng.integers(-128, 128))
            elif trial % 4 == 1:
                bad[pos] = int(row[pos]) + (64 if row[pos] < 0 or trial % 8 == 1 else -64)
                assert -128 <= bad[pos] <= 127
            else:
                bad[pos] = int(rng.integers(-q, q))
            want = oracle.digest_row(p, root, r, bad[:q], bad[q:])
            h = ctypes.c_uint64(0)
            fl = ctypes.c_uint32(0)
            bad = np.ascontiguousarray(bad, dtype=np.int32)
            shim.shim_digest_row(p, root, r, bad.ctypes.data, ctypes.byref(h), ctypes.byref(fl))
            assert (int(h.value), int(fl.value)) == want, (r, pos, bad.tolist())


def test_edge_check_rows(shim):
    for p, root in [(17, 0), (1000, 321), (65537, 65536), (2**31 - 1, 12345)]:
        rng = np.random.default_rng(p)
        ranks = rng.integers(0, p, size=300).astype(np.uint32)
        rows = oracle.schedules_ranks(p, root, ranks)
        xr, xs = ctypes.c_uint64(0), ctypes.c_uint64(0)
        want_r = want_s = 0
        for j, r in enumerate(ranks):
            row = np.ascontiguousarray(rows[j])
            shim.shim_edge_row(p, root, int(r), row.ctypes.data, ctypes.byref(xr), ctypes.byref(xs))
            a, b = oracle.edgecheck(p, root, int(r), int(r) + 1)
            want_r ^= a
            want_s ^= b
        assert (int(xr.value), int(xs.value)) == (want_r, want_s)


def test_replayed_lockstep_stretch_equals_the_search(shim):
    # Consecutive tiles of a wavefront's run mostly arrive at the lockstep stretch of the receive
    # search in the same shared state; the kernels then replay a recorded stretch instead of
    # searching, and take the state after the top levels of the pass over from the tile before.
    # Here a wavefront of 64 lanes runs on the CPU (lane-0 broadcasts, any, minimum and maximum
    # over the 64 lanes' own values), so the checks that decide whether a record may be taken
    # over see what they see on the GPU.  Whatever is replayed must equal Algorithm 5, everywhere
    # a record can be taken over: long stretches of consecutive ranks at both ends and in the
    # middle of several p, from the top down (kernels for p with violations) and from the bottom
    # up (kernels for p = 2^q and 2^q - 1), in one run (long enough for the stretch to be recorded
    # in two parts) and in runs as short as the kernels'.
    replays = 0
    cases = [(2**31 - 1, 0, 2**30 - 30000, 60000), (2**31 - 1, 12345, 2**31 - 1 - 50000, 50000),
             (2**31 - 1, 0, 0, 40000), (1000003, 0, 0, 120000), (1000003, 999999, 880000, 120003),
             (805306373, 7, 402653000, 50000), (2**30 + 1, 2**29, 2**29 - 20000, 40000),
             (65537, 1, 0, 65537), (4099, 0, 0, 4099), (3 * 2**20, 5, 2**20 - 10000, 30000),
             (2**30, 2**29 + 7, 2**29 - 20000, 45000), (2**27 - 1, 5, 2**26 - 25000, 50001)]
    for p, root, a, n in cases:
        want = oracle.schedules(p, root=root, r_begin=a, r_end=a + n, send_mode=1)
        for run_tiles, descending in [(0, True), (0, False), (6, True), (4, False), (3, False)]:
            rows, flags, _, _ = shim_tiles(shim, p, root, a, n, run_tiles, descending)
            replays_here = int(shim.shim_last_replays())
            top_here = int(shim.shim_last_top_replays())
            assert np.array_equal(rows, want), (p, root, a, n, run_tiles, descending)
            assert not flags.any()
            assert int(shim.shim_wave_operations()) > 0
            replays += replays_here
            if p > 10**6 and run_tiles == 0:
                assert replays_here > n // 64 // 4, (p, replays_here)     # the record is actually used
                assert top_here > n // 64 // 4, (p, top_here)
                if p > 2**26:     # long runs record the stretch in two parts: the second is taken alone too
                    assert int(shim.shim_last_mid_replays()) > n // 64 // 50, (p, descending)
    assert replays > 10000


def test_table_of_deep_entries_equals_the_search(shim):
    # With the table of deep entries a rank takes its baseblock, its first receive entries and the
    # state of the search after them from the entry of its rho, and violations of Algorithm 6
    # are answered from the to-processor's entry.  Everything must still equal Algorithms 5 and 6
    # of the oracle: all ranks of several p (small enough for that), and long stretches at both
    # ends, around powers of two and across the root for large p, in runs like the kernels'.
    from_table = generic = ranks = 0
    whole = [16385, 20000, 32767, 32768, 32769, 65537, 100003, 131071]
    cases = [(p, r, 0, p) for p in whole for r in (0, p // 3)]
    cases += [(2**31 - 1, 0, 2**30 - 30000, 60000), (2**31 - 1, 12345, 2**31 - 1 - 50000, 50000),
              (2**31 - 1, 0, 0, 40000), (1000003, 0, 0, 150000), (1000003, 999999, 860000, 140003),
              (805306373, 7, 402653000, 50000), (2**30 + 1, 2**29, 2**29 - 20000, 40000),
              (3 * 2**20, 5, 2**20 - 10000, 30000), (2**30, 2**29 + 7, 2**29 - 20000, 45000),
              (2**27 - 1, 5, 2**26 - 25000, 50001), (2**24 + 1, 0, 2**24 - 40000, 40001),
              (16384 * 3 + 1, 0, 0, 16384 * 3 + 1)]
    for p, root, a, n in cases:
        want = oracle.schedules(p, root=root, r_begin=a, r_end=a + n, send_mode=1)
        for run_tiles, descending in [(0, True), (6, True), (4, False), (2, True)]:
            rows, flags, hashes, _ = shim_tiles(shim, p, root, a, n, run_tiles, descending, use_table=True)
            assert np.array_equal(rows, want), (p, root, a, n, run_tiles, descending)
            assert not flags.any()
            from_table += int(shim.shim_last_from_table())
            generic += int(shim.shim_last_generic())
            ranks += n
        dg, fl = oracle.digest(p, root, a, a + n)
        assert int(np.bitwise_xor.reduce(hashes)) == dg and fl == 0
    assert generic > 0.99 * ranks                   # nearly every rank has an entry
    assert from_table > 100000                      # and violations are answered from the table
    # small p has no levels above the deep ones: the table is not used, the result is the same
    rows, flags, _, _ = shim_tiles(shim, 4099, 5, 0, 4099, 0, True, use_table=True)
    assert np.array_equal(rows, oracle.schedules(4099, root=5)) and int(shim.shim_last_generic()) == 0


def test_level_helpers_against_the_skips(shim):
    # first level whose skip fits into v, and the number of levels with a skip of at least the
    # threshold, against skip[] of Algorithm 2 (level j is skip[q - j])
    rng = np.random.default_rng(3)
    top_skip = int(shim.shim_top_skip())
    ps = [2, 3, 5, 17, 100, 4095, 4096, 4097, 8191, 8192, 65537, 1000003, 2**30 + 1, 2**31 - 1]
    ps += [int(x) for x in rng.integers(2, 2**31 - 1, size=40)]
    for p in ps:
        sk = oracle.skips(p)
        q = len(sk) - 1
        want_top = sum(1 for j in range(1, q + 1) if sk[q - j] >= top_skip)
        assert int(shim.shim_top_level_count(p)) == want_top, p
        vs = {1, 2, 3, p - 1, p // 2, max(1, p // 2 - 1), min(p - 1, p // 2 + 1)}
        vs |= {int(s) for s in sk[:-1]} | {int(s) - 1 for s in sk[:-1] if s > 1} | {min(p - 1, int(s) + 1) for s in sk[:-1]}
        vs |= {int(x) for x in rng.integers(1, p, size=20)}
        for v in sorted(x for x in vs if 1 <= x < p):
            want = next(j for j in range(1, q + 1) if sk[q - j] <= v)
            assert int(shim.shim_first_level_taken(p, v)) == want, (p, v)


def test_plain_and_reorganised_receive_search_agree(shim):
    # the search one list element at a time from the first call on, and the form the kernels run,
    # against each other and against Algorithm 5 of the oracle, rank 1 and the root included
    rng = np.random.default_rng(11)
    cases = [(p, v) for p in range(1, 300) for v in range(p)]
    for p in [1000003, 2**31 - 1, 2**30 + 1, 805306373, 65537, 4099]:
        vs = {0, 1, 2, 3, p - 1, p - 2, p // 2} | {int(x) for x in rng.integers(0, p, size=300)}
        cases += [(p, v) for v in sorted(vs)]
    for p, v in cases:
        q = oracle.q_of(p)
        plain = np.full(max(q, 1), 99, dtype=np.int32)
        fast = np.full(max(q, 1), 99, dtype=np.int32)
        an = ctypes.c_uint32(0)
        counts = shim.shim_recv_two_ways(p, v, plain.ctypes.data, fast.ctypes.data, ctypes.byref(an))
        assert counts == (q | (q << 16)) and an.value == 0, (p, v, counts, an.value)
        want = oracle.recvschedule(p, v)
        assert np.array_equal(plain[:q], want) and np.array_equal(fast[:q], want), (p, v)
