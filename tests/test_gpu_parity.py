"""Parity of the HIP library with the CPU oracle, through the C ABI.

Integer work: every comparison is bit-exact.  All inputs are seeded and
synthetic (paper_2407_18004_amd.workloads).  Small cases are compared element
by element; the full-size workloads are compared on what the oracle can
recompute in seconds (whole tables where it can, seeded samples and
order-free digests otherwise).
"""
import json
import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
import paper_2407_18004_amd as lib  # noqa: E402
from paper_2407_18004_amd import workloads  # noqa: E402
from paper_2407_18004_amd.binding import VERDICT_BYTES, verdicts_from_bytes  # noqa: E402

DEV = "cuda:0"
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("these tests need a GPU (run them with -m gpu on an MI355X)")
    lib.load_library()          # fails loudly if the HIP library is not built


def gpu_table(p, root=0, r_begin=0, r_end=None):
    """[ranks][2q] table through bcast_schedules."""
    if r_end is None:
        r_end = p
    q = lib.bcast_q(p)
    t = torch.full((max(r_end - r_begin, 0), 2 * q), 99, dtype=torch.int32, device=DEV)
    lib.bcast_schedules(p, root, r_begin, r_end, t, t, 2 * q, send_offset=q)
    torch.cuda.synchronize()
    return t.cpu().numpy()


def gpu_digest(p, root, a, b):
    dg = torch.full((1,), -1, dtype=torch.int64, device=DEV)
    fl = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    lib.bcast_schedules_digest(p, root, a, b, dg, fl)
    torch.cuda.synchronize()
    return int(dg.item()) & oracle.U64_MAX, int(fl.item()) & 0xFFFFFFFF


def gpu_edgecheck(p, root, a, b):
    x = torch.full((2,), -1, dtype=torch.int64, device=DEV)
    lib.bcast_schedules_edgecheck(p, root, a, b, x)
    torch.cuda.synchronize()
    xr, xs = (int(t) & oracle.U64_MAX for t in x.cpu().tolist())
    return xr, xs


def gpu_simulate(p, n, roots, sched=None, reduce=False):
    ws = torch.empty(lib.bcast_simulate_workspace(p, n, len(roots)), dtype=torch.uint8, device=DEV)
    vd = torch.full((len(roots) * VERDICT_BYTES,), 0xAB, dtype=torch.uint8, device=DEV)
    (lib.bcast_simulate_reduce if reduce else lib.bcast_simulate)(p, n, roots, sched, ws, vd)
    torch.cuda.synchronize()
    return verdicts_from_bytes(vd.cpu().numpy().tobytes())


def gpu_batched(p, root, ranks, row_off=None):
    n_inst, m = ranks.shape
    if row_off is None:
        row_off = workloads.batched_row_offsets(p, m)
    d = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a).view(dt)).to(DEV)  # noqa: E731
    out = torch.full((int(row_off[-1]),), 77, dtype=torch.int32, device=DEV)
    rej = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    lib.bcast_schedules_batched(n_inst, d(p, np.int32), d(root, np.int32), d(ranks, np.int32), m,
                                d(row_off, np.int64), out, rej)
    torch.cuda.synchronize()
    return out, int(rej.item()), row_off


# ------------------------------------------------------------ small cases --

def test_skips_and_q_host_calls():
    for p in (1, 2, 3, 17, 1000, 65537, 1000003, 2**31 - 1):
        assert lib.bcast_q(p) == oracle.q_of(p)
        assert lib.bcast_skips(p) == oracle.skips(p)


def test_workload1_small_sweep_schedules():
    # every p in [1, 4096], every rank, element by element
    for p in range(1, workloads.SMALL_SWEEP_MAX_P + 1):
        got = gpu_table(p)
        want = oracle.schedules(p, send_mode=1)
        assert np.array_equal(got, want), p


def test_workload1_small_sweep_simulation():
    clean = 0
    for p in range(1, workloads.SMALL_SWEEP_MAX_P + 1):
        q = oracle.q_of(p)
        n = workloads.small_sweep_blocks(q)
        got = gpu_simulate(p, n, [0])[0]
        assert got["flags"] == 0 and got["rounds"] == (n - 1 + q if q else 0), (p, got)
        assert got["first_bad"] == oracle.U64_MAX
        assert got == oracle.simulate(p, n, 0), p
        clean += 1
    assert clean == workloads.SMALL_SWEEP_MAX_P


@pytest.mark.parametrize("p,root,a,b", [
    (1000, 0, 0, 1000), (1000, 999, 3, 997), (1000, 17, 64, 128), (1000, 17, 63, 130),
    (1000, 5, 500, 500), (4097, 4096, 1, 4097), (2, 1, 0, 2), (3, 2, 0, 3), (1, 0, 0, 1),
    (65537, 12345, 65000, 65537), (2**31 - 1, 2**30, 2**31 - 1 - 300, 2**31 - 1),
    (2**31 - 1, 5, 0, 321),
])
def test_ranges_roots_and_ragged_tails(p, root, a, b):
    got = gpu_table(p, root, a, b)
    want = oracle.schedules(p, root=root, r_begin=a, r_end=b, send_mode=0)
    assert np.array_equal(got, want)
    assert gpu_digest(p, root, a, b) == oracle.digest(p, root, a, b, send_mode=0)


def test_output_layouts_agree():
    p, root, a, b = 100003, 77, 1000, 1000 + 64 * 7 + 13
    q = lib.bcast_q(p)
    want = oracle.schedules(p, root=root, r_begin=a, r_end=b)
    n = b - a
    # two separate [ranks][q] tables
    recv = torch.zeros((n, q), dtype=torch.int32, device=DEV)
    send = torch.zeros((n, q), dtype=torch.int32, device=DEV)
    lib.bcast_schedules(p, root, a, b, recv, send, q)
    torch.cuda.synchronize()
    assert np.array_equal(recv.cpu().numpy(), want[:, :q])
    assert np.array_equal(send.cpu().numpy(), want[:, q:])
    # padded rows: ld = 2q + 5, untouched padding
    ld = 2 * q + 5
    tab = torch.full((n, ld), 1234, dtype=torch.int32, device=DEV)
    lib.bcast_schedules(p, root, a, b, tab, tab, ld, send_offset=q)
    torch.cuda.synchronize()
    got = tab.cpu().numpy()
    assert np.array_equal(got[:, :2 * q], want) and (got[:, 2 * q:] == 1234).all()
    # a table that does not start on a 16-byte boundary
    flat = torch.zeros(n * 2 * q + 1, dtype=torch.int32, device=DEV)
    view = flat[1:]
    lib.bcast_schedules(p, root, a, b, view, view, 2 * q, send_offset=q)
    torch.cuda.synchronize()
    assert np.array_equal(flat.cpu().numpy()[1:].reshape(n, 2 * q), want)


@pytest.mark.parametrize("p,root,a,b", [
    (4000037, 123457, 1000, 2200000),     # few violations per rank, long runs of tiles
    (2097153, 0, 0, 2097153),             # p = 2^21 + 1: more than one violation per rank
    (2097153, 2097152, 5, 2097100),
])
def test_long_runs_with_deferred_violations(p, root, a, b):
    # Tables long enough that a wavefront works through several tiles and fills
    # in the violations of Algorithm 6 later, in batches, in all three layouts.
    q = lib.bcast_q(p)
    n = b - a
    want = oracle.schedules(p, root=root, r_begin=a, r_end=b, send_mode=1)
    t = torch.full((n, 2 * q), 99, dtype=torch.int32, device=DEV)
    lib.bcast_schedules(p, root, a, b, t, t, 2 * q, send_offset=q)
    torch.cuda.synchronize()
    assert np.array_equal(t.cpu().numpy(), want)
    del t
    recv = torch.full((n, q), 99, dtype=torch.int32, device=DEV)
    send = torch.full((n, q), 99, dtype=torch.int32, device=DEV)
    lib.bcast_schedules(p, root, a, b, recv, send, q)
    torch.cuda.synchronize()
    assert np.array_equal(recv.cpu().numpy(), want[:, :q])
    assert np.array_equal(send.cpu().numpy(), want[:, q:])
    del recv, send
    ld = 2 * q + 3
    tab = torch.full((n, ld), 1234, dtype=torch.int32, device=DEV)
    lib.bcast_schedules(p, root, a, b, tab, tab, ld, send_offset=q)
    torch.cuda.synchronize()
    got = tab.cpu().numpy()
    assert np.array_equal(got[:, :2 * q], want) and (got[:, 2 * q:] == 1234).all()
    # the same ranks through the digest and the edge check (whole rows deferred there)
    assert gpu_digest(p, root, a, b) == oracle.digest(p, root, a, b, send_mode=1)
    assert gpu_edgecheck(p, root, a, b) == oracle.edgecheck(p, root, a, b, send_mode=1)
    # send by definition on a seeded sample
    ranks = np.sort(workloads.streamed_sample_ranks(512, seed=11, p=n).astype(np.int64)) + a
    assert np.array_equal(want[ranks - a], oracle.schedules_ranks(p, root, ranks.astype(np.uint32), send_mode=0))


def test_seeded_long_ranges_at_odd_offsets():
    # seeded p of every size class, random roots, ranges of 1.2 to 2.6 million ranks that start and
    # end anywhere (so tiles straddle the root, runs start mid-way through a power of two, and
    # the records carried from tile to tile see all alignments): table, digest and edge check
    rng = np.random.default_rng(20240718)
    for case in range(6):
        bits = int(rng.integers(22, 32))
        p = int(rng.integers(2 ** (bits - 1), min(2 ** bits, 2 ** 31 - 1)))
        if case == 0:
            p = 2 ** 23 - 1                      # the variant without violations
        if case == 1:
            p = 2 ** 24                          # a power of two, root in the middle of the range
        root = int(rng.integers(0, p))
        n = int(rng.integers(1_200_000, 2_600_000))
        n = min(n, p)
        a = int(rng.integers(0, p - n + 1))
        if case in (1, 2):                       # put the root inside the range
            a = max(0, min(p - n, root - n // 3))
        b = a + n
        q = lib.bcast_q(p)
        want = oracle.schedules(p, root=root, r_begin=a, r_end=b, send_mode=1)
        t = torch.full((n, 2 * q), 99, dtype=torch.int32, device=DEV)
        lib.bcast_schedules(p, root, a, b, t, t, 2 * q, send_offset=q)
        torch.cuda.synchronize()
        got = t.cpu().numpy()
        del t
        assert np.array_equal(got, want), (p, root, a, b)
        assert gpu_digest(p, root, a, b) == oracle.digest(p, root, a, b, send_mode=1), (p, root, a, b)
        assert gpu_edgecheck(p, root, a, b) == oracle.edgecheck(p, root, a, b, send_mode=1)
        ranks = np.sort(workloads.streamed_sample_ranks(256, seed=case, p=n).astype(np.int64)) + a
        assert np.array_equal(want[ranks - a],
                              oracle.schedules_ranks(p, root, ranks.astype(np.uint32), send_mode=0))


@pytest.mark.parametrize("p,root,a,n", [
    (2**31 - 1, 123456789, 123456789 - 1_500_000, 3_000_000),     # the root in the middle of the range
    (2**31 - 1, 2**31 - 2, 2**31 - 1 - 2_500_000, 2_500_000),     # the last ranks; root = p - 1
    (2**31 - 1, 1, 0, 2_000_001),                                  # the first ranks; ranks 0, 1, 2 special
    (2**30, 2**29 + 7, 2**29 - 1_000_000, 2_100_000),             # a power of two
])
def test_streamed_ranges_of_the_largest_instances(p, root, a, n):
    # digests and edge sums of long ranges where wavefronts carry their records across the root
    b = a + n
    assert gpu_digest(p, root, a, b) == oracle.digest(p, root, a, b, send_mode=1)
    assert gpu_edgecheck(p, root, a, b) == oracle.edgecheck(p, root, a, b, send_mode=1)
    q = lib.bcast_q(p)
    lo, hi = a + n // 2 - 70_000, a + n // 2 + 70_000             # a table of the middle part
    t = torch.full((hi - lo, 2 * q), 99, dtype=torch.int32, device=DEV)
    lib.bcast_schedules(p, root, lo, hi, t, t, 2 * q, send_offset=q)
    torch.cuda.synchronize()
    assert np.array_equal(t.cpu().numpy(), oracle.schedules(p, root=root, r_begin=lo, r_end=hi, send_mode=1))


def test_argument_errors():
    t = torch.zeros((16, 40), dtype=torch.int32, device=DEV)
    with pytest.raises(lib.BcastError) as e:
        lib.bcast_schedules(0, 0, 0, 0, t, t, 40)
    assert e.value.code == lib.BCAST_EINVAL
    for args in [(2**31, 0, 0, 1), (100, 100, 0, 10), (100, 0, 11, 10), (100, 0, 0, 101)]:
        with pytest.raises(lib.BcastError):
            lib.bcast_schedules(*args, t, t, 14, send_offset=7)
    with pytest.raises(lib.BcastError):       # ld < q
        lib.bcast_schedules(100, 0, 0, 10, t, t, 6, send_offset=7)
    with pytest.raises(lib.BcastError):       # rows overlap
        lib.bcast_schedules(100, 0, 0, 10, t, t, 14, send_offset=3)
    with pytest.raises(lib.BcastError):
        lib.bcast_q(0)
    ws = torch.zeros(16, dtype=torch.uint8, device=DEV)
    vd = torch.zeros(VERDICT_BYTES, dtype=torch.uint8, device=DEV)
    with pytest.raises(lib.BcastError) as e:
        lib.bcast_simulate(100, 10, [0], None, ws, vd)
    assert e.value.code == lib.BCAST_ENOMEM
    with pytest.raises(lib.BcastError):
        lib.bcast_simulate(100, 10, [100], None, ws, vd)
    assert lib.bcast_simulate_workspace(0, 1, 1) == 0
    assert lib.bcast_simulate_workspace(100, 2**28 + 1, 1) == 0      # more blocks than BCAST_MAX_N
    with pytest.raises(lib.BcastError) as e:
        lib.bcast_simulate(100, 2**28 + 1, [0], None, ws, vd)
    assert e.value.code == lib.BCAST_EINVAL
    torch.cuda.synchronize()


# ------------------------------------------------- workload 2: one table --

def test_workload2_materialised_instance():
    p = workloads.MATERIALISED_P
    got = gpu_table(p)
    want = oracle.schedules(p, send_mode=1)
    assert got.shape == (p, 40)
    assert np.array_equal(got, want)
    # send by definition on a seeded sample of ranks
    ranks = workloads.streamed_sample_ranks(4096, seed=7, p=p)
    assert np.array_equal(got[ranks], oracle.schedules_ranks(p, 0, ranks, send_mode=0))


# ---------------------------------------------- workload 3: huge streamed --

def streamed_golden():
    """The oracle's digests of the 32 chunks (tests/golden/make_digest_golden.py --streamed)."""
    with open(os.path.join(GOLDEN, "streamed_chunk_digests.json")) as fh:
        gold = json.load(fh)
    assert gold["p"] == workloads.STREAMED_P and gold["chunk"] == workloads.STREAMED_CHUNK
    return gold


def test_workload3_streamed_digests():
    p = workloads.STREAMED_P
    chunks = workloads.streamed_chunks()
    assert len(chunks) == 32
    gold = streamed_golden()
    whole = 0
    per_chunk = []
    for i, (a, b) in enumerate(chunks):
        dg, fl = gpu_digest(p, 0, a, b)
        assert fl == 0, (a, b, fl)
        want = gold["chunks"][i]
        assert (want["r_begin"], want["r_end"]) == (a, b)
        assert f"{dg:016x}" == want["digest"] and want["flags"] == 0, (i, a, b)
        per_chunk.append(dg)
        whole ^= dg
    assert f"{whole:016x}" == gold["digest"]
    # order-free digest: any other split of a chunk gives the same value
    a, b = chunks[5]
    cut = a + 12345677
    assert gpu_digest(p, 0, a, cut)[0] ^ gpu_digest(p, 0, cut, b)[0] == per_chunk[5]
    a, b = chunks[31]
    assert b == p
    # windows the oracle recomputes: start, a chunk boundary, the very end
    w = 1 << 21
    for lo, hi in [(0, w), (chunks[7][0] - w // 2, chunks[7][0] + w // 2), (p - w, p)]:
        assert gpu_digest(p, 0, lo, hi) == oracle.digest(p, 0, lo, hi, send_mode=1)
    # one call over the whole range equals the XOR of the chunks
    assert gpu_digest(p, 0, 0, p) == (whole, 0)


@pytest.mark.parametrize("chunk", [0, 17, 31])
def test_workload3_whole_chunks_against_the_oracle_live(chunk):
    # Launches of the size and shape the benchmark times (2^26 ranks: every wavefront works
    # through a run of several tiles and carries its records from tile to tile), digest and
    # edge sums against the oracle computed here and now: the first chunk (with the root), one
    # from the middle, and the last one, which is a rank short.
    p = workloads.STREAMED_P
    a, b = workloads.streamed_chunks()[chunk]
    assert gpu_digest(p, 0, a, b) == oracle.digest(p, 0, a, b, send_mode=1)
    assert gpu_edgecheck(p, 0, a, b) == oracle.edgecheck(p, 0, a, b, send_mode=1)


@pytest.mark.parametrize("p,root,a,n", [
    (2**30, 2**29 + 7, 2**29 - 2**23 + 11, 2**24 + 5),          # a power of two, the root inside
    (2**27 - 1, 77_000_001, 77_000_001 - 9_000_000, 2**24 + 100_003),   # 2^q - 1, the root inside
    (2**31 - 1, 2**31 - 2, 2**31 - 1 - 2**24 - 63, 2**24 + 63),  # the last ranks, root = p - 1
])
def test_long_launches_without_violations_against_the_oracle(p, root, a, n):
    # p = 2^q and 2^q - 1 take the kernels whose wavefronts work alone; only launches of
    # several million ranks give them runs of three and more tiles, where the records are used
    b = a + n
    assert b <= p
    assert gpu_digest(p, root, a, b) == oracle.digest(p, root, a, b, send_mode=1)
    assert gpu_edgecheck(p, root, a, b) == oracle.edgecheck(p, root, a, b, send_mode=1)


@pytest.mark.parametrize("p,root,a", [
    (2**31 - 1, 0, 0),
    (2**31 - 1, 1_500_000_000, 1_500_000_000 - 5_000_000),
    (2**30, 3, 2**29),
])
def test_long_tables_without_violations_slice_by_slice(p, root, a):
    # one bcast_schedules launch of 2^24 + 77 ranks (4.2 GB at q = 31), compared with the
    # oracle in slices of 2^21 ranks so that the host never holds the whole table
    n = 2**24 + 77
    q = lib.bcast_q(p)
    t = torch.full((n, 2 * q), 99, dtype=torch.int32, device=DEV)
    lib.bcast_schedules(p, root, a, a + n, t, t, 2 * q, send_offset=q)
    torch.cuda.synchronize()
    step = 2**21
    for lo in range(0, n, step):
        hi = min(lo + step, n)
        want = oracle.schedules(p, root=root, r_begin=a + lo, r_end=a + hi, send_mode=1)
        assert np.array_equal(t[lo:hi].cpu().numpy(), want), (p, root, a + lo, a + hi)
    del t


def test_workload3_seeded_rank_sample_against_definition():
    p = workloads.STREAMED_P
    ranks = workloads.streamed_sample_ranks(2**20, seed=42)
    pa = np.array([p], dtype=np.uint32)
    out, rej, _ = gpu_batched(pa, np.array([0], dtype=np.uint32), ranks[None, :])
    assert rej == 0
    got = out.cpu().numpy().reshape(ranks.size, 62)
    want = oracle.schedules_ranks(p, 0, ranks, send_mode=1)
    assert np.array_equal(got, want)
    sub = ranks[:: 16]                      # send by definition (q recv searches per rank)
    assert np.array_equal(got[:: 16], oracle.schedules_ranks(p, 0, sub, send_mode=0))


def test_edge_check_matches_oracle_and_holds_on_whole_instances():
    for p, root, a, b in [(1000, 0, 0, 1000), (1000, 77, 100, 901), (65537, 12345, 0, 65537),
                          (1, 0, 0, 1), (2, 1, 0, 2), (1000003, 5, 400000, 600001),
                          (2**31 - 1, 0, 2**31 - 1 - 2**20, 2**31 - 1), (2**30 + 1, 9, 0, 2**20)]:
        assert gpu_edgecheck(p, root, a, b) == oracle.edgecheck(p, root, a, b), (p, root, a, b)
    for p, root in [(1000, 0), (65537, 12345), (1000003, 0), (2**24 + 1, 3)]:
        xr, xs = gpu_edgecheck(p, root, 0, p)
        assert xr == xs, (p, root)
        xr, xs = gpu_edgecheck(p, root, 0, p - 1)
        assert xr != xs


def test_workload3_edge_check_of_the_whole_instance():
    # Conditions 1 and 2 on all 31 * (2^31 - 1) edges, chunk by chunk
    p = workloads.STREAMED_P
    gold = streamed_golden()
    xr = xs = 0
    seen = []
    for a, b in workloads.streamed_chunks():
        r, s = gpu_edgecheck(p, 0, a, b)
        xr ^= r
        xs ^= s
        want = gold["chunks"][len(seen)]
        assert (f"{r:016x}", f"{s:016x}") == (want["edge_recv"], want["edge_send"]), (a, b)
        seen.append((a, b))
    assert xr == xs
    assert (f"{xr:016x}", f"{xs:016x}") == (gold["edge_recv"], gold["edge_send"])
    w = 1 << 21
    assert gpu_edgecheck(p, 0, 2**30 - w, 2**30 + w) == oracle.edgecheck(p, 0, 2**30 - w, 2**30 + w)


# ------------------------------------------- workload 4: batched instances --

def check_batched(first, n_inst, m, check_every=1):
    p, root, ranks = workloads.batched_instances(n_inst, m, seed=42, first=first)
    out, rej, row_off = gpu_batched(p, root, ranks)
    assert rej == 0
    for i in range(0, n_inst, check_every):
        q = oracle.q_of(int(p[i]))
        got = out[int(row_off[i]): int(row_off[i + 1])].cpu().numpy().reshape(m, 2 * q)
        want = oracle.schedules_ranks(int(p[i]), int(root[i]), ranks[i], send_mode=1)
        assert np.array_equal(got, want), (i, int(p[i]), int(root[i]))
    return out


def test_workload4_batched_small():
    check_batched(0, 300, 200)                 # ragged tiles: 200 = 3*64 + 8
    check_batched(1000, 64, 4096, check_every=4)
    # wavefronts take 16 tiles of an instance in a row: 68 tiles are four such batches and one of
    # four tiles, the last of them ragged; 17 tiles are one batch and a single tile
    check_batched(2000, 40, 4096 + 200, check_every=2)
    check_batched(3000, 48, 1024 + 8, check_every=2)


def test_workload4_batched_rejects_bad_input():
    p = np.array([100, 0, 50, 64], dtype=np.uint32)
    root = np.array([0, 0, 50, 3], dtype=np.uint32)        # instance 2: root >= p
    ranks = np.array([[1, 2, 100, 4], [0, 0, 0, 0], [1, 2, 3, 4], [5, 6, 7, 63]], dtype=np.uint32)
    m = 4
    row_off = workloads.batched_row_offsets(np.array([100, 1, 50, 64], dtype=np.uint32), m)
    out, rej, _ = gpu_batched(p, root, ranks, row_off)
    assert rej == 3                     # rank 100 of instance 0, instances 1 and 2
    got = out.cpu().numpy()
    q0 = 7
    rows0 = got[: m * 2 * q0].reshape(m, 2 * q0)
    want0 = oracle.schedules_ranks(100, 0, np.array([1, 2, 4], dtype=np.uint32))
    assert np.array_equal(rows0[[0, 1, 3]], want0)
    assert (rows0[2] == np.iinfo(np.int32).min).all()
    a, b = int(row_off[1]), int(row_off[3])
    assert (got[a:b] == 77).all()       # rejected instances write nothing
    want3 = oracle.schedules_ranks(64, 3, ranks[3])
    assert np.array_equal(got[int(row_off[3]):].reshape(m, 12), want3)


def test_workload4_batched_full_size():
    # 65,536 instances x 4,096 ranks, about 35 GB of schedules in HBM, all of them
    # compared with the oracle.
    n_inst, m = 65536, 4096
    p, root, _ = workloads.batched_instances(n_inst, m, seed=42, with_ranks=False)
    row_off = workloads.batched_row_offsets(p, m)
    total = int(row_off[-1])
    assert total * 4 > 30e9
    out = torch.empty(total, dtype=torch.int32, device=DEV)
    ranks_d = torch.empty((n_inst, m), dtype=torch.int32, device=DEV)
    step = 4096
    for first in range(0, n_inst, step):
        _, _, ranks = workloads.batched_instances(step, m, seed=42, first=first)
        ranks_d[first:first + step] = torch.from_numpy(ranks.view(np.int32)).to(DEV)
    rej = torch.zeros(1, dtype=torch.int32, device=DEV)
    d = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a).view(dt)).to(DEV)  # noqa: E731
    lib.bcast_schedules_batched(n_inst, d(p, np.int32), d(root, np.int32), ranks_d, m,
                                d(row_off, np.int64), out, rej)
    torch.cuda.synchronize()
    assert int(rej.item()) == 0
    # every row of every instance, element by element: the table comes back in blocks of 2,048
    # instances (about 1.1 GB) and the oracle recomputes each instance's 4,096 rows
    block = 2048
    for first in range(0, n_inst, block):
        got_block = out[int(row_off[first]): int(row_off[first + block])].cpu().numpy()
        _, _, ranks = workloads.batched_instances(block, m, seed=42, first=first)
        base = int(row_off[first])
        for i in range(first, first + block):
            q = oracle.q_of(int(p[i]))
            got = got_block[int(row_off[i]) - base: int(row_off[i + 1]) - base].reshape(m, 2 * q)
            want = oracle.schedules_ranks(int(p[i]), int(root[i]), ranks[i - first], send_mode=1)
            assert np.array_equal(got, want), (i, int(p[i]), int(root[i]))
        print(f"batched: instances [{first}, {first + block}) equal the oracle's", flush=True)


# ------------------------------------------------ workload 5: simulation --

def test_workload5_simulation_single_root():
    p, n, root = workloads.SIMULATION_P, workloads.SIMULATION_N, workloads.SIMULATION_ROOT
    got = gpu_simulate(p, n, [root])[0]
    want = oracle.simulate(p, n, root)
    assert got == want
    assert got["flags"] == 0 and got["rounds"] == n - 1 + 17 == 272


def test_workload5_simulation_64_roots():
    p, n = workloads.SIMULATION_P, workloads.SIMULATION_N
    roots = workloads.simulation_roots(64, seed=42)
    got = gpu_simulate(p, n, roots)
    assert len(got) == 64
    for j, vd in enumerate(got):
        assert vd["flags"] == 0 and vd["rounds"] == 272 and vd["first_bad"] == oracle.U64_MAX
        if j % 16 == 0:
            assert vd == oracle.simulate(p, n, roots[j]), roots[j]


def test_simulation_reports_planted_mistakes_like_the_oracle():
    # mistakes are planted into a schedule table on the host; both sides then
    # replay the same table
    p, n = 1000, 37
    q = oracle.q_of(p)
    roots = [0, 123, 999]
    rng = np.random.default_rng(11)
    tables = []
    for root in roots:
        tab = oracle.schedules(p, root=root)
        for _ in range(5):
            r, c = int(rng.integers(0, p)), int(rng.integers(0, 2 * q))
            tab[r, c] = int(rng.integers(-q, q))
        tables.append(tab)
    tables[2][5, 3] = 10**9
    tables[2][6, q + 2] = -(2**31)
    sched = torch.from_numpy(np.stack(tables)).to(DEV)
    got = gpu_simulate(p, n, roots, sched)
    for j, root in enumerate(roots):
        want = oracle.simulate(p, n, root, tables[j])
        assert got[j] == want, (root, got[j], want)
        assert want["flags"] != 0
    # an explicit correct table passes
    good = torch.from_numpy(np.stack([oracle.schedules(p, root=r) for r in roots])).to(DEV)
    for vd in gpu_simulate(p, n, roots, good):
        assert vd["flags"] == 0


@pytest.mark.parametrize("p", [2, 3, 17, 100, 1000, 4096, 65537])
@pytest.mark.parametrize("n", [1, 2, 31, 64, 100])
def test_simulation_block_counts(p, n):
    root = p // 3
    assert gpu_simulate(p, n, [root])[0] == oracle.simulate(p, n, root)


@pytest.mark.parametrize("p,n", [
    (1000, 32745), (1000, 32746),      # the last n whose entries are staged as 16-bit halves, and the first beyond
    (100, 40000), (17, 100003),
])
def test_simulation_many_blocks(p, n):
    # both ways of staging the entries, with planted mistakes and entries far out of range
    q = oracle.q_of(p)
    root = p // 3
    assert gpu_simulate(p, n, [root])[0] == oracle.simulate(p, n, root)
    assert gpu_simulate(p, n, [root], reduce=True)[0] == oracle.simulate_reduce(p, n, root)
    rng = np.random.default_rng(p + n)
    tab = oracle.schedules(p, root=root)
    for _ in range(4):
        r, c = int(rng.integers(0, p)), int(rng.integers(0, 2 * q))
        tab[r, c] = int(rng.integers(-q, q))
    tab[5, 1] = 2**31 - 1
    tab[6, q + 1] = -(2**31)
    tab[7, 0] = n + 2 * q + 2           # exactly the clamping bound, and one off on either side
    tab[8, q] = n + 2 * q + 1
    tab[9, 2] = -(n + 2 * q + 3)
    sched = torch.from_numpy(tab[None]).to(DEV)
    want = oracle.simulate(p, n, root, tab)
    assert want["flags"] != 0
    assert gpu_simulate(p, n, [root], sched)[0] == want
    assert gpu_simulate(p, n, [root], sched, reduce=True)[0] == oracle.simulate_reduce(p, n, root, tab)


# ------------------------------------------------ reduction by reversal ----

@pytest.mark.parametrize("p", [1, 2, 3, 17, 100, 1000, 4096, 65537])
@pytest.mark.parametrize("n", [1, 2, 31, 64, 100])
def test_reduction_replay_block_counts(p, n):
    root = p // 3
    got = gpu_simulate(p, n, [root], reduce=True)[0]
    assert got == oracle.simulate_reduce(p, n, root)
    assert got["flags"] == 0


def test_reduction_replay_workload5_and_planted_mistakes():
    p, n = workloads.SIMULATION_P, workloads.SIMULATION_N
    roots = workloads.simulation_roots(64, seed=42)
    got = gpu_simulate(p, n, roots, reduce=True)
    for j, vd in enumerate(got):
        assert vd["flags"] == 0 and vd["rounds"] == 272
        if j % 32 == 0:
            assert vd == oracle.simulate_reduce(p, n, roots[j])
    p, n = 1000, 37
    q = oracle.q_of(p)
    roots = [0, 123, 999]
    rng = np.random.default_rng(12)
    tables = []
    for root in roots:
        tab = oracle.schedules(p, root=root)
        for _ in range(5):
            r, c = int(rng.integers(0, p)), int(rng.integers(0, 2 * q))
            tab[r, c] = int(rng.integers(-q, q))
        tables.append(tab)
    tables[1][7, 2] = 10**9
    sched = torch.from_numpy(np.stack(tables)).to(DEV)
    got = gpu_simulate(p, n, roots, sched, reduce=True)
    for j, root in enumerate(roots):
        want = oracle.simulate_reduce(p, n, root, tables[j])
        assert got[j] == want and want["flags"] != 0, (root, got[j], want)


# ------------------------------------------------- doubling (even p) -------

@pytest.mark.parametrize("p", [1, 2, 3, 9, 17, 64, 100, 1000, 4097, 65537, 500002, 2**20 - 1])
def test_doubling_equals_the_schedules_of_2p(p):
    # Observations 1 and 5 on the GPU: table(2p) from table(p), against the oracle's table(2p)
    q = lib.bcast_q(p)
    src = torch.from_numpy(oracle.schedules(p)).to(DEV) if q else None
    dst = torch.full((2 * p, 2 * (q + 1)), 55, dtype=torch.int32, device=DEV)
    lib.bcast_schedules_double(p, src, dst)
    torch.cuda.synchronize()
    assert np.array_equal(dst.cpu().numpy(), oracle.schedules(2 * p))


def test_doubling_chain_from_the_gpu_table_and_errors():
    # 125,001 -> 250,002 -> 500,004 -> 1,000,008 from a table computed on the GPU
    p = 125001
    cur = torch.from_numpy(gpu_table(p)).to(DEV)
    for _ in range(3):
        q = lib.bcast_q(p)
        nxt = torch.empty((2 * p, 2 * (q + 1)), dtype=torch.int32, device=DEV)
        lib.bcast_schedules_double(p, cur, nxt)
        p, cur = 2 * p, nxt
    torch.cuda.synchronize()
    assert p == 1000008
    assert np.array_equal(cur.cpu().numpy(), oracle.schedules(p))
    with pytest.raises(lib.BcastError):
        lib.bcast_schedules_double(2**30, cur, cur)
    with pytest.raises(lib.BcastError):
        lib.bcast_schedules_double(1000008, cur, cur)          # overlap


def test_schedules_by_doubling_equal_the_oracle():
    # table(p) for p = m 2^j as table(m) doubled j times, against the oracle's table(p):
    # powers of two (m = 1), twice an odd number, 3 * 2^20, workload 2's neighbour, odd p
    for p in [1, 2, 4, 6, 12, 18, 64, 1000, 1001, 4096, 65536, 131072, 262146, 999_998, 1_000_004, 3 * 2**20, 5 * 2**18, 2**22,
              2**24]:
        q = lib.bcast_q(p)
        ws = torch.full((lib.bcast_schedules_doubling_workspace(p),), 0x5A, dtype=torch.uint8, device=DEV)
        out = torch.full((p, 2 * q), 77, dtype=torch.int32, device=DEV)
        lib.bcast_schedules_doubling(p, out, ws)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), oracle.schedules(p)), p
    p = 1_000_004
    q = lib.bcast_q(p)
    out = torch.empty((p, 2 * q), dtype=torch.int32, device=DEV)
    small = torch.empty(lib.bcast_schedules_doubling_workspace(p) - 1, dtype=torch.uint8, device=DEV)
    with pytest.raises(lib.BcastError) as e:
        lib.bcast_schedules_doubling(p, out, small)
    assert e.value.code == lib.BCAST_ENOMEM
    with pytest.raises(lib.BcastError):               # the table inside the workspace
        big = torch.empty(p * 2 * q * 4 + lib.bcast_schedules_doubling_workspace(p), dtype=torch.uint8, device=DEV)
        lib.bcast_schedules_doubling(p, big[: p * 2 * q * 4].view(torch.int32), big)
    torch.cuda.synchronize()


def test_baseblock_listing_in_linear_time():
    # the listing of Lemma 4's proof on the GPU against Algorithm 3 of the oracle: every rank of
    # every p <= 4096 (the baseblock is the one non-negative entry of the receive row, which the
    # oracle takes from Algorithm 3; the root has q), direct calls of Algorithm 3 on samples,
    # and all ranks of three large p
    def want_list(p):
        q = oracle.q_of(p)
        b = oracle.schedules(p)[:, :q].max(axis=1, initial=-1).astype(np.int64)
        b[0] = q
        return b
    rng = np.random.default_rng(4)
    for p in list(range(1, 4097)) + [65537, 1_000_003, 2**22, 3 * 2**20 + 1]:
        lst = torch.full((p + 3,), 200, dtype=torch.uint8, device=DEV)
        view = lst[:p] if p % 2 else lst[3:3 + p]          # also from an address that is not aligned
        lib.bcast_baseblocks(p, view)
        torch.cuda.synchronize()
        got = view.cpu().numpy().astype(np.int64)
        assert np.array_equal(got, want_list(p)), p
        for r in {0, min(1, p - 1), p - 1, p // 2} | {int(x) for x in rng.integers(0, p, size=4)}:
            assert got[r] == oracle.baseblock(p, r), (p, r)
        rest = (lst[p:] if p % 2 else lst[:3]).cpu().numpy()
        assert (rest == 200).all()                          # nothing written outside the list
    # p = 2^31 - 1: two gigabytes of baseblocks; powers of two all the way, so b_r is the
    # position of the lowest set bit of r, and samples against Algorithm 3
    p = 2**31 - 1
    lst = torch.empty(p, dtype=torch.uint8, device=DEV)
    lib.bcast_baseblocks(p, lst)
    torch.cuda.synchronize()
    for lo in (0, 2**30 - 5000, p - 2**20):
        got = lst[lo: lo + 2**20].cpu().numpy().astype(np.int64)
        r = np.arange(lo, lo + 2**20, dtype=np.int64)
        want = np.zeros_like(r)
        rr = r.copy()
        rr[rr == 0] = 1
        low = rr & -rr
        want = np.log2(low).astype(np.int64)
        if lo == 0:
            want[0] = 31
        assert np.array_equal(got, want), lo
        for x in rng.integers(lo, lo + 2**20, size=8):
            assert got[int(x) - lo] == oracle.baseblock(p, int(x))


# --------------------------------------- the calls with a workspace (table of deep entries) --

def ws_table(p, root, a, b, ws=None):
    q = lib.bcast_q(p)
    if ws is None:
        ws = torch.full((lib.bcast_schedules_workspace(p),), 0xEE, dtype=torch.uint8, device=DEV)
    t = torch.full((max(b - a, 0), 2 * q), 99, dtype=torch.int32, device=DEV)
    lib.bcast_schedules_ws(p, root, a, b, t, t, 2 * q, ws, send_offset=q)
    torch.cuda.synchronize()
    return t


def ws_digest_and_edges(p, root, a, b, ws):
    dg = torch.full((1,), -1, dtype=torch.int64, device=DEV)
    fl = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    x = torch.full((2,), -1, dtype=torch.int64, device=DEV)
    lib.bcast_schedules_digest_ws(p, root, a, b, dg, fl, ws)
    lib.bcast_schedules_edgecheck_ws(p, root, a, b, x, ws)
    torch.cuda.synchronize()
    xr, xs = (int(t) & oracle.U64_MAX for t in x.cpu().tolist())
    return (int(dg.item()) & oracle.U64_MAX, int(fl.item()) & 0xFFFFFFFF), (xr, xs)


@pytest.mark.parametrize("p,root,a,n", [
    (4000037, 123457, 1000, 2_400_000),       # few violations per rank
    (2**22 + 1, 0, 0, 2**22 + 1),             # more than one violation per rank, all ranks
    (2**22 + 1, 2**22, 5, 2**22 - 100),
    (2**23 - 1, 3, 0, 2**23 - 1),             # the kernels whose wavefronts work alone
    (2**24, 2**23 + 5, 2**23 - 2_000_000, 4_000_001),
    (3 * 2**20 + 1, 77, 0, 3 * 2**20 + 1),    # the smallest skip above the deep levels is odd
    (1000003, 0, 0, 1000003), (20000, 1, 0, 20000), (100, 3, 0, 100), (1, 0, 0, 1),   # below the thresholds
    # fewer than 2^20 ranks: the entries left open go to a segment of the workspace per wavefront; with more
    # than one violation per rank some segments fill up and their wavefronts search for the rest themselves
    (2**19 + 1, 5, 0, 2**19 + 1), (2**20 - 3, 0, 7, 2**20 - 20), (786433, 9, 100000, 600000), (2**17 + 1, 2**16, 0, 2**17 + 1),
])
def test_calls_with_workspace_equal_the_oracle(p, root, a, n):
    b = a + n
    ws = torch.full((lib.bcast_schedules_workspace(p),), 0xEE, dtype=torch.uint8, device=DEV)
    want = oracle.schedules(p, root=root, r_begin=a, r_end=b, send_mode=1)
    assert np.array_equal(ws_table(p, root, a, b, ws).cpu().numpy(), want)
    dg, xs = ws_digest_and_edges(p, root, a, b, ws)
    assert dg == oracle.digest(p, root, a, b, send_mode=1)
    assert xs == oracle.edgecheck(p, root, a, b, send_mode=1)
    # separate tables, and a workspace that is reused without being cleared
    q = lib.bcast_q(p)
    recv = torch.full((n, max(q, 1)), 99, dtype=torch.int32, device=DEV)
    send = torch.full((n, max(q, 1)), 99, dtype=torch.int32, device=DEV)
    if q:
        lib.bcast_schedules_ws(p, root, a, b, recv, send, q, ws)
        torch.cuda.synchronize()
        assert np.array_equal(recv.cpu().numpy(), want[:, :q]) and np.array_equal(send.cpu().numpy(), want[:, q:])


@pytest.mark.parametrize("q", list(range(2, 32)))
def test_digest_and_edge_check_for_every_number_of_rounds(q):
    """Every q: the row layout of the digest kernels, the words they read rows by and the tail of
    the hash change with q (q mod 4, 2q mod 20); p = 2^q - 1, 2^q and an odd p with violations."""
    odd = (1 << (q - 1)) + 1 + 2 * ((q * 2654435761) % max(1, 1 << max(q - 3, 0)))
    for p in (2**q - 1, 2**q, odd):
        if p > workloads.STREAMED_P:                   # 2^31 is past the largest p of the library
            continue
        assert lib.bcast_q(p) == q, (p, q)
        n = min(p, 150_000)
        root = (p * 5) // 7
        a = max(0, min(root - n // 3, p - n))          # the root inside the range
        assert gpu_digest(p, root, a, a + n) == oracle.digest(p, root, a, a + n, send_mode=1), (p, "digest")
        assert gpu_edgecheck(p, root, a, a + n) == oracle.edgecheck(p, root, a, a + n, send_mode=1), (p, "edges")
        if p >= 2**21 + 70_000:                        # with the table of deep entries and records in use
            n = 2**21 + 4321
            a = max(0, min(root - n // 3, p - n))
            ws = torch.full((lib.bcast_schedules_workspace(p),), 0xEE, dtype=torch.uint8, device=DEV)
            dg, xs = ws_digest_and_edges(p, root, a, a + n, ws)
            assert dg == oracle.digest(p, root, a, a + n, send_mode=1), (p, "digest, workspace")
            assert xs == oracle.edgecheck(p, root, a, a + n, send_mode=1), (p, "edges, workspace")


@pytest.mark.parametrize("q", list(range(25, 32)))
def test_long_runs_for_every_large_number_of_rounds(q):
    """Launches long enough for every wavefront to work through a dozen tiles, so that the records a
    wavefront carries from tile to tile (top levels, lockstep stretch in two parts) and the tables in
    the workspace are all in use, for each q that has that many ranks: digest, flags and edge check
    against the oracle, p = 2^q - 1 and an odd p with violations, the root inside the range."""
    n = 2**24 + 2**22 + 12345
    odd = (1 << (q - 1)) + 1 + 2 * ((q * 2654435761) % (1 << (q - 3)))
    for p in (2**q - 1, odd):
        assert lib.bcast_q(p) == q and p > n
        root = (p * 3) // 5
        a = max(0, min(root - n // 2, p - n))
        ws = torch.full((lib.bcast_schedules_workspace(p),), 0xEE, dtype=torch.uint8, device=DEV)
        dg, xs = ws_digest_and_edges(p, root, a, a + n, ws)
        assert dg == oracle.digest(p, root, a, a + n, send_mode=1), (p, "digest")
        assert xs == oracle.edgecheck(p, root, a, a + n, send_mode=1), (p, "edges")
        assert gpu_digest(p, root, a, a + n) == dg, (p, "digest without a workspace")


def test_calls_with_workspace_on_the_streamed_instance():
    p = workloads.STREAMED_P
    gold = streamed_golden()
    ws = torch.empty(lib.bcast_schedules_workspace(p), dtype=torch.uint8, device=DEV)
    whole = 0
    for i, (a, b) in enumerate(workloads.streamed_chunks()):
        dg = torch.zeros(1, dtype=torch.int64, device=DEV)
        fl = torch.ones(1, dtype=torch.int32, device=DEV)
        lib.bcast_schedules_digest_ws(p, 0, a, b, dg, fl, ws)
        torch.cuda.synchronize()
        got = int(dg.item()) & oracle.U64_MAX
        assert f"{got:016x}" == gold["chunks"][i]["digest"] and int(fl.item()) == 0, i
        whole ^= got
    assert f"{whole:016x}" == gold["digest"]
    # whole chunks live, with the edge sums, a root inside the range, and a long table by slices
    for root, a, n in [(0, 17 * 2**26, 2**26), (1_500_000_000, 1_500_000_000 - 30_000_000, 2**26 + 12345)]:
        dg, xs = ws_digest_and_edges(p, root, a, a + n, ws)
        assert dg == oracle.digest(p, root, a, a + n, send_mode=1)
        assert xs == oracle.edgecheck(p, root, a, a + n, send_mode=1)
    n = 2**24 + 77
    for root, a in [(0, 0), (1_500_000_000, 1_500_000_000 - 5_000_000)]:
        t = ws_table(p, root, a, a + n, ws)
        step = 2**21
        for lo in range(0, n, step):
            hi = min(lo + step, n)
            want = oracle.schedules(p, root=root, r_begin=a + lo, r_end=a + hi, send_mode=1)
            assert np.array_equal(t[lo:hi].cpu().numpy(), want), (root, a + lo)
        del t


def gpu_digest_chunks(p, root, a, b, chunk, ws=None):
    n_slots = max(0, -(-(b - a) // chunk))
    dg = torch.full((n_slots + 1,), -1, dtype=torch.int64, device=DEV)       # one more: must stay as it is
    fl = torch.full((n_slots + 1,), -1, dtype=torch.int32, device=DEV)
    lib.bcast_schedules_digest_chunks(p, root, a, b, chunk, dg, fl, ws)
    torch.cuda.synchronize()
    d, f = dg.cpu().tolist(), fl.cpu().tolist()
    assert d[n_slots] == -1 and f[n_slots] == -1
    return [(x & oracle.U64_MAX, y & 0xFFFFFFFF) for x, y in zip(d[:n_slots], f[:n_slots])]


@pytest.mark.parametrize("p,root,a,n,chunk", [
    (1000003, 5, 0, 1000003, 2**17),           # violations; the last chunk ragged
    (1000003, 999999, 123, 700000, 64),        # a chunk per tile: batches of deferred ranks mix chunks
    (2**22 + 1, 7, 1000, 2**22 - 5000, 2**12), # more than one violation per rank; with the workspace: the list of ranks
    (2**23 - 1, 3, 0, 2**23 - 1, 2**20),       # the kernels whose wavefronts work alone
    (2**24, 2**23 + 5, 2**23 - 2_000_000, 4_000_001, 2**16),
    (4099, 0, 0, 4099, 128), (100, 3, 10, 80, 64), (1, 0, 0, 1, 64), (1000, 1, 500, 0, 64),
])
def test_digests_of_all_chunks_in_one_call(p, root, a, n, chunk):
    b = a + n
    want = [oracle.digest(p, root, lo, min(lo + chunk, b), send_mode=1) for lo in range(a, b, chunk)]
    assert gpu_digest_chunks(p, root, a, b, chunk) == want
    ws = torch.full((lib.bcast_schedules_workspace(p),), 0xEE, dtype=torch.uint8, device=DEV)
    assert gpu_digest_chunks(p, root, a, b, chunk, ws) == want
    if n:
        assert gpu_digest_chunks(p, root, a, b, 2**40) == [gpu_digest(p, root, a, b)]      # one chunk


def test_the_flag_for_more_than_four_violations():
    # p = 2^30 + 1, r = 3 * 2^26: five violations of Algorithm 6 (see the oracle's pins)
    p, r = 2**30 + 1, 3 * 2**26
    for a, b in [(r, r + 1), (r - 1000, r + 1000), (r - 64, r)]:
        assert gpu_digest(p, 0, a, b) == oracle.digest(p, 0, a, b, send_mode=1), (a, b)
    assert gpu_digest(p, 0, r - 1000, r + 1000)[1] == 8 and gpu_digest(p, 0, r - 64, r)[1] == 0
    ws = torch.full((lib.bcast_schedules_workspace(p),), 0xEE, dtype=torch.uint8, device=DEV)
    got = gpu_digest_chunks(p, 0, r - 2**21, r + 2**21, 2**20, ws)
    assert got == [oracle.digest(p, 0, lo, lo + 2**20, send_mode=1) for lo in range(r - 2**21, r + 2**21, 2**20)]
    assert [f for _, f in got] == [0, 0, 8, 0]


def test_workload3_all_chunk_digests_in_one_call():
    p = workloads.STREAMED_P
    gold = streamed_golden()
    ws = torch.empty(lib.bcast_schedules_workspace(p), dtype=torch.uint8, device=DEV)
    got = gpu_digest_chunks(p, 0, 0, p, workloads.STREAMED_CHUNK, ws)
    assert [f"{d:016x}" for d, _ in got] == [c["digest"] for c in gold["chunks"]]
    assert all(f == 0 for _, f in got)
    with pytest.raises(lib.BcastError):
        lib.bcast_schedules_digest_chunks(p, 0, 0, p, 100, torch.zeros(1, dtype=torch.int64, device=DEV),
                                          torch.zeros(1, dtype=torch.int32, device=DEV), None)     # not a power of two
    with pytest.raises(lib.BcastError):
        lib.bcast_schedules_digest_chunks(p, 0, 0, p, 32, torch.zeros(1, dtype=torch.int64, device=DEV),
                                          torch.zeros(1, dtype=torch.int32, device=DEV), None)     # below 64


def test_calls_with_workspace_argument_errors():
    p = 4000037
    q = lib.bcast_q(p)
    t = torch.zeros((16, 2 * q), dtype=torch.int32, device=DEV)
    small = torch.zeros(lib.bcast_schedules_workspace(p) - 1, dtype=torch.uint8, device=DEV)
    dg = torch.zeros(1, dtype=torch.int64, device=DEV)
    fl = torch.zeros(1, dtype=torch.int32, device=DEV)
    with pytest.raises(lib.BcastError) as e:
        lib.bcast_schedules_ws(p, 0, 0, 16, t, t, 2 * q, small, send_offset=q)
    assert e.value.code == lib.BCAST_ENOMEM
    with pytest.raises(lib.BcastError) as e:
        lib.bcast_schedules_digest_ws(p, 0, 0, 16, dg, fl, None)
    assert e.value.code == lib.BCAST_EINVAL
    ws = torch.zeros(lib.bcast_schedules_workspace(p), dtype=torch.uint8, device=DEV)
    with pytest.raises(lib.BcastError) as e:
        lib.bcast_schedules_ws(p, p, 0, 16, t, t, 2 * q, ws, send_offset=q)
    assert e.value.code == lib.BCAST_EINVAL
    assert lib.bcast_schedules_workspace(0) == 0
    torch.cuda.synchronize()
