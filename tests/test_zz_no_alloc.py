"""bcast_simulate_noalloc, the entry point for callers that cannot allocate: the
same replay as bcast_simulate on the library's own scratch array.  Its verdicts
must equal those of bcast_simulate (and the oracle's), call after call on the
array the last call left behind, and sizes beyond the array are refused."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
import paper_2407_18004_amd as lib  # noqa: E402
from paper_2407_18004_amd import workloads  # noqa: E402
from paper_2407_18004_amd.binding import VERDICT_BYTES, verdicts_from_bytes  # noqa: E402

DEV = "cuda:0"
SCRATCH_BYTES = 32 * 1024 * 1024        # BCAST_NOALLOC_SCRATCH_BYTES of include/bcast.h


def with_workspace(p, n, roots, sched=None):
    ws = torch.empty(lib.bcast_simulate_workspace(p, n, len(roots)), dtype=torch.uint8, device=DEV)
    vd = torch.full((len(roots) * VERDICT_BYTES,), 0xAB, dtype=torch.uint8, device=DEV)
    lib.bcast_simulate(p, n, roots, sched, ws, vd)
    torch.cuda.synchronize()
    return verdicts_from_bytes(vd.cpu().numpy().tobytes())


def without_allocation(p, n, roots, sched, vd):
    """vd: a verdict buffer allocated beforehand; nothing is allocated around the call."""
    vd.fill_(0xCD)
    # the number of allocations torch's allocator has served so far (frees by the garbage
    # collector of tensors of earlier tests do not touch it)
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    lib.bcast_simulate_noalloc(p, n, roots, sched, vd)
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
    torch.cuda.synchronize()
    return verdicts_from_bytes(vd[: len(roots) * VERDICT_BYTES].cpu().numpy().tobytes())


def test_two_calls_in_a_row_the_second_smaller():
    if not torch.cuda.is_available():
        pytest.fail("this test needs a GPU (run it with -m gpu on an MI355X)")
    lib.load_library()
    vd = torch.empty(8 * VERDICT_BYTES, dtype=torch.uint8, device=DEV)
    # first call: the replay of workload 5 with one root (20 MB of the 32 MiB array)
    p, n, root = workloads.SIMULATION_P, workloads.SIMULATION_N, workloads.SIMULATION_ROOT
    assert lib.bcast_simulate_workspace(p, n, 1) <= SCRATCH_BYTES
    got = without_allocation(p, n, [root], None, vd)
    assert got == with_workspace(p, n, [root])
    assert got[0] == oracle.simulate(p, n, root) and got[0]["flags"] == 0
    # second call, smaller, on what the first one left in the array: three roots, more blocks
    # than one possession word holds, and a caller's table with planted mistakes
    p2, n2, roots2 = 1000, 37, [0, 123, 999]
    q2 = oracle.q_of(p2)
    rng = np.random.default_rng(3)
    tables = []
    for r in roots2:
        tab = oracle.schedules(p2, root=r)
        for _ in range(4):
            tab[int(rng.integers(0, p2)), int(rng.integers(0, 2 * q2))] = int(rng.integers(-q2, q2))
        tables.append(tab)
    sched = torch.from_numpy(np.stack(tables)).to(DEV)
    got2 = without_allocation(p2, n2, roots2, sched, vd)
    assert got2 == with_workspace(p2, n2, roots2, sched)
    for j, r in enumerate(roots2):
        assert got2[j] == oracle.simulate(p2, n2, r, tables[j]) and got2[j]["flags"] != 0
    # third: the table computed in the call again, smaller still, clean
    got3 = without_allocation(4099, 41, [0, 4098], None, vd)
    assert got3 == with_workspace(4099, 41, [0, 4098])
    assert all(v["flags"] == 0 for v in got3)
    # and the first instance once more, now over the remains of smaller ones
    assert without_allocation(p, n, [root], None, vd)[0] == got[0]


def test_sizes_beyond_the_array_are_refused():
    lib.load_library()
    vd = torch.full((64 * VERDICT_BYTES,), 0x11, dtype=torch.uint8, device=DEV)
    p, n = workloads.SIMULATION_P, workloads.SIMULATION_N
    roots = workloads.simulation_roots(64, seed=42)
    assert lib.bcast_simulate_workspace(p, n, 64) > SCRATCH_BYTES
    with pytest.raises(lib.BcastError) as e:
        lib.bcast_simulate_noalloc(p, n, roots, None, vd)
    assert e.value.code == lib.BCAST_ENOMEM
    with pytest.raises(lib.BcastError) as e:
        lib.bcast_simulate_noalloc(p, 0, [0], None, vd)
    assert e.value.code == lib.BCAST_EINVAL
    with pytest.raises(lib.BcastError) as e:
        lib.bcast_simulate_noalloc(100, 10, [100], None, vd)
    assert e.value.code == lib.BCAST_EINVAL
    torch.cuda.synchronize()
    assert bool((vd == 0x11).all())          # nothing was launched
    # close to the limit from both sides (q = 17: 276 bytes per processor with one block)
    fits, too_big = 120_001, 131_072
    assert 0 < lib.bcast_simulate_workspace(fits, 1, 1) <= SCRATCH_BYTES < lib.bcast_simulate_workspace(too_big, 1, 1)
    with pytest.raises(lib.BcastError) as e:
        lib.bcast_simulate_noalloc(too_big, 1, [5], None, vd)
    assert e.value.code == lib.BCAST_ENOMEM
    got = verdicts_from_bytes(_run(fits, 1, [5], vd))
    assert got[0] == oracle.simulate(fits, 1, 5)


def _run(p, n, roots, vd):
    lib.bcast_simulate_noalloc(p, n, roots, None, vd)
    torch.cuda.synchronize()
    return vd[: len(roots) * VERDICT_BYTES].cpu().numpy().tobytes()
