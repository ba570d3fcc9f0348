"""The seeded input generators (no schedule arithmetic): internal consistency on the CPU."""
import numpy as np
import pytest

from paper_2407_18004_amd import workloads as w


def test_counter_random_is_the_splitmix64_finaliser():
    # SplitMix64's published first outputs for seed 0 are mix(0), mix(golden), ... : the finaliser
    # applied to 0 (after adding the golden-ratio increment) is 0xE220A8397B1DCDAF
    assert int(w._mix(np.asarray(0, dtype=np.uint64))) == 0xE220A8397B1DCDAF
    a = w.counter_random(42, 3, np.arange(8))
    b = np.array([int(w.counter_random(42, 3, i)) for i in range(8)], dtype=np.uint64)
    assert (a == b).all()                          # any element can be drawn on its own


@pytest.mark.parametrize("first,n_inst,m", [(0, 64, 256), (65_000, 37, 4096), (123, 5, 1)])
def test_ranks_drawn_with_torch_equal_the_numpy_draws(first, n_inst, m):
    p, root, ranks = w.batched_instances(n_inst, m, seed=42, first=first)
    got = w.batched_ranks_on_device(p, m, 42, first, "cpu").numpy().view(np.uint32)
    assert got.shape == ranks.shape
    assert (got == ranks).all()
    assert (ranks < p[:, None]).all() and (root < p).all()
    assert p.min() >= 2 and int(p.max()) < 2**31


def test_batched_offsets_and_chunks():
    p = np.array([2, 3, 4, 5, 1 << 20, (1 << 31) - 1], dtype=np.uint32)
    assert w.q_of(p).tolist() == [1, 2, 2, 3, 20, 31]
    off = w.batched_row_offsets(p, 4)
    assert off.tolist() == [0, 8, 24, 40, 64, 224, 472]
    chunks = w.streamed_chunks()
    assert chunks[0] == (0, 2**26) and chunks[-1][1] == 2**31 - 1 and len(chunks) == 32
    assert all(a[1] == b[0] for a, b in zip(chunks, chunks[1:]))
