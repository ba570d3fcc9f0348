"""The built HIP library loads and exports every function include/bcast.h
declares.  Host-only entry points are also called; nothing here needs a GPU."""
import ctypes
import os

import pytest

import paper_2407_18004_amd as lib


@pytest.fixture(scope="module")
def built():
    if not os.path.exists(lib.library_path()):
        from paper_2407_18004_amd import build
        build.build()
    return lib.load_library()


def test_every_declared_symbol_is_exported(built):
    names = lib.exported_symbols()
    assert set(names) >= {"bcast_q", "bcast_skips", "bcast_schedules", "bcast_schedules_digest",
                          "bcast_schedules_batched", "bcast_schedules_edgecheck", "bcast_schedules_double", "bcast_simulate_workspace",
                          "bcast_simulate", "bcast_simulate_reduce", "bcast_strerror"}
    for name in names:
        assert isinstance(getattr(built, name), ctypes._CFuncPtr), name


def test_host_only_entry_points(built):
    assert lib.bcast_q(1) == 0 and lib.bcast_q(2) == 1 and lib.bcast_q(2**31 - 1) == 31
    assert lib.bcast_skips(17) == [1, 2, 3, 5, 9, 17]          # Table 1
    assert lib.bcast_skips(11) == [1, 2, 3, 6, 11]             # proof of Lemma 4
    with pytest.raises(lib.BcastError):
        lib.bcast_q(0)
    with pytest.raises(lib.BcastError):
        lib.bcast_q(2**31)
    assert lib.bcast_strerror(0) == "ok"
    assert lib.bcast_simulate_workspace(65537, 256, 64) >= 64 * 8 * 65537 * 4
    assert lib.bcast_simulate_workspace(10, 0, 1) == 0
    # the workspace of the *_ws calls: the two tables of deep entries (2,050 entries of 16 bytes and 32 rows
    # of 2,050 16-bit words), then room for the open entries either as one list of p / 8 + 4,096 or as a
    # segment of 64 per wavefront of a short launch (at most 8,192 of them, one per tile and four more)
    tables = 2050 * 16 + 32 * 2050 * 2
    sizes = [lib.bcast_schedules_workspace(p) for p in (1, 100, 65537, 1000003, 2**24 + 1, 2**31 - 1)]
    assert sizes == sorted(sizes) and lib.bcast_schedules_workspace(2**31) == 0
    assert sizes[0] >= tables + 8 * 4096 and sizes[0] < tables + 64 * 1024
    assert sizes[3] >= tables + 8192 * (64 * 8 + 4)            # p = 1,000,003: 15,626 tiles, 8,192 segments
    assert sizes[5] >= tables + 8 * 2**22 and sizes[5] < tables + 8 * 2**22 + 2**20


def test_verdict_struct_layout():
    from paper_2407_18004_amd.binding import Verdict
    assert ctypes.sizeof(Verdict) == 48
    assert Verdict.first_bad.offset == 40


def test_missing_library_is_an_error(monkeypatch, tmp_path):
    from paper_2407_18004_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(ImportError):
        binding.load_library()
