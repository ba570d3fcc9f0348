#!/usr/bin/env python3
"""Benchmark of the schedule hot path on one MI355X.

One step = one pass of the whole path (skips, baseblock, receive search, send
walk with violations, invariant flags and digest) over every rank of the huge
streamed instance p = 2^31 - 1, root 0, in 32 chunks of 2^26 ranks, each chunk
with a digest and flags of its own, all of them from one call of
bcast_schedules_digest_chunks.  Nothing crosses PCIe inside the timed
region: the inputs are scalars and each chunk leaves 12 bytes in HBM.  The 32
chunk digests are compared with the ones the CPU oracle wrote
(tests/golden/streamed_chunk_digests.json).

Prints ONE JSON line.  `roofline` prices the dominant kernel (k_digest, plain
integer VALU work) against the chip's 32-bit lane-operation rate, on two bases:
a fixed count of the algorithm's operations per rank (`frac`) and the
lane-operations the kernel actually executes (`frac_executed`).  The
materialised tables are timed as well and priced against HBM write bandwidth
under `materialised`.  `cpu_baseline` is the CPU oracle timed on this
machine's cores on a bounded sample of the same instance.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "rank-schedules/sec (recv+send, q=ceil(log2 p)) at p=2^31-1"
UNIT = "rank-schedules/s"

# MI355X: 256 CUs x 4 SIMDs x 32 lanes per cycle x 2.4 GHz 32-bit lane-operations (the rate
# behind the published 157.3 TFLOP/s of fp32 vector FMA = 2 x 78.6).  Only additions, logic,
# shifts and moves on vector registers issue at that rate; compares, selects, min/max, multiplies,
# three-operand forms and anything with a scalar-register operand take twice as long.
PEAK_LANE_OPS = 256 * 4 * 32 * 2.4e9
PEAK_HBM = 8.0e12

# Operations of the algorithm per rank-schedule at q = 31, counted on the paper's algorithms as a
# sequential program would run them (no sharing between ranks): Algorithm 3 4 per level (124);
# Algorithm 4 10 per list element looked at and 8 per recursive call, 67.6 and 22.5 of them per
# rank as the oracle counts them at p = 2^31 - 1 (856); the mapping of Algorithm 5 3 per round
# (93); Algorithm 6 10 per round (300); packing 2.5 per entry and 8 SplitMix64 of 30 (395).
ALGORITHMIC_LANE_OPS_Q31 = 124 + 856 + 93 + 300 + 395


def load_counters() -> dict:
    """Per-kernel figures taken from rocprofv3 counters (profiles/bench_counters.json, which
    names the summaries it was computed from): active VALU lane-operations per rank-schedule
    and HBM bytes per launch.  Empty if the file is missing."""
    path = os.path.join(ROOT, "profiles", "bench_counters.json")
    try:
        with open(path) as fh:
            return json.load(fh).get("kernels", {})
    except (OSError, ValueError):
        return {}


def load_golden_digests() -> dict | None:
    path = os.path.join(ROOT, "tests", "golden", "streamed_chunk_digests.json")
    try:
        with open(path) as fh:
            return json.load(fh)
    except (OSError, ValueError):
        return None


def run(args) -> dict:
    import torch

    import paper_2407_18004_amd as lib
    from paper_2407_18004_amd import workloads

    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU")
    lib.load_library()
    dev = "cuda:0"
    torch.cuda.set_device(0)

    p = workloads.STREAMED_P
    q = lib.bcast_q(p)
    chunks = workloads.streamed_chunks()
    n_chunks = len(chunks)
    dg = torch.zeros(n_chunks, dtype=torch.int64, device=dev)
    fl = torch.zeros(n_chunks, dtype=torch.int32, device=dev)
    dgs = [dg[i:i + 1] for i in range(n_chunks)]
    fls = [fl[i:i + 1] for i in range(n_chunks)]
    ws = torch.empty(lib.bcast_schedules_workspace(p), dtype=torch.uint8, device=dev)
    chunk_ranks = chunks[0][1] - chunks[0][0]

    # One call computes the digests and flags of all chunks (bcast_schedules_digest_chunks: one
    # launch works through the whole instance and writes a result per chunk); with
    # --calls-per-chunk every chunk is a call of bcast_schedules_digest_ws, one after the other.
    def step(events=None, per_chunk=False):
        if events is not None:
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
        if per_chunk:
            for i, (a, b) in enumerate(chunks):
                lib.bcast_schedules_digest_ws(p, 0, a, b, dgs[i], fls[i], ws)
        else:
            lib.bcast_schedules_digest_chunks(p, 0, 0, p, chunk_ranks, dg, fl, ws)
        if events is not None:
            e1.record()
            events.append((e0, e1))

    if args.copy_probe:                 # known traffic: 256 MiB read + 256 MiB written per copy
        src = torch.zeros(64 * 1024 * 1024, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step(per_chunk=args.calls_per_chunk)
    torch.cuda.synchronize()
    events = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(events, per_chunk=args.calls_per_chunk)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = p / (ms_per_step * 1e-3)
    flags_or = int(torch.bitwise_or(fl[0], fl.max()).item()) if n_chunks else 0
    assert int(fl.abs().sum().item()) == 0, "invariant flags raised on the GPU"
    per_chunk = [x & ((1 << 64) - 1) for x in dg.cpu().tolist()]
    whole = 0
    for x in per_chunk:
        whole ^= x
    gold = load_golden_digests()
    equals_oracle = None
    if gold is not None:
        equals_oracle = (gold["digest"] == f"{whole:016x}" and
                         [c["digest"] for c in gold["chunks"]] == [f"{x:016x}" for x in per_chunk])
        assert equals_oracle, "chunk digests differ from the oracle's"

    # for comparison, outside the timed region: the same step as one call per chunk
    other_ms = None
    if not args.calls_per_chunk and not args.no_compare:
        step(per_chunk=True)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for _ in range(2):
            step(per_chunk=True)
        torch.cuda.synchronize()
        other_ms = (time.perf_counter() - t2) * 1e3 / 2
        per_chunk_again = [x & ((1 << 64) - 1) for x in dg.cpu().tolist()]
        assert per_chunk_again == per_chunk, "one call and 32 calls give different chunk digests"

    launch_ms = [a.elapsed_time(b) for a, b in events]
    avg_launch_ms = sum(launch_ms) / len(launch_ms)
    ranks_per_launch = p                        # an event pair encloses a whole step
    # `achieved`: operations of the algorithm per rank (fixed, see ALGORITHMIC_LANE_OPS_Q31) x ranks
    # per step / live duration of the step between HIP events on the launch stream (the event pairs
    # enclose the small kernels of the call or calls, which clear the results and build the table of
    # deep entries, as well; k_digest is all but 20 us of it).  `achieved_executed`:
    # the same with the 32-bit lane-operations the kernel's active lanes execute per rank
    # (SQ_THREAD_CYCLES_VALU / ranks, measured with rocprofv3) in place of the fixed count.
    counters = load_counters()
    ops_exec = counters.get("k_digest", {}).get("active_valu_lane_ops_per_rank")
    per_s = ranks_per_launch / (avg_launch_ms * 1e-3)
    achieved = ALGORITHMIC_LANE_OPS_Q31 * per_s
    achieved_exec = ops_exec * per_s if ops_exec else None
    roofline = {
        "kernel": "k_digest", "bound": "alu",
        "achieved": achieved / 1e12, "peak": PEAK_LANE_OPS / 1e12, "unit": "Tlane-op/s",
        "frac": achieved / PEAK_LANE_OPS,
        "basis": "operations of Algorithms 3-6 and the digest per rank, counted once (fixed)",
        "lane_ops_per_rank": ALGORITHMIC_LANE_OPS_Q31,
        "achieved_executed": achieved_exec / 1e12 if achieved_exec else None,
        "frac_executed": achieved_exec / PEAK_LANE_OPS if achieved_exec else None,
        "lane_ops_per_rank_executed": ops_exec,
        "traffic": counters.get("k_digest", {}).get("hbm_bytes_per_launch"),
        "avg_launch_ms": avg_launch_ms, "launches": len(launch_ms),
        "ranks_per_launch": ranks_per_launch,
    }

    out = {
        "metric": METRIC, "value": value, "unit": UNIT, "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32", "data": "synthetic",
        "config": {"workload": "streamed instance p=2^31-1, root=0, all ranks in 32 chunks of "
                               "2^26, digest+flags per chunk (" +
                               ("bcast_schedules_digest_ws" if args.calls_per_chunk else "bcast_schedules_digest_chunks") + ")",
                   "p": p, "q": q, "chunks": n_chunks,
                   "calls_per_step": n_chunks if args.calls_per_chunk else 1,
                   "ms_per_step_with_a_call_per_chunk": other_ms, "digest": f"{whole:016x}",
                   "flags": flags_or, "digests_equal_oracle": equals_oracle},
        "roofline": roofline,
    }
    if not args.headline_only:
        out["materialised"] = bench_materialised(torch, lib, workloads, dev, args, counters)
        out["other_workloads"] = bench_other(torch, lib, workloads, dev, counters)
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(p)
    return out


def bench_materialised(torch, lib, workloads, dev, args, counters) -> dict:
    """The [p][2q] table of p = 1,000,003 (q = 20): 8q bytes written per rank; and, for the
    rate the kernels reach once a launch is long enough, 2^25 ranks of p = 2^31 - 1."""
    p = workloads.MATERIALISED_P
    q = lib.bcast_q(p)
    table = torch.empty((p, 2 * q), dtype=torch.int32, device=dev)
    reps = max(20, 4 * args.steps)
    ws2 = torch.empty(lib.bcast_schedules_workspace(p), dtype=torch.uint8, device=dev)
    # with a workspace: what the search leaves open of the send part is filled in from the
    # table's own receive rows by a second kernel (the whole call is timed: three kernels)
    med = _median_ms(torch, lambda: lib.bcast_schedules_ws(p, 0, 0, p, table, table, 2 * q, ws2,
                                                           send_offset=q), reps)
    # without: the same entries by searches at the end of every workgroup
    med_search = _median_ms(torch, lambda: lib.bcast_schedules(p, 0, 0, p, table, table, 2 * q,
                                                               send_offset=q), reps)
    nbytes = 8.0 * q * p
    del table, ws2
    pl, nl = workloads.STREAMED_P, 1 << 25
    ql = lib.bcast_q(pl)
    big = torch.empty((nl, 2 * ql), dtype=torch.int32, device=dev)
    ws = torch.empty(lib.bcast_schedules_workspace(pl), dtype=torch.uint8, device=dev)
    med_l = _median_ms(torch, lambda: lib.bcast_schedules_ws(pl, 0, 0, nl, big, big, 2 * ql, ws,
                                                             send_offset=ql), 7)
    med_plain = _median_ms(torch, lambda: lib.bcast_schedules(pl, 0, 0, nl, big, big, 2 * ql,
                                                              send_offset=ql), 5)
    del big
    bytes_l = 8.0 * ql * nl
    large = {"workload": "ranks [0, 2^25) of p=2^31-1, int32 [2^25][62] table (bcast_schedules_ws)",
             "kernel": "k_schedules", "median_launch_ms": med_l,
             "rank_schedules_per_s": nl / (med_l * 1e-3),
             "roofline": {"bound": "hbm", "achieved": bytes_l / (med_l * 1e-3) / 1e9,
                          "peak": PEAK_HBM / 1e9, "unit": "GB/s",
                          "frac": bytes_l / (med_l * 1e-3) / PEAK_HBM,
                          "traffic": counters.get("k_schedules_long", {}).get("hbm_bytes_per_launch")},
             "without_workspace_ms": med_plain}
    return {
        "long_launch": large,
        "workload": "p=1000003 root=0 all ranks, int32 [p][40] table (bcast_schedules_ws)",
        "kernel": "k_schedules + k_fill_open", "median_launch_ms": med, "launches": reps,
        "without_workspace_ms": med_search,
        "rank_schedules_per_s": p / (med * 1e-3),
        "roofline": {"bound": "hbm", "achieved": nbytes / (med * 1e-3) / 1e9,
                     "peak": PEAK_HBM / 1e9, "unit": "GB/s",
                     "frac": nbytes / (med * 1e-3) / PEAK_HBM,
                     "traffic": counters.get("k_schedules", {}).get("hbm_bytes_per_launch")},
    }


def _median_ms(torch, fn, reps: int) -> float:
    fn()
    torch.cuda.synchronize()
    evs = []
    for _ in range(reps):
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        evs.append((e0, e1))
    torch.cuda.synchronize()
    ms = sorted(a.elapsed_time(b) for a, b in evs)
    return ms[len(ms) // 2]


def bench_other(torch, lib, workloads, dev, counters) -> dict:
    """The workloads that are not rank ranges (all 65,536 batched instances, the broadcast
    replay) and the generation by doubling."""
    import numpy as np
    from paper_2407_18004_amd.binding import VERDICT_BYTES
    n_inst, m = 65536, 4096
    p, root, _ = workloads.batched_instances(n_inst, m, seed=42, with_ranks=False)
    row_off = workloads.batched_row_offsets(p, m)
    d = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a).view(dt)).to(dev)  # noqa: E731
    dp, droot, doff = d(p, np.int32), d(root, np.int32), d(row_off, np.int64)
    dranks = torch.empty((n_inst, m), dtype=torch.int32, device=dev)
    block = 8192
    for first in range(0, n_inst, block):
        dranks[first:first + block] = workloads.batched_ranks_on_device(p[first:first + block], m, 42,
                                                                        first, dev)
    out = torch.empty(int(row_off[-1]), dtype=torch.int32, device=dev)
    rej = torch.zeros(1, dtype=torch.int32, device=dev)
    ms_b = _median_ms(torch, lambda: lib.bcast_schedules_batched(n_inst, dp, droot, dranks, m, doff,
                                                                 out, rej), 3)
    assert int(rej.item()) == 0
    nbytes = 4.0 * int(row_off[-1]) + 4.0 * n_inst * m
    del out, dranks
    ps, n = workloads.SIMULATION_P, workloads.SIMULATION_N
    roots = workloads.simulation_roots(64, seed=42)
    q = lib.bcast_q(ps)
    ws = torch.empty(lib.bcast_simulate_workspace(ps, n, 64), dtype=torch.uint8, device=dev)
    vd = torch.zeros(64 * VERDICT_BYTES, dtype=torch.uint8, device=dev)
    ms_1 = _median_ms(torch, lambda: lib.bcast_simulate(ps, n, [workloads.SIMULATION_ROOT], None,
                                                        ws, vd), 5)
    ms_64 = _median_ms(torch, lambda: lib.bcast_simulate(ps, n, roots, None, ws, vd), 5)
    rounds = n - 1 + q
    del ws
    # doubling (Observations 1 and 5): one step, and whole tables of even p against the search
    ph = 500_002
    qh = lib.bcast_q(ph)
    half = torch.empty((ph, 2 * qh), dtype=torch.int32, device=dev)
    lib.bcast_schedules(ph, 0, 0, ph, half, half, 2 * qh, send_offset=qh)
    full = torch.empty((2 * ph, 2 * (qh + 1)), dtype=torch.int32, device=dev)
    ms_d = _median_ms(torch, lambda: lib.bcast_schedules_double(ph, half, full), 20)
    bytes_d = 4.0 * half.numel() + 4.0 * full.numel()
    del half, full
    even = {}
    for pe, name in ((1_000_004, "p=1,000,004 = 4 x 250,001"), (3 * 2**20, "p=3 x 2^20")):
        qe = lib.bcast_q(pe)
        tab = torch.empty((pe, 2 * qe), dtype=torch.int32, device=dev)
        wse = torch.empty(lib.bcast_schedules_doubling_workspace(pe), dtype=torch.uint8, device=dev)
        ms_e = _median_ms(torch, lambda: lib.bcast_schedules_doubling(pe, tab, wse), 10)
        ms_s = _median_ms(torch, lambda: lib.bcast_schedules(pe, 0, 0, pe, tab, tab, 2 * qe,
                                                             send_offset=qe), 10)
        even[name] = {"by_doubling_ms": ms_e, "by_search_ms": ms_s,
                      "by_doubling_GB_per_s": 8.0 * qe * pe / (ms_e * 1e-3) / 1e9}
        del tab, wse
    # digests of an instance with violations of Algorithm 6 in nearly every rank, and the edge check
    pv = 2**30 + 1
    wsv = torch.empty(lib.bcast_schedules_workspace(pv), dtype=torch.uint8, device=dev)
    dgv = torch.zeros(2, dtype=torch.int64, device=dev)
    flv = torch.zeros(1, dtype=torch.int32, device=dev)
    ms_v = _median_ms(torch, lambda: lib.bcast_schedules_digest_ws(pv, 0, 2**26, 2**27, dgv[:1], flv, wsv), 5)
    assert int(flv.item()) == 0
    pe_ = workloads.STREAMED_P
    ms_x = _median_ms(torch, lambda: lib.bcast_schedules_edgecheck_ws(pe_, 0, 2**26, 2**27, dgv, wsv), 5)
    ms_xv = _median_ms(torch, lambda: lib.bcast_schedules_edgecheck_ws(pv, 0, 2**26, 2**27, dgv, wsv), 5)
    pb = workloads.STREAMED_P
    lst = torch.empty(pb, dtype=torch.uint8, device=dev)
    ms_l = _median_ms(torch, lambda: lib.bcast_baseblocks(pb, lst), 5)
    del lst
    return {
        "doubling": {"workload": "table of p=1,000,004 from the table of p=500,002 "
                                 "(bcast_schedules_double)", "kernel": "k_double",
                     "median_launch_ms": ms_d, "rank_schedules_per_s": 2 * ph / (ms_d * 1e-3),
                     "roofline": {"bound": "hbm", "achieved": bytes_d / (ms_d * 1e-3) / 1e9,
                                  "peak": PEAK_HBM / 1e9, "unit": "GB/s",
                                  "frac": bytes_d / (ms_d * 1e-3) / PEAK_HBM},
                     "whole_tables_of_even_p": even},
        "digest_with_violations": {"workload": "ranks [2^26, 2^27) of p=2^30+1 (1.6 violations of "
                                               "Algorithm 6 per rank), digest+flags (bcast_schedules_digest_ws)",
                                   "kernel": "k_digest<true,false>", "median_launch_ms": ms_v,
                                   "rank_schedules_per_s": 2**26 / (ms_v * 1e-3)},
        "edgecheck": {"workload": "ranks [2^26, 2^27), Conditions 1 and 2 as two XOR sums "
                                  "(bcast_schedules_edgecheck_ws)", "kernel": "k_digest<.,true>",
                      "p=2^31-1_ms": ms_x, "p=2^30+1_ms": ms_xv,
                      "rank_schedules_per_s_p=2^31-1": 2**26 / (ms_x * 1e-3)},
        "baseblock_listing": {"workload": "all baseblocks of p=2^31-1, one byte each, by the "
                                          "linear-time listing (bcast_baseblocks)",
                              "median_call_ms": ms_l,
                              "GB_per_s_moved": 2.0 * pb / (ms_l * 1e-3) / 1e9},
        "batched": {"workload": "65,536 seeded instances x 4,096 ranks (workload 4 in full)",
                    "kernel": "k_batched", "median_launch_ms": ms_b,
                    "rank_schedules_per_s": n_inst * m / (ms_b * 1e-3),
                    "roofline": {"bound": "hbm", "achieved": nbytes / (ms_b * 1e-3) / 1e9,
                                 "peak": PEAK_HBM / 1e9, "unit": "GB/s",
                                 "frac": nbytes / (ms_b * 1e-3) / PEAK_HBM,
                                 "traffic": counters.get("k_batched", {}).get("hbm_bytes_per_launch")}},
        "simulate": {"workload": "p=65537 n=256 (272 rounds), schedules computed in the call",
                     "kernel": "k_schedules + k_simulate",
                     "one_root_ms": ms_1, "64_roots_ms": ms_64,
                     "processor_rounds_per_s_64_roots": 64.0 * ps * rounds / (ms_64 * 1e-3)},
    }


def cpu_baseline(p: int) -> dict:
    """The oracle (Algorithms 5 and 6 in plain C, OpenMP over ranks) on this
    machine's cores, on a prefix of the same instance sized for some 12 s, and
    on one core on a prefix sized for some 6 s."""
    import oracle
    threads = oracle.default_threads()
    probe = 1 << 22
    t0 = time.perf_counter()
    oracle.digest(p, 0, 0, probe, send_mode=1, threads=threads)
    rate = probe / (time.perf_counter() - t0)
    n = int(min(p, max(probe, rate * 12.0)))
    t0 = time.perf_counter()
    oracle.digest(p, 0, 0, n, send_mode=1, threads=threads)
    dt = time.perf_counter() - t0
    probe1 = 1 << 20
    t0 = time.perf_counter()
    oracle.digest(p, 0, 0, probe1, send_mode=1, threads=1)
    rate1 = probe1 / (time.perf_counter() - t0)
    n1 = int(min(p, max(probe1, rate1 * 6.0)))
    t0 = time.perf_counter()
    oracle.digest(p, 0, 0, n1, send_mode=1, threads=1)
    dt1 = time.perf_counter() - t0
    return {"value": n / dt, "unit": UNIT, "cores": threads, "kind": "oracle",
            "sample": f"ranks [0, {n}) of p=2^31-1, digest+flags, {dt:.1f} s",
            "one_core": {"value": n1 / dt1, "unit": UNIT, "cores": 1,
                         "sample": f"ranks [0, {n1}) of p=2^31-1, digest+flags, {dt1:.1f} s"}}


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--no-compare", action="store_true",
                    help="skip the untimed steps with a call per chunk that are run for comparison")
    ap.add_argument("--calls-per-chunk", action="store_true",
                    help="a call of bcast_schedules_digest_ws per chunk instead of one call for all chunks")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--headline-only", action="store_true",
                    help="time the streamed instance only (no tables, no other workloads)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain 256 MiB device copy (scale for the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        raise SystemExit("bench.py: this build runs on one GPU only (rank-schedules are independent; "
                         "nothing is exchanged between GPUs). Run it with --gpus 1.")
    print(json.dumps(run(args)), flush=True)


if __name__ == "__main__":
    main()
