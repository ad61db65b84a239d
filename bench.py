#!/usr/bin/env python3
"""Benchmark of the shm355 hot path on one MI355X.

Headline (the JSON line's `value`): configuration 2's work-group put -- 8 logical PEs, each
putting a 256 MiB float32 message to PE (p+1) mod 8 with 1024 work-groups of 256 threads through
direct loads/stores, launched as one grid on the team stream.  One step = one such put by all
eight PEs.  Inputs are seeded synthetic data resident in HBM before the timed region.

The same line carries `roofline` (the put kernel against the HBM copy roofline, timed with HIP
events on the stream it runs on), `cpu_baseline` (the oracle's work-group put timed on this host,
context only) and `extras` with the other configurations: the put sweep over message sizes,
work-group counts and both transfer paths with the measured crossover, the ping/flag latency, the
pipelined ring, the atomic storm (ops/s) and the two collectives.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MiB = 1 << 20
GiB = 1 << 30
HBM_PEAK_GBS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def event_pair(torch):
    return torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)


def time_on_stream(torch, stream, fn, iters):
    """Average milliseconds per call of fn, between two events recorded on `stream`."""
    e0, e1 = event_pair(torch)
    e0.record(stream)
    for _ in range(iters):
        fn()
    e1.record(stream)
    e1.synchronize()
    return e0.elapsed_time(e1) / iters


def paper_timing(torch, run_trial):
    """The paper's method (section "Performance Evaluation"): double the iteration count of the
    warm-up until one batch takes more than 2 ms, then ten trials, best one.  run_trial(iters)
    returns milliseconds per iteration."""
    iters = 1
    while True:
        ms = run_trial(iters)
        if ms * iters > 2.0 or iters >= 4096:
            break
        iters *= 2
    return min(run_trial(iters) for _ in range(10))


def concurrent_pe_trial(torch, g, launch_pe, npes, iters):
    """All PEs start together on their own streams; time = common start to the latest end."""
    start = torch.cuda.Event(enable_timing=True)
    ends = [torch.cuda.Event(enable_timing=True) for _ in range(npes)]
    torch.cuda.synchronize()
    start.record(g.streams[0])
    for p in range(1, npes):
        g.streams[p].wait_event(start)
    for _ in range(iters):
        for p in range(npes):
            launch_pe(p)
    for p in range(npes):
        ends[p].record(g.streams[p])
    torch.cuda.synchronize()
    return max(start.elapsed_time(e) for e in ends) / iters


def headline(torch, S, synth, g, args):
    npes, n, n_wg = 8, args.size_mib * MiB, args.n_wg
    src, dst = g.malloc(n), g.malloc(n)
    log(f"[bench] generating and uploading {npes} x {args.size_mib} MiB of seeded float32 N(0,1)")
    data0 = None
    for p in range(npes):
        d = synth.c2_source(p, n)
        g.write(p, src, d)
        if p == 0:
            data0 = d
    g.set_team_sync(False)

    def step():
        g.launch_wg_put_all(1, dst, src, n, n_wg, S.SHM_PATH_LDST)

    for _ in range(args.warmup):
        step()
    g.barrier_all()
    torch.cuda.synchronize()
    e0, e1 = event_pair(torch)
    t0 = time.perf_counter()
    e0.record(g.streams[0])
    for _ in range(args.steps):
        step()
    e1.record(g.streams[0])
    g.barrier_all()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    wall_ms = (t1 - t0) * 1e3 / args.steps
    kern_ms = e0.elapsed_time(e1) / args.steps
    g.set_team_sync(True)
    ok = bool(np.array_equal(g.read(1, dst, 4096), data0[:4096]) and
              np.array_equal(g.read(1, dst + n - 4096, 4096), data0[n - 4096:]))
    payload = npes * n
    res = {
        "wall_ms": wall_ms, "kernel_ms": kern_ms, "payload_bytes": payload,
        "value_gbs": payload / wall_ms / 1e6,
        "achieved_gbs": 2 * payload / kern_ms / 1e6,
        "spot_check_ok": ok,
    }
    g.free(src), g.free(dst)
    return res, data0


def cpu_put_baseline(oracle_mod, data0, n, n_wg, budget_s=12.0):
    """The oracle's work-group put, one host core, on a bounded sample of the same workload:
    one PE's message at full size, repeated until the time budget is used."""
    o = oracle_mod.ShmemOracle(2, 2 * n)
    o.write(0, 0, data0)
    t_end = time.perf_counter() + budget_s
    best, reps = float("inf"), 0
    while reps < 3 or (time.perf_counter() < t_end and reps < 20):
        t0 = time.perf_counter()
        o.wg_put(0, n, 0, n, 1, n_wg)
        best = min(best, time.perf_counter() - t0)
        reps += 1
    assert np.array_equal(o.heap[1][n:n + 4096], data0[:4096])
    return {"value": n / best / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"one PE's {n >> 20} MiB message with {n_wg} group slices, best of {reps} (numpy, single thread); "
                      f"host has {os.cpu_count()} logical CPUs"}


def put_sweep(torch, S, g, args):
    """Configuration 2: message sizes 8 B .. 256 MiB, 8 PEs concurrently on their own streams."""
    npes = 8
    max_n = args.sweep_max_mib * MiB
    src, dst = g.malloc(max_n), g.malloc(max_n)
    sizes = [1 << k for k in range(3, 29) if (1 << k) <= max_n]
    rows = []
    curves = [("ldst", w) for w in (1, 4, 64, 1024)] + [("sdma", 0)]
    for n in sizes:
        row = {"bytes": n}
        for kind, n_wg in curves:
            path = S.SHM_PATH_LDST if kind == "ldst" else S.SHM_PATH_SDMA
            ms = paper_timing(torch, lambda iters: concurrent_pe_trial(
                torch, g, lambda p: g.launch_wg_put(p, (p + 1) % npes, dst, src, n, max(n_wg, 1), path), npes, iters))
            key = f"ldst_wg{n_wg}" if kind == "ldst" else "sdma"
            row[key + "_us"] = ms * 1e3
            row[key + "_gbs"] = npes * n / ms / 1e6
        rows.append(row)
        log("[sweep] " + " ".join(f"{k}={v:.4g}" if isinstance(v, float) else f"{k}={v}" for k, v in row.items() if not k.endswith("_us")))
    # team-launch curve for the largest work-group count (one grid for all PEs)
    g.set_team_sync(False)
    for row in rows:
        n = row["bytes"]
        ms = paper_timing(torch, lambda iters: time_on_stream(
            torch, g.streams[0], lambda: g.launch_wg_put_all(1, dst, src, n, 1024, S.SHM_PATH_LDST), iters))
        row["team_wg1024_us"], row["team_wg1024_gbs"] = ms * 1e3, npes * n / ms / 1e6
    g.set_team_sync(True)
    # crossover per work-group count: first size from which the engine is at least as fast, for good
    cross = {}
    for n_wg in (1, 4, 64, 1024):
        key, c = f"ldst_wg{n_wg}_gbs", None
        for i, row in enumerate(rows):
            if key in row and all(r["sdma_gbs"] >= r[key] for r in rows[i:] if key in r):
                c = row["bytes"]
                break
        cross[str(n_wg)] = c
        g.set_cutover(n_wg, c if c is not None else (1 << 64) - 1)
    g.free(src), g.free(dst)
    return {"pes": npes, "timing": "warm-up doubling to >2 ms, best of 10 (events: common start to latest end)",
            "rows": rows, "crossover_bytes": cross,
            "crossover_note": "smallest message from which the copy-engine path stays at least as fast as "
                              "loads/stores; null = loads/stores win at every measured size"}


def pingflag(torch, S, synth, args):
    g = S.Shm.on_torch(2, MiB)
    payload = synth.c1_payload(4096)
    n = payload.nbytes
    data, back, flag = g.malloc(n), g.malloc(n), g.calloc(8, 8)
    g.write(0, data, payload)
    zero = np.zeros(8, np.uint8)
    best_wall, best_dev = float("inf"), float("inf")
    for i in range(30):
        g.write(1, flag, zero)
        torch.cuda.synchronize()
        e0, e1 = event_pair(torch)
        t0 = time.perf_counter()
        e0.record(g.streams[0])
        g.launch_pingflag(data, back, n, flag)
        e1.record(g.streams[1])
        g.barrier_all()
        t1 = time.perf_counter()
        if i >= 5:
            best_wall = min(best_wall, (t1 - t0) * 1e6)
            best_dev = min(best_dev, e0.elapsed_time(e1) * 1e3)
    ok = bool(np.array_equal(g.read(1, back, n, np.int32), payload))
    g.finalize()
    return {"bytes": n, "device_us": best_dev, "host_round_trip_us": best_wall, "ok": ok,
            "note": "PE0: 16 KiB work-group put, quiet, flag; PE1 (own stream): wait, get back; best of 25"}


def ring(torch, S, synth, g, args):
    npes, n_chunks, nel = 8, 64, 524288
    cb = 2 * nel
    src, slot, acc, sig = g.malloc(cb * n_chunks), g.malloc(cb * n_chunks), g.malloc(4 * nel), g.calloc(8, 8)
    for p in range(npes):
        g.write(p, src, synth.c3_chunks(p, n_chunks, nel))
    zero = np.zeros(8, np.uint8)
    out = {}
    for n_prod, n_cons in ((32, 32), (16, 32), (32, 64), (64, 64)):
        best = float("inf")
        for i in range(12):
            for p in range(npes):
                g.write(p, sig, zero)
            torch.cuda.synchronize()
            e0, e1 = event_pair(torch)
            e0.record(g.streams[0])
            g.launch_ring_pipeline(src, slot, sig, acc, cb, n_chunks, n_prod, n_cons)
            e1.record(g.streams[0])
            g.barrier_all()
            if i >= 2:
                best = min(best, e0.elapsed_time(e1))
        algo = npes * (n_chunks * 3 * cb + 4 * nel)
        out[f"prod{n_prod}_cons{n_cons}"] = {"ms": best, "payload_gbs": npes * n_chunks * cb / best / 1e6,
                                           "algorithmic_gbs": algo / best / 1e6, "frac_hbm": algo / best / 1e6 / HBM_PEAK_GBS}
    for off in (src, slot, acc, sig):
        g.free(off)
    return out


def storm(torch, S, synth, args):
    npes, n_ctr, n_items, ops = 16, 1024, 1 << 20, 64
    g = S.Shm.on_torch(npes, MiB)
    ctr = g.calloc(8 * n_ctr, 256)
    targets = torch.from_numpy(synth.c4_targets(n_items, ops, npes, n_ctr).view(np.int16)).cuda()
    checksum = torch.zeros(n_items // 256, dtype=torch.int64, device="cuda")
    out = {}
    for name, kind in (("fetch_add", S.SHM_STORM_FETCH_ADD), ("add_no_return", S.SHM_STORM_ADD),
                       ("plain_store_ceiling", S.SHM_STORM_PLAIN_STORE)):
        best = float("inf")
        for i in range(7):
            torch.cuda.synchronize()
            e0, e1 = event_pair(torch)
            e0.record(g.streams[0])
            g.launch_amo_storm(ctr, n_ctr, targets, n_items, ops, kind, None, checksum if kind == S.SHM_STORM_FETCH_ADD else None)
            e1.record(g.streams[0])
            g.barrier_all()
            if i >= 2:
                best = min(best, e0.elapsed_time(e1))
        out[name] = {"ms": best, "gops": n_items * ops / best / 1e6}
    g.finalize()
    out["ops"] = n_items * ops
    return out


def collectives(torch, S, synth, g, args):
    npes, nel = 8, 16 * MiB
    fsrc, fdst = g.malloc(4 * nel), g.malloc(4 * nel * npes)
    rsrc, rdst = g.malloc(4 * nel), g.malloc(4 * nel)
    for p in range(npes):
        g.write(p, fsrc, synth.c5_fcollect_source(p, nel))
        g.write(p, rsrc, synth.c5_reduce_source(p, nel))
    out = {}

    def best_of(fn, stream_timed=True):
        best = float("inf")
        for i in range(8):
            torch.cuda.synchronize()
            e0, e1 = event_pair(torch)
            e0.record(g.streams[0])
            fn()
            e1.record(g.streams[0])
            g.barrier_all()
            if i >= 2:
                best = min(best, e0.elapsed_time(e1))
        return best

    fc_bytes = npes * 4 * nel + npes * npes * 4 * nel            # each source read once, every block written 8 times
    for n_wg in (256, 1024):
        ms = best_of(lambda: g.launch_fcollect(fdst, fsrc, 4 * nel, n_wg, S.SHM_PATH_LDST))
        out[f"fcollect_ldst_wg{n_wg}"] = {"ms": ms, "algorithmic_gbs": fc_bytes / ms / 1e6, "frac_hbm": fc_bytes / ms / 1e6 / HBM_PEAK_GBS}
    ms = best_of(lambda: g.launch_fcollect(fdst, fsrc, 4 * nel, 1024, S.SHM_PATH_SDMA))
    sd_bytes = 2 * npes * npes * 4 * nel
    out["fcollect_sdma"] = {"ms": ms, "algorithmic_gbs": sd_bytes / ms / 1e6, "frac_hbm": sd_bytes / ms / 1e6 / HBM_PEAK_GBS,
                            "note": "64 engine copies of 64 MiB: 8 GiB of traffic for the same result"}
    dup_bytes = npes * npes * 4 * nel + npes * 4 * nel
    spl_bytes = npes * 4 * nel + npes * 4 * nel
    for n_wg in (256, 1024):
        ms = best_of(lambda: g.launch_reduce_sum_f32(rdst, rsrc, nel, n_wg, S.SHM_REDUCE_DUPLICATE))
        out[f"reduce_duplicate_wg{n_wg}"] = {"ms": ms, "algorithmic_gbs": dup_bytes / ms / 1e6, "frac_hbm": dup_bytes / ms / 1e6 / HBM_PEAK_GBS}
        ms = best_of(lambda: g.launch_reduce_sum_f32(rdst, rsrc, nel, n_wg, S.SHM_REDUCE_SPLIT))
        out[f"reduce_split_wg{n_wg}"] = {"ms": ms, "algorithmic_gbs": spl_bytes / ms / 1e6, "frac_hbm": spl_bytes / ms / 1e6 / HBM_PEAK_GBS}
    for off in (fsrc, fdst, rsrc, rdst):
        g.free(off)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--size-mib", type=int, default=256, help="message size per PE of the headline put")
    ap.add_argument("--n-wg", type=int, default=1024, help="work-groups per PE of the headline put")
    ap.add_argument("--sweep-max-mib", type=int, default=256)
    ap.add_argument("--no-extras", action="store_true", help="headline only (used for profiling runs)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (its PEs are logical partitions of that GPU's HBM); "
              "--gpus must be 1", file=sys.stderr)
        return 2

    import torch
    from paper_2409_20476_amd import shm as S, synth
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2

    g = S.Shm.on_torch(8, GiB)
    head, data0 = headline(torch, S, synth, g, args)
    log(f"[bench] headline: {head}")
    n = args.size_mib * MiB

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import shmem_oracle
        cpu = cpu_put_baseline(shmem_oracle, data0, n, args.n_wg)
        log(f"[bench] cpu baseline: {cpu}")
    del data0

    extras = {}
    if not args.no_extras:
        extras["config1_pingflag"] = pingflag(torch, S, synth, args)
        log(f"[bench] c1: {extras['config1_pingflag']}")
        extras["config2_put_sweep"] = put_sweep(torch, S, g, args)
        log(f"[bench] crossover: {extras['config2_put_sweep']['crossover_bytes']}")
        extras["config3_ring"] = ring(torch, S, synth, g, args)
        log(f"[bench] c3: {extras['config3_ring']}")
        extras["config4_amo_storm"] = storm(torch, S, synth, args)
        log(f"[bench] c4: {extras['config4_amo_storm']}")
        extras["config5_collectives"] = collectives(torch, S, synth, g, args)
        log(f"[bench] c5: {extras['config5_collectives']}")
    g.finalize()

    traffic = None
    tpath = os.path.join(ROOT, "profiles", "shmk_wg_rma_traffic.json")
    if os.path.exists(tpath) and args.size_mib == 256 and args.n_wg == 1024:
        with open(tpath) as f:
            traffic = json.load(f).get("hbm_bytes_per_launch")

    line = {
        "metric": "work-group put GB/s vs msg size (% of HBM copy roofline); AMO ops/s",
        "value": head["value_gbs"], "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["wall_ms"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": f"config 2: 8 logical PEs, work-group put of {args.size_mib} MiB float32 N(0,1) per PE to PE (p+1) mod 8, "
                               f"{args.n_wg} work-groups x 256 threads per PE, direct load/store, one team grid",
                   "pes": 8, "bytes_per_pe": n, "n_wg_per_pe": args.n_wg, "path": "ldst"},
        "value_note": "payload bytes delivered per second, all 8 PEs together; % of roofline counts read + written bytes",
        "pct_of_hbm_copy_roofline": 100.0 * 2 * head["value_gbs"] / HBM_PEAK_GBS,
        "spot_check_ok": head["spot_check_ok"],
        "roofline": {"bound": "hbm", "kernel": "shmk_wg_rma", "achieved": head["achieved_gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": head["achieved_gbs"] / HBM_PEAK_GBS, "traffic": traffic,
                     "algorithmic_bytes_per_launch": 2 * head["payload_bytes"], "kernel_ms": head["kernel_ms"]},
        "cpu_baseline": cpu,
    }
    if extras:
        if "config4_amo_storm" in extras:
            line["amo_ops_per_s"] = extras["config4_amo_storm"]["fetch_add"]["gops"] * 1e9
        line["extras"] = extras
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
