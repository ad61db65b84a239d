#!/usr/bin/env python3
"""Benchmark of the shm355 hot path on one MI355X.

Headline (the JSON line's `value`): configuration 2's work-group put -- 8 logical PEs, each
putting a 256 MiB float32 message to PE (p+1) mod 8 with 1024 work-groups of 256 threads through
direct loads/stores, launched as one grid on the team stream.  One step = one such put by all
eight PEs.  Inputs are seeded synthetic data resident in HBM before the timed region.

The LAST line of stdout is one compact JSON object (a few KB): the headline, `roofline` (the put
kernel against the HBM copy roofline, timed with HIP events on the stream it runs on),
`cpu_baseline` (the oracle's work-group put timed on this host, context only), `amo_ops_per_s`, and
`configs`, a short summary per configuration with the oracle's time beside each GPU figure.  The
full measurements (the put sweep over message sizes, work-group counts and transfer paths, the
ping/flag latency, the pipelined ring, the atomic storm, the collectives, the sweeps of the paper's
other experiments) go to a JSON file (`--extras-out`; see its default) and, in
short form, to stderr.
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
    # every delivered byte against its source, on the device (torch only compares), plus PE 1's first
    # and last 4 KiB against the host's copy of PE 0's seeded data
    H = g.heap_tensor.numel() // npes
    ok = all(torch.equal(g.heap_tensor[((p + 1) % npes) * H + dst:((p + 1) % npes) * H + dst + n],
                         g.heap_tensor[p * H + src:p * H + src + n]) for p in range(npes))
    ok = bool(ok and np.array_equal(g.read(1, dst, 4096), data0[:4096]) and
              np.array_equal(g.read(1, dst + n - 4096, 4096), data0[n - 4096:]))
    payload = npes * n
    res = {
        "wall_ms": wall_ms, "kernel_ms": kern_ms, "payload_bytes": payload,
        "value_gbs": payload / wall_ms / 1e6,
        "achieved_gbs": 2 * payload / kern_ms / 1e6,
        "check_ok": ok, "kernel": "shmk_wg_rma_tiles",
    }
    g.free(src), g.free(dst)
    return res, data0


def best_of_3(fn):
    best = float("inf")
    for _ in range(3):
        t0 = time.perf_counter()
        fn()
        best = min(best, time.perf_counter() - t0)
    return best


def cpu_config_baselines(oracle_mod, synth):
    """The oracle, as it stands, timed on this host right after the GPU measurement of each
    configuration: one core (numpy copies and adds are single-threaded), best of 3, on a bounded
    sample of the configuration's workload.  Context only.  Returns {extra name: function}."""
    O = oracle_mod

    def c1():
        o = O.ShmemOracle(2, MiB)
        payload = synth.c1_payload(4096)
        n = payload.nbytes
        data, back, flag = o.malloc(n), o.malloc(n), o.calloc(8, 8)
        o.write(0, data, payload)

        def once():
            o.write(1, flag, np.zeros(8, np.uint8))
            o.wg_put(0, data, data, n, 1, 1)
            o.quiet(0)
            o.put_signal(0, data, data, 0, flag, 1, O.SIGNAL_SET, 1)
            o.signal_wait_until(1, flag, O.CMP_EQ, 1)
            o.wg_get(1, back, data, n, 0, 1)
        t = min(best_of_3(once) for _ in range(20))
        assert np.array_equal(o.read(1, back, n, np.int32), payload)
        return {"us": t * 1e6, "sample": "the whole configuration (16 KiB put, quiet, flag, wait, get back), best of 60"}

    def c3():
        npes, n_chunks, nel = 8, 8, 524288          # 8 of the 64 chunks per PE
        cb = 2 * nel
        o = O.ShmemOracle(npes, 2 * cb * n_chunks + 4 * nel + (1 << 16))
        src, slot, acc, sig = o.malloc(cb * n_chunks), o.malloc(cb * n_chunks), o.malloc(4 * nel), o.calloc(8, 8)
        for p in range(npes):
            o.write(p, src, synth.c3_chunks(p, n_chunks, nel))

        def once():
            for p in range(npes):
                o.write(p, sig, np.zeros(8, np.uint8))
            o.ring_pipeline(src, slot, sig, acc, cb, n_chunks, 32, 1)
        t = best_of_3(once)
        payload = npes * n_chunks * cb
        return {"ms_scaled_to_64_chunks": t * 1e3 * 64 / n_chunks, "payload_gbs": payload / t / 1e9,
                "sample": f"8 PEs x {n_chunks} of the 64 chunks of 1 MiB, best of 3"}

    def c4():
        npes, n_ctr, n_items, ops = 16, 1024, 1 << 17, 64     # 2^23 of the 2^26 operations
        o = O.ShmemOracle(npes, MiB)
        ctr = o.calloc(8 * n_ctr, 256)
        targets = synth.c4_targets(n_items, ops, npes, n_ctr)
        t = best_of_3(lambda: o.amo_storm(ctr, n_ctr, targets))
        return {"mops": n_items * ops / t / 1e6, "sample": f"{n_items * ops} of the 2^26 fetch-adds (array form of the oracle), best of 3"}

    def c5():
        npes, nel = 8, 2 * MiB                              # 2 Mi of the 16 Mi elements per PE
        o = O.ShmemOracle(npes, 4 * nel * (npes + 3) + (1 << 16))
        fsrc, fdst, rsrc, rdst = o.malloc(4 * nel), o.malloc(4 * nel * npes), o.malloc(4 * nel), o.malloc(4 * nel)
        for p in range(npes):
            o.write(p, fsrc, synth.c5_fcollect_source(p, nel))
            o.write(p, rsrc, synth.c5_reduce_source(p, nel))
        tf = best_of_3(lambda: o.fcollect(fdst, fsrc, 4 * nel))
        tr = best_of_3(lambda: o.reduce_sum_f32(rdst, rsrc, nel))
        scale = 16 * MiB / nel
        return {"fcollect_ms_scaled": tf * 1e3 * scale, "fcollect_algorithmic_gbs": (npes + npes * npes) * 4 * nel / tf / 1e9,
                "reduce_ms_scaled": tr * 1e3 * scale, "reduce_melems_per_s": nel / tr / 1e6,
                "sample": f"8 PEs x {nel >> 20} Mi of the 16 Mi elements, times scaled by {scale:g}, best of 3"}

    def wrap(fn):
        def run():
            r = fn()
            r.update({"cores": 1, "kind": "oracle", "host_logical_cpus": os.cpu_count()})
            return r
        return run
    return {"config1_pingflag": wrap(c1), "config3_ring": wrap(c3), "config4_amo_storm": wrap(c4), "config5_collectives": wrap(c5)}


def cpu_put_baseline(oracle_mod, data0, n, n_wg, budget_s=6.0):
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


def host_timed_trial(torch, g, launch_pe, npes, iters):
    """Host clock from the first enqueue to completion of everything on all PEs (what a caller of
    the library sees; also the only clock that covers copy-engine transfers, which are not in a
    stream)."""
    g.barrier_all()
    t0 = time.perf_counter()
    for _ in range(iters):
        for p in range(npes):
            launch_pe(p)
    g.barrier_all()
    return (time.perf_counter() - t0) * 1e3 / iters


def in_kernel_put_us(torch, S, g, npes, dst, src, n, n_wg, ticks, khz):
    """Microseconds per put as seen by the issuing kernel (device clock inside the kernel, no launch
    cost): every PE's kernel repeats its put `reps` times, all eight kernels overlapping."""
    def run(reps):
        ticks[:, 0] = -1          # UINT64_MAX
        ticks[:, 1] = 0
        torch.cuda.synchronize()
        for p in range(npes):
            g.launch_wg_put_timed(p, (p + 1) % npes, dst, src, n, n_wg, reps, ticks[p])
        g.barrier_all()
        t = ticks.cpu().numpy().astype(np.uint64)
        per_put = float(np.mean((t[:, 1] - t[:, 0]).astype(np.float64))) / reps / khz * 1e3
        span = float(t[:, 1].max() - t[:, 0].min()) / reps / khz * 1e3      # all PEs: first start to last end
        return per_put, span
    est = run(4)[0]
    reps = int(min(512, max(4, 300.0 / max(est, 0.05))))
    return min(run(reps) for _ in range(5))


def crossover_at_other_queue_count(queues):
    """The hardware-queue count is read when the HIP runtime initialises, so the crossover at the other
    count (8 PE streams on 4 queues run in two rounds; on 8 queues all at once) is measured by a child
    process running this file's sweep alone."""
    import subprocess
    cmd = [sys.executable, os.path.abspath(__file__), "--hw-queues", str(queues), "--extras", "config2_put_sweep", "--size-mib", "16",
           "--steps", "2", "--warmup", "1", "--no-cpu-baseline", "--no-other-queue-count", "--extras-out", ""]
    try:
        proc = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
        last = proc.stdout.strip().splitlines()[-1]
        return {"hip_hardware_queues": queues, "crossover_bytes": json.loads(last)["configs"]["c2"]["crossover_bytes_ldst_to_sdma_by_wg_per_pe"]}
    except Exception as e:          # the figure is an extra: its absence must not cost the headline
        log(f"[bench] crossover at {queues} hardware queues not measured: {e!r}")
        return None


def placement_spread(torch, S, g, args):
    """The team put at nine placements of the destination relative to the source (HBM channel
    hashing can make a copy's rate depend on it), at the headline size and at 64 MiB per PE:
    percent of the HBM copy roofline, HIP events."""
    npes = 8
    shifts = (0, 4096, 8192, 65536, MiB, MiB + 4096, 2 * MiB, 16 * MiB + 8192, 64 * MiB - 4096)
    out = {"note": "8 PEs x 1024 groups, destination = source + message size + shift"}
    g.set_team_sync(False)
    for n in (256 * MiB, 64 * MiB):
        region = g.malloc(2 * n + 64 * MiB)
        pcts = {}
        for sh in shifts:
            dst = region + n + sh
            ms = min(time_on_stream(torch, g.streams[0], lambda: g.launch_wg_put_all(1, dst, region, n, 1024, S.SHM_PATH_LDST), 5)
                     for _ in range(4))
            pcts[str(sh)] = 100.0 * 2 * npes * n / ms / 1e6 / HBM_PEAK_GBS
        g.free(region)
        v = sorted(pcts.values())
        suffix = "" if n == 256 * MiB else f"_{n // MiB}mib"
        out["pct_by_destination_shift_bytes" + suffix] = pcts
        out["pct_min_med_max" + suffix] = [v[0], v[len(v) // 2], v[-1]]
    # ... and at sixteen random placements (seeded; offsets in steps of 2 MiB, the last four of 64 KiB) anywhere in a
    # 1000 MiB region, for the form the launcher takes for 128 groups per PE or more (pieces by ticket) and the one it takes for fewer (127: group-owned tiles)
    import random
    rnd = random.Random(20476)
    span = 1000 * MiB
    region = g.malloc(span)
    for n in (256 * MiB, 64 * MiB):
        rows = {"tickets_wg1024": [], "tiles_wg127": []}
        for k in range(16):
            gran = 2 * MiB if k < 12 else 64 * 1024
            while True:
                so, do = (rnd.randrange(0, (span - n) // gran) * gran for _ in range(2))
                if so + n <= do or do + n <= so:
                    break
            for key, n_wg in (("tickets_wg1024", 1024), ("tiles_wg127", 127)):
                ms = min(time_on_stream(torch, g.streams[0],
                                        lambda: g.launch_wg_put_all(1, region + do, region + so, n, n_wg, S.SHM_PATH_LDST), 4) for _ in range(3))
                rows[key].append(100.0 * 2 * npes * n / ms / 1e6 / HBM_PEAK_GBS)
        out[f"random_placements_pct_min_mean_max_{n // MiB}mib"] = {k: [min(v), sum(v) / len(v), max(v)] for k, v in rows.items()}
    # ... and at byte addresses off the 1 KiB boundaries the buffers above lie on (128 MiB per PE): destination and
    # source the same number of bytes past a boundary, the destination alone, and the two 8 bytes apart
    odd = {}
    n = 128 * MiB
    for key, da, sa in (("on_boundaries", 0, 0), ("both_8_bytes_past", 8, 8), ("both_16_bytes_past", 16, 16), ("dst_16_bytes_past", 16, 0),
                        ("dst_256_bytes_past", 256, 0), ("src_16_bytes_past", 0, 16), ("8_bytes_apart", 8, 0)):
        ms = min(time_on_stream(torch, g.streams[0],
                                lambda: g.launch_wg_put_all(1, region + 512 * MiB + da, region + sa, n, 1024, S.SHM_PATH_LDST), 4) for _ in range(3))
        odd[key] = 100.0 * 2 * npes * n / ms / 1e6 / HBM_PEAK_GBS
    out["odd_addresses_pct_128mib"] = odd
    # ... and whether repeating a transfer on the same buffers flatters it: the same put through buffer pairs taken
    # in turn (7 pairs of 64 MiB, 3 of 128 MiB: 0.9-1.8 GiB per PE round before a byte is touched again, against a
    # memory-side cache of 256 MiB) beside the put repeated on one pair
    fresh = {}
    for n in (64 * MiB, 128 * MiB):
        pairs = span // (2 * n)
        for key, n_wg in (("tickets_wg1024", 1024), ("tiles_wg127", 127)):
            def same():
                g.launch_wg_put_all(1, region + n, region, n, n_wg, S.SHM_PATH_LDST)

            def in_turn():
                for i in range(pairs):
                    g.launch_wg_put_all(1, region + (2 * i + 1) * n, region + 2 * i * n, n, n_wg, S.SHM_PATH_LDST)
            ms_same = min(time_on_stream(torch, g.streams[0], same, 2 * pairs) for _ in range(3))
            ms_turn = min(time_on_stream(torch, g.streams[0], in_turn, 2) for _ in range(3)) / pairs
            fresh[f"{key}_{n // MiB}mib"] = {"same_pair_pct": 100.0 * 2 * npes * n / ms_same / 1e6 / HBM_PEAK_GBS,
                                             "pairs_in_turn_pct": 100.0 * 2 * npes * n / ms_turn / 1e6 / HBM_PEAK_GBS, "pairs": pairs}
    out["fresh_buffers"] = fresh
    g.free(region)
    g.set_team_sync(True)
    return out


def hbm_ceilings(torch, S, g, args):
    """One-direction and copy ceilings of this chip measured with the library's own access forms
    (16-byte nontemporal loads and stores in the launch shape of the headline put): what a kernel
    that only reads, only writes, or copies can reach."""
    npes, n = 8, 256 * MiB
    a, b = g.malloc(n), g.malloc(n)
    g.set_team_sync(False)
    out = {}

    def probe(kind, n_wg):
        return min(time_on_stream(torch, g.streams[0], lambda: g.launch_stream_probe(kind, b, a, n, n_wg), 5) for _ in range(5))

    # each direction in three access orders: group-owned tiles, a front that sweeps the block, and the put's own walk
    # (32 KiB pieces by ticket); the best one is that direction's ceiling
    for name, kinds in (("read_only", (("tiles", S.SHM_PROBE_READ, (1024,)), ("front", S.SHM_PROBE_READ_FRONT, (64, 256, 1024)),
                                       ("tickets", S.SHM_PROBE_READ_TICKETS, (128,)))),
                        ("write_only", (("tiles", S.SHM_PROBE_WRITE, (1024,)), ("front", S.SHM_PROBE_WRITE_FRONT, (64, 256, 1024)),
                                        ("tickets", S.SHM_PROBE_WRITE_TICKETS, (128,))))):
        forms = {f"{form}_wg{w}": probe(kind, w) for form, kind, wgs in kinds for w in wgs}
        best = min(forms, key=forms.get)
        ms = forms[best]
        out[name] = {"ms": ms, "gbs": npes * n / ms / 1e6, "frac_hbm": npes * n / ms / 1e6 / HBM_PEAK_GBS, "form": best,
                     "frac_hbm_by_form": {k: npes * n / v / 1e6 / HBM_PEAK_GBS for k, v in forms.items()}}
    ms = probe(S.SHM_PROBE_COPY, 1024)
    out["copy"] = {"ms": ms, "gbs": 2 * npes * n / ms / 1e6, "frac_hbm": 2 * npes * n / ms / 1e6 / HBM_PEAK_GBS}
    g.set_team_sync(True)
    g.free(a), g.free(b)
    r, w = out["read_only"]["gbs"], out["write_only"]["gbs"]
    return {"kernels": out, "copy_bus_time_limit_frac_hbm": 2.0 / (1.0 / r + 1.0 / w) / HBM_PEAK_GBS,
            "note": "8 PEs x 256 MiB; read_only / write_only: the best of three access orders (group-owned 64 KiB tiles; a front of "
                    "n_wg x 4 KiB per PE sweeping the block; the put's own walk, 32 KiB pieces by ticket); copy = the put itself; copy_bus_time_limit = "
                    "2 / (1/read + 1/write): a copy whose reads and writes share the bus without overlapping or disturbing each other"}


def put_sweep(torch, S, g, args):
    """Configuration 2: message sizes 8 B .. 256 MiB, 8 PEs concurrently, each on its own stream
    (or engine), through loads/stores with 1, 4, 64, 1024 work-groups, through the SDMA copy
    engines, and through hipMemcpyAsync (a runtime copy kernel on one device)."""
    npes = 8
    max_n = args.sweep_max_mib * MiB
    src, dst = g.malloc(max_n), g.malloc(max_n)
    sizes = [1 << k for k in range(3, 29) if (1 << k) <= max_n]
    ticks = torch.zeros((npes, 2), dtype=torch.int64, device="cuda")
    khz = g.wall_clock_khz()
    rows = []
    wgs = (1, 4, 64, 1024)
    never = (1 << 64) - 1
    defaults = {str(w): (None if g.get_cutover(w) >= never else g.get_cutover(w)) for w in wgs}     # before the sweep retunes them
    for n in sizes:
        row = {"bytes": n}
        for n_wg in wgs:
            us, span = in_kernel_put_us(torch, S, g, npes, dst, src, n, n_wg, ticks, khz)
            row[f"ldst_wg{n_wg}_us"], row[f"ldst_wg{n_wg}_gbs"] = us, npes * n / span / 1e3
            launch = lambda p: g.launch_wg_put(p, (p + 1) % npes, dst, src, n, n_wg, S.SHM_PATH_LDST)
            ms = paper_timing(torch, lambda iters: host_timed_trial(torch, g, launch, npes, iters))
            row[f"ldst_wg{n_wg}_host_us"] = ms * 1e3
        for key, path in (("sdma", S.SHM_PATH_SDMA), ("memcpy", S.SHM_PATH_MEMCPY)):
            launch = lambda p: g.launch_wg_put(p, (p + 1) % npes, dst, src, n, 1, path)
            ms = paper_timing(torch, lambda iters: host_timed_trial(torch, g, launch, npes, iters))
            row[key + "_us"], row[key + "_gbs"] = ms * 1e3, npes * n / ms / 1e6
        rows.append(row)
        log("[sweep] " + " ".join(f"{k}={v:.4g}" if isinstance(v, float) else f"{k}={v}" for k, v in row.items() if k.endswith("_gbs") or k == "bytes"))
    # team-launch curve for the largest work-group count (one grid for all PEs)
    g.set_team_sync(False)
    for row in rows:
        n = row["bytes"]
        ms = paper_timing(torch, lambda iters: time_on_stream(
            torch, g.streams[0], lambda: g.launch_wg_put_all(1, dst, src, n, 1024, S.SHM_PATH_LDST), iters))
        row["team_wg1024_event_us"], row["team_wg1024_event_gbs"] = ms * 1e3, npes * n / ms / 1e6
    # the get of the same shape at the largest size: every PE reads its neighbour's block
    n = rows[-1]["bytes"]
    ms = paper_timing(torch, lambda iters: time_on_stream(
        torch, g.streams[0], lambda: g.launch_wg_get_all(1, dst, src, n, 1024, S.SHM_PATH_LDST), iters))
    team_get = {"bytes": n, "us": ms * 1e3, "gbs": npes * n / ms / 1e6, "frac_hbm": 2 * npes * n / ms / 1e6 / HBM_PEAK_GBS}
    g.set_team_sync(True)

    def crossover(faster):
        for i, row in enumerate(rows):
            if all(faster(r) for r in rows[i:]):
                return row["bytes"]
        return None

    # all 8 PEs transfer at once: compare what they move together per second, either way
    cross_dev = {str(w): crossover(lambda r, w=w: r["sdma_gbs"] >= r[f"ldst_wg{w}_gbs"]) for w in wgs}
    cross_one = {str(w): crossover(lambda r, w=w: r["sdma_us"] <= r[f"ldst_wg{w}_us"]) for w in wgs}
    cross_host = {str(w): crossover(lambda r, w=w: r["sdma_us"] <= r[f"ldst_wg{w}_host_us"]) for w in wgs}
    for w in wgs:
        c = cross_dev[str(w)]
        g.set_cutover(w, c if c is not None else (1 << 64) - 1)
    auto = [{"bytes": r["bytes"], **{f"wg{w}": ("sdma" if g.choose_path(r["bytes"], w) == S.SHM_PATH_SDMA else "ldst") for w in wgs}}
            for r in rows]
    g.free(src), g.free(dst)
    placement = placement_spread(torch, S, g, args) if max_n >= 256 * MiB else None
    queues = int(os.environ.get("GPU_MAX_HW_QUEUES", "4"))
    other = None
    if not args.no_other_queue_count:
        other = crossover_at_other_queue_count(8 if queues < 8 else 4)
    return {"pes": npes, "hip_hardware_queues": queues, "library_default_cutover_bytes": defaults,
            "crossover_other_queue_count": other, **({"placement": placement} if placement else {}),
            "timing": "8 PEs concurrently. ldst_wgK_us: device clock inside the issuing kernel, per put incl. its quiet, mean over "
                      "PEs (a put issued from a running kernel, as in the paper's experiment; ldst_wgK_gbs uses the span from "
                      "the first PE's start to the last PE's end); ldst_wgK_host_us, sdma_us, memcpy_us: host "
                      "clock from first enqueue to completion on all PEs, warm-up doubling to >2 ms then best of 10; "
                      "team_wg1024_event_us: HIP events around one grid for all PEs; gbs = payload of all 8 PEs",
            "rows": rows, "team_get_wg1024_event": team_get, "crossover_bytes": cross_dev, "crossover_bytes_one_pe_kernel_time": cross_one,
            "crossover_bytes_host_launched": cross_host, "auto_path": auto,
            "crossover_note": "smallest message from which the SDMA copy engines stay at least as fast as loads/stores by that "
                              "many work-groups per PE, all 8 PEs transferring at once. crossover_bytes compares the bytes all "
                              "PEs move per second (SDMA: host submit to completion of all; loads/stores: first kernel start "
                              "to last kernel end on the device); _one_pe_kernel_time compares the engines' completion "
                              "time with ONE PE's in-kernel put time; _host_launched with host-launched put kernels. "
                              "null = loads/stores win at every measured size"}


def reverse_offload(torch, S, args):
    """The paper's reverse-offload ring and its cutover experiment: round trip and request rate of the
    ring, and one work-group (64 / 256 / 1024 work-items) putting 8 B .. 128 MiB from inside a kernel,
    once with loads/stores and once by asking the host proxy for a copy engine."""
    g = S.Shm.on_torch(2, 512 * MiB)
    g.proxy_start()
    khz = g.wall_clock_khz()
    t = torch.zeros(2, dtype=torch.int64, device="cuda")

    def timed(launch):
        t[0], t[1] = -1, 0
        torch.cuda.synchronize()
        launch()
        g.quiet(0)
        a, b = (int(v) & ((1 << 64) - 1) for v in t.tolist())
        return (b - a) / khz * 1e3

    out = {"round_trip_us": {}, "request_rate_mreq_s": {}}
    for n_wg in (1, 8, 64):
        out["round_trip_us"][str(n_wg)] = min(timed(lambda: g.launch_offload_nop(0, n_wg, 500, True, t)) for _ in range(3)) / 500
    for n_wg in (1, 8, 64, 256):
        out["request_rate_mreq_s"][str(n_wg)] = max(n_wg * 2001 / timed(lambda: g.launch_offload_nop(0, n_wg, 2000, False, t))
                                                    for _ in range(3))
    src, dst = g.malloc(128 * MiB), g.malloc(128 * MiB)
    rows = []
    for k in range(3, 28):
        n = 1 << k
        row = {"bytes": n}
        reps = 4 if n >= 8 * MiB else 20
        for wg in (1, 16, 64, 128, 256, 1024):
            if wg < 64 and n > (4 * MiB if wg == 16 else MiB):
                continue                       # a few lanes move 0.3-4 GB/s: the curve is flat long before this
            row[f"ldst_wi{wg}_us"] = min(timed(lambda: g.launch_put_device_initiated(0, 1, dst, src, n, 1, 0, 0, reps, t, wg))
                                         for _ in range(3)) / reps
        row["engine_us"] = min(timed(lambda: g.launch_put_device_initiated(0, 1, dst, src, n, 1, 1, 0, reps, t, 256))
                               for _ in range(3)) / reps
        rows.append(row)
    cross = {}
    for wg in (1, 16, 64, 128, 256, 1024):
        key = f"ldst_wi{wg}_us"
        have = [r for r in rows if key in r]           # the few-lane curves stop early; sizes beyond are the engine's
        cross[str(wg)] = next((r["bytes"] for i, r in enumerate(have) if all(q["engine_us"] <= q[key] for q in have[i:])), None)
    # the cutover taken inside the kernel, with the threshold just measured for 256 work-items
    cut = cross["256"] or (1 << 62)
    for row in rows:
        n = row["bytes"]
        reps = 4 if n >= 8 * MiB else 20
        row["auto_wi256_us"] = min(timed(lambda: g.launch_put_device_initiated(0, 1, dst, src, n, 1, 2, cut, reps, t, 256))
                                   for _ in range(3)) / reps
    requests, copies = g.proxy_stats()
    g.proxy_stop()
    g.finalize()
    out.update({"single_group_put": rows, "cutover_bytes_by_work_items": cross, "proxy_requests": requests, "proxy_copies": copies,
                "note": "device clock inside the kernel, per put including completion (loads/stores: group quiet; engine: the "
                        "host's completion message); round trips: one wave per group waiting for each answer; rate: "
                        "fire-and-forget, one host thread"})
    return out


def single_thread_and_strided(torch, S, args):
    """The paper's first experiment (put/get called by ONE work-item, bandwidth against size; here to
    the caller's own partition and to another PE's), the strided forms, the get through the ring, and
    the transfer whose first bytes go by loads/stores while the copy engine starts."""
    g = S.Shm.on_torch(2, 512 * MiB)
    g.proxy_start()
    khz = g.wall_clock_khz()
    t = torch.zeros(2, dtype=torch.int64, device="cuda")

    def timed(launch):
        t[0], t[1] = -1, 0
        torch.cuda.synchronize()
        launch()
        g.quiet(0)
        a, b = (int(v) & ((1 << 64) - 1) for v in t.tolist())
        return (b - a) / khz * 1e3

    src, dst = g.malloc(128 * MiB), g.malloc(128 * MiB)
    out = {}
    rows = []
    for k in range(3, 23):
        n = 1 << k
        reps = max(1, min(50, (1 << 20) // n))
        row = {"bytes": n}
        for name, pe, is_get in (("put_other_pe", 1, False), ("get_other_pe", 1, True), ("put_same_pe", 0, False)):
            us = min(timed(lambda: g.launch_thread_rma(0, pe, dst, src, n, is_get, reps, t)) for _ in range(3)) / reps
            row[f"{name}_us"] = us
            row[f"{name}_gbs"] = n / us / 1e3
        rows.append(row)
    out["one_work_item"] = rows
    # strided: 4 Mi elements moved by 64 groups (host clock on the stream: whole launch)
    strided = []
    nel = 1 << 20
    for elem in (4, 16):
        for ds, ss in ((1, 1), (2, 1), (1, 2), (4, 4), (16, 16)):
            for name, fn in (("iput", g.launch_iput), ("iget", g.launch_iget)):
                best = float("inf")
                for i in range(5):
                    e0, e1 = event_pair(torch)
                    torch.cuda.synchronize()
                    e0.record(g.streams[0])
                    fn(0, 1, dst, src, ds, ss, nel, elem, 64)
                    e1.record(g.streams[0])
                    g.quiet(0)
                    if i:
                        best = min(best, e0.elapsed_time(e1) * 1e3)
                strided.append({"op": name, "elem_bytes": elem, "dst_stride": ds, "src_stride": ss, "elements": nel, "us": best,
                                "payload_gbs": nel * elem / best / 1e3})
    out["strided_64_groups"] = strided
    # one group of 256: get by loads/stores, by the engine, and the covered put/get against both
    rows = []
    for k in range(16, 28):
        n = 1 << k
        reps = 4 if n >= 8 * MiB else 10
        row = {"bytes": n}
        for name, is_get, mode, cover in (("put_ldst", False, 0, 0), ("put_engine", False, 1, 0), ("put_covered_256k", False, 4, 256 * 1024),
                                          ("put_covered_512k", False, 4, 512 * 1024), ("get_ldst", True, 0, 0), ("get_engine", True, 1, 0),
                                          ("get_nbi_quiet", True, 3, 0), ("get_covered_256k", True, 4, 256 * 1024)):
            row[f"{name}_us"] = min(timed(lambda: g.launch_rma_device_initiated(0, 1, dst, src, n, 1, is_get, mode, 0, cover,
                                                                                 S.SHM_NO_CONSUME, reps, t, 256))
                                    for _ in range(3)) / reps
        rows.append(row)
    out["one_group_256_work_items"] = rows
    g.proxy_stop()
    g.finalize()
    out["note"] = ("device clock inside the kernel; one work-item keeps 32 16-byte loads in flight, so its bandwidth is bytes in "
                   "flight over memory latency; covered = copy engine for all but the first 256/512 KiB, which the group moves "
                   "itself while the engine starts")
    return out


def collective_sweeps(torch, S, args):
    """The paper's collective experiments: fcollect against elements, work-groups and PEs with the
    host copy paths beside it; broadcast against the number of PEs; the device-side sync."""
    out = {"fcollect": {}, "broadcast_us_by_pes": {}, "sync_us_by_pes": {}, "barrier_us_by_pes": {}}
    t = torch.zeros(2, dtype=torch.int64, device="cuda")
    def host_path_us(g, launch):
        def trial(iters):
            g.barrier_all()
            t0 = time.perf_counter()
            for _ in range(iters):
                launch()
            g.barrier_all()
            return (time.perf_counter() - t0) * 1e3 / iters
        return paper_timing(torch, trial) * 1e3

    def sweep(g, launch, sizes):
        """launch(n, n_wg, path); per size the three group counts by loads/stores and the two host-started paths."""
        rows = []
        for n in sizes:
            row = {"bytes_per_pe": n}
            for n_wg in (1, 4, 64):
                ms = paper_timing(torch, lambda iters: time_on_stream(torch, g.streams[0], lambda: launch(n, n_wg, S.SHM_PATH_LDST), iters))
                row[f"ldst_wg{n_wg}_us"] = ms * 1e3
            row["memcpy_us"] = host_path_us(g, lambda: launch(n, 1, S.SHM_PATH_MEMCPY))
            row["sdma_us"] = host_path_us(g, lambda: launch(n, 1, S.SHM_PATH_SDMA))
            for n_wg in (1, 4, 64):      # the tuned collective: the library's own choice, host clock
                row[f"auto_wg{n_wg}_us"] = host_path_us(g, lambda: launch(n, n_wg, S.SHM_PATH_AUTO))
            rows.append(row)
        cut = {}
        for n_wg in (1, 4, 64):
            key = f"ldst_wg{n_wg}_us"
            cut[str(n_wg)] = next((r["bytes_per_pe"] for i, r in enumerate(rows)
                                   if all(min(q["memcpy_us"], q["sdma_us"]) <= q[key] for q in rows[i:])), None)
        return {"rows": rows, "cutover_bytes_per_pe": cut}

    out["broadcast"] = {}
    for npes in (4, 8, 12):
        g = S.Shm.on_torch(npes, 512 * MiB)
        g.set_team_sync(False)
        src, dst = g.malloc(16 * MiB), g.malloc(16 * MiB * npes)
        out["fcollect"][str(npes)] = sweep(g, lambda n, n_wg, path: g.launch_fcollect(dst, src, n, n_wg, path), [1 << k for k in range(4, 25)])
        out["broadcast"][str(npes)] = sweep(g, lambda n, n_wg, path: g.launch_broadcast(dst, src, n, 0, n_wg, path),
                                            [1 << k for k in range(10, 25, 2)])
        g.finalize()
    for npes in (2, 4, 8, 12, 16):
        g = S.Shm.on_torch(npes, 64 * MiB)
        g.set_team_sync(False)
        src, dst = g.malloc(MiB), g.malloc(MiB)
        out["broadcast_us_by_pes"][str(npes)] = {
            str(n): paper_timing(torch, lambda iters: time_on_stream(
                torch, g.streams[0], lambda: g.launch_broadcast(dst, src, n, 0, 2, S.SHM_PATH_LDST), iters)) * 1e3
            for n in (4096, 65536, MiB)}
        for key, quiet in (("sync_us_by_pes", 0), ("barrier_us_by_pes", 1)):
            best = float("inf")
            for _ in range(3):
                t[0], t[1] = -1, 0
                torch.cuda.synchronize()
                g.launch_sync_all(200, quiet, t)
                g.barrier_all()
                a, b = (int(v) & ((1 << 64) - 1) for v in t.tolist())
                best = min(best, (b - a) / g.wall_clock_khz() * 1e3 / 200)
            out[key][str(npes)] = best
        g.finalize()
    # host time per small team launch under the three ways of ordering it against the PE streams
    out["team_launch_host_us"] = {}
    for npes in (2, 8, 16):
        g = S.Shm.on_torch(npes, 8 * MiB)
        src, dst = g.malloc(4096), g.malloc(4096 * npes)
        row = {}
        for name, mode in (("full", S.SHM_TEAM_SYNC_FULL), ("tracked", S.SHM_TEAM_SYNC_TRACKED), ("off", S.SHM_TEAM_SYNC_OFF)):
            g.set_team_sync(mode)
            for _ in range(50):
                g.launch_fcollect(dst, src, 64, 1)
            g.barrier_all()
            t0 = time.perf_counter()
            for _ in range(1000):
                g.launch_fcollect(dst, src, 64, 1)
            g.barrier_all()
            row[name] = (time.perf_counter() - t0) / 1000 * 1e6
        out["team_launch_host_us"][str(npes)] = row
        g.finalize()
    out["note"] = ("fcollect / broadcast: ldst_wgK_us = one grid with K groups of 256 threads per PE (root only for broadcast; HIP events, "
                   "launch included); memcpy_us / sdma_us = npes^2 (broadcast: npes) host-started copies, host clock; auto_wgK_us = "
                   "SHM_PATH_AUTO with the library's per-collective thresholds, host clock; cutover = smallest block from which a host "
                   "copy path stays at least as fast. broadcast_us_by_pes: root PE 0, 2 groups (the paper uses 128 work-items). "
                   "sync / barrier: device clock inside one kernel of npes groups, per operation. team_launch_host_us: host time per fcollect of "
                   "64 bytes in a loop of 1000, by team sync mode and number of PEs")
    return out


def graph_replay(torch, S, args):
    """Launch-bound loops recorded once as a HIP graph: 64 small puts issued one by one and as one replay."""
    g = S.Shm.on_torch(2, 64 * MiB)
    src, dst = g.malloc(MiB), g.malloc(MiB)
    out = {}
    for n, n_wg in ((8, 1), (4096, 1), (65536, 4)):
        count = 64
        issue = lambda: [g.launch_wg_put(0, 1, dst, src, n, n_wg) for _ in range(count)]
        eager_us = paper_timing(torch, lambda iters: time_on_stream(torch, g.streams[0], issue, iters)) * 1e3 / count
        graph = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=g.streams[0]):
            issue()
        torch.cuda.synchronize()

        def replay_trial(iters):
            e0, e1 = event_pair(torch)
            with torch.cuda.stream(g.streams[0]):
                e0.record()
                for _ in range(iters):
                    graph.replay()
                e1.record()
            e1.synchronize()
            return e0.elapsed_time(e1) / iters
        replay_us = paper_timing(torch, replay_trial) * 1e3 / count
        out[f"{n}B_wg{n_wg}"] = {"eager_us_per_put": eager_us, "graph_us_per_put": replay_us}
        del graph
    g.finalize()
    out["note"] = "64 work-group puts PE 0 -> PE 1 on one stream; eager = 64 launches, graph = one replay of the recorded 64"
    return out


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
    src, slot, acc, sig = g.malloc(cb * n_chunks), g.malloc(cb * n_chunks), g.malloc(4 * nel), g.calloc(8 * 64, 8)
    for p in range(npes):
        g.write(p, src, synth.c3_chunks(p, n_chunks, nel))
    zero = np.zeros(8 * 64, np.uint8)
    out = {}
    g.set_team_sync(False)      # all PE streams are idle here; time the grid, not the stream join/fork events
    for n_prod, n_cons, n_sig in ((8, 32, 1), (16, 32, 1), (32, 32, 1), (32, 32, 32), (64, 64, 64)):
        best = float("inf")
        for i in range(12):
            for p in range(npes):
                g.write(p, sig, zero)
            torch.cuda.synchronize()
            e0, e1 = event_pair(torch)
            e0.record(g.streams[0])
            g.launch_ring_pipeline(src, slot, sig, acc, cb, n_chunks, n_prod, n_cons, n_sig)
            e1.record(g.streams[0])
            g.barrier_all()
            if i >= 2:
                best = min(best, e0.elapsed_time(e1))
        algo = npes * (n_chunks * 3 * cb + 4 * nel)
        out[f"prod{n_prod}_cons{n_cons}_sig{n_sig}"] = {"ms": best, "payload_gbs": npes * n_chunks * cb / best / 1e6,
                                           "algorithmic_gbs": algo / best / 1e6, "frac_hbm": algo / best / 1e6 / HBM_PEAK_GBS}
    g.set_team_sync(True)
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
    g.set_team_sync(False)
    returning = (S.SHM_STORM_FETCH_ADD, S.SHM_STORM_FETCH_ADD_WG)
    for name, kind in (("fetch_add", S.SHM_STORM_FETCH_ADD), ("add_no_return", S.SHM_STORM_ADD),
                       ("plain_store_ceiling", S.SHM_STORM_PLAIN_STORE), ("fetch_add_batched_by_work_group", S.SHM_STORM_FETCH_ADD_WG)):
        best = float("inf")
        for i in range(7):
            torch.cuda.synchronize()
            e0, e1 = event_pair(torch)
            e0.record(g.streams[0])
            g.launch_amo_storm(ctr, n_ctr, targets, n_items, ops, kind, None, checksum if kind in returning else None)
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
    g.set_team_sync(False)      # streams are idle; the MEMCPY and SDMA forms below order themselves with barrier_all

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
    for n_wg in (32, 256, 1024):           # 32 groups per PE = one group per compute unit
        ms = best_of(lambda: g.launch_fcollect(fdst, fsrc, 4 * nel, n_wg, S.SHM_PATH_LDST))
        out[f"fcollect_ldst_wg{n_wg}"] = {"ms": ms, "algorithmic_gbs": fc_bytes / ms / 1e6, "frac_hbm": fc_bytes / ms / 1e6 / HBM_PEAK_GBS}
    sd_bytes = 2 * npes * npes * 4 * nel
    for key, path, note in (("fcollect_memcpy", S.SHM_PATH_MEMCPY, "64 runtime copies of 64 MiB on the 8 PE streams, host clock: "
                                                                   "8 GiB of traffic for the same result"),
                            ("fcollect_sdma", S.SHM_PATH_SDMA, "64 SDMA engine copies of 64 MiB, host clock")):
        best = float("inf")
        for i in range(4):
            g.barrier_all()
            t0 = time.perf_counter()
            g.launch_fcollect(fdst, fsrc, 4 * nel, 1024, path)
            g.barrier_all()
            if i >= 1:
                best = min(best, (time.perf_counter() - t0) * 1e3)
        out[key] = {"ms": best, "traffic_gbs": sd_bytes / best / 1e6, "note": note}
    dup_bytes = npes * npes * 4 * nel + npes * 4 * nel
    spl_bytes = npes * 4 * nel + npes * 4 * nel
    # The duplicate form loads every source npes times, but the npes readers of one share run side by
    # side on one XCD and all but the first are served by that L2: the kernel is bound by L2 hit
    # bandwidth, and what it must take from HBM is each source once plus the results (= spl_bytes).
    dup_note = "bound: l2 (npes loads per element, all but one served by the XCD's L2); frac_hbm_min_traffic = (each source once + results) / time / 8 TB/s"
    for n_wg in (256, 1024):
        ms = best_of(lambda: g.launch_reduce_sum_f32(rdst, rsrc, nel, n_wg, S.SHM_REDUCE_DUPLICATE))
        out[f"reduce_duplicate_wg{n_wg}"] = {"ms": ms, "bound": "l2", "algorithmic_load_store_gbs": dup_bytes / ms / 1e6,
                                             "frac_hbm_min_traffic": spl_bytes / ms / 1e6 / HBM_PEAK_GBS, "note": dup_note}
        ms = best_of(lambda: g.launch_reduce_sum_f32(rdst, rsrc, nel, n_wg, S.SHM_REDUCE_SPLIT))
        out[f"reduce_split_wg{n_wg}"] = {"ms": ms, "algorithmic_gbs": spl_bytes / ms / 1e6, "frac_hbm": spl_bytes / ms / 1e6 / HBM_PEAK_GBS}
    # the reduction matrix on the same 64 MiB per PE: one operator per element width (HBM-bound, so the
    # type only changes the arithmetic per byte)
    matrix = {}
    for name, dtype, op, width in (("uint8_xor", S.SHM_UINT8, S.SHM_OP_XOR, 1), ("int8_max", S.SHM_INT8, S.SHM_OP_MAX, 1),
                                   ("int16_sum", S.SHM_INT16, S.SHM_OP_SUM, 2), ("int32_sum", S.SHM_INT32, S.SHM_OP_SUM, 4),
                                   ("float32_sum", S.SHM_FLOAT32, S.SHM_OP_SUM, 4), ("float32_max", S.SHM_FLOAT32, S.SHM_OP_MAX, 4),
                                   ("int64_prod", S.SHM_INT64, S.SHM_OP_PROD, 8), ("float64_sum", S.SHM_FLOAT64, S.SHM_OP_SUM, 8)):
        ms = best_of(lambda: g.launch_reduce(rdst, rsrc, 4 * nel // width, dtype, op, 1024, S.SHM_REDUCE_DUPLICATE))
        ms2 = best_of(lambda: g.launch_reduce(rdst, rsrc, 4 * nel // width, dtype, op, 1024, S.SHM_REDUCE_SPLIT))
        matrix[name] = {"duplicate_ms": ms, "duplicate_frac_hbm_min_traffic": spl_bytes / ms / 1e6 / HBM_PEAK_GBS,
                        "split_ms": ms2, "split_frac_hbm": spl_bytes / ms2 / 1e6 / HBM_PEAK_GBS}
    out["reduce_matrix_wg1024"] = matrix
    g.set_team_sync(True)
    for off in (fsrc, fdst, rsrc, rdst):
        g.free(off)
    return out


def kernel_source_sha256():
    """Hash of the device sources every kernel is built from: a profile summary made for other
    sources says nothing about the kernels measured now."""
    import hashlib
    h = hashlib.sha256()
    for name in ("shm_device.hpp", "shm_kernels.hpp", "shm_release_algo.hpp"):
        with open(os.path.join(ROOT, "paper_2409_20476_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def traffic_from_profile(args):
    """HBM bytes per launch of the headline kernel from the committed rocprofv3 counter summary
    (FETCH_SIZE and WRITE_SIZE cannot be read from inside this process).  Reported only when the
    summary was made for the device sources as they are now; otherwise null."""
    tpath = os.path.join(ROOT, "profiles", "shmk_wg_rma_tiles_config2_256MiB_hbm_counters.txt")
    if not (os.path.exists(tpath) and args.size_mib == 256 and args.n_wg == 1024):
        return None, "not measured in this run"
    import re
    text = open(tpath).read()
    m = re.search(r"^hbm_bytes_per_launch:\s*(\d+)", text, re.M)
    sha = re.search(r"^kernel_source_sha256:\s*([0-9a-f]{64})", text, re.M)
    if not m or not sha or sha.group(1) != kernel_source_sha256():
        return None, "the committed counter summary was made for other kernel sources; not measured in this run"
    return int(m.group(1)), "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary under profiles/, made for these kernel sources (hash checked)"


def rnd(x, digits=4):
    """Short numbers for the compact line."""
    if isinstance(x, float):
        return float(f"{x:.{digits}g}")
    if isinstance(x, dict):
        return {k: rnd(v, digits) for k, v in x.items()}
    if isinstance(x, (list, tuple)):
        return [rnd(v, digits) for v in x]
    return x


def summarise(extras, cpu_legs):
    """One short entry per configuration for the compact line: the GPU figure, its fraction of the HBM
    roofline where that is the bound, and the oracle's time on this host beside it."""
    out = {}
    pct = lambda payload_gbs: 100.0 * 2 * payload_gbs / HBM_PEAK_GBS        # a copy reads and writes every byte
    if "config1_pingflag" in extras:
        r = extras["config1_pingflag"]
        out["c1"] = {"device_us": r["device_us"], "host_round_trip_us": r["host_round_trip_us"], "ok": r["ok"],
                     "cpu_oracle_us": cpu_legs.get("config1_pingflag", {}).get("us")}
    if "config2_put_sweep" in extras:
        r = extras["config2_put_sweep"]
        rows = {q["bytes"] >> 20: q for q in r["rows"] if q["bytes"] >= 64 * MiB}
        out["c2"] = {
            "pct_of_hbm_roofline_by_mib": {
                "team_grid_wg1024": {str(q["bytes"] >> 20): pct(q["team_wg1024_event_gbs"]) for q in r["rows"] if q["bytes"] >= 8 * MiB},
                "per_pe_streams_wg1024": {str(m): pct(8 * q["bytes"] / q["ldst_wg1024_host_us"] / 1e3) for m, q in rows.items()},
                "per_pe_streams_wg64": {str(m): pct(8 * q["bytes"] / q["ldst_wg64_host_us"] / 1e3) for m, q in rows.items()},
                "put_plus_quiet_inside_kernel_wg1024": {str(m): pct(q["ldst_wg1024_gbs"]) for m, q in rows.items()},
                "sdma_engines": {str(m): pct(q["sdma_gbs"]) for m, q in rows.items()},
            },
            "crossover_bytes_ldst_to_sdma_by_wg_per_pe": r["crossover_bytes"],
            "hip_hardware_queues": r["hip_hardware_queues"],
            "crossover_other_queue_count": r.get("crossover_other_queue_count"),
            "library_default_cutover_bytes": r.get("library_default_cutover_bytes"),
        }
        if "placement" in r:
            out["c2"]["placement_pct_min_med_max"] = r["placement"]["pct_min_med_max"]
            out["c2"]["placement_pct_min_med_max_64mib"] = r["placement"].get("pct_min_med_max_64mib")
            out["c2"]["same_pair_vs_pairs_in_turn_pct"] = {k: [v["same_pair_pct"], v["pairs_in_turn_pct"]]
                                                           for k, v in r["placement"].get("fresh_buffers", {}).items()}
            out["c2"]["odd_addresses_pct_128mib"] = r["placement"].get("odd_addresses_pct_128mib")
            out["c2"]["random_placements_pct_min_mean_max"] = {k.rsplit("_", 1)[1]: v for k, v in r["placement"].items()
                                                               if k.startswith("random_placements")}
    if "hbm_ceilings" in extras:
        hc = extras["hbm_ceilings"]
        out["hbm_ceilings_pct"] = {**{k: v["frac_hbm"] * 100 for k, v in hc["kernels"].items()},
                                   "copy_bus_time_limit": hc["copy_bus_time_limit_frac_hbm"] * 100,
                                   "forms": {k: v["form"] for k, v in hc["kernels"].items() if "form" in v}}
    if "config3_ring" in extras:
        r = extras["config3_ring"]
        shapes = {k: q for k, q in r.items() if k.startswith("prod")}
        best = min(shapes.values(), key=lambda q: q["ms"])
        cpu = cpu_legs.get("config3_ring", {})
        out["c3"] = {"ms": best["ms"], "frac_hbm": best["frac_hbm"], "payload_gbs": best["payload_gbs"],
                     "ms_by_shape": {k: q["ms"] for k, q in shapes.items()},
                     "cpu_oracle_ms_scaled": cpu.get("ms_scaled_to_64_chunks"), "cpu_oracle_payload_gbs": cpu.get("payload_gbs")}
    if "config4_amo_storm" in extras:
        r = extras["config4_amo_storm"]
        out["c4"] = {"fetch_add_gops": r["fetch_add"]["gops"], "ms": r["fetch_add"]["ms"],
                     "add_no_return_gops": r["add_no_return"]["gops"], "plain_store_ceiling_gops": r["plain_store_ceiling"]["gops"],
                     "batched_by_work_group_gops": r["fetch_add_batched_by_work_group"]["gops"],
                     "cpu_oracle_mops": cpu_legs.get("config4_amo_storm", {}).get("mops")}
    if "config5_collectives" in extras:
        r = extras["config5_collectives"]
        fc = min((v for k, v in r.items() if k.startswith("fcollect_ldst_wg")), key=lambda q: q["ms"])
        sp = min((v for k, v in r.items() if k.startswith("reduce_split_wg")), key=lambda q: q["ms"])
        du = min((v for k, v in r.items() if k.startswith("reduce_duplicate_wg")), key=lambda q: q["ms"])
        cpu = cpu_legs.get("config5_collectives", {})
        out["c5"] = {"fcollect_ms": fc["ms"], "fcollect_frac_hbm": fc["frac_hbm"],
                     "reduce_split_ms": sp["ms"], "reduce_split_frac_hbm": sp["frac_hbm"],
                     "reduce_duplicate_ms": du["ms"], "reduce_duplicate_bound": "l2",
                     "reduce_duplicate_frac_hbm_min_traffic": du["frac_hbm_min_traffic"],
                     "cpu_oracle_fcollect_ms_scaled": cpu.get("fcollect_ms_scaled"), "cpu_oracle_reduce_ms_scaled": cpu.get("reduce_ms_scaled")}
    if "reverse_offload" in extras:
        r = extras["reverse_offload"]
        out["reverse_offload"] = {"round_trip_us": r["round_trip_us"].get("1"), "mreq_per_s": max(r["request_rate_mreq_s"].values()),
                                  "in_kernel_cutover_bytes_by_work_items": r["cutover_bytes_by_work_items"]}
    return rnd(out)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--size-mib", type=int, default=256, help="message size per PE of the headline put")
    ap.add_argument("--n-wg", type=int, default=1024, help="work-groups per PE of the headline put")
    ap.add_argument("--sweep-max-mib", type=int, default=256)
    ap.add_argument("--no-extras", action="store_true", help="headline only (used for profiling runs)")
    ap.add_argument("--hw-queues", type=int, default=0,
                    help="set GPU_MAX_HW_QUEUES for this run, 1..32 (HIP's default is 4: the kernels of 8 PE streams then run in "
                         "two rounds and the per-PE curves of the sweep halve; 8 gives every PE stream a queue); 0 = leave the "
                         "environment as it is")
    ap.add_argument("--extras", default="all", help="comma-separated names of the extra measurements to run (default: all)")
    ap.add_argument("--extras-out", default=os.path.join(ROOT, "gpurun_out", "bench_extras.json"),
                    help="file that receives the full measurements as JSON ('' = do not write)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-queue-count", action="store_true",
                    help="do not start the child process that measures the crossover at the other hardware-queue count")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a plain 2 GiB tensor copy five times (reference reading for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (its PEs are logical partitions of that GPU's HBM); "
              "--gpus must be 1", file=sys.stderr)
        return 2
    if args.hw_queues and not 1 <= args.hw_queues <= 32:
        print("bench.py: --hw-queues must be 1..32", file=sys.stderr)
        return 2

    if args.hw_queues:       # read by the HIP runtime when it initialises, i.e. before torch touches the GPU
        os.environ["GPU_MAX_HW_QUEUES"] = str(args.hw_queues)
    from paper_2409_20476_amd import build as shm_build
    shm_build.ensure_built()            # loads what is built; compiles only if nothing is
    import torch
    from paper_2409_20476_amd import shm as S, synth
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2

    if args.calibration_copy:
        a = torch.zeros(2 * GiB, dtype=torch.uint8, device="cuda")
        b = torch.ones(2 * GiB, dtype=torch.uint8, device="cuda")
        for _ in range(5):
            a.copy_(b)
        torch.cuda.synchronize()
        del a, b
        torch.cuda.empty_cache()

    g = S.Shm.on_torch(8, GiB)
    head, data0 = headline(torch, S, synth, g, args)
    log(f"[bench] headline: {head}")
    n = args.size_mib * MiB

    cpu, cpu_fns, cpu_legs = None, {}, {}
    if not args.no_cpu_baseline:
        from oracle import shmem_oracle
        cpu = cpu_put_baseline(shmem_oracle, data0, n, args.n_wg)
        log(f"[bench] cpu baseline: {cpu}")
        cpu_fns = cpu_config_baselines(shmem_oracle, synth)
    del data0

    extras = {}
    table = [
        ("config1_pingflag", lambda: pingflag(torch, S, synth, args), lambda r: f"c1: {r}"),
        ("config2_put_sweep", lambda: put_sweep(torch, S, g, args), lambda r: f"crossover: {r['crossover_bytes']}"),
        ("hbm_ceilings", lambda: hbm_ceilings(torch, S, g, args), lambda r: f"ceilings: {r['kernels']}"),
        ("reverse_offload", lambda: reverse_offload(torch, S, args),
         lambda r: f"reverse offload: rtt {r['round_trip_us']} rate {r['request_rate_mreq_s']} cutover {r['cutover_bytes_by_work_items']}"),
        ("single_thread_and_strided", lambda: single_thread_and_strided(torch, S, args),
         lambda r: f"one work-item put GB/s: {[(q['bytes'], round(q['put_other_pe_gbs'], 3)) for q in r['one_work_item'][::4]]}"),
        ("collective_sweeps", lambda: collective_sweeps(torch, S, args),
         lambda r: f"sync us by PEs {r['sync_us_by_pes']} barrier {r['barrier_us_by_pes']} fcollect cutover "
                   f"{dict((k, v['cutover_bytes_per_pe']) for k, v in r['fcollect'].items())}"),
        ("graph_replay", lambda: graph_replay(torch, S, args), lambda r: f"graph replay: {r}"),
        ("config3_ring", lambda: ring(torch, S, synth, g, args), lambda r: f"c3: {r}"),
        ("config4_amo_storm", lambda: storm(torch, S, synth, args), lambda r: f"c4: {r}"),
        ("config5_collectives", lambda: collectives(torch, S, synth, g, args), lambda r: f"c5: {r}"),
    ]
    wanted = None if args.extras == "all" else set(args.extras.split(","))
    unknown = (wanted or set()) - {name for name, _, _ in table}
    if unknown:
        print(f"bench.py: unknown extras {sorted(unknown)}; known: {[name for name, _, _ in table]}", file=sys.stderr)
        return 2
    for name, run, describe in table:
        if args.no_extras or (wanted is not None and name not in wanted):
            continue
        extras[name] = run()
        log(f"[bench] {describe(extras[name])}")
        if name in cpu_fns:              # the oracle's time for the same configuration, right after the GPU's
            cpu_legs[name] = cpu_fns[name]()
            extras[name]["cpu_baseline"] = cpu_legs[name]
            log(f"[bench] {name} cpu baseline: {cpu_legs[name]}")
    g.finalize()

    traffic, traffic_source = traffic_from_profile(args)
    line = {
        "metric": "work-group put GB/s vs msg size (% of HBM copy roofline); AMO ops/s",
        "value": rnd(head["value_gbs"], 6), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": rnd(head["wall_ms"], 6),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": f"config 2: 8 logical PEs, work-group put of {args.size_mib} MiB float32 N(0,1) per PE to PE (p+1) mod 8, "
                               f"{args.n_wg} work-groups x 256 threads per PE, direct load/store, one team grid",
                   "pes": 8, "bytes_per_pe": n, "n_wg_per_pe": args.n_wg, "path": "ldst",
                   "hip_hardware_queues": int(os.environ.get("GPU_MAX_HW_QUEUES", "4"))},
        "value_note": "payload bytes delivered per second, all 8 PEs together; % of roofline counts read + written bytes",
        "pct_of_hbm_copy_roofline": rnd(100.0 * 2 * head["value_gbs"] / HBM_PEAK_GBS),
        "check_ok": head["check_ok"],
        "roofline": {"bound": "hbm", "kernel": head["kernel"], "achieved": rnd(head["achieved_gbs"], 6), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": rnd(head["achieved_gbs"] / HBM_PEAK_GBS), "traffic": traffic, "traffic_source": traffic_source,
                     "algorithmic_bytes_per_launch": 2 * head["payload_bytes"], "kernel_ms": rnd(head["kernel_ms"], 6)},
        "cpu_baseline": rnd(cpu) if cpu else None,
    }
    if extras:
        if "config4_amo_storm" in extras:
            line["amo_ops_per_s"] = rnd(extras["config4_amo_storm"]["fetch_add"]["gops"] * 1e9)       # the scalar device API
            line["amo_ops_per_s_batched_by_work_group"] = rnd(extras["config4_amo_storm"]["fetch_add_batched_by_work_group"]["gops"] * 1e9)
        line["configs"] = summarise(extras, cpu_legs)
        if args.extras_out:
            try:
                os.makedirs(os.path.dirname(args.extras_out) or ".", exist_ok=True)
                with open(args.extras_out, "w") as f:
                    json.dump({"headline": line, "extras": extras}, f)
                line["extras_file"] = os.path.relpath(args.extras_out, ROOT)
            except OSError as e:
                log(f"[bench] could not write {args.extras_out}: {e}")
    text = json.dumps(line, separators=(",", ":"))
    if len(text) > 6000:                 # the reader of this line keeps only the end of stdout
        line.pop("configs", None)
        line["configs_dropped"] = "summary too long; see extras_file"
        text = json.dumps(line, separators=(",", ":"))
    sys.stdout.flush()
    print(text, flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
