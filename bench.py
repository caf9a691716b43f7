#!/usr/bin/env python3
"""Throughput of the analyzer hot path on one MI355X.

A step = one pass of the whole path over one synthetic trace that is already
resident in HBM: ccld_ingest (device columns -> keyed window), ccld_analyze_window
(sort, per-collective statistics, flags, blame, Eq. 1-4 groups, hang alerts) and
ccld_rank_blame.  The default workload is the 4,096-rank trace (TP8 x PP8 x DP64,
20,000 collectives per rank, about 82M records) in a seeded random order.

Prints ONE JSON line with the records/s of the whole step, the roofline figures
of the dominant kernel (the radix-sort scatter pass, timed with HIP events on the
library's stream inside the timed region) and the CPU oracle's rate on a bounded
sample of the same trace.
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

HBM_PEAK_GBS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def kernel_sources_digest() -> str:
    """sha256 over the sources of the kernels the trace workload launches (ingest, sort, collectives,
    flags, blame, groups, alerts): the counters in profiles/ only describe these kernels."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2605_04478_amd", "csrc")
    for name in ("device_utils.h", "radix_sort.h", "radix_sort.hip", "select.h", "segments.hip", "window.hip",
                 "window_kernels.h"):
        h.update(name.encode())
        h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()


def measured_traffic(kernel: str):
    """HBM bytes per launch of `kernel` from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
    recorded in profiles/window_config3_traffic.json, or None if the kernels have changed since."""
    path = os.path.join(ROOT, "profiles", "window_config3_traffic.json")
    try:
        rec = json.load(open(path))
        if rec.get("csrc_sha256") != kernel_sources_digest():
            return None
        k = rec["kernels"].get(kernel)
        return None if k is None else k["fetch_bytes"] + k["write_bytes"]
    except (OSError, ValueError, KeyError):
        return None


def measured_step_traffic():
    """HBM bytes of one whole step (every kernel of the counter runs times its launches per step), or None if the
    kernels have changed since the counters were taken."""
    path = os.path.join(ROOT, "profiles", "window_config3_traffic.json")
    try:
        rec = json.load(open(path))
        if rec.get("csrc_sha256") != kernel_sources_digest():
            return None
        return sum((k["fetch_bytes"] + k["write_bytes"]) * k["launches"] for k in rec["kernels"].values())
    except (OSError, ValueError, KeyError):
        return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--cycles", type=int, default=2000, help="10-op cycles per rank (2000 = the 82M-record trace)")
    ap.add_argument("--no-shuffle", action="store_true", help="keep the generator's time-major record order")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-time-major", action="store_true",
                    help="skip the secondary figure on the generator's record order (keeps a profile to the timed steps)")
    ap.add_argument("--cpu-cycles", type=int, default=2000, help="cycles of the trace given to the CPU oracle")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--placement", choices=("sort", "dense"), default="sort",
                    help="how the timed steps bring a collective's records together (ccld_params.placement)")
    ap.add_argument("--host-batch", action="store_true",
                    help="also time two steps whose batch starts in pinned host memory (PCIe-inclusive rate)")
    ap.add_argument("--workload", choices=("trace", "stream", "hang", "rates", "frames"), default="trace",
                    help="trace: the 4,096-rank trace (default, the headline metric); stream: sliding window at "
                         "16,384 ranks, per-step latency; hang: hang location on 17M snapshot rows")
    ap.add_argument("--stream-steps", type=int, default=600)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (torch) so that rocprofv3 --pmc FETCH_SIZE / "
                         "WRITE_SIZE readings can be scaled by a kernel of known traffic")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this analyzer runs on ONE GPU (no sharding, no collectives); run it with --gpus 1")
        return 2

    import numpy as np
    import torch
    from paper_2605_04478_amd import ccld, tracegen as tg

    if not torch.cuda.is_available():
        log("bench.py: no GPU")
        return 2
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.workload == "stream":
        return bench_stream(args, torch, np, ccld, tg)
    if args.workload == "hang":
        return bench_hang(args, torch, np, ccld, tg)
    if args.workload == "rates":
        return bench_rates(args, torch, np, ccld, tg)
    if args.workload == "frames":
        return bench_frames(args, torch, np, ccld, tg)

    spec = tg.config3(n_cycles=args.cycles, seed=args.seed)
    t0 = time.time()
    tr = tg.generate(spec)
    n = tr.n
    log(f"generated {n} records ({spec.layout.n_ranks} ranks, {tr.topo.n_comms} communicators) in {time.time() - t0:.1f}s")

    an = ccld.Analyzer(tr.topo, max_window_records=n, device="cuda:0",
                       placement=ccld.PLACEMENT_DENSE if args.placement == "dense" else ccld.PLACEMENT_SORT)
    cols = an.to_device(tr.cols)
    cols_time_major = None
    if not args.no_shuffle:
        g = torch.Generator(device=dev)
        g.manual_seed(args.seed + 1)
        perm = torch.randperm(n, device=dev, generator=g)
        cols_time_major = cols          # kept for a secondary figure: the order a probe fleet would deliver
        cols = {k: v[perm].contiguous() for k, v in cols.items()}
        del perm
    torch.cuda.synchronize()
    now = int(tr.cols["t_exit"].max()) + 1
    n_seg_expected = n // 4 + 1024
    buffers = an.alloc_window_result(n, seg_cap=n_seg_expected, flag_cap=max(n // 8, 1 << 16),
                                     group_cap=min(an.n_comms * 1024, 1 << 22))
    # every result table stays in HBM (the counts come back with each call's status)
    blame_buffers = (torch.empty(5 * an.n_ranks, dtype=torch.int64, device=dev),
                     torch.empty(an.n_ranks, dtype=torch.int32, device=dev))
    log(f"workspace {an.workspace_bytes / 2**30:.2f} GiB; inputs resident in HBM")

    # Every step analyses operation counters the analyzer has not seen before (the counters of step i are
    # those of the trace plus i times the operations per rank), as successive windows of a running job do;
    # re-analysing one window would let the per-group watermarks skip work.  Up to twelve windows are kept
    # resident (warm-up, timed steps, the steps of the per-class table); longer runs cycle through them.
    n_windows = max(1, min(args.warmup + 2 * args.steps, 12))
    seq_windows = [cols["seq"] + i * spec.n_slots for i in range(n_windows)]
    step_no = [0]

    def step():
        w = dict(cols)
        w["seq"] = seq_windows[step_no[0] % n_windows]
        step_no[0] += 1
        an.reset_window()
        an.ingest(w)
        res = an.analyze_window(now, buffers=buffers)
        an.rank_blame(to_host=False, buffers=blame_buffers)
        return res

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)                  # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    res = None
    for _ in range(args.warmup):
        res = step()
    torch.cuda.synchronize()
    # the timed region carries events around the dominant kernel class only (a record costs about 9 us on
    # the stream); the per-class table comes from a second, untimed set of steps
    DOMINANT = "segments"
    an.profile_enable(True, only=DOMINANT)
    t_start = time.perf_counter()
    for _ in range(args.steps):
        res = step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t_start
    prof_timed, passes = an.profile_read()
    an.profile_enable(True)
    for _ in range(args.steps):
        res = step()
    torch.cuda.synchronize()
    prof, _ = an.profile_read()
    an.profile_enable(False)
    assert res is not None and res.status == "OK", res
    time_major_ms = None
    if cols_time_major is not None and not args.no_time_major:
        for timed in (False, True):
            torch.cuda.synchronize()
            t_t = time.perf_counter()
            for _ in range(2):
                an.reset_window()
                an.ingest(cols_time_major)
                r3 = an.analyze_window(now, buffers=buffers)
                an.rank_blame(to_host=False, buffers=blame_buffers)
            torch.cuda.synchronize()
            if timed:
                time_major_ms = (time.perf_counter() - t_t) / 2 * 1e3
        assert r3.status == "OK" and int(r3.n_flag) == int(res.n_flag)
    pcie = None
    if args.host_batch:
        # the same batch handed over as host arrays (pinned): the library stages it over PCIe first
        host = {}
        udt = {"rank": np.uint32, "comm": np.uint32, "seq": np.uint64, "op": np.uint8, "bytes": np.uint64,
               "t_enter": np.int64, "t_exit": np.int64}
        for k, v in cols.items():
            t = torch.empty(v.shape, dtype=v.dtype, pin_memory=True)
            t.copy_(v)
            host[k] = t.numpy().view(udt[k])          # the binding's dtypes: no copy out of the pinned pages
        torch.cuda.synchronize()
        t_h = time.perf_counter()
        for _ in range(2):
            an.reset_window()
            an.ingest(host)
            r2 = an.analyze_window(now, buffers=buffers)
            an.rank_blame(to_host=False, buffers=blame_buffers)
        torch.cuda.synchronize()
        pcie = n / ((time.perf_counter() - t_h) / 2)
        assert r2.status == "OK" and int(r2.n_flag) == int(res.n_flag)
        del host
    ms_per_step = dt / args.steps * 1e3
    value = n / (dt / args.steps)

    # Algorithmic HBM bytes per step of each kernel class (what the method has to move):
    #  ingest   reads the 41-byte SoA record, writes an 8-byte key and a 32-byte payload row
    #  hist     reads the 8-byte key once per pass
    #  scatter  pass 1 reads the key and writes key + index (20 B); later passes move key + index (24 B);
    #           when key bits + index bits <= 64 the passes move one packed word (16 B) and the last
    #           pass writes key + index (8 B in, 12 B out)
    #  seg_heads reads the sorted key once (collective heads per tile)
    #  segments reads key + index, gathers the 32-byte row, writes a 21-column int64 row per
    #           collective, its detection-group key and range (16 B) and one flag byte per record
    n_seg = int(res.n_seg)
    bl = lambda v: int(v).bit_length()
    # key = (communicator, operation counter, member slot inside the communicator)
    key_bits = bl(tr.topo.n_comms - 1) + bl(int(np.max(tr.topo.size)) - 1) + bl(int(tr.cols["seq"].max()))
    packed = passes >= 2 and key_bits + bl(n - 1) <= 64      # key and index travel as one 64-bit word
    scatter_bytes = (16.0 * (passes - 1) + 20.0) if packed else (20.0 + 24.0 * (passes - 1))
    alg = {"ingest": n * 81.0, "sort_hist": n * 8.0 * passes, "sort_scatter": n * scatter_bytes,
           "seg_heads": n * 8.0, "segments": n * (12.0 + 32.0 + 1.0) + n_seg * (21 * 8.0 + 16.0)}
    kernels = {k: {"ms_per_step": round(v[0] / args.steps, 4), "launches_per_step": v[1] / args.steps}
               for k, v in prof.items() if v[1]}
    for k, b in alg.items():
        if k in kernels and kernels[k]["ms_per_step"] > 0:
            kernels[k]["algorithmic_GBps"] = round(b / (kernels[k]["ms_per_step"] * 1e-3) / 1e9, 1)
    dominant = max(alg, key=lambda k: prof[k][0])
    # the dominant class as timed inside the timed region (falls back to the untimed table if another class
    # has overtaken it)
    d_ms, d_cnt = prof_timed[dominant] if dominant == DOMINANT and prof_timed[dominant][1] else prof[dominant]
    launches_per_step = max(d_cnt // args.steps, 1)
    alg_bytes_per_launch = alg[dominant] / launches_per_step
    d_avg_ms = d_ms / max(d_cnt, 1)
    achieved = alg_bytes_per_launch / (d_avg_ms * 1e-3) / 1e9 if d_avg_ms > 0 else 0.0
    kname = {"ingest": "k_ingest", "sort_hist": "k_radix_hist", "sort_scatter": "k_radix_scatter",
             "seg_heads": "k_keys_pass", "segments": "k_seg_wave"}[dominant]
    traffic = measured_traffic(kname)
    # the whole step against the HBM peak: algorithmic bytes of the priced classes, and the counted traffic
    step_alg = sum(alg[k] for k in alg if k in kernels)
    step_traffic = measured_step_traffic()
    whole_step = {"algorithmic_bytes": step_alg, "algorithmic_GBps": round(step_alg / (ms_per_step * 1e-3) / 1e9, 1),
                  "traffic_bytes": step_traffic,
                  "traffic_GBps": None if step_traffic is None else round(step_traffic / (ms_per_step * 1e-3) / 1e9, 1),
                  "traffic_frac_of_peak": None if step_traffic is None
                  else round(step_traffic / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 3)}

    cpu = None
    if not args.no_cpu:
        from oracle import ccld_oracle as orc
        R = spec.layout.n_ranks
        m = min(args.cpu_cycles, args.cycles) * 10 * R
        sample = {k: v[:m] for k, v in tr.cols.items()}
        o = orc.Oracle(tr.topo)
        t1 = time.perf_counter()
        ro = o.analyze_window(sample, now)
        t_cpu = time.perf_counter() - t1
        assert ro.status == "OK"
        cpu = {"value": m / t_cpu, "unit": "records/s", "cores": 1, "kind": "oracle",
               "sample": f"first {min(args.cpu_cycles, args.cycles)} cycles of the same trace "
                         f"({m} records, {len(ro.seg['comm'])} collectives), {t_cpu:.1f} s single-threaded"}

    out = {
        "metric": "trace records analyzed/sec (and HBM GB/s, % peak) at 4,096 ranks; 1 MI355X",
        "value": value, "unit": "records/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int64", "data": "synthetic",
        "config": {"workload": f"config 3: 4,096 ranks TP8xPP8xDP64, {args.cycles * 10} collectives/rank, "
                               f"{n} records, {'shuffled' if not args.no_shuffle else 'time-major'} order; "
                               "step = ingest + analyze_window + rank_blame, every step on operation counters "
                               "not seen before",
                   "records": n, "collectives": int(res.n_seg), "flags": int(res.n_flag),
                   "groups": int(res.n_group), "pcie_inclusive_records_per_s": pcie, "time_major_order_ms_per_step": time_major_ms, "sort_passes": passes, "sort_key_bits": key_bits,
                   "sort_packed_words": bool(packed)},
        "roofline": {"bound": "hbm", "kernel": kname, "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "avg_launch_ms": d_avg_ms, "launches": d_cnt,
                     "algorithmic_bytes_per_launch": alg_bytes_per_launch, "whole_step": whole_step},
        "kernels": kernels,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    an.close()
    return 0


def bench_stream(args, torch, np, ccld, tg) -> int:
    """16,384 ranks, one-second batches of about 2M records, window of 10 batches kept on the device,
    a slow rank re-drawn every 30 batches and one hang at batch 300; per-step latency of
    ingest + analyze_window + rank_blame (the batch is already in HBM when the clock starts)."""
    ss = tg.config5(n_steps=args.stream_steps, seed=args.seed, hang_step=min(300, args.stream_steps // 2))
    topo = ss.layout.topology()
    per = ss.slots_per_step * ss.layout.n_ranks
    W = 10
    an = ccld.Analyzer(topo, max_window_records=W * per, max_batch_records=per, window_batches=W,
                       hang_threshold_ns=5_000_000_000, device="cuda:0")
    buffers = an.alloc_window_result(W * per, seg_cap=W * per // 4 + 1024, flag_cap=W * per // 8 + 1024,
                                     group_cap=min(an.n_comms * 1024, 1 << 22))
    blame_buffers = (torch.empty(5 * an.n_ranks, dtype=torch.int64, device="cuda:0"),
                     torch.empty(an.n_ranks, dtype=torch.int32, device="cuda:0"))
    lat, alerts, first_alert, leaders = [], 0, None, []
    for step in range(ss.n_steps):
        b = tg.stream_batch(ss, step)
        cols = an.to_device(b.cols)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        an.ingest(cols)
        res = an.analyze_window(ss.now_ns(step), buffers=buffers)
        blame, order = an.rank_blame(to_host=False, buffers=blame_buffers)
        torch.cuda.synchronize()
        lat.append(time.perf_counter() - t0)
        assert res.status == "OK", res.status
        if res.n_alert:
            alerts += 1
            first_alert = step if first_alert is None else first_alert
        if step % ss.epoch_steps == ss.epoch_steps - 1:
            leaders.append(int(order[0]) == ss.slow_rank(step))
    lat = np.asarray(lat[W:]) * 1e3                  # full windows only
    out = {"metric": "streaming analysis at 16,384 ranks: per-step analyze latency and records/s", "unit": "records/s",
           "value": float(per / (lat.mean() * 1e-3)), "n_gpus": 1, "steps": int(lat.shape[0]), "warmup": W,
           "ms_per_step": float(lat.mean()), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "int64", "data": "synthetic",
           "config": {"workload": f"config 5: 16,384 ranks TP8xPP16xDP128, {per} new records per 1 s step, "
                                  f"window of {W} steps ({W * per} records) resident on the device",
                      "latency_ms": {"p50": float(np.percentile(lat, 50)), "p95": float(np.percentile(lat, 95)),
                                     "max": float(lat.max())},
                      "window_records_per_s": float(W * per / (lat.mean() * 1e-3)),
                      "steps_with_hang_alert": alerts, "first_alert_step": first_alert, "hang_step": ss.hang_step,
                      "slow_rank_led_blame_at_epoch_end": f"{sum(leaders)}/{len(leaders)}"}}
    print(json.dumps(out), flush=True)
    an.close()
    return 0


def bench_hang(args, torch, np, ccld, tg) -> int:
    """Hang location at 4,096 ranks: 16,777,216 snapshot rows resident in HBM."""
    ht = tg.generate_hang(tg.config4(seed=args.seed))
    an = ccld.Analyzer(ht.topo, max_window_records=1024, max_snapshot_rows=ht.n, device="cuda:0")
    cols = an.snapshots_to_device(ht.cols)
    torch.cuda.synchronize()
    res = None
    for _ in range(args.warmup):
        res = an.locate_hang(cols, 64, 16)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        res = an.locate_hang(cols, 64, 16)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps
    roots = res.root
    ok = list(roots["rank"]) == [ht.root_rank] and list(roots["comm"]) == [ht.root_comm]
    out = {"metric": "hang location at 4,096 ranks: snapshot rows analysed/sec", "unit": "rows/s", "value": ht.n / dt,
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt * 1e3, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "int64", "data": "synthetic",
           "config": {"workload": "config 4: 4,096 ranks x {TP,PP,DP,world} x 16 channels x 64 snapshots "
                                  f"({ht.n} rows, 32 B each), one frozen rank in one DP ring",
                      "root_found": bool(ok), "hung_communicators": int(res.n_hung_comm),
                      "algorithmic_GBps": ht.n * 48.0 / dt / 1e9}}
    print(json.dumps(out), flush=True)
    an.close()
    return 0


def bench_rates(args, torch, np, ccld, tg) -> int:
    """SendRate / RecvRate at 4,096 ranks: 16,777,216 snapshot rows resident in HBM."""
    spec = tg.RateSpec(layout=tg.Layout3D(tp=8, pp=8, dp=64, world=True), n_snapshots=64, n_channels=16, seed=args.seed)
    tr = tg.generate_rates(spec)
    an = ccld.Analyzer(tr.topo, max_window_records=1024, max_snapshot_rows=tr.n, device="cuda:0")
    cols = an.snapshots_to_device(tr.cols)
    torch.cuda.synchronize()
    res = None
    for _ in range(args.warmup):
        res = an.progress_rates(cols, 64, 16)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        res = an.progress_rates(cols, 64, 16)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps
    pair, comm = res.pair, res.comm
    mine = np.unique(pair["comm"][pair["rank"] == tr.slow_rank])
    ok = all(int(comm["root"][c]) == tr.slow_rank for c in mine)
    out = {"metric": "progress rates at 4,096 ranks: snapshot rows analysed/sec", "unit": "rows/s", "value": tr.n / dt,
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt * 1e3, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "int64", "data": "synthetic",
           "config": {"workload": "4,096 ranks x {TP,PP,DP,world} x 16 channels x 64 samples "
                                  f"({tr.n} rows, 32 B each), one slow rank",
                      "slow_rank_is_minimal_rate_member_of_its_communicators": bool(ok),
                      "algorithmic_GBps": tr.n * 48.0 / dt / 1e9}}
    print(json.dumps(out), flush=True)
    an.close()
    return 0


def bench_frames(args, torch, np, ccld, tg) -> int:
    """Probing Frame decoding at 4,096 ranks: one 1184-byte frame per rank and snapshot, resident in HBM."""
    lay = tg.Layout3D(tp=8, pp=8, dp=64, world=True)
    ht = tg.generate_hang(tg.config4(seed=args.seed, layout=lay, n_channels=8, n_snapshots=8), shuffle=False)
    an = ccld.Analyzer(ht.topo, max_window_records=1024, max_snapshot_rows=ht.n, device="cuda:0")
    c = ht.cols
    frames_d, ranks_d = [], []
    for s in range(8):
        m = c["snap"] == s
        fr, rk = tg.encode_frames(ht.topo, {k: v[m] for k, v in c.items()}, 8, kernel_counter=3 * s)
        frames_d.append(torch.from_numpy(fr.view(np.uint8).reshape(-1).copy()).to("cuda:0"))
        ranks_d.append(torch.from_numpy(rk.view(np.int32).copy()).to("cuda:0"))
    torch.cuda.synchronize()
    for s in range(8):
        st, _ = an.decode_frames(frames_d[s], ranks_d[s], s, 8)
        assert st == "OK"
    torch.cuda.synchronize()
    reps = max(args.steps, 1) * 8
    t0 = time.perf_counter()
    for i in range(reps):
        an.decode_frames(frames_d[i % 8], ranks_d[i % 8], 8 + i, 8)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / reps
    n_frames = lay.n_ranks
    out = {"metric": "Probing Frame decoding at 4,096 ranks: frames decoded/sec", "unit": "frames/s", "value": n_frames / dt,
           "n_gpus": 1, "steps": reps, "warmup": 8, "ms_per_step": dt * 1e3, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "int64", "data": "synthetic",
           "config": {"workload": f"{n_frames} frames of 1184 bytes per snapshot -> {int(ht.topo.size.sum()) * 8} snapshot rows",
                      "algorithmic_GBps": (n_frames * 1184.0 + int(ht.topo.size.sum()) * 8 * 32.0) / dt / 1e9}}
    print(json.dumps(out), flush=True)
    an.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
