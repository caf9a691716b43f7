#!/usr/bin/env python3
"""Throughput of the analyzer hot path on one MI355X.

Default workload ("trace"): a step is one pass of the whole path over one synthetic trace that is already
resident in HBM: ccld_ingest (device columns -> keyed window), ccld_analyze_window (placement by sort or by
dense grid, per-collective statistics, flags, blame, Eq. 1-4 groups, hang alerts) and ccld_rank_blame, on the
4,096-rank trace (TP8 x PP8 x DP64, 20,000 collectives per rank, about 82M records) in a seeded random order.

Prints ONE JSON line: records/s of the whole step; "roofline" for the kernel class that takes the most time
(the per-collective statistics kernel), timed with HIP events on the library's stream inside the timed region and
priced with the method's algorithmic bytes per record (the bytes of this implementation's own layout are given
beside them); "kernels", the per-class table of a second set of steps; "cpu_baseline", the CPU oracle timed on a
bounded sample of the same trace in a seeded random order (the GPU analyses the same arrays and must agree).

Other workloads (--workload stream | hang | rates | frames) print the same kind of line for the sliding-window
analysis at 16,384 ranks, the hang location and the progress rates on 16.8M snapshot rows, and the decoding of
Probing Frames.  --traffic-from turns the CSVs of two rocprofv3 --pmc runs into profiles/window_config3_traffic.json.
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
                 "window_kernels.h", "dense.h", "dense.hip"):
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


def roofline(kernel, alg_bytes_per_launch, avg_ms, launches, traffic=None, **extra):
    """The roofline object of the JSON line: algorithmic bytes per launch over the average launch duration."""
    achieved = alg_bytes_per_launch / (avg_ms * 1e-3) / 1e9 if avg_ms > 0 else 0.0
    out = {"bound": "hbm", "kernel": kernel, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
           "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "avg_launch_ms": avg_ms, "launches": launches,
           "algorithmic_bytes_per_launch": alg_bytes_per_launch}
    out.update(extra)
    return out


def traffic_from_counters(fetch_dir: str, write_dir: str) -> int:
    """Reads the counter CSVs of the two runs
         rocprofv3 --pmc FETCH_SIZE --output-format csv -d <fetch_dir> -o run -- python3 bench.py --steps 1 --warmup 0 --no-cpu --no-time-major --no-dense --calibrate-copy
         rocprofv3 --pmc WRITE_SIZE --output-format csv -d <write_dir> -o run -- python3 bench.py --steps 1 --warmup 0 --no-cpu --no-time-major --no-dense --calibrate-copy
    and writes profiles/window_config3_traffic.json: per kernel the bytes per launch (counter value in KiB x 1024 x scale),
    averaged over the launches of the kernel's largest grid; scale = what the 1 GiB -> 1 GiB calibration copy
    (__amd_rocclr_copyBuffer) should read or write over what the counter shows for it."""
    import csv
    import glob
    import re
    STEPS_IN_RUN = 2          # --steps 1 --warmup 0: the timed step and the step of the per-class table
    per = {}
    scale = {}
    for d, counter in ((fetch_dir, "FETCH_SIZE"), (write_dir, "WRITE_SIZE")):
        files = glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True)
        if not files:
            log(f"no counter CSV under {d}")
            return 2
        rows = [r for r in csv.DictReader(open(files[0])) if r["Counter_Name"] == counter]
        copies = [float(r["Counter_Value"]) for r in rows if "copyBuffer" in r["Kernel_Name"] and float(r["Counter_Value"]) > 256 * 1024]
        scale[counter] = (1 << 20) / max(copies) if copies else 1.0
        for r in rows:
            m = re.match(r"(?:void )?ccld::(k_\w+)", r["Kernel_Name"])
            if not m:
                continue
            groups = int(r["Grid_Size"]) // max(int(r["Workgroup_Size"]), 1)
            per.setdefault(m.group(1), {}).setdefault(counter, []).append((groups, float(r["Counter_Value"])))
    kernels = {}
    for k, c in per.items():
        g = max(x[0] for x in c.get("FETCH_SIZE", [(0, 0)]) + c.get("WRITE_SIZE", [(0, 0)]))
        f = [v for gg, v in c.get("FETCH_SIZE", []) if gg == g]
        w = [v for gg, v in c.get("WRITE_SIZE", []) if gg == g]
        kernels[k] = {"workgroups": g, "launches": max(len(f), len(w)) // STEPS_IN_RUN,      # per step
                      "fetch_bytes": int(sum(f) / max(len(f), 1) * 1024 * scale["FETCH_SIZE"]),
                      "write_bytes": int(sum(w) / max(len(w), 1) * 1024 * scale["WRITE_SIZE"])}
    rec = {"csrc_sha256": kernel_sources_digest(), "workload": "config 3, 81,920,000 records, shuffled, one step",
           "scale": scale, "kernels": kernels}
    path = os.path.join(ROOT, "profiles", "window_config3_traffic.json")
    json.dump(rec, open(path, "w"), indent=1, sort_keys=True)
    for k in sorted(kernels):
        v = kernels[k]
        log(f"{k:22s} groups {v['workgroups']:7d} launches {v['launches']:2d} fetch {v['fetch_bytes'] / 1e9:7.3f} GB write {v['write_bytes'] / 1e9:7.3f} GB")
    log(f"scale {scale}; wrote {path}")
    return 0


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
    ap.add_argument("--no-dense", action="store_true",
                    help="skip the secondary figure with the other placement (ccld_params.placement)")
    ap.add_argument("--cpu-cycles", type=int, default=1000,
                    help="cycles of the trace given to the CPU oracle (in a seeded random order, as the timed steps)")
    ap.add_argument("--traffic-from", nargs=2, metavar=("FETCH_DIR", "WRITE_DIR"), default=None,
                    help="no GPU work: turn two rocprofv3 --pmc output folders into profiles/window_config3_traffic.json")
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
    if args.traffic_from:
        return traffic_from_counters(*args.traffic_from)
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
    # root-cause / secondary separation of the late entries of the last analysis (not part of the step)
    torch.cuda.synchronize()
    t_c = time.perf_counter()
    for _ in range(3):
        st_c, chain, _ = an.flag_chains(res)
    torch.cuda.synchronize()
    chains_ms = (time.perf_counter() - t_c) / 3 * 1e3
    chains_info = {"ms": chains_ms, "with_parent": int((chain["parent"] >= 0).sum()), "max_depth": int(chain["depth"].max())}
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
    other_ms = None
    if not args.no_dense:
        # the same steps with the other placement (its own context and workspace)
        other = "dense" if args.placement == "sort" else "sort"
        an2 = ccld.Analyzer(tr.topo, max_window_records=n, device="cuda:0",
                            placement=ccld.PLACEMENT_DENSE if other == "dense" else ccld.PLACEMENT_SORT)
        for timed in (False, True):
            torch.cuda.synchronize()
            t_t = time.perf_counter()
            for i in range(3):
                w = dict(cols)
                w["seq"] = seq_windows[i % n_windows]
                an2.reset_window()
                an2.ingest(w)
                r4 = an2.analyze_window(now, buffers=buffers)
                an2.rank_blame(to_host=False, buffers=blame_buffers)
            torch.cuda.synchronize()
            if timed:
                other_ms = {"placement": other, "ms_per_step": (time.perf_counter() - t_t) / 3 * 1e3, "path_taken": int(r4.path)}
        assert r4.status == "OK" and int(r4.n_flag) == int(res.n_flag) and int(r4.n_seg) == int(res.n_seg)
        an2.close()
        del an2
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

    # HBM bytes per step of each kernel class, priced twice.
    # "alg": what the method has to move per record, whatever the layout (N records, S collectives, P sort passes):
    #  ingest       pack + first histogram: communicator, counter and rank in (16 B), one 8-byte key out
    #  sort_scatter pass 1 reads the key and writes key + index (20 B); later passes move key + index (24 B)
    #  segments     key + index (12 B) and the record's op, bytes, t_enter, t_exit (25 B) in; 13 int64 columns
    #               of statistics per collective out (104 B)
    #  the histogram re-reads, the head marking and the dense partition are this implementation's own passes:
    #  no algorithmic bytes
    # "layout": what this implementation's data layout moves:
    #  ingest       reads the 41-byte SoA record, writes an 8-byte key and a 32-byte payload row
    #  sort_hist    reads the 8-byte key once per pass
    #  sort_scatter as above; when key bits + index bits <= 64 the passes move one packed word (16 B) and the
    #               last pass writes key + index (8 B in, 12 B out)
    #  seg_heads    reads the sorted key once (collective heads per tile)
    #  segments     reads key + index, gathers the 32-byte row, writes a 21-column int64 row per collective, its
    #               detection-group key and range (16 B) and one flag byte per record
    #  dense_partition reads and writes the 32-byte row
    n_seg = int(res.n_seg)
    bl = lambda v: int(v).bit_length()
    # key = (communicator, operation counter, member slot inside the communicator)
    key_bits = bl(tr.topo.n_comms - 1) + bl(int(np.max(tr.topo.size)) - 1) + bl(int(tr.cols["seq"].max()))
    dense = int(res.path) == 1
    packed = passes >= 2 and key_bits + bl(n - 1) <= 64      # key and index travel as one 64-bit word
    scatter_bytes = (16.0 * (passes - 1) + 20.0) if packed else (20.0 + 24.0 * (passes - 1))
    if dense:
        alg = {"ingest": n * 24.0, "segments": n * 25.0 + n_seg * 104.0}
        layout = {"ingest": n * 81.0, "dense_partition": n * 64.0, "segments": n * (32.0 + 12.0 + 1.0) + n_seg * (21 * 8.0 + 16.0)}
    else:
        alg = {"ingest": n * 24.0, "sort_scatter": n * (20.0 + 24.0 * (passes - 1)), "segments": n * 37.0 + n_seg * 104.0}
        layout = {"ingest": n * 81.0, "sort_hist": n * 8.0 * passes, "sort_scatter": n * scatter_bytes,
                  "seg_heads": n * 8.0, "segments": n * (12.0 + 32.0 + 1.0) + n_seg * (21 * 8.0 + 16.0)}
    kernels = {k: {"ms_per_step": round(v[0] / args.steps, 4), "launches_per_step": v[1] / args.steps}
               for k, v in prof.items() if v[1]}
    for k, v in kernels.items():
        if v["ms_per_step"] > 0:
            if k in alg:
                v["algorithmic_GBps"] = round(alg[k] / (v["ms_per_step"] * 1e-3) / 1e9, 1)
            if k in layout:
                v["layout_GBps"] = round(layout[k] / (v["ms_per_step"] * 1e-3) / 1e9, 1)
    dominant = max(alg, key=lambda k: prof[k][0])
    # the dominant class as timed inside the timed region (falls back to the untimed table if another class
    # has overtaken it)
    d_ms, d_cnt = prof_timed[dominant] if dominant == DOMINANT and prof_timed[dominant][1] else prof[dominant]
    launches_per_step = max(d_cnt // args.steps, 1)
    d_avg_ms = d_ms / max(d_cnt, 1)
    kname = {"ingest": "k_ingest_staged", "sort_scatter": "k_radix_scatter",
             "segments": "k_dense_stats" if dense else "k_seg_wave"}[dominant]
    traffic = measured_traffic(kname)
    # the whole step: algorithmic and layout bytes over the step time; the counted bytes are what the L2 exchanged
    # with the fabric (memory-side cache and HBM together), so they are not set against the HBM peak
    step_alg, step_layout = sum(alg.values()), sum(layout.values())
    step_traffic = measured_step_traffic()
    gbps = lambda b: round(b / (ms_per_step * 1e-3) / 1e9, 1)
    whole_step = {"algorithmic_bytes": step_alg, "algorithmic_GBps": gbps(step_alg),
                  "algorithmic_frac_of_peak": round(gbps(step_alg) / HBM_PEAK_GBS, 3),
                  "layout_bytes": step_layout, "layout_GBps": gbps(step_layout),
                  "l2_fabric_bytes_counted": step_traffic,
                  "l2_fabric_GBps_counted": None if step_traffic is None else gbps(step_traffic)}

    cpu = None
    if not args.no_cpu:
        # the oracle on a bounded sample: the first cycles of the same trace in a seeded random order; the GPU
        # analyses the same arrays first and both must report the same numbers of collectives and flags
        from oracle import ccld_oracle as orc
        cyc = min(args.cpu_cycles, args.cycles)
        m = min(cyc * 10 * spec.layout.n_ranks, n)            # the trace is slot-major: whole collectives only
        rng = np.random.default_rng(args.seed + 2)
        pm = rng.permutation(m)
        sample = {k: np.ascontiguousarray(v[:m][pm]) for k, v in tr.cols.items()}
        now_s = int(sample["t_exit"][sample["t_exit"] != tg.INFLIGHT].max()) + 1
        an.reset_window()
        an.ingest(an.to_device(sample))
        rg = an.analyze_window(now_s, buffers=buffers)
        o = orc.Oracle(tr.topo)
        t1 = time.perf_counter()
        ro = o.analyze_window(sample, now_s)
        t_cpu = time.perf_counter() - t1
        assert ro.status == "OK" and rg.status == "OK"
        assert int(rg.n_seg) == len(ro.seg["comm"]) and int(rg.n_flag) == len(ro.flag["comm"]), "GPU and oracle disagree on the sample"
        cpu = {"value": m / t_cpu, "unit": "records/s", "cores": 1, "kind": "oracle",
               "sample": f"first {cyc} cycles of the same trace in a seeded random order ({m} records, "
                         f"{len(ro.seg['comm'])} collectives, {len(ro.flag['comm'])} flags: the same counts as the GPU "
                         f"on these arrays), {t_cpu:.1f} s single-threaded"}

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
                   "groups": int(res.n_group), "placement": "dense" if dense else "sort",
                   "pcie_inclusive_records_per_s": pcie, "time_major_order_ms_per_step": time_major_ms,
                   "other_placement": other_ms, "flag_chains": chains_info,
                   "sort_passes": passes, "sort_key_bits": key_bits, "sort_packed_words": bool(packed)},
        "roofline": roofline(kname, alg[dominant] / launches_per_step, d_avg_ms, d_cnt, traffic,
                             layout_bytes_per_launch=layout[dominant] / launches_per_step,
                             layout_GBps=layout[dominant] / launches_per_step / (d_avg_ms * 1e-3) / 1e9 if d_avg_ms > 0 else 0.0,
                             whole_step=whole_step),
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
    DOMINANT = "segments"
    kept, segs = [], []                 # the first W batches, for the oracle leg; collectives per full window
    for step in range(ss.n_steps):
        if step == W:                   # full windows from here on: time the dominant class inside the timed steps
            an.profile_enable(True, only=DOMINANT)
        b = tg.stream_batch(ss, step)
        if step < W and not args.no_cpu:
            kept.append(b.cols)
        cols = an.to_device(b.cols)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        an.ingest(cols)
        res = an.analyze_window(ss.now_ns(step), buffers=buffers)
        blame, order = an.rank_blame(to_host=False, buffers=blame_buffers)
        torch.cuda.synchronize()
        lat.append(time.perf_counter() - t0)
        assert res.status == "OK", res.status
        if step >= W:
            segs.append(int(res.n_seg))
        if step == W - 1:
            first_window = (int(res.n_seg), int(res.n_flag), int(res.n_records))
        if res.n_alert:
            alerts += 1
            first_alert = step if first_alert is None else first_alert
        if step % ss.epoch_steps == ss.epoch_steps - 1:
            leaders.append(int(order[0]) == ss.slow_rank(step))
    lat = np.asarray(lat[W:]) * 1e3                  # full windows only
    prof, _ = an.profile_read()
    an.profile_enable(False)
    d_ms, d_cnt = prof[DOMINANT]
    # the statistics pass covers the whole window every step: per record key + index (12 B) and op, bytes,
    # t_enter, t_exit (25 B) in, 104 B of statistics per collective out
    alg = W * per * 37.0 + float(np.mean(segs)) * 104.0
    layout = W * per * 45.0 + float(np.mean(segs)) * 184.0
    d_avg = d_ms / max(d_cnt, 1)
    cpu = None
    if not args.no_cpu:
        # the oracle on the first full window (the W batches concatenated in arrival order): the same records the
        # GPU analysed at step W - 1
        from oracle import ccld_oracle as orc
        win = {k: np.concatenate([c[k] for c in kept]) for k in kept[0]}
        o = orc.Oracle(topo, {"hang_threshold_ns": 5_000_000_000})
        t1 = time.perf_counter()
        ro = o.analyze_window(win, ss.now_ns(W - 1))
        t_cpu = time.perf_counter() - t1
        assert ro.status == "OK" and (len(ro.seg["comm"]), len(ro.flag["comm"]), int(win["rank"].shape[0])) == first_window, \
            "GPU and oracle disagree on the first full window"
        cpu = {"value": per / t_cpu, "unit": "records/s", "cores": 1, "kind": "oracle",
               "sample": f"one step: the first full window ({first_window[2]} records, {first_window[0]} collectives, "
                         f"{first_window[1]} flags: the same counts as the GPU at that step), {t_cpu:.1f} s single-threaded; "
                         "value = new records per step / that time, as for the GPU"}
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
                      "slow_rank_led_blame_at_epoch_end": f"{sum(leaders)}/{len(leaders)}"},
           "roofline": roofline("k_seg_wave + k_seg_multi<2> + k_seg_lengths (the statistics of the whole window)", alg, d_avg, d_cnt,
                                layout_bytes_per_launch=layout,
                                note="one launch = the statistics pass of one step; the step as a whole is bound by "
                                     "launch latency (about 60 launches for 2M new records), not by HBM"),
           "cpu_baseline": cpu}
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
    an.profile_enable(True, only="hang_place")
    t0 = time.perf_counter()
    for _ in range(args.steps):
        res = an.locate_hang(cols, 64, 16)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps
    prof, _ = an.profile_read()
    an.profile_enable(False)
    p_ms, p_cnt = prof["hang_place"]
    cpu = None
    if not args.no_cpu:
        from oracle import ccld_oracle as orc
        t1 = time.perf_counter()
        ro = orc.Oracle(ht.topo).locate_hang(ht.cols, 64, 16)
        t_cpu = time.perf_counter() - t1
        assert ro.status == "OK" and list(ro.root["rank"]) == list(res.root["rank"]) and list(ro.root["comm"]) == list(res.root["comm"])
        cpu = {"value": ht.n / t_cpu, "unit": "rows/s", "cores": 1, "kind": "oracle",
               "sample": f"the same {ht.n} rows (same roots as the GPU), {t_cpu:.1f} s single-threaded"}
    roots = res.root
    ok = list(roots["rank"]) == [ht.root_rank] and list(roots["comm"]) == [ht.root_comm]
    out = {"metric": "hang location at 4,096 ranks: snapshot rows analysed/sec", "unit": "rows/s", "value": ht.n / dt,
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt * 1e3, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "int64", "data": "synthetic",
           "config": {"workload": "config 4: 4,096 ranks x {TP,PP,DP,world} x 16 channels x 64 snapshots "
                                  f"({ht.n} rows, 32 B each), one frozen rank in one DP ring",
                      "root_found": bool(ok), "hung_communicators": int(res.n_hung_comm),
                      "whole_pass_algorithmic_GBps": ht.n * 32.0 / dt / 1e9},
           # placement of the rows in the (member, channel, snapshot) grid: every 32-byte row is touched once by the
           # method; this implementation clears the grid (16 B per cell), regroups the rows by region (32 B in,
           # 20 B out) and places them (20 B in, 16 B out)
           "roofline": roofline("grid fill + k_hang_part + k_hang_place_regions (placement of the snapshot rows)",
                                ht.n * 32.0, p_ms / max(p_cnt, 1), p_cnt, layout_bytes_per_launch=ht.n * (16.0 + 52.0 + 36.0)),
           "cpu_baseline": cpu}
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
    an.profile_enable(True, only="hang_place")
    t0 = time.perf_counter()
    for _ in range(args.steps):
        res = an.progress_rates(cols, 64, 16)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps
    prof, _ = an.profile_read()
    an.profile_enable(False)
    p_ms, p_cnt = prof["hang_place"]
    cpu = None
    if not args.no_cpu:
        from oracle import ccld_oracle as orc
        t1 = time.perf_counter()
        ro = orc.Oracle(tr.topo).progress_rates(tr.cols, 64, 16)
        t_cpu = time.perf_counter() - t1
        assert ro.status == "OK" and np.array_equal(ro.comm["root"], res.comm["root"])
        cpu = {"value": tr.n / t_cpu, "unit": "rows/s", "cores": 1, "kind": "oracle",
               "sample": f"the same {tr.n} rows (same minimal-rate members as the GPU), {t_cpu:.1f} s single-threaded"}
    pair, comm = res.pair, res.comm
    mine = np.unique(pair["comm"][pair["rank"] == tr.slow_rank])
    ok = all(int(comm["root"][c]) == tr.slow_rank for c in mine)
    out = {"metric": "progress rates at 4,096 ranks: snapshot rows analysed/sec", "unit": "rows/s", "value": tr.n / dt,
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt * 1e3, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "int64", "data": "synthetic",
           "config": {"workload": "4,096 ranks x {TP,PP,DP,world} x 16 channels x 64 samples "
                                  f"({tr.n} rows, 32 B each), one slow rank",
                      "slow_rank_is_minimal_rate_member_of_its_communicators": bool(ok),
                      "whole_pass_algorithmic_GBps": tr.n * 32.0 / dt / 1e9},
           "roofline": roofline("grid fill + k_hang_part + k_hang_place_regions (placement of the sampled rows)",
                                tr.n * 32.0, p_ms / max(p_cnt, 1), p_cnt, layout_bytes_per_launch=tr.n * (16.0 + 52.0 + 36.0)),
           "cpu_baseline": cpu}
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
    an.profile_enable(True, only="frames")
    t0 = time.perf_counter()
    for i in range(reps):
        an.decode_frames(frames_d[i % 8], ranks_d[i % 8], 8 + i, 8)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / reps
    prof, _ = an.profile_read()
    an.profile_enable(False)
    f_ms, f_cnt = prof["frames"]
    n_frames = lay.n_ranks
    n_rows_out = int(ht.topo.size.sum()) * 8
    cpu = None
    if not args.no_cpu:
        from oracle import ccld_oracle as orc
        o = orc.Oracle(ht.topo)
        o.frames_begin(8)
        host = [(f.cpu().numpy(), r.cpu().numpy().view(np.uint32)) for f, r in zip(frames_d, ranks_d)]
        t1 = time.perf_counter()
        k = 0
        while time.perf_counter() - t1 < 10.0:
            st, _rows = o.decode_frames(host[k % 8][0], host[k % 8][1], k)
            assert st == "OK"
            k += 1
        t_cpu = time.perf_counter() - t1
        o.frames_end()
        cpu = {"value": k * n_frames / t_cpu, "unit": "frames/s", "cores": 1, "kind": "oracle",
               "sample": f"{k} snapshots of the same {n_frames} frames, {t_cpu:.1f} s single-threaded"}
    out = {"metric": "Probing Frame decoding at 4,096 ranks: frames decoded/sec", "unit": "frames/s", "value": n_frames / dt,
           "n_gpus": 1, "steps": reps, "warmup": 8, "ms_per_step": dt * 1e3, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "int64", "data": "synthetic",
           "config": {"workload": f"{n_frames} frames of 1184 bytes per snapshot -> {int(ht.topo.size.sum()) * 8} snapshot rows",
                      "whole_call_algorithmic_GBps": (n_frames * 1184.0 + n_rows_out * 32.0) / dt / 1e9},
           # frames in (1184 B each), snapshot rows out (32 B each); three small launches per snapshot
           "roofline": roofline("k_frames<check> + k_frames<apply> + k_frame_rows (one snapshot's frames)",
                                n_frames * 1184.0 + n_rows_out * 32.0, f_ms / max(f_cnt, 1), f_cnt,
                                note="4.8 MB per call: bound by launch latency and the status read-back, not by HBM"),
           "cpu_baseline": cpu}
    print(json.dumps(out), flush=True)
    an.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
