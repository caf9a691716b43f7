"""GPU parity on randomly drawn inputs: topologies (communicators of 1 to thousands of members in any
member order, ring and tree), partial and tied rounds, stragglers, operations in flight, missing
and very large operation counters, one to three windows with state carried over, host and device
batches, random analyzer parameters; and snapshot series of random progress (healthy, not-entered,
inconsistent and all-stalled communicators, missing and repeated rows) through the hang and the
progress-rate passes; and random Probing Frames (any blocks written, communicators repeated in a
frame, bad ranks, communicators and counts) through the frame decoder.  Every table is compared with the oracle's, bit-exactly."""
import collections

import numpy as np
import pytest

from oracle import ccld_oracle as orc
from paper_2605_04478_amd import tracegen as tg
from tests.helpers import INFLIGHT, T0, toy_cols
from tests.test_gpu_window import compare

pytestmark = pytest.mark.gpu

FAR = T0 + 10**15


def rand_case(seed):
    rng = np.random.default_rng(seed)
    big = rng.random() < 0.15
    R = int(rng.integers(600, 5000)) if big else int(rng.integers(1, 90))
    n_comms = int(rng.integers(1, 9))
    comms, algo, parents = [], [], []
    for c in range(n_comms):
        u = rng.random()
        if u < 0.15:
            sz = 1
        elif u < 0.5:
            sz = int(rng.integers(1, min(R, 9) + 1))
        elif u < 0.85:
            sz = int(rng.integers(1, min(R, 70) + 1))
        else:
            sz = int(rng.integers(1, R + 1))
        mem = rng.choice(R, sz, replace=False)
        if rng.random() < 0.5:
            mem = np.sort(mem)
        comms.append([int(x) for x in mem])
        tree = rng.random() < 0.3
        algo.append(1 if tree else 0)
        par, pp = [-1], 0
        for q in range(1, sz):
            pp = int(rng.integers(pp, min(q, pp + 2)))          # non-decreasing parents: BFS order
            par.append(pp)
        parents.append(par if tree else None)
    topo = tg.make_topology(R, comms, algo=algo, tree_parent=parents if any(p is not None for p in parents) else None)
    budget = 60000 if not big else 150000
    rows = []
    tie = rng.random() < 0.5
    for c, mem in enumerate(comms):
        seq0 = int(rng.choice([0, 0, 1, 1000, 2**33, 2**47]))
        n_seq = max(1, min(int(rng.integers(1, 400)), budget // (n_comms * len(mem))))
        kind_op = int(rng.integers(0, 4))
        for s in range(n_seq):
            if rng.random() < 0.05:
                continue                                   # a counter value missing entirely
            n = len(mem) if rng.random() < 0.7 else int(rng.integers(1, len(mem) + 1))
            ranks = mem if n == len(mem) else list(rng.choice(mem, n, replace=False))
            base = T0 + s * 100_000 + int(rng.integers(0, 1000))
            te = base + (rng.integers(0, 4, n) if tie else rng.integers(0, 30_000, n))
            if rng.random() < 0.2:
                te[int(rng.integers(0, n))] += int(rng.integers(1, 10**9))          # straggler
            dur = rng.integers(0, 5, n) if tie else rng.integers(1000, 60_000, n)
            if rng.random() < 0.1:
                dur = dur * int(rng.integers(2, 40))
            tx = te + dur
            infl = rng.random(n) < (0.3 if rng.random() < 0.1 else 0.01)
            nbytes = int(rng.choice([0, 1, 3, 4, 8, 1 << 10, 1 << 20, 1 << 33]))
            for r, a, b, f in zip(ranks, te, tx, infl):
                op = kind_op if rng.random() > 0.002 else int(rng.integers(0, 8))
                rows.append((int(r), c, seq0 + s, op, nbytes if rng.random() > 0.002 else nbytes + 8, int(a),
                             INFLIGHT if f else int(b)))
    params = {}
    if rng.random() < 0.7:
        params = dict(hang_threshold_ns=int(rng.choice([1, 50_000, 10**7, 300 * 10**9])),
                      lag_floor_ns=int(rng.choice([1, 2, 1000, 300_000])),
                      tbase_init_ns=int(rng.choice([1, 2, 2000, 50_000, 2**61])),
                      kmad_num=int(rng.integers(1, 10)), kmad_den=int(rng.integers(1, 4)),
                      tbase_rounds=int(rng.choice([1, 2, 7, 100])), repeat_threshold=int(rng.integers(1, 4)),
                      tbase_warmup_ns=int(rng.choice([0, 10**6, 120 * 10**9])),
                      theta_num=int(rng.integers(1, 7)), theta_den=int(rng.integers(1, 3)),
                      barrier_bytes=int(rng.choice([0, 4, 9])))
    return topo, rows, params, rng


def run(seed):
    topo, rows, params, rng = rand_case(seed)
    if not rows:
        return 0
    cols = toy_cols(rows)
    n = len(rows)
    # shuffle, then 1-3 windows split by time order of the counter, analysed in turn with state carried
    perm = rng.permutation(n)
    cols = {k: v[perm] for k, v in cols.items()}
    n_win = int(rng.integers(1, 4))
    order = np.argsort(cols["t_enter"], kind="stable")
    cuts = [0] + sorted(int(x) for x in rng.integers(0, n + 1, n_win - 1)) + [n]
    from paper_2605_04478_amd import ccld
    # one context that sorts and one that tries the dense placement first, each with its own detection state
    ans = [ccld.Analyzer(topo, max_window_records=n, placement=pl, **params) for pl in (0, 1)]
    o = orc.Oracle(topo, params)
    now = int(rng.choice([FAR, T0 + 10**6, T0 + 10**8]))
    for w in range(n_win):
        sel = order[cuts[w]:cuts[w + 1]]
        sel = sel[rng.permutation(len(sel))]
        sl = {k: v[sel] for k, v in cols.items()}
        on_dev = rng.random() < 0.7
        ref = o.analyze_window(sl, now)
        for pl, an in enumerate(ans):
            an.reset_window()
            an.ingest(an.to_device(sl) if on_dev else sl)
            g = an.analyze_window(now, n_records=max(len(sel), 1), per_record=True, alert_cap=len(sel) + 1,
                                  cand_cap=max(65536, 8 * len(sel)))
            blame = order_ = None
            if ref.status == "OK":
                blame, order_ = an.rank_blame()
            compare(g, ref, blame, order_, what=f"seed{seed} window{w} n={len(sel)} status={ref.status} placement={pl}")
            assert pl == 1 or g.path == 0
    for an in ans:
        an.close()
    return n


@pytest.mark.parametrize("block", range(4))
def test_random_cases_match_the_oracle(block):
    total = 0
    for seed in range(block * 30, block * 30 + 30):
        total += run(seed)
    assert total > 0


# ---- windows of several batches: each ingest drops the oldest batch -------------------------------
def run_stream(seed):
    topo, rows, params, rng = rand_case(seed)
    if not rows:
        return 0
    cols = toy_cols(rows)
    n = len(rows)
    order = np.argsort(cols["t_enter"], kind="stable")
    wb = int(rng.integers(1, 6))
    n_b = int(rng.integers(1, 9))
    cuts = [0] + sorted(int(x) for x in rng.integers(0, n + 1, n_b - 1)) + [n]
    batches = []
    for i in range(n_b):
        sel = order[cuts[i]:cuts[i + 1]]
        sel = sel[rng.permutation(len(sel))]
        batches.append({k: v[sel] for k, v in cols.items()})
    max_b = max(max(len(b["rank"]) for b in batches), 1)
    params = dict(params, window_batches=wb)
    from paper_2605_04478_amd import ccld
    an = ccld.Analyzer(topo, max_window_records=max(wb * max_b, 1), max_batch_records=max_b, **params)
    o = orc.Oracle(topo, params)
    for i, b in enumerate(batches):
        on_dev = rng.random() < 0.7
        an.ingest(an.to_device(b) if on_dev else b)
        if rng.random() < 0.3 and i + 1 < n_b:
            continue                                    # several ingests between analyses
        win = batches[max(0, i - wb + 1): i + 1]
        wc = {k: np.concatenate([w[k] for w in win]) for k in b}
        nw = len(wc["rank"])
        g = an.analyze_window(FAR, n_records=max(nw, 1), per_record=True, alert_cap=nw + 1, cand_cap=max(65536, 8 * nw))
        ref = o.analyze_window(wc, FAR)
        blame = order_ = None
        if ref.status == "OK":
            blame, order_ = an.rank_blame()
        compare(g, ref, blame, order_, what=f"seed{seed} step{i} wb={wb} n={nw} status={ref.status}")
    an.close()
    return n


def test_random_windows_of_several_batches_match_the_oracle():
    total = 0
    for seed in range(1000, 1040):
        total += run_stream(seed)
    assert total > 0


# ---- snapshot series: ccld_locate_hang and ccld_progress_rates ------------------------------------
def rand_topo(rng):
    big = rng.random() < 0.1
    R = int(rng.integers(200, 1500)) if big else int(rng.integers(1, 40))
    n_comms = int(rng.integers(1, 7))
    comms, algo, parents = [], [], []
    for c in range(n_comms):
        u = rng.random()
        sz = 1 if u < 0.1 else int(rng.integers(1, min(R, 9) + 1)) if u < 0.6 else int(rng.integers(1, R + 1))
        mem = rng.choice(R, sz, replace=False)
        if rng.random() < 0.5:
            mem = np.sort(mem)
        comms.append([int(x) for x in mem])
        tree = rng.random() < 0.3
        algo.append(1 if tree else 0)
        par, pp = [-1], 0
        for q in range(1, sz):
            pp = int(rng.integers(pp, min(q, pp + 2)))
            par.append(pp)
        parents.append(par if tree else None)
    return tg.make_topology(R, comms, algo=algo, tree_parent=parents if any(p is not None for p in parents) else None), comms


def rand_rows(rng, comms, n_snap, n_ch):
    cols = {k: [] for k in tg.SNAP_COLUMNS}
    for c, mem in enumerate(comms):
        m = len(mem)
        mode = rng.choice(["healthy", "h1", "h2", "h3", "rand"])
        freeze = int(rng.integers(0, n_snap + 1))
        seq_now = int(rng.choice([0, 5, 1000, 2**40]))
        # per slot / channel series
        s_idx = np.arange(n_snap)
        for q, r in enumerate(mem):
            behind = mode == "h1" and rng.random() < 0.3
            moving = mode == "h2" and rng.random() < 0.4
            for ch in range(n_ch):
                inc_s = rng.integers(0, 3, n_snap) * (rng.random(n_snap) < 0.6)
                inc_r = rng.integers(0, 3, n_snap) * (rng.random(n_snap) < 0.6)
                if rng.random() < 0.1:
                    inc_s[:] = 0
                    inc_r[:] = 0
                if mode != "healthy" and not moving and mode != "rand":
                    inc_s[freeze:] = 0
                    inc_r[freeze:] = 0
                seq_inc = (rng.random(n_snap) < 0.05).astype(np.int64)
                if mode in ("h1", "h2", "h3"):
                    seq_inc[freeze:] = 0
                seq = seq_now + np.cumsum(seq_inc)
                if behind:
                    seq = np.minimum(seq, seq_now)
                sent = np.cumsum(inc_s)
                recv = np.cumsum(inc_r)
                # counters restart with every new operation
                for t in np.nonzero(seq_inc)[0]:
                    sent[t:] -= sent[t]
                    recv[t:] -= recv[t]
                cols["snap"].append(s_idx)
                cols["rank"].append(np.full(n_snap, r))
                cols["comm"].append(np.full(n_snap, c))
                cols["channel"].append(np.full(n_snap, ch))
                cols["seq_posted"].append(seq)
                cols["chunks_sent"].append(sent)
                cols["chunks_recv"].append(recv)
    dt = {"snap": np.uint32, "rank": np.uint32, "comm": np.uint32, "channel": np.uint32,
          "seq_posted": np.uint64, "chunks_sent": np.uint32, "chunks_recv": np.uint32}
    out = {k: np.concatenate(v).astype(dt[k]) for k, v in cols.items()}
    p = rng.permutation(out["snap"].shape[0])
    return {k: v[p] for k, v in out.items()}


def cmp_tables(g, o, names, what):
    assert g.status == o.status, (what, g.status, o.status)
    if o.status != "OK":
        return
    for name in names:
        gt, ot = getattr(g, name), getattr(o, name)
        for k in ot:
            assert np.array_equal(gt[k], ot[k]), (what, name, k, gt[k][:8], ot[k][:8])


def run_hang(seed):
    rng = np.random.default_rng(seed)
    topo, comms = rand_topo(rng)
    cells = int(topo.size.sum())
    n_ch = int(rng.integers(1, 9))
    n_snap = int(rng.integers(1, max(2, min(140, 400000 // (cells * n_ch)))))
    cols = rand_rows(rng, comms, n_snap, n_ch)
    fault = rng.random()
    n = cols["snap"].shape[0]
    if fault < 0.05 and n > 1:                                   # a missing row
        keep = np.ones(n, bool); keep[int(rng.integers(0, n))] = False
        cols = {k: v[keep] for k, v in cols.items()}
    elif fault < 0.1:                                            # a repeated row
        j = int(rng.integers(0, n))
        cols = {k: np.concatenate([v, v[j:j + 1]]) for k, v in cols.items()}
    params = dict(stall_snapshots=int(rng.choice([1, 2, 5, 30])), fifo_depth=int(rng.choice([1, 2, 8])))
    rows = int(cols["snap"].shape[0])
    from paper_2605_04478_amd import ccld
    an = ccld.Analyzer(topo, max_window_records=1024, max_snapshot_rows=max(cells * n_snap * n_ch, rows, 1), **params)
    o = orc.Oracle(topo, params)
    what = f"seed{seed} snaps={n_snap} ch={n_ch} rows={rows}"
    on_dev = rng.random() < 0.7
    src = an.snapshots_to_device(cols) if on_dev else cols
    g = an.locate_hang(src, n_snap, n_ch, root_cap=cells + 1)
    ref = o.locate_hang(cols, n_snap, n_ch)
    cmp_tables(g, ref, ("root", "pair", "comm"), what + " hang")
    if ref.status == "OK":
        assert g.n_root == len(ref.root["rank"]) and g.n_hung_comm == int(ref.comm["hung"].sum()), what
    g2 = an.progress_rates(src, n_snap, n_ch)
    ref2 = o.progress_rates(cols, n_snap, n_ch)
    cmp_tables(g2, ref2, ("pair", "comm"), what + " rates")
    an.close()
    return rows, ref.status, (len(ref.root["rank"]) if ref.status == "OK" else 0)


@pytest.mark.parametrize("block", range(3))
def test_random_snapshot_series_match_the_oracle(block):
    seen = set()
    # seed 230 names more roots than the window holds records: the root list is sorted in buffers
    # sized for the larger of the two
    for seed in list(range(block * 40, block * 40 + 40)) + ([230] if block == 0 else []):
        seen.add(run_hang(seed)[1])
    assert "OK" in seen


# ---- Probing Frames: ccld_decode_frames -------------------------------------------------------------
def run_frames(seed):
    rng = np.random.default_rng(seed)
    topo, comms = rand_topo(rng)
    R = topo.n_ranks
    n_ch = int(rng.integers(1, 9))
    n_snap = int(rng.integers(1, 12))
    of_rank = collections.defaultdict(list)
    for c, mem in enumerate(comms):
        for r in mem:
            of_rank[r].append(c)
    cells = int(topo.size.sum())
    from paper_2605_04478_amd import ccld
    from tests.test_gpu_frames import both
    an = ccld.Analyzer(topo, max_window_records=16, max_snapshot_rows=max(cells * n_ch * 2, 40 * (min(R, 300) + 2)))
    o = orc.Oracle(topo)
    o.frames_begin(n_ch)
    st_seen = collections.Counter()
    for s in range(n_snap):
        k = int(rng.integers(0, min(R, 300) + 1))
        ranks = rng.choice(R, k, replace=False).astype(np.uint32)
        if rng.random() < 0.03 and k > 0:
            ranks = np.concatenate([ranks, ranks[:1]])          # the same rank twice
        frames = np.zeros(len(ranks), dtype=tg.FRAME_DTYPE)
        frames["mode"] = 1
        frames["n_channels"] = n_ch if rng.random() > 0.02 else int(rng.integers(0, 12))
        frames["counter"] = rng.integers(0, 2**40, len(ranks))
        frames["kernel_index"] = frames["counter"] % 8
        bad = (int(rng.integers(0, max(len(ranks), 1))), int(rng.integers(0, 8))) if rng.random() < 0.12 else None
        for i, r in enumerate(ranks):
            mine = of_rank.get(int(r), [])
            for b in range(8):
                if rng.random() < 0.5 and bad != (i, b):
                    continue
                u = rng.random() if bad == (i, b) else 0.0
                if not mine and bad != (i, b):
                    continue
                if mine and u < 0.4:
                    cm = int(rng.choice(mine))
                elif u < 0.7:
                    cm = int(rng.integers(0, topo.n_comms))      # maybe not a member
                else:
                    cm = topo.n_comms + int(rng.integers(0, 3))  # unknown communicator
                frames["block"]["comm"][i, b] = cm
                frames["block"]["ext"][i, b] = 1 if rng.random() > 0.05 else 0
                frames["block"]["counter"][i, b] = int(rng.integers(0, 50)) if rng.random() < 0.8 else int(rng.integers(0, 2**50))
                cnt = rng.integers(0, 2**32, (8, 2), dtype=np.uint64) if rng.random() < 0.5 else rng.integers(0, 9, (8, 2)).astype(np.uint64)
                if bad == (i, b) and u < 0.2:
                    cnt[int(rng.integers(0, 8)), 0] = 2**32 + 5
                frames["block"]["count"][i, b] = cnt
        if rng.random() < 0.01 and len(ranks):
            ranks = ranks.copy(); ranks[0] = R + 3               # rank out of range
        fr = frames.view(np.uint8).reshape(len(ranks), tg.FRAME_BYTES)
        st, _ = both(an, o, fr, ranks, s, n_ch, on_device=bool(rng.random() < 0.5), what=f"seed{seed} snap{s}")
        st_seen[st] += 1
        if rng.random() < 0.05:
            an.reset_frames(); o.frames_begin(n_ch)
    an.close()
    return st_seen


def test_random_frames_match_the_oracle():
    seen = collections.Counter()
    for seed in range(80):
        seen += run_frames(seed)
    assert seen["OK"] > 100 and len(seen) > 2
