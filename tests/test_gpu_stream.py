"""GPU parity for streaming analysis: a sliding window of one-second batches kept on the device,
a slow rank that rotates, and a hang that appears mid-stream; every step is compared with the
CPU oracle run on the concatenated window."""
import numpy as np
import pytest

from oracle import ccld_oracle as orc
from paper_2605_04478_amd import tracegen as tg
from tests.test_gpu_window import compare

pytestmark = pytest.mark.gpu


def test_streaming_window_matches_oracle_every_step():
    from paper_2605_04478_amd import ccld
    ss = tg.config5(n_steps=26, layout=tg.Layout3D(tp=4, pp=4, dp=16), epoch_steps=6, hang_step=11)
    topo = ss.layout.topology()
    W = 10
    per = ss.slots_per_step * ss.layout.n_ranks
    params = dict(hang_threshold_ns=5_000_000_000, window_batches=W)
    an = ccld.Analyzer(topo, max_window_records=W * per, max_batch_records=per, **params)
    o = orc.Oracle(topo, dict(hang_threshold_ns=5_000_000_000))
    batches = []
    alerts_seen, located = [], set()
    hang_rank, hang_comm, hang_seq = ss.hang_site()
    for step in range(ss.n_steps):
        b = tg.stream_batch(ss, step)
        batches.append(b.cols)
        an.ingest(an.to_device(b.cols))
        win = batches[max(0, step - W + 1): step + 1]
        cols = {k: np.concatenate([w[k] for w in win]) for k in b.cols}
        now = ss.now_ns(step)
        g = an.analyze_window(now, n_records=W * per, per_record=True)
        ref = o.analyze_window(cols, now)
        blame, order = an.rank_blame()
        compare(g, ref, blame, order, what=f"step{step}")
        if g.n_alert:
            alerts_seen.append(step)
            a = g.alert
            assert list(a["comm"]) == [hang_comm] and list(a["seq"]) == [hang_seq] and list(a["class"]) == [1]
            assert list(g.cand) == [hang_rank]
        # the slow rank of the current epoch leads the blame once its epoch fills most of the window
        if step % ss.epoch_steps == ss.epoch_steps - 1:
            located.add((int(order[0]), ss.slow_rank(step)))
    # the hang is in flight for longer than 5 s from step hang+5 until its records leave the window
    assert alerts_seen == list(range(ss.hang_step + 5, ss.hang_step + W))
    assert all(a == b for a, b in located) and len(located) >= 3


def test_kept_window_order_survives_odd_sequences():
    """Windows of several batches keep the previous window's order and merge the new records into it.
    Here the sequence of calls varies: several ingests between two analyses, an empty batch, batches
    of very different sizes, a hang location in between (it borrows the sort buffers), a reset, and
    operation counters that move the window's key format from step to step."""
    from paper_2605_04478_amd import ccld
    from tests.test_gpu_window import FAR
    from tests.test_oracle_hang import snap_rows
    spec = tg.config2(n_cycles=40)
    tr = tg.generate(spec)
    R = spec.layout.n_ranks
    sizes = [7, 1, 0, 12, 3, 3, 25, 2, 9, 9, 4, 30, 1, 1, 6]           # collectives per rank in each batch
    starts = np.cumsum([0] + sizes)
    batches = [{k: v[starts[i] * R:starts[i + 1] * R] for k, v in tr.cols.items()} for i in range(len(sizes))]
    wb = 4
    cap = max(sum(sizes[i:i + wb]) for i in range(len(sizes))) * R + 13
    n_cells = int(tr.topo.size.sum()) * 4
    an = ccld.Analyzer(tr.topo, max_window_records=cap, max_batch_records=max(sizes) * R, window_batches=wb,
                       max_snapshot_rows=n_cells, stall_snapshots=2)
    o = orc.Oracle(tr.topo, dict(window_batches=wb, stall_snapshots=2))
    rng = np.random.default_rng(5)
    held = []
    for i, b in enumerate(batches):
        p = rng.permutation(len(b["rank"]))
        b = {k: v[p] for k, v in b.items()}
        if i == 11:                                          # start over: the kept order must not be used
            an.reset_window()
            held = []
        an.ingest(an.to_device(b))
        held = (held + [b])[-wb:]
        if i in (1, 5, 9):                                   # no analysis after these ingests
            continue
        if i == 7:                                           # the hang pass sorts its roots in the same buffers
            rows = snap_rows(tr.topo, 4, 1, lambda s, c, q, ch: (3, 5, 5) if q else (2, 9, 9))
            h = an.locate_hang(an.snapshots_to_device(rows), 4, 1, root_cap=n_cells)
            assert h.status == "OK" and h.n_root > 0
        cols = {k: np.concatenate([w[k] for w in held]) for k in b}
        n = len(cols["rank"])
        g = an.analyze_window(FAR, n_records=max(n, 1), per_record=True)
        ref = o.analyze_window(cols, FAR)
        blame, order = an.rank_blame()
        compare(g, ref, blame, order, what=f"batch{i}")
    an.close()
