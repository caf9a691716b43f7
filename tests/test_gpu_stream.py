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
