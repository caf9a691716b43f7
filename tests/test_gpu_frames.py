"""GPU parity: ccld_decode_frames through the C ABI against the CPU oracle (identical rows and
statuses), and hang location from rows decoded on the device."""
import numpy as np
import pytest

from oracle import ccld_oracle as orc
from paper_2605_04478_amd import tracegen as tg
from tests.helpers import ring_topology
from tests.test_oracle_frames import G, pack_frame

pytestmark = pytest.mark.gpu
UNSIGNED = {"snap": np.uint32, "rank": np.uint32, "comm": np.uint32, "channel": np.uint32,
            "seq_posted": np.uint64, "chunks_sent": np.uint32, "chunks_recv": np.uint32}


def host(rows):
    return {k: v.cpu().numpy().view(UNSIGNED[k]) for k, v in rows.items()}


def both(an, o, frames, ranks, snap, n_ch, on_device=False, what=""):
    so, ro = o.decode_frames(frames, ranks, snap)
    if on_device:
        import torch
        fd = torch.from_numpy(np.ascontiguousarray(frames).view(np.uint8).reshape(-1).copy()).to(an.device)
        rd = torch.from_numpy(np.ascontiguousarray(ranks, dtype=np.uint32).view(np.int32).copy()).to(an.device)
        sg, rg = an.decode_frames(fd, rd, snap, n_ch)
    else:
        sg, rg = an.decode_frames(frames, ranks, snap, n_ch)
    assert sg == so, (what, sg, so)
    if so == "OK":
        rg = host(rg)
        for k in ro:
            assert np.array_equal(rg[k], ro[k]), (what, k)
    return so, rg


def test_hand_packed_frames_errors_and_carry_forward():
    from paper_2605_04478_amd import ccld
    topo = ring_topology(3, comms=[[0, 1, 2], [2, 0]])
    an = ccld.Analyzer(topo, max_window_records=16, max_snapshot_rows=4096)
    o = orc.Oracle(topo)
    o.frames_begin(2)
    f0 = pack_frame([(5, 0, True, 40, [(7, 6), (9, 8)]), (6, 1, True, 11, [(1, 2), (3, 4)]),
                     (2, 1, False, 99, [(50, 50), (50, 50)])], n_channels=2)
    f1 = pack_frame([(0, 0, True, 41, [(2, 1), (0, 0)]), (7, 0, True, 42, [(1, 0), (1, 1)])], n_channels=2)
    f2 = pack_frame([(1, 0, True, 43, [(5, 5), (6, 6)])], n_channels=1)
    for s, (fr, rk) in enumerate([(f0, 0), (f1, 0), (f0, 0), (f2, 0), (f1, 2)]):
        both(an, o, np.stack([fr]), np.asarray([rk]), s, 2, on_device=bool(s % 2), what=f"step{s}")
    bad = [(pack_frame([(0, 9, True, 6, [(1, 1)])], 2), 1), (pack_frame([(0, 1, True, 6, [(1, 1)])], 2), 1),
           (pack_frame([(0, 0, True, 6, [(1, 1)])], 2), 7), (pack_frame([(0, 0, True, 6, [(1, 1)])], 9), 1),
           (pack_frame([(0, 0, True, 6, [(2**32, 1)])], 2), 1)]
    for i, (fr, rk) in enumerate(bad):
        st, _ = both(an, o, np.stack([fr]), np.asarray([rk]), 9, 2, what=f"bad{i}")
        assert st != "OK"
    st, _ = both(an, o, np.stack([f0, f0]), np.asarray([0, 0]), 9, 2, what="dup")
    assert st == "E_DUPLICATE_KEY"
    both(an, o, np.zeros((0, G["frame_bytes"]), np.uint8), np.zeros(0, np.uint32), 10, 2, what="after-errors")
    an.reset_frames()
    o.frames_begin(2)
    both(an, o, np.stack([f2]), np.asarray([1]), 11, 2, what="after-reset")
    # equal operation counters in three blocks (the block further back wins), the largest 32-bit count, and a range
    # error that outranks two frames of one rank
    an.reset_frames()
    o.frames_begin(2)
    f3 = pack_frame([(1, 0, True, 50, [(1, 1), (1, 1)]), (6, 0, True, 50, [(2, 2), (2, 2)]), (3, 0, True, 50, [(3, 3), (3, 3)])],
                    n_channels=2)
    edge = pack_frame([(0, 0, True, 51, [(2**32 - 1, 2**32 - 1), (2, 2)])], n_channels=2)
    _, rows = both(an, o, np.stack([f3]), np.asarray([0]), 12, 2, what="equal counters")
    m = (rows["rank"] == 0) & (rows["comm"] == 0)
    assert list(rows["chunks_sent"][m]) == [2, 2]
    both(an, o, np.stack([edge]), np.asarray([1]), 13, 2, on_device=True, what="largest count")
    nine = pack_frame([(0, 0, True, 6, [(1, 1)])], 9)
    st, _ = both(an, o, np.stack([nine, f2, f2]), np.asarray([0, 1, 1]), 14, 2, what="range+dup")
    assert st == "E_RANGE"
    an.close()


@pytest.mark.parametrize("lay,n_ch", [(tg.Layout3D(tp=2, pp=2, dp=4, world=True), 4),
                                      (tg.Layout3D(tp=4, pp=2, dp=8, world=True), 8)])
def test_hang_series_decoded_on_the_device(lay, n_ch):
    from paper_2605_04478_amd import ccld
    n_snap = 40
    ht = tg.generate_hang(tg.config4(layout=lay, n_channels=n_ch, n_snapshots=n_snap, hang_snapshot=5), shuffle=False)
    n_rows = ht.n
    an = ccld.Analyzer(ht.topo, max_window_records=16, max_snapshot_rows=n_rows)
    o = orc.Oracle(ht.topo)
    o.frames_begin(n_ch)
    rng = np.random.default_rng(4)
    c = ht.cols
    prev = None
    dev_rows = {k: [] for k in c}
    for s in range(n_snap):
        m = c["snap"] == s
        rows = {k: v[m] for k, v in c.items()}
        order = np.lexsort((rows["channel"], rows["comm"], rows["rank"]))
        state = np.stack([rows[k][order].astype(np.int64) for k in ("seq_posted", "chunks_sent", "chunks_recv")])
        state = state.reshape(3, ht.topo.n_ranks, 4, n_ch)
        changed = np.ones((ht.topo.n_ranks, 4), bool) if prev is None else (state != prev).any(axis=(0, 3))
        keep = changed | (rng.random(changed.shape) < 0.5)
        prev = state
        frames, ranks = tg.encode_frames(ht.topo, rows, n_ch, keep=keep, kernel_counter=3 * s)
        p = rng.permutation(len(ranks))
        st, rg = both(an, o, frames[p], ranks[p], s, n_ch, on_device=bool(s % 2), what=f"snap{s}")
        assert st == "OK"
        for k in dev_rows:
            dev_rows[k].append(rg[k])
    cols = {k: np.concatenate(v) for k, v in dev_rows.items()}
    g = an.locate_hang(an.snapshots_to_device(cols), n_snap, n_ch)
    assert g.status == "OK" and list(g.root["rank"]) == [ht.root_rank] and list(g.root["comm"]) == [ht.root_comm]
    an.close()
