"""GPU parity: ccld_progress_rates through the C ABI against the CPU oracle (bit-exact tables), and
the communication-slow root that ccld_analyze_window reports afterwards."""
import numpy as np
import pytest

from oracle import ccld_oracle as orc
from paper_2605_04478_amd import tracegen as tg
from tests.helpers import T0, ring_topology, rounds_with_durations, toy_cols
from tests.test_oracle_rates import series_cols

pytestmark = pytest.mark.gpu
NO_RANK = 0xFFFFFFFF


def run_both(topo, cols, n_snap, n_ch, on_device=True, what=""):
    from paper_2605_04478_amd import ccld
    n_cells = int(topo.size.sum()) * n_snap * n_ch
    an = ccld.Analyzer(topo, max_window_records=1024, max_snapshot_rows=max(n_cells, int(cols["snap"].shape[0]), 1))
    g = an.progress_rates(an.snapshots_to_device(cols) if on_device else cols, n_snap, n_ch)
    o = orc.Oracle(topo).progress_rates(cols, n_snap, n_ch)
    assert g.status == o.status, (what, g.status, o.status)
    if o.status == "OK":
        assert g.n_pair == len(o.pair["rank"]) and g.n_comm == len(o.comm["comm"]), what
        for name in ("pair", "comm"):
            gt, ot = getattr(g, name), getattr(o, name)
            for k in ot:
                assert np.array_equal(gt[k], ot[k]), (what, name, k, gt[k][:8], ot[k][:8])
    an.close()
    return g, o


@pytest.mark.parametrize("n_snap,n_ch", [(64, 4), (65, 1), (130, 3), (7, 2), (1, 1), (200, 2)])
def test_generated_series_parity(n_snap, n_ch):
    # series shorter than, equal to and longer than one wavefront of samples, with runs that cross
    # the 64-sample chunks
    lay = tg.Layout3D(tp=4, pp=2, dp=4, world=True)
    tr = tg.generate_rates(tg.RateSpec(layout=lay, n_snapshots=n_snap, n_channels=n_ch, seed=n_snap))
    g, o = run_both(tr.topo, tr.cols, n_snap, n_ch, what=f"rates{n_snap}x{n_ch}")
    if n_snap >= 64:
        mine = np.unique(o.pair["comm"][o.pair["rank"] == tr.slow_rank])
        assert all(g.comm["root"][c] == tr.slow_rank for c in mine)


def test_random_series_with_long_runs_and_idle_channels():
    rng = np.random.default_rng(4)
    topo = ring_topology(6, comms=[[0, 1, 2, 3, 4, 5], [4, 1, 3], [2, 5]])
    n_snap, n_ch = 150, 3
    series = {}
    for c, members in enumerate([[0, 1, 2, 3, 4, 5], [4, 1, 3], [2, 5]]):
        for r in members:
            for ch in range(n_ch):
                s, q, sent, recv = [], 10, 0, 0
                for t in range(n_snap):
                    if rng.random() < 0.04:
                        q, sent, recv = q + int(rng.integers(1, 3)), 0, 0
                    if ch != 2 or r % 2 == 0:                  # channel 2 of odd ranks never moves
                        sent += int(rng.integers(0, 3)) * int(rng.random() < 0.5)
                        recv += int(rng.integers(0, 2))
                    s.append((q, sent, recv))
                series[(r, c, ch)] = s
    run_both(topo, series_cols(series), n_snap, n_ch, what="random-series")
    run_both(topo, series_cols(series), n_snap, n_ch, on_device=False, what="random-series-host")


def test_ranks_in_more_than_four_communicators():
    # the membership lookup leaves its packed row: placement falls back to searching the member list
    rng = np.random.default_rng(9)
    comms = [[3, 0, 2, 1], [0, 1], [2, 0], [0, 3], [1, 0, 3], [2, 3]]
    topo = ring_topology(4, comms=comms)
    series = {}
    for c, members in enumerate(comms):
        for r in members:
            q, sent, recv, s = 3, 0, 0, []
            for t in range(40):
                if rng.random() < 0.15:
                    q, sent, recv = q + 1, 0, 0
                sent += int(rng.integers(0, 3)); recv += int(rng.integers(0, 2))
                s.append((q, sent, recv))
            series[(r, c, 0)] = s
    run_both(topo, series_cols(series), 40, 1, what="five-comms")


def test_paper_example_and_validation():
    topo = ring_topology(2)
    series = {(0, 0, 0): [(7, s, 0) for s in [0, 5, 8, 8, 8, 8, 8, 8]] + [(8, 0, 0)],
              (1, 0, 0): [(7, s, 0) for s in [0, 1, 2, 3, 5, 6, 7, 8]] + [(8, 0, 0)]}
    g, o = run_both(topo, series_cols(series), 9, 1, what="example")
    assert list(g.pair["changes_send"]) == [2, 7] and g.comm["root"][0] == 1
    cols = series_cols(series)
    gap = {k: v[:-1] for k, v in cols.items()}
    run_both(topo, gap, 9, 1, what="gap")
    dup = {k: np.concatenate([v, v[:1]]) for k, v in cols.items()}
    run_both(topo, dup, 9, 1, what="dup")
    bad = {k: v.copy() for k, v in cols.items()}
    bad["rank"][3] = 5
    run_both(topo, bad, 9, 1, what="member")


def test_communication_slow_root_follows_the_rate_pass():
    from paper_2605_04478_amd import ccld
    topo = ring_topology(4)
    rows = rounds_with_durations([[1000, 1010, 1005, 1001]] * 3 + [[9000, 9100, 9050, 9020]])
    cols = toy_cols(rows)
    series = {(r, 0, 0): [(1, 0, 0), (1, 8, 8), (2, 0, 0)] for r in range(4)}
    series[(3, 0, 0)] = [(1, 2, 8), (1, 8, 8), (2, 0, 0)]
    an = ccld.Analyzer(topo, max_window_records=64, max_snapshot_rows=64, tbase_init_ns=1000)
    o = orc.Oracle(topo, {"tbase_init_ns": 1000})
    for with_rates in (False, True):
        if with_rates:
            assert an.progress_rates(series_cols(series), 3, 1).status == "OK"
            o.progress_rates(series_cols(series), 3, 1)
        an.reset_window()
        an.ingest(an.to_device(cols))
        g = an.analyze_window(T0 + 10**10)
        w = o.analyze_window(cols, T0 + 10**10)
        assert np.array_equal(g.group["class"], w.group["class"]) and g.group["class"][0] == 2
        assert np.array_equal(g.group["root_s2"], w.group["root_s2"])
        assert g.group["root_s2"][0] == (3 if with_rates else NO_RANK)
    an.close()


def test_silent_runs_and_the_receive_side_parity():
    topo = ring_topology(2)
    silent = {(0, 0, 0): [(5, 3, 0), (5, 3, 0), (6, 0, 0), (6, 0, 0), (7, 2, 0), (7, 2, 0), (8, 0, 0)],
              (1, 0, 0): [(5, 1, 0), (5, 2, 0), (6, 1, 0), (6, 2, 0), (7, 1, 0), (7, 2, 0), (8, 0, 0)]}
    g, o = run_both(topo, series_cols(silent), 7, 1, what="silent run")
    assert list(g.pair["ops_send"]) == [2, 3] and list(g.pair["changes_send"]) == [2, 6]
    fast, slow = [1, 4, 4, 4], [1, 2, 3, 4]
    recv = {(0, 0, 0): [(3, s, v) for s, v in zip(fast, fast)] + [(4, 0, 0)],
            (1, 0, 0): [(3, s, v) for s, v in zip(fast, slow)] + [(4, 0, 0)]}
    g, o = run_both(topo, series_cols(recv), 5, 1, what="receive side")
    assert g.comm["root_send"][0] == 0 and g.comm["root_recv"][0] == 1 and g.comm["root"][0] == 1



def test_location_needs_a_slow_window_and_the_rate_root_is_for_communication_only_parity():
    from paper_2605_04478_amd import ccld
    topo = ring_topology(2)
    prm = dict(tbase_init_ns=1000, repeat_threshold=2)
    an = ccld.Analyzer(topo, max_window_records=64, max_snapshot_rows=64, **prm)
    o = orc.Oracle(topo, prm)
    series = {(0, 0, 0): [(1, 0, 0), (1, 8, 8), (2, 0, 0)], (1, 0, 0): [(1, 2, 8), (1, 8, 8), (2, 0, 0)]}
    assert an.progress_rates(series_cols(series), 3, 1).status == "OK"
    o.progress_rates(series_cols(series), 3, 1)
    want = [(1, 1, 0, 1), (1, 2, 1, 1), (0, 2, 0, 0)]                 # slow, repeats, locate, class per window
    for s, durs in enumerate([[9000, 1000], [9000, 1000], [1200, 1100]]):
        cols = toy_cols(rounds_with_durations([durs], seq0=s))
        an.reset_window()
        an.ingest(an.to_device(cols))
        g = an.analyze_window(T0 + 10**12)
        w = o.analyze_window(cols, T0 + 10**12)
        for k in w.group:
            assert np.array_equal(g.group[k], w.group[k]), (s, k)
        assert (g.group["slow"][0], g.group["repeats"][0], g.group["locate"][0], g.group["class"][0]) == want[s]
        assert g.group["root_s2"][0] == NO_RANK
    an.close()
