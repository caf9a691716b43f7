"""Pins of the oracle's SendRate / RecvRate pass (Section 4.1.2, "Slow Diagnostic Metrics", and
the communication-slow root of Eq. 4): the paper's worked example, closed forms by construction,
invariances, and recovery of the generator's slow rank."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import ccld_oracle as orc
from paper_2605_04478_amd import tracegen as tg
from tests.helpers import T0, ring_topology, rounds_with_durations, toy_cols

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "sendrate_example.txt")
NO_RANK = 0xFFFFFFFF


def golden():
    out = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if line:
            k, v = [x.strip() for x in line.split("=")]
            out[k] = Fraction(v)
    return out


def series_cols(series, n_channels=1):
    """series[(rank, comm, channel)] = list of (seq, sent, recv) per snapshot -> snapshot columns."""
    rows = []
    for (r, c, ch), samples in series.items():
        for t, (q, s, v) in enumerate(samples):
            rows.append((t, r, c, ch, q, s, v))
    g = lambda i, dt: np.asarray([x[i] for x in rows], dtype=dt)
    return {"snap": g(0, np.uint32), "rank": g(1, np.uint32), "comm": g(2, np.uint32), "channel": g(3, np.uint32),
            "seq_posted": g(4, np.uint64), "chunks_sent": g(5, np.uint32), "chunks_recv": g(6, np.uint32)}


def rates(topo, series, n_snap, n_ch=1, oracle=None):
    o = oracle or orc.Oracle(topo)
    r = o.progress_rates(series_cols(series), n_snap, n_ch)
    assert r.status == "OK"
    return r


def test_paper_example_two_versus_seven_changes():
    g = golden()
    total = int(g["sends_per_operation"])
    # rank 0: the 8 sends show up as 2 value changes; rank 1: as 7; one more sample of the next
    # operation closes the run
    normal = [0, 5, 8, 8, 8, 8, 8, 8]
    slow = [0, 1, 2, 3, 5, 6, 7, 8]
    assert normal[-1] == slow[-1] == total
    topo = ring_topology(2)
    series = {(0, 0, 0): [(7, s, 0) for s in normal] + [(8, 0, 0)],
              (1, 0, 0): [(7, s, 0) for s in slow] + [(8, 0, 0)]}
    r = rates(topo, series, 9)
    ops, chg = r.pair["ops_send"], r.pair["changes_send"]
    assert list(chg) == [int(g["normal_value_changes"]), int(g["slow_value_changes"])]
    assert Fraction(int(ops[0]), int(chg[0])) == g["normal_rate"]
    assert Fraction(int(ops[1]), int(chg[1])) == g["slow_rate"]
    assert r.comm["root_send"][0] == 1 and r.comm["root"][0] == 1
    assert r.comm["root_recv"][0] == NO_RANK            # nobody received anything: no RecvRate


def test_changes_equal_the_samples_an_operation_keeps_moving():
    # closed form by construction: rank r's count moves at k_r consecutive samples of each operation
    topo = ring_topology(4)
    ks = [1, 2, 5, 3]
    n_ops, period = 4, 8
    series = {}
    for r, k in enumerate(ks):
        s = []
        for j in range(n_ops + 1):                       # the last operation stays open
            for u in range(period):
                s.append((100 + j, (16 * min(u, k)) // k, (16 * min(u, k + 1)) // (k + 1)))
        series[(r, 0, 0)] = s
    r = rates(topo, series, (n_ops + 1) * period)
    assert list(r.pair["ops_send"]) == [n_ops] * 4 and list(r.pair["ops_recv"]) == [n_ops] * 4
    assert list(r.pair["changes_send"]) == [n_ops * k for k in ks]
    assert list(r.pair["changes_recv"]) == [n_ops * (k + 1) for k in ks]
    assert r.comm["root_send"][0] == 2 and r.comm["root_recv"][0] == 2 and r.comm["root"][0] == 2


def test_open_run_is_ignored_and_first_sample_counts_against_zero():
    topo = ring_topology(2)
    # rank 0: operation 5 observed from its second chunk on (first sample already non-zero: a change),
    # then operation 6 unfinished; rank 1: only ever one operation counter -> everything is open
    series = {(0, 0, 0): [(5, 3, 0), (5, 3, 0), (5, 8, 1), (6, 1, 0), (6, 4, 0), (6, 6, 0)],
              (1, 0, 0): [(6, 0, 0), (6, 1, 0), (6, 2, 0), (6, 3, 0), (6, 4, 0), (6, 5, 0)]}
    r = rates(topo, series, 6)
    assert list(r.pair["ops_send"]) == [1, 0] and list(r.pair["changes_send"]) == [2, 0]
    assert list(r.pair["ops_recv"]) == [1, 0] and list(r.pair["changes_recv"]) == [1, 0]
    assert r.comm["root"][0] == 0


def test_sampling_twice_as_often_changes_nothing():
    tr = tg.generate_rates(tg.RateSpec(layout=tg.Layout3D(tp=2, pp=2, dp=2), n_snapshots=40, n_channels=2, seed=3),
                           shuffle=False)
    o1 = orc.Oracle(tr.topo)
    a = o1.progress_rates(tr.cols, 40, 2)
    # every snapshot repeated: samples 2t and 2t+1 show the same counts
    c2 = {k: np.concatenate([v, v]) for k, v in tr.cols.items()}
    c2["snap"] = np.concatenate([tr.cols["snap"] * 2, tr.cols["snap"] * 2 + 1]).astype(np.uint32)
    b = orc.Oracle(tr.topo).progress_rates(c2, 80, 2)
    for k in a.pair:
        assert np.array_equal(a.pair[k], b.pair[k]), k
    for k in a.comm:
        assert np.array_equal(a.comm[k], b.comm[k]), k


def test_channels_add_up():
    # the same two series once on two channels of one pair, once on one channel of two pairs
    topo2 = ring_topology(2)
    s_a = [(1, 0, 0), (1, 4, 2), (1, 8, 8), (2, 0, 0)]
    s_b = [(1, 0, 0), (1, 1, 0), (1, 5, 3), (2, 0, 0)]
    two_channels = {(0, 0, 0): s_a, (0, 0, 1): s_b, (1, 0, 0): s_a, (1, 0, 1): s_a}
    o = orc.Oracle(topo2)
    r = o.progress_rates(series_cols(two_channels), 4, 2)
    assert r.status == "OK"
    assert list(r.pair["changes_send"]) == [2 + 2, 2 + 2] and list(r.pair["ops_send"]) == [2, 2]
    assert list(r.pair["changes_recv"]) == [2 + 1, 2 + 2] and list(r.pair["ops_recv"]) == [2, 2]
    assert r.comm["root_recv"][0] == 1                   # 2/4 < 2/3


def test_row_order_and_generator_truth():
    spec = tg.RateSpec(layout=tg.Layout3D(tp=4, pp=2, dp=4), n_snapshots=64, n_channels=4, seed=5)
    a = tg.generate_rates(spec, shuffle=False)
    b = tg.generate_rates(spec, shuffle=True)
    ra = orc.Oracle(a.topo).progress_rates(a.cols, 64, 4)
    rb = orc.Oracle(b.topo).progress_rates(b.cols, 64, 4)
    for k in ra.pair:
        assert np.array_equal(ra.pair[k], rb.pair[k]), k
    # the slow rank has the smallest rate in every communicator it belongs to, in both directions
    mine = np.unique(ra.pair["comm"][ra.pair["rank"] == a.slow_rank])
    assert len(mine) == 3
    for c in mine:
        assert ra.comm["root_send"][c] == a.slow_rank and ra.comm["root_recv"][c] == a.slow_rank
        assert ra.comm["root"][c] == a.slow_rank
    # a healthy run names somebody, but nobody stands out: every rate is at least 1/3
    h = tg.generate_rates(tg.RateSpec(layout=spec.layout, n_snapshots=64, n_channels=4, seed=5, slow_rank=-1))
    rh = orc.Oracle(h.topo).progress_rates(h.cols, 64, 4)
    assert np.all(3 * rh.pair["ops_send"] >= rh.pair["changes_send"])
    assert np.all(rh.pair["changes_send"] >= rh.pair["ops_send"])


def test_validation_matches_hang_location():
    topo = ring_topology(2)
    ok = {(0, 0, 0): [(1, 0, 0), (2, 0, 0)], (1, 0, 0): [(1, 0, 0), (2, 0, 0)]}
    cols = series_cols(ok)
    o = orc.Oracle(topo)
    assert o.progress_rates(cols, 2, 1).status == "OK"
    bad = {k: v.copy() for k, v in cols.items()}
    bad["comm"][0] = 9
    assert o.progress_rates(bad, 2, 1).status == "E_UNKNOWN_COMM"
    gap = {k: v[:-1] for k, v in cols.items()}
    assert o.progress_rates(gap, 2, 1).status == "E_SNAPSHOT_GAP"
    dup = {k: np.concatenate([v, v[:1]]) for k, v in cols.items()}
    assert o.progress_rates(dup, 2, 1).status == "E_DUPLICATE_KEY"


def test_communication_slow_root_uses_the_rate_pass():
    # Eq. 4 with P < alpha: one round where every rank's duration is long and nearly equal
    topo = ring_topology(4)
    rows = rounds_with_durations([[1000, 1010, 1005, 1001]] * 3 + [[9000, 9100, 9050, 9020]])
    o = orc.Oracle(topo, {"tbase_init_ns": 1000})
    w = o.analyze_window(toy_cols(rows), T0 + 10**10)
    assert w.group["class"][0] == 2 and w.group["root_s2"][0] == NO_RANK and w.group["root_s1"][0] == NO_RANK
    series = {(r, 0, 0): [(1, 0, 0), (1, 8, 8), (2, 0, 0)] for r in range(4)}
    series[(3, 0, 0)] = [(1, 2, 8), (1, 8, 8), (2, 0, 0)]       # two changes: 2 (against zero), then 8
    o.progress_rates(series_cols(series), 3, 1)
    w = o.analyze_window(toy_cols(rows), T0 + 10**10)
    assert w.group["class"][0] == 2 and w.group["root_s2"][0] == 3


def test_equal_rates_name_the_smaller_rank():
    """Ranks 1 and 2 both show 3 changes per operation (rate 1/3), rank 0 shows 1, rank 3 shows 2:
    the minimal rate is shared, the smaller rank is reported.  2/6 equals 1/3 as well."""
    topo = ring_topology(4)
    fast = [(1, 0, 0), (1, 8, 8), (1, 8, 8), (1, 8, 8), (2, 0, 0)]
    three = [(1, 0, 0), (1, 2, 2), (1, 5, 5), (1, 8, 8), (2, 0, 0)]
    two = [(1, 0, 0), (1, 4, 4), (1, 8, 8), (1, 8, 8), (2, 0, 0)]
    series = {(0, 0, 0): fast, (1, 0, 0): three, (2, 0, 0): three, (3, 0, 0): two}
    r = rates(topo, series, 5)
    assert list(r.pair["ops_send"]) == [1, 1, 1, 1] and list(r.pair["changes_send"]) == [1, 3, 3, 2]
    assert r.comm["root_send"][0] == 1 and r.comm["root_recv"][0] == 1 and r.comm["root"][0] == 1
    # rank 0 with two operations of three changes each: 2/6 == 1/3, now rank 0 is the smallest of the tied ranks
    twice = [(1, 0, 0), (1, 2, 2), (1, 5, 5), (1, 8, 8), (2, 1, 1), (2, 4, 4), (2, 8, 8), (3, 0, 0)]
    pad = lambda s: s[:-1] + [s[-2]] * 3 + [s[-1]]
    series = {(0, 0, 0): twice, (1, 0, 0): pad(three), (2, 0, 0): pad(three), (3, 0, 0): pad(two)}
    r = rates(topo, series, 8)
    assert list(r.pair["ops_send"]) == [2, 1, 1, 1] and list(r.pair["changes_send"]) == [6, 3, 3, 2]
    assert r.comm["root_send"][0] == 0 and r.comm["root"][0] == 0


def test_an_operation_without_any_change_is_not_an_observed_operation():
    """Rank 0 sends in operations 5 and 7 but not in 6 (one change each, three runs): two observed operations, two
    changes.  Counting the silent run as an operation would make it 3/2."""
    topo = ring_topology(2)
    series = {(0, 0, 0): [(5, 3, 0), (5, 3, 0), (6, 0, 0), (6, 0, 0), (7, 2, 0), (7, 2, 0), (8, 0, 0)],
              (1, 0, 0): [(5, 1, 0), (5, 2, 0), (6, 1, 0), (6, 2, 0), (7, 1, 0), (7, 2, 0), (8, 0, 0)]}
    r = rates(topo, series, 7)
    assert list(r.pair["ops_send"]) == [2, 3] and list(r.pair["changes_send"]) == [2, 6]


def test_the_root_is_the_member_whose_smaller_rate_is_minimal_send_or_receive():
    """Rank 1 sends as fast as rank 0 but receives slowly: it is the RecvRate root and, its RecvRate being the
    smallest rate of all, the communicator's root."""
    topo = ring_topology(2)
    fast = [1, 4, 4, 4]
    slow = [1, 2, 3, 4]
    series = {(0, 0, 0): [(3, s, v) for s, v in zip(fast, fast)] + [(4, 0, 0)],
              (1, 0, 0): [(3, s, v) for s, v in zip(fast, slow)] + [(4, 0, 0)]}
    r = rates(topo, series, 5)
    assert list(r.pair["changes_send"]) == [2, 2] and list(r.pair["changes_recv"]) == [2, 4]
    assert r.comm["root_send"][0] == 0 and r.comm["root_recv"][0] == 1 and r.comm["root"][0] == 1

