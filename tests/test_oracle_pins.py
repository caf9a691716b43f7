"""Pins of the CPU oracle's window analysis: each test checks the oracle
against something fixed by the paper or by mathematics (closed forms of Eq. 1-4,
the paper's limiting cases and constants, brute-force definitions, library
routines on special cases, invariants, recovery of injected faults)."""
import os

import numpy as np
import pytest
import scipy.stats

from oracle import ccld_oracle as orc
from paper_2605_04478_amd import tracegen as tg
from tests.helpers import INFLIGHT, T0, concat_cols, ring_topology, rounds_with_durations, toy_cols

NO_RANK = orc.NO_RANK
FAR = T0 + 10**15      # a "now" that is later than everything


def analyze(topo, cols, now=FAR, **params):
    o = orc.Oracle(topo, params)
    return o.analyze_window(cols, now), o


def test_defaults_match_constants_stated_in_paper():
    vals = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "paper_constants.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = [x.strip() for x in line.split("=")]
                vals[k] = float(v)
    P = orc.DEFAULT_PARAMS
    assert P["hang_threshold_ns"] == vals["hang_threshold_minutes"] * 60e9
    assert P["tbase_rounds"] == vals["tbase_rounds"]
    assert P["tbase_warmup_ns"] == vals["tbase_warmup_minutes"] * 60e9
    assert P["theta_num"] / P["theta_den"] == vals["theta_slow"]
    assert P["alpha_num"] / P["ab_den"] == vals["alpha"]
    assert P["beta_num"] / P["ab_den"] == vals["beta"]
    assert P["barrier_bytes"] == vals["barrier_bytes"]


# --------------------------------------------------------------------------
# grouping
# --------------------------------------------------------------------------
def test_grouping_equals_lexicographic_sort():
    tr = tg.generate(tg.config2(n_cycles=20)).shuffled(3)
    r, _ = analyze(tr.topo, tr.cols)
    assert r.status == "OK"
    c = tr.cols
    ref = np.lexsort((c["rank"], c["seq"], c["comm"]))
    assert np.array_equal(r.perm, ref.astype(np.uint64))
    # one segment per distinct (comm, seq), in order
    pairs = np.unique(np.stack([c["comm"].astype(np.int64), c["seq"].astype(np.int64)], 1), axis=0)
    assert np.array_equal(r.seg["comm"], pairs[:, 0]) and np.array_equal(r.seg["seq"], pairs[:, 1])
    assert r.seg["n"].sum() == tr.n


def _same(a: orc.WindowResult, b: orc.WindowResult):
    for name in ("rec", "seg", "flag", "group", "alert", "blame"):
        da, db = getattr(a, name), getattr(b, name)
        for k in da:
            assert np.array_equal(da[k], db[k]), (name, k)
    assert np.array_equal(a.cand, b.cand) and np.array_equal(a.order, b.order)


def test_results_do_not_depend_on_record_order():
    tr = tg.generate(tg.config2(n_cycles=30))
    # make it interesting: some in-flight records, one missing member
    cols = {k: v.copy() for k, v in tr.cols.items()}
    last = cols["seq"] == cols["seq"][cols["comm"] == 70].max()
    cols["t_exit"][(cols["comm"] == 70) & last] = INFLIGHT
    keep = ~((cols["comm"] == 3) & (cols["seq"] == 5) & (cols["rank"] == tr.topo.members_of(3)[2]))
    cols = {k: v[keep] for k, v in cols.items()}
    base, _ = analyze(tr.topo, cols, hang_threshold_ns=1_000_000)
    assert len(base.alert["comm"]) >= 1 and len(base.flag["comm"]) > 0
    n = cols["rank"].shape[0]
    for s in range(10):
        p = np.random.default_rng(s).permutation(n)
        r, _ = analyze(tr.topo, {k: v[p] for k, v in cols.items()}, hang_threshold_ns=1_000_000)
        _same(base, r)
        # same records in the same sorted order
        assert np.array_equal(p[r.perm.astype(np.int64)], base.perm.astype(np.int64))


# --------------------------------------------------------------------------
# order statistics
# --------------------------------------------------------------------------
def _count_def_median(x):
    """The lower median by its counting definition, without sorting."""
    k = (len(x) - 1) // 2
    for v in x:
        if np.sum(x < v) <= k < np.sum(x <= v):
            return int(v)
    raise AssertionError


def test_median_and_mad_against_counting_definition_and_library():
    rng = np.random.default_rng(7)
    R = 17
    topo = ring_topology(R)
    rows, present = [], {}
    for s in range(300):
        n = int(rng.integers(1, R + 1))
        ranks = np.sort(rng.choice(R, n, replace=False))
        te = T0 + rng.integers(0, 12, n)            # many ties
        tx = te + rng.integers(0, 9, n)
        present[s] = (te.copy(), tx.copy())
        for r, a, b in zip(ranks, te, tx):
            rows.append((int(r), 0, s, 0, 1024, int(a), int(b)))
    r, _ = analyze(topo, toy_cols(rows))
    assert r.status == "OK" and len(r.seg["seq"]) == 300
    for s in range(300):
        te, tx = present[s]
        for name, x in (("enter", te), ("exit", tx)):
            med = _count_def_median(x)
            mad = _count_def_median(np.abs(x - med))
            assert r.seg[name + "_med"][s] == med
            assert r.seg[name + "_mad"][s] == mad
            assert r.seg[name + "_min"][s] == x.min() and r.seg[name + "_max"][s] == x.max()
            assert r.seg[name + "_min"][s] <= med <= r.seg[name + "_max"][s]
            if len(x) % 2 == 1:       # odd n: the lower median is the textbook median
                assert med - T0 == int(np.median(x - T0))
                assert mad == int(scipy.stats.median_abs_deviation(x - T0))
            if np.sum(x == med) * 2 > len(x):
                assert mad == 0
        d = tx - te
        assert r.seg["dur_min"][s] == d.min() and r.seg["dur_max"][s] == d.max()


def test_duration_extremes_break_ties_towards_smallest_rank():
    topo = ring_topology(4)
    rows = [(0, 0, 0, 0, 64, T0, T0 + 50), (1, 0, 0, 0, 64, T0, T0 + 10), (2, 0, 0, 0, 64, T0 + 5, T0 + 15),
            (3, 0, 0, 0, 64, T0 + 1, T0 + 51)]
    r, _ = analyze(topo, toy_cols(rows))
    assert r.seg["dur_min"][0] == 10 and r.seg["argmin_rank"][0] == 1
    assert r.seg["dur_max"][0] == 50 and r.seg["argmax_rank"][0] == 0


# --------------------------------------------------------------------------
# Eq. 1 - Eq. 4 closed forms
# --------------------------------------------------------------------------
US = 1000


def test_eq1_baseline_is_mean_of_first_m_round_maxima():
    topo = ring_topology(4)
    durs = [[10 * US, 5 * US, 5 * US, 5 * US], [20 * US] * 4, [30 * US, 1, 1, 1], [40 * US] * 4,
            [50 * US] * 4, [60 * US] * 4]
    rows = rounds_with_durations(durs)
    o = orc.Oracle(topo, dict(tbase_rounds=4, tbase_init_ns=1000))
    # first window: rounds 0..3 -> r <= m, the configured baseline applies
    first = toy_cols(rows[:16])
    r = o.analyze_window(first, FAR)
    assert r.group["m"][0] == 4 and r.group["frozen"][0] == 0
    assert r.group["static"][0] == 1 and r.group["tbase"][0] == 1000
    # re-analysing the same rounds changes nothing (watermark)
    r = o.analyze_window(first, FAR)
    assert r.group["m"][0] == 4 and r.group["frozen"][0] == 0
    # second window: rounds 4, 5 -> baseline = (10+20+30+40)/4 us
    r = o.analyze_window(toy_cols(rows[16:]), FAR)
    assert r.group["frozen"][0] == 1 and r.group["m"][0] == 4
    assert r.group["static"][0] == 0 and r.group["tbase"][0] == 25 * US
    # a window that still holds baseline rounds only: the configured value again
    r = o.analyze_window(first, FAR)
    assert r.group["static"][0] == 1 and r.group["tbase"][0] == 1000


def test_eq1_mean_is_floored():
    topo = ring_topology(2)
    rows = rounds_with_durations([[10, 1], [11, 1], [12, 1], [100, 100]])
    r, _ = analyze(topo, toy_cols(rows), tbase_rounds=3, tbase_init_ns=5)
    assert r.group["m"][0] == 3 and r.group["frozen"][0] == 1
    rows2 = rounds_with_durations([[10, 1], [11, 1], [13, 1], [100, 100]])
    r2, _ = analyze(topo, toy_cols(rows2), tbase_rounds=3, tbase_init_ns=5)
    # (10+11+12)/3 = 11 ; (10+11+13)/3 = 11.33 -> 11 ; r* = round 2 (largest range), which is a baseline round
    assert r.group["static"][0] == 1 and r2.group["static"][0] == 1
    # force r* to be the post-baseline round by giving it the largest range
    rows3 = rounds_with_durations([[10, 1], [11, 1], [13, 1], [100, 1]])
    r3, _ = analyze(topo, toy_cols(rows3), tbase_rounds=3, tbase_init_ns=5)
    assert r3.group["static"][0] == 0 and r3.group["tbase"][0] == 11


def test_eq1_m_is_limited_by_the_warmup_span():
    topo = ring_topology(2)
    # rounds every 50 s; warm-up span 120 s -> rounds at 0, 50, 100 s count, the one at 150 s freezes
    rows = rounds_with_durations([[10 * US, 1]] * 3 + [[70 * US, 1]] * 2, spacing_ns=50_000_000_000)
    r, _ = analyze(topo, toy_cols(rows), tbase_init_ns=7)
    assert r.group["m"][0] == 3 and r.group["frozen"][0] == 1
    assert r.group["static"][0] == 0 and r.group["tbase"][0] == 10 * US
    # fewer than tbase_rounds rounds, all inside the span: never frozen
    r, _ = analyze(topo, toy_cols(rows[:6]), tbase_init_ns=7)
    assert r.group["m"][0] == 3 and r.group["frozen"][0] == 0 and r.group["static"][0] == 1


def test_eq2_selects_largest_range_not_longest_round():
    topo = ring_topology(4)
    rows = rounds_with_durations([[100 * US] * 4, [10 * US, 50 * US, 20 * US, 30 * US], [90 * US] * 4])
    r, _ = analyze(topo, toy_cols(rows), tbase_init_ns=1000)
    assert r.group["rstar_seq"][0] == 1
    assert r.group["tmax"][0] == 50 * US and r.group["tmin"][0] == 10 * US
    # tie on the range -> the earliest round
    rows = rounds_with_durations([[5, 5, 5, 5], [10, 50, 20, 30], [60, 20, 30, 40]])
    r, _ = analyze(topo, toy_cols(rows), tbase_init_ns=1000)
    assert r.group["rstar_seq"][0] == 1


@pytest.mark.parametrize("tmax,slow", [(4000, 0), (4001, 1), (3999, 0), (500, 0)])
def test_eq3_threshold_is_strict(tmax, slow):
    topo = ring_topology(2)
    rows = rounds_with_durations([[tmax, max(tmax - 10, 0)]])
    r, _ = analyze(topo, toy_cols(rows), tbase_init_ns=1000)      # R = (Tmax-1000)/1000 vs theta = 3
    assert r.group["slow"][0] == slow


@pytest.mark.parametrize("tmin,cls", [
    (1000, 1),   # T_min -> T_base : P = 1, purely slow computation
    (5000, 2),   # T_min -> T_max  : P = 0, purely slow communication
    (3000, 3),   # P = 0.5, equal contribution
    (2600, 3),   # P = 0.6 exactly is not > beta
    (2599, 1),
    (3400, 3),   # P = 0.4 exactly is not < alpha
    (3401, 2),
])
def test_eq4_classification(tmin, cls):
    topo = ring_topology(3)
    rows = rounds_with_durations([[5000, tmin, 5000]])
    r, _ = analyze(topo, toy_cols(rows), tbase_init_ns=1000)
    assert r.group["slow"][0] == 1 and r.group["class"][0] == cls
    # computation-slow / mixed: the rank with minimal communication time is the root
    want = NO_RANK if cls == 2 else (1 if tmin < 5000 else 0)
    assert r.group["root_s1"][0] == want
    assert r.group["root_s2"][0] == NO_RANK


def test_repetition_counter_triggers_location_on_recurrence_only():
    topo = ring_topology(2)
    o = orc.Oracle(topo, dict(tbase_init_ns=1000, repeat_threshold=2))
    w1 = toy_cols(rounds_with_durations([[9000, 1000]], seq0=0))
    w2 = toy_cols(rounds_with_durations([[9000, 1000]], seq0=1))
    r = o.analyze_window(w1, FAR)
    assert r.group["slow"][0] == 1 and r.group["repeats"][0] == 1 and r.group["locate"][0] == 0
    r = o.analyze_window(w1, FAR)          # same round seen again: not a recurrence
    assert r.group["repeats"][0] == 1 and r.group["locate"][0] == 0
    r = o.analyze_window(w2, FAR)
    assert r.group["repeats"][0] == 2 and r.group["locate"][0] == 1


def test_detection_groups_split_by_operation_and_size_class():
    topo = ring_topology(2)
    rows = (rounds_with_durations([[100, 90]], op=tg.OP_ALLREDUCE, nbytes=1 << 20, seq0=0)
            + rounds_with_durations([[100, 90]], op=tg.OP_ALLGATHER, nbytes=1 << 20, seq0=1)
            + rounds_with_durations([[100, 90]], op=tg.OP_ALLREDUCE, nbytes=(1 << 21) - 1, seq0=2)
            + rounds_with_durations([[100, 90]], op=tg.OP_ALLREDUCE, nbytes=1 << 21, seq0=3))
    r, _ = analyze(topo, toy_cols(rows))
    got = list(zip(r.group["op"], r.group["cls"], r.group["n_usable"]))
    assert got == [(0, 20, 2), (0, 21, 1), (1, 20, 1)]


# --------------------------------------------------------------------------
# usability, barriers, hang alerts
# --------------------------------------------------------------------------
def test_barrier_rounds_are_never_flagged_or_alerted():
    topo = ring_topology(4)
    rows = []
    for s, nb in enumerate([0, 1, 3]):        # all-reduce of less than 4 bytes
        rows += [(r, 0, s, tg.OP_ALLREDUCE, nb, T0, T0 + 10) for r in range(3)]
        rows.append((3, 0, s, tg.OP_ALLREDUCE, nb, T0 + 10**9, INFLIGHT if s == 2 else T0 + 10**9 + 5))
    rows += [(r, 0, 3, tg.OP_ALLREDUCE, 4, T0, T0 + 10) for r in range(4)]   # 4 bytes: not a barrier
    r, _ = analyze(topo, toy_cols(rows), hang_threshold_ns=10)
    assert list(r.seg["state"] & orc.SEG_BARRIER) == [4, 4, 4, 0]
    assert list(r.seg["state"] & orc.SEG_USABLE) == [0, 0, 0, 8]
    assert len(r.flag["rank"]) == 0 and len(r.alert["comm"]) == 0
    assert len(r.group["comm"]) == 1 and r.group["n_usable"][0] == 1
    # the same late rank on a real operation is flagged
    rows2 = [(r, 0, 0, tg.OP_ALLREDUCE, 4096, T0, T0 + 10**9 + 5) for r in range(3)]
    rows2.append((3, 0, 0, tg.OP_ALLREDUCE, 4096, T0 + 10**9, T0 + 10**9 + 5))
    r2, _ = analyze(topo, toy_cols(rows2))
    assert list(r2.flag["rank"]) == [3] and list(r2.flag["kind"]) == [orc.FLAG_LATE_ENTER]
    assert r2.flag["lag_enter"][0] == 10**9


def test_inconsistent_or_incomplete_rounds_are_not_used():
    topo = ring_topology(3)
    late = 10**9
    rows = [(0, 0, 0, 0, 4096, T0, T0 + late + 9), (1, 0, 0, 0, 4096, T0, T0 + late + 9),
            (2, 0, 0, 0, 8192, T0 + late, T0 + late + 9)]                       # sizes differ
    rows += [(0, 0, 1, 0, 4096, T0, T0 + late + 9), (2, 0, 1, 0, 4096, T0 + late, T0 + late + 9)]  # rank 1 missing
    rows += [(0, 0, 2, 0, 4096, T0, T0 + late + 9), (1, 0, 2, 1, 4096, T0, T0 + late + 9),
             (2, 0, 2, 0, 4096, T0 + late, T0 + late + 9)]                      # operations differ
    r, _ = analyze(topo, toy_cols(rows))
    assert list(r.seg["state"]) == [orc.SEG_COMPLETE, orc.SEG_CONSISTENT, orc.SEG_COMPLETE]
    assert len(r.flag["rank"]) == 0 and len(r.group["comm"]) == 0
    assert list(r.seg["n"]) == [3, 2, 3]


def _hang_rows(kind):
    base = [(r, 0, 6, 0, 4096, T0 + r, T0 + 100) for r in range(4)]            # an earlier, healthy round
    t = T0 + 1000
    if kind == "H1":      # rank 2 never posted operation 7
        return base + [(r, 0, 7, 0, 4096, t + r, INFLIGHT) for r in (0, 1, 3)]
    if kind == "H2":      # everyone entered; ranks 2, 3 ran something else and left
        return base + [(0, 0, 7, 0, 4096, t, INFLIGHT), (1, 0, 7, 0, 4096, t + 1, INFLIGHT),
                       (2, 0, 7, 1, 4096, t + 2, t + 50), (3, 0, 7, 1, 4096, t + 3, t + 60)]
    return base + [(r, 0, 7, 0, 4096, t + 3 - r, INFLIGHT) for r in range(4)]  # H3: all hung


@pytest.mark.parametrize("kind,cls,cands", [("H1", 1, [2]), ("H2", 2, [2, 3]), ("H3", 3, [])])
def test_hang_alert_branches(kind, cls, cands):
    topo = ring_topology(4)
    cols = toy_cols(_hang_rows(kind))
    thr = 5_000
    first_enter = T0 + 1000
    r, _ = analyze(topo, cols, now=first_enter + thr, hang_threshold_ns=thr)
    assert len(r.alert["comm"]) == 0                      # duration == threshold: not exceeded
    r, _ = analyze(topo, cols, now=first_enter + thr + 1, hang_threshold_ns=thr)
    assert list(r.alert["seq"]) == [7] and list(r.alert["class"]) == [cls]
    assert r.alert["age"][0] == thr + 1
    assert list(r.cand[r.alert["cand_off"][0]: r.alert["cand_off"][0] + r.alert["n_cand"][0]]) == cands
    assert r.seg["inflight"][1] == {"H1": 3, "H2": 2, "H3": 4}[kind]


# --------------------------------------------------------------------------
# validation
# --------------------------------------------------------------------------
def test_validation_statuses():
    topo = ring_topology(4, comms=[[0, 1], [2, 3]])
    ok = [(0, 0, 0, 0, 8, T0, T0 + 1), (1, 0, 0, 0, 8, T0, T0 + 1)]
    assert analyze(topo, toy_cols(ok))[0].status == "OK"
    assert analyze(topo, toy_cols(ok + [(0, 2, 0, 0, 8, T0, T0 + 1)]))[0].status == "E_UNKNOWN_COMM"
    assert analyze(topo, toy_cols(ok + [(2, 0, 1, 0, 8, T0, T0 + 1)]))[0].status == "E_RANK_NOT_MEMBER"
    assert analyze(topo, toy_cols(ok + [(1, 0, 0, 0, 8, T0 + 5, T0 + 9)]))[0].status == "E_DUPLICATE_KEY"
    assert analyze(topo, toy_cols(ok + [(1, 0, 1, 0, 8, T0 + 5, T0 + 4)]))[0].status == "E_RANGE"
    assert analyze(topo, toy_cols(ok + [(1, 0, 1, 16, 8, T0 + 5, T0 + 9)]))[0].status == "E_RANGE"
    both = ok + [(0, 2, 0, 0, 8, T0, T0 + 1), (2, 0, 1, 0, 8, T0, T0 + 1)]
    assert analyze(topo, toy_cols(both))[0].status == "E_UNKNOWN_COMM"
    assert analyze(topo, toy_cols(both[::-1]))[0].status == "E_UNKNOWN_COMM"
    empty, _ = analyze(topo, toy_cols([]))
    assert empty.status == "OK" and len(empty.seg["comm"]) == 0 and empty.blame["n_records"].sum() == 0
    # a record before the epoch is out of range; a non-member outranks a range error, whatever the order
    assert analyze(topo, toy_cols(ok + [(1, 0, 1, 0, 8, -1, T0)]))[0].status == "E_RANGE"
    mixed = ok + [(1, 0, 1, 0, 8, T0 + 5, T0 + 4), (2, 0, 1, 0, 8, T0, T0 + 1)]
    assert analyze(topo, toy_cols(mixed))[0].status == "E_RANK_NOT_MEMBER"
    assert analyze(topo, toy_cols(mixed[::-1]))[0].status == "E_RANK_NOT_MEMBER"


# --------------------------------------------------------------------------
# injected faults are recovered, clean traces raise nothing
# --------------------------------------------------------------------------
def test_config1_flags_equal_injected_delays_exactly():
    tr = tg.generate(tg.config1()).shuffled(11)
    r, _ = analyze(tr.topo, tr.cols)
    inj = tr.inj_delay > 0
    want = sorted(zip(tr.cols["seq"][inj].tolist(), tr.cols["rank"][inj].tolist()))
    got = sorted(zip(r.flag["seq"].tolist(), r.flag["rank"].tolist()))
    assert got == want and len(want) > 20
    assert np.all(r.flag["kind"] == orc.FLAG_LATE_ENTER)
    assert np.all(np.abs(r.flag["lag_enter"] - 2_000_000) < 150_000)      # 2 ms +- skew and jitter
    # blame: only rank 5, first in the order, counts add up
    assert r.order[0] == 5 and r.blame["n_late_enter"][5] == len(want)
    assert r.blame["n_late_enter"].sum() == len(want) and r.blame["n_late_exit"].sum() == 0
    assert r.blame["sum_lag_enter"][5] == r.flag["lag_enter"].sum()
    assert np.all(r.blame["n_records"] == 1000)
    # the paper's rule sees it too: a slow group, computation-slow, root = the late rank
    slow = r.group["slow"] == 1
    assert slow.any() and np.all(r.group["class"][slow] == 1) and np.all(r.group["root_s1"][slow] == 5)


def test_clean_traces_raise_no_flags():
    for spec in (tg.config1(faults=False), tg.config2(n_cycles=40, faults=False),
                 tg.config3(n_cycles=10, faults=False, layout=tg.Layout3D(tp=8, pp=2, dp=8))):
        tr = tg.generate(spec)
        r, _ = analyze(tr.topo, tr.cols)
        assert r.status == "OK"
        assert len(r.flag["rank"]) == 0 and len(r.alert["comm"]) == 0
        assert np.all(r.seg["state"] == (orc.SEG_COMPLETE | orc.SEG_CONSISTENT | orc.SEG_USABLE))


def test_config2_slow_ranks_and_slow_link_are_located():
    spec = tg.config2(n_cycles=100)
    tr = tg.generate(spec).shuffled(5)
    r, _ = analyze(tr.topo, tr.cols)
    slow = sorted(s.rank for s in spec.slow_ranks)
    link = sorted(spec.slow_groups[0].ranks)
    assert sorted(np.nonzero(r.blame["n_late_enter"])[0].tolist()) == slow
    assert sorted(np.nonzero(r.blame["n_late_exit"])[0].tolist()) == link
    # record level: every flagged entry was injected; every injected delay well above the floor is flagged
    key = lambda c, s, k: set(zip(c.tolist(), s.tolist(), k.tolist()))
    fe = r.flag["kind"] & 1 > 0
    flagged = key(r.flag["comm"][fe], r.flag["seq"][fe], r.flag["rank"][fe])
    inj = tr.inj_delay > 0
    assert flagged <= key(tr.cols["comm"][inj], tr.cols["seq"][inj], tr.cols["rank"][inj])
    big = tr.inj_delay > 300_000 + 4 * 50_000 + 20_000
    assert key(tr.cols["comm"][big], tr.cols["seq"][big], tr.cols["rank"][big]) <= flagged
    fx = r.flag["kind"] & 2 > 0
    st = tr.stretched
    assert key(r.flag["comm"][fx], r.flag["seq"][fx], r.flag["rank"][fx]) <= \
        key(tr.cols["comm"][st], tr.cols["seq"][st], tr.cols["rank"][st])
    assert set(r.order[:5].tolist()) == set(slow + link)
    assert r.blame["n_late_enter"].sum() == fe.sum() and r.blame["n_late_exit"].sum() == fx.sum()
    assert r.blame["sum_lag_exit"].sum() == r.flag["lag_exit"][fx].sum()


def test_config3_shape_faults_are_located_on_a_small_layout():
    spec = tg.config3(n_cycles=60, layout=tg.Layout3D(tp=8, pp=4, dp=16))
    tr = tg.generate(spec)
    r, _ = analyze(tr.topo, tr.cols)
    slow = sorted(s.rank for s in spec.slow_ranks)
    nic = sorted(x for g in spec.slow_groups for x in g.ranks)
    top = set(np.nonzero(r.blame["n_late_enter"] >= 2)[0].tolist())
    assert top == set(slow)
    assert set(np.nonzero(r.blame["n_late_exit"] >= 2)[0].tolist()) == set(nic)


# ---- dependent schedules: a delay travels to the peers' later operations ---------------------------
def test_propagating_schedule_keeps_faulty_ranks_on_top_and_clean_runs_clean():
    # every group of a kind runs the same operation at the same step (one SPMD program): without
    # that, groups finish at different times and their members meet late without any fault
    spec = tg.config2(n_cycles=120)
    spec.same_size_per_kind = True
    tr = tg.generate(spec)
    pr = tg.propagate(tr, gap_ns=2_000_000)
    R = spec.layout.n_ranks
    # the replay keeps every record's own entry offset and transfer time: only the schedule moves
    assert np.all(pr.cols["t_exit"] >= pr.cols["t_enter"])
    e0 = tr.cols["t_enter"].reshape(-1, R)
    e1 = pr.cols["t_enter"].reshape(-1, R)
    assert np.array_equal(e1[0] - e0[0], np.full(R, 2_000_000))          # first slot: shifted by the gap only
    assert np.all(np.diff(e1, axis=0) > 0)                               # a rank's operations stay ordered
    faulty = sorted([s.rank for s in spec.slow_ranks] + [r for g in spec.slow_groups for r in g.ranks])
    o = orc.Oracle(pr.topo)
    w = o.analyze_window(pr.shuffled(1).cols, int(pr.cols["t_exit"].max()) + 1)
    assert w.status == "OK"
    n_flags = w.blame["n_late_enter"] + w.blame["n_late_exit"]
    # secondary flags reach far more ranks than were faulty, yet the faulty ranks lead the blame order
    assert int((n_flags > 0).sum()) > 10 * len(faulty)
    assert sorted(int(r) for r in w.order[:len(faulty)]) == faulty
    # without faults nothing is flagged although every collective now waits for its slowest member
    cspec = tg.config2(n_cycles=60, faults=False)
    cspec.same_size_per_kind = True
    clean = tg.propagate(tg.generate(cspec), gap_ns=2_000_000)
    wc = orc.Oracle(clean.topo).analyze_window(clean.cols, int(clean.cols["t_exit"].max()) + 1)
    assert wc.status == "OK" and len(wc.flag["rank"]) == 0


# --------------------------------------------------------------------------
# the late test, one leg at a time (expected values written out by hand from the definition:
# late iff lag > floor and lag * kmad_den > kmad_num * MAD, both strict)
# --------------------------------------------------------------------------
def _one_round(enters, exits, nbytes=1 << 20):
    return [(r, 0, 0, tg.OP_ALLREDUCE, nbytes, T0 + int(e), T0 + int(x)) for r, (e, x) in enumerate(zip(enters, exits))]


@pytest.mark.parametrize("side", ["enter", "exit"])
def test_late_needs_both_the_floor_and_the_mad_multiple(side):
    topo = ring_topology(5)
    kind = orc.FLAG_LATE_ENTER if side == "enter" else orc.FLAG_LATE_EXIT
    base = 10_000_000          # the other side: everyone at the same time, never late

    def run(offsets, **params):
        if side == "enter":
            rows = _one_round(offsets, [base] * 5)
        else:
            rows = _one_round([0] * 5, [base + o for o in offsets])
        r, _ = analyze(topo, toy_cols(rows), **params)
        assert r.status == "OK" and r.seg["state"][0] & orc.SEG_USABLE
        return r

    # spread values: median 400,000, deviations {0, 200k, 200k, 400k, 400k} -> MAD 200,000.
    # rank 4: lag 400,000 exceeds the floor (300,000) but 2 * 400,000 <= 9 * 200,000: not late
    r = run([0, 200_000, 400_000, 600_000, 800_000])
    assert r.seg[side + "_med"][0] - T0 - (base if side == "exit" else 0) == 400_000
    assert r.seg[side + "_mad"][0] == 200_000
    assert list(r.rec["lag_" + side]) == [-400_000, -200_000, 0, 200_000, 400_000]
    assert len(r.flag["rank"]) == 0 and r.rec["flag"].sum() == 0
    # equality of the MAD leg: median 400,000, MAD 200,000, lag 900,000: 2 * 900,000 == 9 * 200,000 -> not late
    r = run([0, 200_000, 400_000, 600_000, 1_300_000])
    assert r.seg[side + "_mad"][0] == 200_000 and r.rec["lag_" + side][4] == 900_000
    assert len(r.flag["rank"]) == 0
    # one nanosecond more: late
    r = run([0, 200_000, 400_000, 600_000, 1_300_001])
    assert list(r.flag["rank"]) == [4] and list(r.flag["kind"]) == [kind]
    assert r.flag["lag_" + side][0] == 900_001
    # the multiple itself: with kmad = 2/1 the same round flags at 400,001 and not at 400,000
    r = run([0, 200_000, 400_000, 600_000, 800_000], kmad_num=2, kmad_den=1)
    assert len(r.flag["rank"]) == 0
    r = run([0, 200_000, 400_000, 600_000, 800_001], kmad_num=2, kmad_den=1)
    assert list(r.flag["rank"]) == [4]
    # the ratio is num/den, not den/num: 1/3 flags lag 400,000 (3 * 400,000 > 200,000), 3/1 does not
    assert list(run([0, 200_000, 400_000, 600_000, 800_000], kmad_num=1, kmad_den=3).flag["rank"]) == [4]
    assert len(run([0, 200_000, 400_000, 600_000, 800_000], kmad_num=3, kmad_den=1).flag["rank"]) == 0
    # the floor leg alone: MAD 0 (four equal values), lag == floor -> not late, floor + 1 -> late
    r = run([0, 0, 0, 0, 300_000])
    assert r.seg[side + "_mad"][0] == 0 and len(r.flag["rank"]) == 0
    r = run([0, 0, 0, 0, 300_001])
    assert list(r.flag["rank"]) == [4] and list(r.flag["kind"]) == [kind]
    assert r.blame["n_late_" + side][4] == 1 and r.blame["sum_lag_" + side][4] == 300_001
    other = "exit" if side == "enter" else "enter"
    assert r.blame["n_late_" + other].sum() == 0


def test_blame_order_is_flags_then_summed_lag_then_rank():
    """order[] = (number of flags descending, summed lag descending, rank ascending)."""
    topo = ring_topology(6)
    dur = 10_000_000
    late = {0: {2: 400_000},               # round -> {rank: entry delay}
            1: {2: 400_000},
            2: {1: 500_000},
            3: {3: 700_000},
            4: {4: 500_000}}
    rows = []
    for j in range(5):
        t = T0 + j * 1_000_000_000
        for r in range(6):
            rows.append((r, 0, j, tg.OP_ALLREDUCE, 1 << 20, t + late[j].get(r, 0), t + dur))
    r, _ = analyze(topo, toy_cols(rows))
    assert list(r.blame["n_late_enter"]) == [0, 1, 2, 1, 1, 0] and r.blame["n_late_exit"].sum() == 0
    assert list(r.blame["sum_lag_enter"]) == [0, 500_000, 800_000, 700_000, 500_000, 0]
    # rank 2 has two flags; ranks 3, 1, 4 one each with lags 700k > 500k = 500k (1 before 4); then 0, 5
    assert list(r.order) == [2, 3, 1, 4, 0, 5]
    # the lag that orders is the sum of both kinds: rank 4 also leaves late by 300,001 ns in its round
    rows2 = [(rk, c, s, op, nb, te, tx + (300_001 if (s == 4 and rk == 4) else 0)) for rk, c, s, op, nb, te, tx in rows]
    r2, _ = analyze(topo, toy_cols(rows2))
    assert list(r2.blame["n_late_exit"]) == [0, 0, 0, 0, 1, 0]
    assert list(r2.order) == [4, 2, 3, 1, 0, 5]        # ranks 4 and 2 have two flags each; 800,001 > 800,000


def test_round_with_an_operation_in_flight_is_not_usable():
    """Every member has a record but one operation has not completed: the round is neither complete
    nor usable, it raises no flag and forms no detection group."""
    topo = ring_topology(4)
    t = T0
    rows = [(0, 0, 0, tg.OP_ALLREDUCE, 1 << 20, t, t + 1000), (1, 0, 0, tg.OP_ALLREDUCE, 1 << 20, t, t + 1000),
            (2, 0, 0, tg.OP_ALLREDUCE, 1 << 20, t + 900_000, INFLIGHT), (3, 0, 0, tg.OP_ALLREDUCE, 1 << 20, t, t + 1000)]
    r, _ = analyze(topo, toy_cols(rows), now=t + 10**9)
    assert r.seg["n"][0] == 4 and r.seg["inflight"][0] == 1
    assert r.seg["state"][0] == orc.SEG_CONSISTENT
    assert len(r.group["comm"]) == 0 and len(r.flag["rank"]) == 0 and r.rec["flag"].sum() == 0
    assert list(r.rec["lag_enter"]) == [0, 0, 0, 0]
    # statistics cover the three completed records only
    assert r.seg["enter_max"][0] == t and r.seg["exit_med"][0] == t + 1000 and r.seg["dur_max"][0] == 1000
    # the same round completed: usable, one group, rank 2 late on entry
    rows[2] = (2, 0, 0, tg.OP_ALLREDUCE, 1 << 20, t + 900_000, t + 900_500)
    r, _ = analyze(topo, toy_cols(rows), now=t + 10**9)
    assert r.seg["state"][0] == orc.SEG_COMPLETE | orc.SEG_CONSISTENT | orc.SEG_USABLE
    assert len(r.group["comm"]) == 1 and list(r.flag["rank"]) == [2]


def test_eq1_round_exactly_at_the_end_of_the_warmup_span_still_counts():
    """Rounds start 0, 60 and 120 s after the first one with a 120 s span: all three are averaged
    (m = 3); one nanosecond later the third round already ends the warm-up (m = 2)."""
    topo = ring_topology(2)
    span = 120_000_000_000
    for extra, m, base in ((0, 3, (100 + 200 + 600) // 3), (1, 2, (100 + 200) // 2)):
        rows = []
        for j, (t, d) in enumerate(((0, 100), (span // 2, 200), (span + extra, 600), (span + 10**9, 700),
                                    (span + 2 * 10**9, 100_000))):
            # the last round alone has a spread, so Eq. 2 selects it and the averaged baseline shows
            rows += [(r, 0, j, tg.OP_ALLREDUCE, 1 << 20, T0 + t, T0 + t + (1 if (j == 4 and r == 1) else d))
                     for r in range(2)]
        r, _ = analyze(topo, toy_cols(rows), tbase_warmup_ns=span, tbase_rounds=100)
        assert r.group["rstar_seq"][0] == 4
        assert r.group["frozen"][0] == 1 and r.group["m"][0] == m
        assert r.group["static"][0] == 0 and r.group["tbase"][0] == base


def test_only_an_allreduce_of_a_few_bytes_is_a_barrier():
    """The 4-byte all-reduce is the barrier (Section 4.2.1); an all-gather of the same size is an ordinary round."""
    topo = ring_topology(2)
    rows = (rounds_with_durations([[9000, 1000]], op=tg.OP_ALLREDUCE, nbytes=3, seq0=0)
            + rounds_with_durations([[9000, 1000]], op=tg.OP_ALLGATHER, nbytes=3, seq0=1))
    r, _ = analyze(topo, toy_cols(rows), tbase_init_ns=1000)
    assert list(r.seg["state"] & orc.SEG_BARRIER) == [orc.SEG_BARRIER, 0]
    assert list(r.seg["state"] & orc.SEG_USABLE) == [0, orc.SEG_USABLE]
    assert list(r.group["op"]) == [tg.OP_ALLGATHER] and r.group["slow"][0] == 1


def test_a_missing_member_means_not_entered_even_when_others_have_finished():
    """Rank 2 never posted operation 7, rank 3 has already left it, ranks 0 and 1 are still inside: the member
    without a record is the candidate (first branch of the hang decision tree), not the ranks that finished."""
    topo = ring_topology(4)
    t = T0 + 1000
    rows = [(r, 0, 6, 0, 4096, T0 + r, T0 + 100) for r in range(4)]
    rows += [(0, 0, 7, 0, 4096, t, INFLIGHT), (1, 0, 7, 0, 4096, t + 1, INFLIGHT), (3, 0, 7, 0, 4096, t + 2, t + 90)]
    r, _ = analyze(topo, toy_cols(rows), now=t + 10_000, hang_threshold_ns=5_000)
    assert list(r.alert["class"]) == [1]
    assert list(r.cand[r.alert["cand_off"][0]: r.alert["cand_off"][0] + r.alert["n_cand"][0]]) == [2]


def test_the_warmup_span_is_measured_between_earliest_entries():
    """Rounds every 60 s, warm-up span 120 s; in the first round one rank enters 1 s after the other.  Measured
    from the first round's earliest entry the round at 120 s still belongs to the baseline (Eq. 1); measured from
    its latest entry the span would even reach a round at 121 s, which it must not."""
    topo = ring_topology(2)
    S = 1_000_000_000

    def rounds(third_at):
        rows = []
        for j, start in enumerate([0, 60 * S, third_at, 240 * S]):
            for rk in range(2):
                te = T0 + start + (S if (j == 0 and rk == 1) else 0)
                rows.append((rk, 0, j, tg.OP_ALLREDUCE, 1 << 20, te, te + 10 * US))
        return rows
    r, _ = analyze(topo, toy_cols(rounds(120 * S)), tbase_init_ns=7)
    assert r.group["m"][0] == 3 and r.group["frozen"][0] == 1
    r, _ = analyze(topo, toy_cols(rounds(120 * S + S // 2)), tbase_init_ns=7)
    assert r.group["m"][0] == 2 and r.group["frozen"][0] == 1


def test_location_needs_a_slow_window_and_the_rate_root_is_for_communication_only():
    from tests.test_oracle_rates import series_cols
    topo = ring_topology(2)
    o = orc.Oracle(topo, dict(tbase_init_ns=1000, repeat_threshold=2))
    series = {(0, 0, 0): [(1, 0, 0), (1, 8, 8), (2, 0, 0)], (1, 0, 0): [(1, 2, 8), (1, 8, 8), (2, 0, 0)]}
    o.progress_rates(series_cols(series), 3, 1)                          # rank 1 has the minimal rate
    for s in (0, 1):
        r = o.analyze_window(toy_cols(rounds_with_durations([[9000, 1000]], seq0=s)), FAR)
    assert r.group["repeats"][0] == 2 and r.group["locate"][0] == 1
    # computation-slow (P = 1): the communication-side root stays empty although a rate pass has run
    assert r.group["class"][0] == 1 and r.group["root_s1"][0] == 1 and r.group["root_s2"][0] == NO_RANK
    # the next window is healthy: nothing to locate, whatever the counter says
    r = o.analyze_window(toy_cols(rounds_with_durations([[1200, 1100]], seq0=2)), FAR)
    assert r.group["slow"][0] == 0 and r.group["repeats"][0] == 2 and r.group["locate"][0] == 0
