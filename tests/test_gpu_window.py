"""GPU parity: ccld_ingest / ccld_analyze_window / ccld_rank_blame through the C ABI
against the CPU oracle, element by element and bit-exact (everything is int64)."""
import numpy as np
import pytest

from oracle import ccld_oracle as orc
from paper_2605_04478_amd import tracegen as tg
from tests.helpers import INFLIGHT, T0, ring_topology, rounds_with_durations, toy_cols

pytestmark = pytest.mark.gpu

FAR = T0 + 10**15


def _analyzer(topo, n, **params):
    from paper_2605_04478_amd import ccld
    return ccld.Analyzer(topo, max_window_records=max(n, 1), **params)


def compare(g, o, blame=None, order=None, per_record=True, what=""):
    """g: ccld.WindowResult, o: oracle WindowResult."""
    assert g.status == o.status, (what, g.status, o.status)
    if o.status != "OK":
        return
    assert g.n_seg == len(o.seg["comm"]), what
    assert g.n_flag == len(o.flag["comm"]), what
    assert g.n_group == len(o.group["comm"]), what
    assert g.n_alert == len(o.alert["comm"]), what
    assert g.n_cand == len(o.cand), what
    for name in ("seg", "flag", "group", "alert"):
        gt, ot = getattr(g, name), getattr(o, name)
        for k in ot:
            assert np.array_equal(gt[k], ot[k]), (what, name, k, np.nonzero(gt[k] != ot[k])[0][:5])
    assert np.array_equal(g.cand, o.cand), what
    if per_record:
        pr = g.per_record()
        assert np.array_equal(pr["perm"].astype(np.uint64), o.perm), what
        assert np.array_equal(pr["lag_enter"], o.rec["lag_enter"]), what
        assert np.array_equal(pr["lag_exit"], o.rec["lag_exit"]), what
        assert np.array_equal(pr["rec_flag"].astype(np.int64), o.rec["flag"]), what
    if blame is not None:
        for k in o.blame:
            assert np.array_equal(blame[k], o.blame[k]), (what, "blame", k)
        assert np.array_equal(order, o.order), (what, "order")


def run_both(topo, cols, now=FAR, on_device=True, what="", expect_path=None, **params):
    """Both placements of the library (dense placement where the window allows it, and the sort) against
    the oracle; returns the result of the dense-placement context."""
    n = int(cols["rank"].shape[0])
    o = orc.Oracle(topo, params).analyze_window(cols, now)
    first = None
    for placement in (1, 0):                   # CCLD_PLACEMENT_DENSE, CCLD_PLACEMENT_SORT
        an = _analyzer(topo, n, placement=placement, **params)
        an.ingest(an.to_device(cols) if on_device else cols)
        g = an.analyze_window(now, n_records=n, per_record=True)
        blame = order = None
        if o.status == "OK":
            blame, order = an.rank_blame()
        compare(g, o, blame, order, what=f"{what} placement={placement}")
        if placement == 0:
            assert g.path == 0
        elif expect_path is not None and o.status == "OK":
            assert g.path == expect_path, (what, g.path)
        an.close()
        first = first or g
    return first, o


def test_config1_parity():
    tr = tg.generate(tg.config1()).shuffled(1)
    g, o = run_both(tr.topo, tr.cols, what="config1")
    assert g.n_flag == int((tr.inj_delay > 0).sum()) and g.n_seg == 1000


def test_config1_host_batch_parity():
    tr = tg.generate(tg.config1(n_slots=300)).shuffled(2)
    run_both(tr.topo, tr.cols, on_device=False, what="config1-host")


def _disturb(tr):
    """In-flight operations, a missing member, inconsistent and barrier rounds, early exits."""
    c = {k: v.copy() for k, v in tr.cols.items()}
    topo = tr.topo
    last70 = c["seq"][c["comm"] == 70].max()
    c["t_exit"][(c["comm"] == 70) & (c["seq"] == last70)] = INFLIGHT                      # all hung
    m = (c["comm"] == 71) & (c["seq"] == c["seq"][c["comm"] == 71].max())
    idx = np.nonzero(m)[0]
    c["t_exit"][idx[: len(idx) // 2]] = INFLIGHT                                          # some completed
    keep = ~((c["comm"] == 3) & (c["seq"] == c["seq"][c["comm"] == 3].max()) &
             (c["rank"] == topo.members_of(3)[2]))
    m2 = (c["comm"] == 3) & (c["seq"] == c["seq"][c["comm"] == 3].max())
    c["t_exit"][m2] = INFLIGHT                                                            # one member never entered
    c["bytes"][(c["comm"] == 5) & (c["seq"] == 4) & (c["rank"] == topo.members_of(5)[1])] += 1
    c["op"][(c["comm"] == 6) & (c["seq"] == 2) & (c["rank"] == topo.members_of(6)[0])] = tg.OP_BROADCAST
    c["bytes"][(c["comm"] == 7) & (c["seq"] == 9)] = 2                                    # a barrier
    c["t_exit"][(c["comm"] == 7) & (c["seq"] == 11)] = INFLIGHT
    c["bytes"][(c["comm"] == 7) & (c["seq"] == 11)] = 0                                   # a hung barrier
    return {k: v[keep] for k, v in c.items()}


def test_config2_parity_with_disturbances():
    tr = tg.generate(tg.config2(n_cycles=100)).shuffled(4)
    cols = _disturb(tr)
    now = int(cols["t_enter"].max()) + 10_000_000
    g, o = run_both(tr.topo, cols, now=now, what="config2", hang_threshold_ns=1_000_000)
    assert g.n_alert >= 3 and g.n_flag > 100 and g.n_group > 100
    assert sorted(set(o.alert["class"].tolist())) == [1, 2, 3]


def test_config3_layout_parity():
    tr = tg.generate(tg.config3(n_cycles=40, layout=tg.Layout3D(tp=8, pp=4, dp=64))).shuffled(5)
    g, o = run_both(tr.topo, tr.cols, what="config3-small")
    assert g.n_flag > 0


def test_propagating_schedule_parity():
    """A dependent schedule (delays travel to the peers' later operations): tens of thousands of
    secondary flags on every rank; the faulty ranks still lead the blame order."""
    spec = tg.config2(n_cycles=60)
    spec.same_size_per_kind = True
    tr = tg.propagate(tg.generate(spec), gap_ns=2_000_000).shuffled(2)
    g, o = run_both(tr.topo, tr.cols, now=int(tr.cols["t_exit"].max()) + 1, what="propagating")
    faulty = sorted([s.rank for s in spec.slow_ranks] + [r for grp in spec.slow_groups for r in grp.ranks])
    assert g.n_flag > 1000
    assert sorted(int(r) for r in o.order[:len(faulty)]) == faulty


@pytest.mark.parametrize("R,n_seq", [(70, 400), (700, 60)])
def test_random_partial_rounds_with_ties(R, n_seq):
    rng = np.random.default_rng(3)
    topo = ring_topology(R, comms=[list(range(R)), list(range(0, R, 2)), [1, 3, 5]])
    rows = []
    for c, members in enumerate([list(range(R)), list(range(0, R, 2)), [1, 3, 5]]):
        for s in range(n_seq):
            n = int(rng.integers(1, len(members) + 1)) if rng.random() < 0.5 else len(members)
            ranks = rng.choice(members, n, replace=False)
            te = T0 + s * 1000 + rng.integers(0, 6, n)
            tx = te + rng.integers(0, 5, n)
            infl = rng.random(n) < 0.05
            for r, a, b, f in zip(ranks, te, tx, infl):
                rows.append((int(r), c, s, int(rng.integers(0, 2)) if rng.random() < 0.01 else 0,
                             64 << int(rng.integers(0, 3)), int(a), INFLIGHT if f else int(b)))
    cols = toy_cols(rows)
    run_both(topo, cols, now=T0 + 10**6, what="ties", hang_threshold_ns=500_000, lag_floor_ns=1,
             tbase_init_ns=2, kmad_num=1, kmad_den=1)


@pytest.mark.parametrize("size,rounds", [(65, 6), (128, 6), (257, 9), (512, 4), (513, 4), (1500, 5), (2048, 3),
                                         (2049, 3), (3000, 3), (16384, 3), (16385, 2), (20000, 2)])
def test_large_communicators_cross_tiles(size, rounds):
    """Collectives at both edges of every size class: one wavefront with several values per lane (65-512), one
    workgroup sorting in LDS (513-2,048 with 256 threads, up to 16,384 with 1,024), counting selection (beyond),
    spanning tile boundaries."""
    rng = np.random.default_rng(size)
    topo = ring_topology(size, comms=[list(range(size)), [0, 1, 2, 3]])
    rows = []
    for s in range(rounds):
        te = T0 + s * 10**7 + rng.integers(0, 2000, size)
        tx = te + 10**6 + rng.integers(0, 3000, size)
        late = rng.choice(size, 3, replace=False)
        te[late] += 5_000_000
        tx[late] = np.maximum(tx[late], te[late] + 10)
        for r in range(size):
            if s == rounds - 1 and r % 97 == 5:
                continue            # last round incomplete
            rows.append((r, 0, s, 0, 4096, int(te[r]), int(tx[r])))
        for r in range(4):
            rows.append((r, 1, s, 0, 1 << 20, int(te[r]), int(tx[r])))
    cols = toy_cols(rows)
    p = np.random.default_rng(1).permutation(len(rows))
    cols = {k: v[p] for k, v in cols.items()}
    g, o = run_both(topo, cols, what=f"large{size}", tbase_init_ns=1000)
    assert g.n_flag >= 3 * (rounds - 1)


def test_edge_sizes():
    topo = ring_topology(4)
    run_both(topo, toy_cols([]), what="empty")
    run_both(topo, toy_cols([(2, 0, 0, 0, 8, T0, T0 + 5)]), what="single")
    run_both(topo, toy_cols([(r, 0, 0, 0, 8, T0 + r, T0 + 5 + r) for r in range(4)]), what="one-round")
    # exact multiples of the tile sizes and one more
    for n_rounds in (256, 257, 512, 513):
        rows = rounds_with_durations([[100, 200, 300, 400 + j] for j in range(n_rounds)])
        run_both(topo, toy_cols(rows), what=f"rounds{n_rounds}", tbase_init_ns=10)


def test_many_communicators_per_rank_and_unsorted_members():
    """Ranks in more than four communicators (the membership lookup leaves its packed 16-byte row)
    and member lists that are not in ascending rank order (keys carry the rank's position among
    the sorted members, outputs carry ranks)."""
    rng = np.random.default_rng(11)
    comms = [[5, 2, 7, 0, 3], [7, 6, 5, 4, 3, 2, 1, 0], [1, 3, 5, 7], [0, 2, 4, 6], [6, 1, 4], [3, 7], [2, 5, 0, 6, 1]]
    topo = ring_topology(8, comms=comms)
    rows = []
    for c, members in enumerate(comms):
        for s in range(60):
            te = T0 + s * 10**7 + rng.integers(0, 2000, len(members))
            tx = te + 10**6 + rng.integers(0, 3000, len(members))
            if s % 7 == 3:
                k = int(rng.integers(0, len(members)))
                te[k] += 5_000_000
                tx[k] = max(tx[k], te[k] + 10)
            for r, a, b in zip(members, te, tx):
                if s == 59 and r == members[0]:
                    continue
                rows.append((r, c, s, 0, 1 << 16, int(a), INFLIGHT if s == 59 else int(b)))
    cols = toy_cols(rows)
    p = rng.permutation(len(rows))
    cols = {k: v[p] for k, v in cols.items()}
    g, o = run_both(topo, cols, now=T0 + 10**12, what="many-comms", tbase_init_ns=1000)
    assert g.n_flag > 0 and g.n_alert > 0


@pytest.mark.parametrize("seq0", [0, 7, 10**6 + 3, 2**40 + 12345])
def test_large_operation_counters(seq0):
    """Counters of a long-running job: the sort keys carry them relative to the window's smallest
    one; one communicator (no communicator field in the key) and several."""
    rng = np.random.default_rng(5)
    for comms in ([[0, 1, 2, 3]], [[0, 1, 2, 3], [2, 0], [1, 3, 2]]):
        topo = ring_topology(4, comms=comms)
        rows = []
        for c, members in enumerate(comms):
            for j in range(90):
                s = seq0 + 3 * c + j + (5 if j > 60 else 0)           # a gap in the counters
                te = T0 + j * 10**7 + rng.integers(0, 2000, len(members))
                tx = te + 10**6 + rng.integers(0, 3000, len(members))
                if j % 9 == 4:
                    te[0] += 4_000_000
                    tx[0] = max(tx[0], te[0] + 10)
                for r, a, b in zip(members, te, tx):
                    rows.append((r, c, s, 0, 1 << 16, int(a), int(b)))
        cols = toy_cols(rows)
        p = rng.permutation(len(rows))
        cols = {k: v[p] for k, v in cols.items()}
        g, o = run_both(topo, cols, what=f"seq0={seq0}", tbase_init_ns=1000)
        assert g.n_flag > 0 and int(g.seg["seq"].min()) == seq0


def test_stragglers_seconds_behind_their_collective():
    """Arrival and completion times spread over more than 32 bits of nanoseconds inside one
    collective (values around +/- 2^31 ns and several seconds)."""
    rng = np.random.default_rng(8)
    topo = ring_topology(8, comms=[list(range(8)), [0, 2, 4, 6]])
    rows = []
    for c, members in enumerate([list(range(8)), [0, 2, 4, 6]]):
        for s in range(300):
            te = T0 + s * 10**10 + rng.integers(0, 2000, len(members))
            tx = te + 10**6 + rng.integers(0, 3000, len(members))
            kind = s % 6
            k = int(rng.integers(0, len(members)))
            if kind == 1:
                te[k] += 5 * 10**9; tx[k] = te[k] + 10**6                  # enters 5 s late
            elif kind == 2:
                tx[k] += 3 * 10**9                                         # leaves 3 s late
            elif kind == 3:
                te[k] -= 2**31 + 5; tx[k] = max(tx[k], te[k] + 1)           # just outside the offset range, early
            elif kind == 4:
                te[k] += 2**31 - 3; tx[k] = te[k] + 10**6                   # just inside / at the edge
            for r, a, b in zip(members, te, tx):
                rows.append((r, c, s, 0, 1 << 16, int(a), int(b)))
    cols = toy_cols(rows)
    p = rng.permutation(len(rows))
    cols = {k: v[p] for k, v in cols.items()}
    g, o = run_both(topo, cols, what="wide", tbase_init_ns=1000)
    assert g.n_flag > 100


def test_validation_parity():
    topo = ring_topology(4, comms=[[0, 1], [2, 3]])
    ok = [(0, 0, 0, 0, 8, T0, T0 + 1), (1, 0, 0, 0, 8, T0, T0 + 1)]
    cases = {"unknown": ok + [(0, 2, 0, 0, 8, T0, T0 + 1)],
             "member": ok + [(2, 0, 1, 0, 8, T0, T0 + 1)],
             "dup": ok + [(1, 0, 0, 0, 8, T0 + 5, T0 + 9)],
             "range": ok + [(1, 0, 1, 0, 8, T0 + 5, T0 + 4)],
             "op": ok + [(1, 0, 1, 16, 8, T0 + 5, T0 + 9)],
             "both": ok + [(0, 2, 0, 0, 8, T0, T0 + 1), (2, 0, 1, 0, 8, T0, T0 + 1)],
             "before-epoch": ok + [(1, 0, 1, 0, 8, -1, T0)],
             "member+range": ok + [(1, 0, 1, 0, 8, T0 + 5, T0 + 4), (2, 0, 1, 0, 8, T0, T0 + 1)],
             "range+member": ok + [(2, 0, 1, 0, 8, T0, T0 + 1), (1, 0, 1, 0, 8, T0 + 5, T0 + 4)]}
    want = {"unknown": "E_UNKNOWN_COMM", "member": "E_RANK_NOT_MEMBER", "dup": "E_DUPLICATE_KEY",
            "range": "E_RANGE", "op": "E_RANGE", "both": "E_UNKNOWN_COMM", "before-epoch": "E_RANGE",
            "member+range": "E_RANK_NOT_MEMBER", "range+member": "E_RANK_NOT_MEMBER"}
    for name, rows in cases.items():
        g, o = run_both(topo, toy_cols(rows), what=name)
        assert g.status == want[name] and g.n_seg == 0


def test_state_across_windows_matches_oracle():
    """Eq. 1 baseline, watermarks and the repetition counter persist from window to window."""
    spec = tg.config1(n_slots=600)
    tr = tg.generate(spec)
    from paper_2605_04478_amd import ccld
    an = ccld.Analyzer(tr.topo, max_window_records=tr.n, tbase_rounds=20)
    o = orc.Oracle(tr.topo, dict(tbase_rounds=20))
    R = spec.layout.n_ranks
    for w, (a, b) in enumerate([(0, 150), (100, 300), (300, 450), (450, 600)]):     # overlapping, then disjoint
        sl = {k: v[a * R:b * R] for k, v in tr.cols.items()}
        an.reset_window()
        an.ingest(an.to_device(sl))
        g = an.analyze_window(FAR, n_records=(b - a) * R, per_record=True)
        ref = o.analyze_window(sl, FAR)
        blame, order = an.rank_blame()
        compare(g, ref, blame, order, what=f"window{w}")
    assert ref.group["frozen"].max() == 1 and ref.group["repeats"].max() >= 2


def test_sliding_window_of_batches():
    """window_batches = 3: each ingest drops the oldest batch; the analysis covers the last three."""
    spec = tg.config2(n_cycles=30)
    tr = tg.generate(spec)
    R = spec.layout.n_ranks
    per = 40 * R
    batches = [{k: v[i:i + per] for k, v in tr.cols.items()} for i in range(0, tr.n, per)]
    from paper_2605_04478_amd import ccld
    an = ccld.Analyzer(tr.topo, max_window_records=3 * per + 17, max_batch_records=per, window_batches=3)
    o = orc.Oracle(tr.topo)
    for i, b in enumerate(batches):
        an.ingest(an.to_device(b))
        win = batches[max(0, i - 2): i + 1]
        cols = {k: np.concatenate([w[k] for w in win]) for k in b}
        g = an.analyze_window(FAR, n_records=3 * per, per_record=True)
        ref = o.analyze_window(cols, FAR)
        blame, order = an.rank_blame()
        compare(g, ref, blame, order, what=f"step{i}")


def test_truncated_tables_keep_exact_counts():
    tr = tg.generate(tg.config1(n_slots=400))
    from paper_2605_04478_amd import ccld
    an = ccld.Analyzer(tr.topo, max_window_records=tr.n)
    an.ingest(an.to_device(tr.cols))
    ref = orc.Oracle(tr.topo).analyze_window(tr.cols, FAR)
    g = an.analyze_window(FAR, n_records=tr.n, flag_cap=5, group_cap=2)
    assert g.status == "W_TRUNCATED"
    assert g.n_flag == len(ref.flag["comm"]) and g.n_group == len(ref.group["comm"])
    assert np.array_equal(g.flag["rank"], ref.flag["rank"][:5])
    assert np.array_equal(g.group["tmax"], ref.group["tmax"][:2])
    blame, order = an.rank_blame()
    assert np.array_equal(blame["n_late_enter"], ref.blame["n_late_enter"])


def test_long_detection_groups_take_the_workgroup_pass():
    """Groups of more than 4,096 rounds are evaluated by a workgroup each, the others by a wavefront
    each; both kinds side by side, over two windows (baseline and repetition state carried)."""
    from paper_2605_04478_amd import ccld
    rng = np.random.default_rng(11)
    R = 6
    topo = ring_topology(R, comms=[list(range(R)), [0, 2, 4]])
    rows = []
    plan = [(0, 9000, 1 << 20), (0, 5000, 1 << 12), (0, 10, 1 << 26), (1, 4500, 1 << 20), (1, 100, 1 << 8)]
    span = 20_000_000_000
    # every group's rounds are spread over the whole time span, so both windows hold a part of each;
    # operation counters of a communicator follow the time order
    events = []
    for g, (comm, rounds, nbytes) in enumerate(plan):
        for j in range(rounds):
            events.append((T0 + (j * span) // rounds + g, comm, nbytes))
    events.sort()
    seq_next = {0: 0, 1: 0}
    for t, comm, nbytes in events:
        members = [0, 1, 2, 3, 4, 5] if comm == 0 else [0, 2, 4]
        s = seq_next[comm]
        seq_next[comm] += 1
        base = 50_000 + int(rng.integers(0, 2_000))
        slow = members[int(rng.integers(0, len(members)))] if rng.random() < 0.002 else -1   # one rank several times slower
        for r in members:
            te = t + int(rng.integers(0, 1_000))
            d = base * (8 if r == slow else 1) + int(rng.integers(0, 500))
            rows.append((r, comm, s, 0, nbytes, te, te + d))
    cols = toy_cols(rows)
    order = np.argsort(cols["t_enter"], kind="stable")
    half = len(rows) // 2
    an = ccld.Analyzer(topo, max_window_records=len(rows), tbase_rounds=50, tbase_warmup_ns=10**12)
    o = orc.Oracle(topo, dict(tbase_rounds=50, tbase_warmup_ns=10**12))
    seen_long = False
    for w, sel in enumerate([order[:half], order[half:]]):
        sel = sel[rng.permutation(len(sel))]
        sl = {k: v[sel] for k, v in cols.items()}
        an.reset_window()
        an.ingest(an.to_device(sl))
        g = an.analyze_window(FAR, n_records=len(sel), per_record=True)
        ref = o.analyze_window(sl, FAR)
        blame, order_ = an.rank_blame()
        compare(g, ref, blame, order_, what=f"long-groups window{w}")
        seen_long = seen_long or int(ref.group["n_usable"].max()) > 4096
        assert int(ref.group["slow"].sum()) >= 1
    assert seen_long
    an.close()


def test_blame_of_a_rank_with_tens_of_thousands_of_flags():
    """A rank that is late in every one of 12,000 collectives owns a run of flags long enough to be
    summed by several workgroups; two other ranks are late now and then."""
    rng = np.random.default_rng(5)
    R, rounds = 8, 12_000
    topo = ring_topology(R)
    rows = []
    for s in range(rounds):
        t = T0 + s * 1_000_000
        for r in range(R):
            te = t + int(rng.integers(0, 2_000))
            if r == 3:
                te += 400_000 + int(rng.integers(0, 50_000))
            elif r in (1, 6) and rng.random() < 0.01:
                te += 300_000
            rows.append((r, 0, s, 0, 1 << 20, te, te + 60_000 + int(rng.integers(0, 3_000))))
    cols = toy_cols(rows)
    p = rng.permutation(len(rows))
    cols = {k: v[p] for k, v in cols.items()}
    g, o = run_both(topo, cols, what="long blame run")
    assert int(o.blame["n_late_enter"][3]) + int(o.blame["n_late_exit"][3]) > 8192
    assert int(o.order[0]) == 3


# --------------------------------------------------------------------------
# dense placement: taken when the window fills a dense grid, abandoned for the sort otherwise
# --------------------------------------------------------------------------
def test_dense_placement_is_taken_on_dense_windows():
    tr = tg.generate(tg.config1(n_slots=300)).shuffled(3)
    g, o = run_both(tr.topo, tr.cols, what="dense config1", expect_path=1)
    tr = tg.generate(tg.config3(n_cycles=30, layout=tg.Layout3D(tp=8, pp=4, dp=64))).shuffled(6)
    g, o = run_both(tr.topo, tr.cols, what="dense config3 layout", expect_path=1)
    assert g.n_flag > 0
    # members without a record, operations in flight, inconsistent and barrier rounds stay on the dense path
    tr = tg.generate(tg.config2(n_cycles=60)).shuffled(4)
    cols = _disturb(tr)
    g, o = run_both(tr.topo, cols, now=int(cols["t_enter"].max()) + 10_000_000, what="dense disturbed",
                    expect_path=1, hang_threshold_ns=1_000_000)
    assert g.n_alert >= 3


def test_dense_placement_falls_back_to_the_sort():
    tr = tg.generate(tg.config2(n_cycles=40)).shuffled(7)
    c = tr.cols
    # a round without any record in the middle of a communicator's counters
    keep = ~((c["comm"] == 9) & (c["seq"] == 17))
    g, o = run_both(tr.topo, {k: v[keep] for k, v in c.items()}, what="hole", expect_path=0)
    assert g.n_seg == len(o.seg["comm"])
    # counters that are far apart: one communicator's records renumbered from a large counter on
    far = {k: v.copy() for k, v in c.items()}
    m = (far["comm"] == 3) & (far["seq"] >= 20)
    far["seq"][m] += 10**12
    run_both(tr.topo, far, what="far apart", expect_path=0)
    # the same at the window's edge is still dense: every communicator has its own first counter
    off = {k: v.copy() for k, v in c.items()}
    off["seq"][off["comm"] == 3] += 10**6
    off["seq"][off["comm"] == 4] += 5
    run_both(tr.topo, off, what="offset counters", expect_path=1)


def test_dense_placement_duplicates_and_small_sizes():
    # communicators of 1, 2, 3, 5, 6, 12 and 33 members over 62 ranks
    comms = [[0], [1, 2], [3, 4, 5], list(range(6, 11)), list(range(11, 17)), list(range(17, 29)), list(range(29, 62))]
    topo = tg.make_topology(62, comms)
    rng = np.random.default_rng(11)
    rows = []
    for c, mem in enumerate(comms):
        for s in range(700 if len(mem) < 6 else 90):
            t = T0 + s * 1_000_000 + int(rng.integers(0, 1000))
            present = [r for r in mem if rng.random() > 0.03] or mem[:1]
            for r in present:
                te = t + int(rng.integers(0, 400_000) if rng.random() < 0.1 else rng.integers(0, 50))
                rows.append((r, c, 1000 + s, c % 3, 4096, te, te + 5000 + int(rng.integers(0, 9))))
    cols = toy_cols(rows)
    p = rng.permutation(len(rows))
    cols = {k: v[p] for k, v in cols.items()}
    g, o = run_both(topo, cols, what="sizes", expect_path=1, tbase_init_ns=1000, lag_floor_ns=1000)
    assert g.n_flag > 0 and g.n_group > 3
    # one record twice: a data error on both paths
    dup = {k: np.concatenate([v, v[5:6]]) for k, v in cols.items()}
    g, o = run_both(topo, dup, what="dup")
    assert g.status == "E_DUPLICATE_KEY"
    # the detection state survives the abandoned attempts and the error: a context that has seen them agrees
    # with one that has not
    from paper_2605_04478_amd import ccld
    keep = ~((cols["comm"] == 5) & (cols["seq"] == 1010))
    hole = {k: v[keep] for k, v in cols.items()}
    an = ccld.Analyzer(topo, max_window_records=len(rows) + 1, tbase_init_ns=1000, lag_floor_ns=1000, placement=1)
    orc_ = orc.Oracle(topo, dict(tbase_init_ns=1000, lag_floor_ns=1000))
    for step, w in enumerate((cols, dup, hole, cols)):
        an.reset_window()
        an.ingest(an.to_device(w))
        gg = an.analyze_window(FAR, n_records=len(rows) + 1, per_record=True)
        oo = orc_.analyze_window(w, FAR)
        blame = order = None
        if oo.status == "OK":
            blame, order = an.rank_blame()
        compare(gg, oo, blame, order, what=f"state step {step}")
        assert gg.path == (0 if step == 2 else 1) or oo.status != "OK"
    an.close()


def test_dense_placement_wide_spreads_take_the_64_bit_pass():
    """Offsets inside a collective that do not fit 30 bits (members seconds apart, operations that run for
    seconds, times near the ends of the int64 range) go through the 64-bit form of the statistics."""
    topo = tg.make_topology(24, [list(range(8)), list(range(8, 24))])
    rng = np.random.default_rng(5)
    rows = []
    for c, mem in enumerate(([*range(8)], [*range(8, 24)])):
        for s in range(300):
            t = T0 + s * 10_000_000_000
            kind = s % 6
            for r in mem:
                te = t + int(rng.integers(0, 2000))
                dur = 50_000 + int(rng.integers(0, 100))
                if kind == 1 and r == mem[3]:
                    te += 3_000_000_000                      # one member three seconds late
                if kind == 2:
                    dur += 2_500_000_000                     # everybody runs for seconds
                if kind == 3 and r == mem[0]:
                    te -= 1_100_000_000                      # the first member far ahead of the others
                if kind == 4 and r == mem[-1]:
                    dur = 2**31 + 5                          # just past 31 bits
                if kind == 5 and r == mem[1]:
                    dur = 2**30 - 1 - 2000                   # just inside the 32-bit form
                rows.append((r, c, s, 0, 1 << 20, te, te + dur))
    # times at the top of the range
    big = 2**62
    for r in range(8):
        rows.append((r, 0, 300, 0, 1 << 20, big + r, big + r + 7 + (2**40 if r == 2 else 0)))
    cols = toy_cols(rows)
    p = rng.permutation(len(rows))
    cols = {k: v[p] for k, v in cols.items()}
    g, o = run_both(topo, cols, now=2**62 + 2**41, what="wide", expect_path=1, tbase_init_ns=1000)
    assert g.n_flag > 100


def test_barrier_operation_missing_member_and_warmup_origin_parity():
    """An all-gather of three bytes is no barrier; a member without a record makes a hang alert of the first kind
    also when other members have finished; the warm-up span of Eq. 1 starts at the first round's earliest entry."""
    topo = ring_topology(2)
    rows = (rounds_with_durations([[9000, 1000]], op=tg.OP_ALLREDUCE, nbytes=3, seq0=0)
            + rounds_with_durations([[9000, 1000]], op=tg.OP_ALLGATHER, nbytes=3, seq0=1))
    g, o = run_both(topo, toy_cols(rows), what="barrier-op", tbase_init_ns=1000)
    assert list(g.group["op"]) == [tg.OP_ALLGATHER] and g.group["slow"][0] == 1
    topo4 = ring_topology(4)
    t = T0 + 1000
    rows = [(r, 0, 6, 0, 4096, T0 + r, T0 + 100) for r in range(4)]
    rows += [(0, 0, 7, 0, 4096, t, INFLIGHT), (1, 0, 7, 0, 4096, t + 1, INFLIGHT), (3, 0, 7, 0, 4096, t + 2, t + 90)]
    g, o = run_both(topo4, toy_cols(rows), now=t + 10_000, what="missing+finished", hang_threshold_ns=5_000)
    assert list(g.alert["class"]) == [1] and list(g.cand[:1]) == [2]
    S = 1_000_000_000
    for third_at, m in ((120 * S, 3), (120 * S + S // 2, 2)):
        rows = []
        for j, start in enumerate([0, 60 * S, third_at, 240 * S]):
            for rk in range(2):
                te = T0 + start + (S if (j == 0 and rk == 1) else 0)
                rows.append((rk, 0, j, tg.OP_ALLREDUCE, 1 << 20, te, te + 10_000))
        g, o = run_both(topo, toy_cols(rows), what=f"warmup{m}", tbase_init_ns=7)
        assert g.group["m"][0] == m and g.group["frozen"][0] == 1



def test_tiles_of_many_short_collectives_beside_longer_ones():
    # pairs: 512 collectives per tile of 1,024 sorted records, of which the statistics kernel stages the table rows
    # of the first 144 and writes the others directly; after them eight-member rounds (128 per tile, all staged)
    # and rounds of 5 (fewer than eight members: never staged by the dense placement); some members missing, one
    # operation in flight, so that rows with empty statistics pass through both ways
    rng = np.random.default_rng(11)
    pairs = [[2 * i, 2 * i + 1] for i in range(24)]
    comms = pairs + [list(range(48, 56)), list(range(56, 64)), [0, 9, 18, 27, 36], list(range(40, 48))]
    topo = ring_topology(64, comms=comms)
    rows = []
    for c, members in enumerate(comms):
        for s in range(130):
            t = T0 + s * 1_000_000 + c * 1000
            for r in members:
                if rng.random() < 0.02:
                    continue                                   # a member without a record
                e = t + int(rng.integers(0, 5000))
                rows.append((r, c, s, tg.OP_ALLREDUCE, 1 << 20, e, e + int(rng.integers(1000, 90000))))
    cols = toy_cols(rows)
    cols["t_exit"][rng.integers(0, len(rows), 40)] = INFLIGHT
    perm = rng.permutation(len(rows))
    cols = {k: v[perm] for k, v in cols.items()}
    g, o = run_both(topo, cols, what="short-and-long", lag_floor_ns=1000, tbase_init_ns=1000)
    assert g.n_seg > 24 * 130 and g.n_flag > 0
