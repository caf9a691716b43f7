"""GPU parity: ccld_locate_hang through the C ABI against the CPU oracle (bit-exact tables)."""
import numpy as np
import pytest

from oracle import ccld_oracle as orc
from paper_2605_04478_amd import tracegen as tg
from tests.helpers import ring_topology
from tests.test_oracle_hang import snap_rows

pytestmark = pytest.mark.gpu


def run_both(topo, cols, n_snap, n_ch, on_device=True, what="", **params):
    from paper_2605_04478_amd import ccld
    n_cells = int(topo.size.sum()) * n_snap * n_ch
    an = ccld.Analyzer(topo, max_window_records=1024, max_snapshot_rows=max(n_cells, int(cols["snap"].shape[0]), 1),
                       **params)
    g = an.locate_hang(an.snapshots_to_device(cols) if on_device else cols, n_snap, n_ch)
    o = orc.Oracle(topo, params).locate_hang(cols, n_snap, n_ch)
    assert g.status == o.status, (what, g.status, o.status)
    if o.status == "OK":
        assert g.n_root == len(o.root["rank"]), what
        assert g.n_hung_comm == int(o.comm["hung"].sum()), what
        for name in ("root", "pair", "comm"):
            gt, ot = getattr(g, name), getattr(o, name)
            for k in ot:
                assert np.array_equal(gt[k], ot[k]), (what, name, k, gt[k][:8], ot[k][:8])
    an.close()
    return g, o


def test_cluster_hang_parity_small_layouts():
    for seed, lay in enumerate([tg.Layout3D(tp=4, pp=2, dp=8, world=True), tg.Layout3D(tp=2, pp=2, dp=4, world=True),
                                tg.Layout3D(tp=8, pp=2, dp=16, world=True)]):
        ht = tg.generate_hang(tg.config4(layout=lay, seed=seed, n_channels=5, n_snapshots=70))
        g, o = run_both(ht.topo, ht.cols, 70, 5, what=f"hang{seed}")
        assert list(g.root["rank"]) == [ht.root_rank] and list(g.root["comm"]) == [ht.root_comm]
        hh = tg.generate_hang(tg.config4(layout=lay, seed=seed, n_channels=5, n_snapshots=70, healthy=True))
        g, o = run_both(hh.topo, hh.cols, 70, 5, what=f"healthy{seed}")
        assert g.n_root == 0 and g.n_hung_comm == 0


def test_host_rows_parity():
    ht = tg.generate_hang(tg.config4(layout=tg.Layout3D(tp=2, pp=2, dp=4, world=True), n_channels=3))
    run_both(ht.topo, ht.cols, 64, 3, on_device=False, what="host")


def test_decision_tree_branches_parity():
    topo = ring_topology(4)
    h1 = lambda s, c, q, ch: (50, 9, 9) if (s < 3 or q == 2) else (51, 1, 0)
    h2 = lambda s, c, q, ch: (51, 10 + s, 10 + s) if q in (1, 3) else (51, 4, 3)
    cyc = {0: (5, 5), 1: (5, 5), 2: (5, 5), 3: (5, 6)}
    sr = {0: (9, 9), 1: (7, 7), 2: (8, 8), 3: (9, 9)}
    for name, st in (("h1", h1), ("h2", h2), ("cycle", lambda s, c, q, ch: (9, *cyc[q])),
                     ("h3", lambda s, c, q, ch: (9, *sr[q]))):
        g, o = run_both(topo, snap_rows(topo, 10, 2, st), 10, 2, what=name, stall_snapshots=4)
        assert g.n_root >= 1


@pytest.mark.parametrize("n", [2, 5, 8, 300])
def test_simulated_rings_parity(n):
    topo = ring_topology(n)
    for frozen in sorted({0, n // 2, n - 1}):
        c0 = np.array([3, 11])
        S, R = tg.ring_steady_state(n, frozen, c0, 1 << 20, 3)
        st = lambda s, c, q, ch: (4, 60, 60) if s < 2 else (5, int(S[q, ch]), int(R[q, ch]))
        g, o = run_both(topo, snap_rows(topo, 9, 2, st), 9, 2, what=f"ring{n}/{frozen}", stall_snapshots=4, fifo_depth=3)
        assert list(g.root["rank"]) == [frozen]


def test_tree_parity():
    topo = tg.make_topology(7, [list(range(7))], algo=[tg.ALGO_TREE], tree_parent=[[-1, 0, 0, 1, 1, 2, 2]])
    ok = {0: (20, 4), 1: (12, 12), 2: (12, 12), 3: (6, 2), 4: (6, 2), 5: (6, 2), 6: (6, 2)}
    bad = dict(ok); bad[5] = (3, 1)
    run_both(topo, snap_rows(topo, 8, 1, lambda s, c, q, ch: (3, *ok[q])), 8, 1, what="tree-ok", stall_snapshots=3)
    g, _ = run_both(topo, snap_rows(topo, 8, 1, lambda s, c, q, ch: (3, *bad[q])), 8, 1, what="tree-bad", stall_snapshots=3)
    assert list(g.root["rank"]) == [5]


def test_statuses_parity():
    topo = ring_topology(4, comms=[[0, 1], [2, 3]])
    cols = snap_rows(topo, 3, 2, lambda s, c, q, ch: (1, 1, 1))
    cases = {"ok": cols, "gap": {k: v[:-1] for k, v in cols.items()},
             "dup": {k: np.concatenate([v[:-1], v[:1]]) for k, v in cols.items()}}
    for name, col, val in (("comm", "comm", 9), ("member", "rank", 3), ("chan", "channel", 2), ("snap", "snap", 3)):
        b = {k: v.copy() for k, v in cols.items()}
        b[col][0] = val
        cases[name] = b
    b = {k: v.copy() for k, v in cols.items()}
    b["channel"][0] = 2; b["rank"][5] = 3
    cases["member+range"] = b
    want = {"ok": "OK", "gap": "E_SNAPSHOT_GAP", "dup": "E_DUPLICATE_KEY", "comm": "E_UNKNOWN_COMM",
            "member": "E_RANK_NOT_MEMBER", "chan": "E_RANGE", "snap": "E_RANGE", "member+range": "E_RANK_NOT_MEMBER"}
    for name, c in cases.items():
        g, o = run_both(topo, c, 3, 2, what=name)
        assert g.status == want[name]


def test_too_few_snapshots_parity():
    topo = ring_topology(3)
    cols = snap_rows(topo, 4, 1, lambda s, c, q, ch: (1, q, 0))
    run_both(topo, cols, 4, 1, what="few3", stall_snapshots=3)
    run_both(topo, cols, 4, 1, what="few4", stall_snapshots=4)


def test_a_row_that_holds_the_fill_pattern_is_still_a_row():
    """The quick placement starts the grid from an all-ones fill and takes a cell that still holds it for an
    empty one; a real row with exactly that content makes it repeat the placement with the presence bitmap."""
    topo = ring_topology(3)
    full = (2**64 - 1, 2**32 - 1, 2**32 - 1)
    state = lambda s, c, q, ch: full if (s == 2 and q == 1 and ch == 0) else (7 + (s > 4), 3 + s, 2 + s)
    g, o = run_both(topo, snap_rows(topo, 9, 2, state), 9, 2, what="all-ones-row", stall_snapshots=3)
    assert g.status == "OK"


def test_large_grids_take_the_two_step_placement_with_the_same_results_and_statuses():
    """Grids of a million cells and more are regrouped by region before they are placed; duplicates (a region
    that receives more rows than it has cells, or a cell left at the fill) must still end in the exact pass."""
    lay = tg.Layout3D(tp=4, pp=4, dp=32, world=True)                    # 512 ranks, 2,048 member slots
    ht = tg.generate_hang(tg.config4(layout=lay, seed=5, n_channels=10, n_snapshots=60))
    n = int(ht.cols["snap"].shape[0])
    assert n == 2048 * 10 * 60 and n >= 1 << 20
    g, o = run_both(ht.topo, ht.cols, 60, 10, what="large")
    assert g.status == "OK" and list(g.root["rank"]) == [ht.root_rank]
    rng = np.random.default_rng(1)
    cases = {}
    b = {k: v.copy() for k, v in ht.cols.items()}
    i, j = rng.choice(n, 2, replace=False)
    for k in b:
        b[k][i] = b[k][j]                                              # one cell twice, one cell missing
    cases["dup"] = (b, "E_DUPLICATE_KEY")
    b = {k: v.copy() for k, v in ht.cols.items()}
    first = np.nonzero((b["comm"] == b["comm"][0]) & (b["rank"] == b["rank"][0]) & (b["channel"] == b["channel"][0]))[0]
    donors = rng.choice(n, 70_000, replace=False)                      # one region receives 70,000 rows more than it holds
    for k in b:
        b[k][donors] = b[k][first[0]]
    cases["overflow"] = (b, "E_DUPLICATE_KEY")
    b = {k: v.copy() for k, v in ht.cols.items()}
    b["channel"][int(rng.integers(n))] = 10
    cases["range"] = (b, "E_RANGE")
    b = {k: v.copy() for k, v in ht.cols.items()}
    b["comm"][int(rng.integers(n))] = ht.topo.n_comms
    cases["comm"] = (b, "E_UNKNOWN_COMM")
    cases["gap"] = ({k: v[:-1] for k, v in ht.cols.items()}, "E_SNAPSHOT_GAP")
    for name, (c, want) in cases.items():
        g, o = run_both(ht.topo, c, 60, 10, what=name)
        assert g.status == want, (name, g.status)


def test_tree_of_16384_members_parity():
    """A binary tree over 16,384 ranks (heap order: contiguous layers): a clean stall, and one with two ranks of
    one layer behind their peers by different amounts (only the one furthest behind is a root)."""
    n = 16384
    parent = [-1] + [(i - 1) // 2 for i in range(1, n)]
    topo = tg.make_topology(n, [list(range(n))], algo=[tg.ALGO_TREE], tree_parent=[parent])
    depth = np.floor(np.log2(np.arange(n) + 1)).astype(int)
    ok = lambda s, c, q, ch: (3, 40 - 2 * int(depth[q]) + ch, 10 + int(depth[q]))
    run_both(topo, snap_rows(topo, 6, 2, ok), 6, 2, what="tree16k-ok", stall_snapshots=3)
    behind = {9000: 7, 12000: 3}
    bad = lambda s, c, q, ch: (3, 40 - 2 * int(depth[q]) + ch - (behind.get(q, 0) if ch == 0 else 0), 10 + int(depth[q]))
    g, _ = run_both(topo, snap_rows(topo, 6, 2, bad), 6, 2, what="tree16k-bad", stall_snapshots=3)
    assert list(g.root["rank"]) == [9000]


def test_operation_counter_is_the_largest_over_the_channels_parity():
    topo = ring_topology(2)
    state = lambda s, c, q, ch: (8 if (q == 0 and ch == 0) else 7, 4, 4)
    g, o = run_both(topo, snap_rows(topo, 6, 2, state), 6, 2, what="seq-over-channels", stall_snapshots=3)
    assert list(g.pair["seq"]) == [8, 7] and list(g.root["rank"]) == [1]


def test_decision_tree_order_and_victim_filter_scope_parity():
    topo = ring_topology(4)

    def st(s, c, q, ch):
        if q == 3:
            return (6, 5, 5)
        if q == 0:
            return (7, 10 + s, 10 + s)
        return (7, 2, 1)
    g, o = run_both(topo, snap_rows(topo, 8, 1, st), 8, 1, what="not-entered first", stall_snapshots=3)
    assert list(g.root["rank"]) == [3] and list(g.root["class"]) == [1]
    topo3 = ring_topology(3)
    g, o = run_both(topo3, snap_rows(topo3, 8, 1, lambda s, c, q, ch: (100 + s, 3 + q, 3)), 8, 1, what="healthy", stall_snapshots=3)
    assert g.comm["root_by_count"][0] == 0xFFFFFFFF
    topo = ring_topology(4, comms=[[0, 1], [0, 2, 3]])

    def st1(s, c, q, ch):
        if c == 0:
            return (5, 3, 2) if q == 0 else (5, 5, 3)
        return (8, 4, 4) if q == 2 else (9, 1, 1)
    g, o = run_both(topo, snap_rows(topo, 8, 1, st1), 8, 1, what="hardware root stays", stall_snapshots=3)
    assert list(zip(g.root["rank"], g.root["comm"], g.root["class"])) == [(0, 0, 3), (3, 1, 1)]
    topo = ring_topology(3, comms=[[0, 1], [1, 2]])

    def st2(s, c, q, ch):
        if c == 0:
            return (5, 1, 0) if q == 0 else (4, 6, 6)
        return (7, 2, 2)
    g, o = run_both(topo, snap_rows(topo, 8, 1, st2), 8, 1, what="idle communicator blocks nobody", stall_snapshots=3)
    assert list(zip(g.root["rank"], g.root["comm"], g.root["class"])) == [(1, 0, 1)]

