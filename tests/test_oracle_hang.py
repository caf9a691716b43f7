"""Pins of the CPU oracle's hang location: the paper's three-branch decision tree on
hand-built states, recovery of the injected root on simulated rings (every frozen position),
agreement of the wait-for walk with the fewest-counts rule, healthy runs, error statuses."""
import numpy as np
import pytest

from oracle import ccld_oracle as orc
from paper_2605_04478_amd import tracegen as tg
from tests.helpers import ring_topology

NO_RANK = orc.NO_RANK


def snap_rows(topo, n_snap, n_ch, state):
    """state(s, comm, slot, ch) -> (seq_posted, chunks_sent, chunks_recv)"""
    cols = {k: [] for k in tg.SNAP_COLUMNS}
    for c in range(topo.n_comms):
        for q, r in enumerate(topo.members_of(c)):
            for ch in range(n_ch):
                for s in range(n_snap):
                    seq, a, b = state(s, c, q, ch)
                    for k, v in zip(tg.SNAP_COLUMNS, (s, int(r), c, ch, seq, a, b)):
                        cols[k].append(v)
    dt = {"snap": np.uint32, "rank": np.uint32, "comm": np.uint32, "channel": np.uint32,
          "seq_posted": np.uint64, "chunks_sent": np.uint32, "chunks_recv": np.uint32}
    return {k: np.asarray(v, dtype=dt[k]) for k, v in cols.items()}


def locate(topo, cols, n_snap, n_ch, **params):
    return orc.Oracle(topo, params).locate_hang(cols, n_snap, n_ch)


def roots(r):
    return list(zip(r.root["rank"].tolist(), r.root["comm"].tolist(), r.root["class"].tolist()))


def test_healthy_progress_has_no_root():
    topo = ring_topology(4)
    r = locate(topo, snap_rows(topo, 12, 2, lambda s, c, q, ch: (100 + s, 7, 7)), 12, 2, stall_snapshots=5)
    assert r.status == "OK" and roots(r) == [] and r.comm["hung"].sum() == 0
    assert r.pair["stalled"].sum() == 0
    # finished and idle: stalled but consistent -> not hung
    r = locate(topo, snap_rows(topo, 12, 2, lambda s, c, q, ch: (100, 7, 7)), 12, 2, stall_snapshots=5)
    assert r.pair["stalled"].sum() == 4 and r.comm["hung"].sum() == 0 and roots(r) == []
    assert list(r.pair["onset"]) == [0, 0, 0, 0]


def test_not_entered_rank_is_the_root():
    """H1: the rank whose operation counter did not increment."""
    topo = ring_topology(4)

    def st(s, c, q, ch):
        if s < 3 or q == 2:
            return (50, 9, 9)                     # rank 2 never posts operation 51
        return (51, 1, 0)
    r = locate(topo, snap_rows(topo, 10, 2, st), 10, 2, stall_snapshots=4)
    assert roots(r) == [(2, 0, 1)]
    assert list(r.pair["entered"]) == [1, 1, 0, 1] and r.comm["seq_max"][0] == 51
    assert list(r.pair["hops"]) == [-1, -1, 0, -1]
    assert list(r.pair["onset"]) == [3, 3, 0, 3]


def test_non_hang_ranks_are_the_root_of_an_inconsistent_hang():
    """H2: all entered, some ranks keep progressing (they run a different operation)."""
    topo = ring_topology(4)

    def st(s, c, q, ch):
        if q in (1, 3):
            return (51, 10 + s, 10 + s)            # still moving
        return (51, 4, 3)
    r = locate(topo, snap_rows(topo, 10, 1, st), 10, 1, stall_snapshots=4)
    assert roots(r) == [(1, 0, 2), (3, 0, 2)]
    assert list(r.pair["stalled"]) == [1, 0, 1, 0]


def test_all_hung_fewest_counts_is_the_root():
    """H3: every rank entered and stalled; a pure wait-for cycle falls back to the rank with the
    fewest SendCount/RecvCount (ties: fewer received, then smaller rank)."""
    topo = ring_topology(4)
    sr = {0: (9, 9), 1: (7, 7), 2: (8, 8), 3: (9, 9)}       # everybody has R >= S_pred?  1: 7 < 9 no
    # make a pure cycle: each rank received everything its predecessor sent
    cyc = {0: (5, 5), 1: (5, 5), 2: (5, 5), 3: (5, 6)}
    r = locate(topo, snap_rows(topo, 8, 1, lambda s, c, q, ch: (9, *cyc[q])), 8, 1, stall_snapshots=3, fifo_depth=8)
    assert r.comm["hung"][0] == 1 and r.comm["class"][0] == 3
    assert list(r.pair["waits_on"]) == [3, 0, 1, 2]
    assert roots(r) == [(0, 0, 3)] and r.comm["root_by_count"][0] == 0
    # not a cycle: rank 1 neither starved (7 < 9) nor back-pressured (7 - 8 < 8)
    r = locate(topo, snap_rows(topo, 8, 1, lambda s, c, q, ch: (9, *sr[q])), 8, 1, stall_snapshots=3, fifo_depth=8)
    assert roots(r) == [(1, 0, 3)] and r.comm["root_by_count"][0] == 1
    assert list(r.pair["waits_on"]) == [3, NO_RANK, 1, 2]
    assert list(r.pair["hops"]) == [3, 0, 1, 2]


@pytest.mark.parametrize("n", [2, 3, 5, 8])
def test_simulated_ring_hang_recovers_every_frozen_position(n):
    topo = ring_topology(n)
    for frozen in range(n):
        for depth in (1, 3, 8):
            c0 = np.array([3, 11, 40])
            S, R = tg.ring_steady_state(n, frozen, c0, 1 << 20, depth)

            def st(s, c, q, ch):
                if s < 2:
                    return (4, 60, 60)
                return (5, int(S[q, ch]), int(R[q, ch]))
            r = locate(topo, snap_rows(topo, 9, 3, st), 9, 3, stall_snapshots=4, fifo_depth=depth)
            assert roots(r) == [(frozen, 0, 3)], (n, frozen, depth)
            assert r.comm["root_by_count"][0] == frozen           # the walk agrees with the fewest counts
            hops = r.pair["hops"]
            assert hops[frozen] == 0 and (np.delete(hops, frozen) > 0).all()
            # brute-force walk over the reported edges ends at the frozen rank
            for q in range(n):
                cur, steps = q, 0
                while r.pair["waits_on"][cur] != NO_RANK:
                    cur = int(r.pair["waits_on"][cur]); steps += 1
                    assert steps <= n
                assert cur == frozen and steps == hops[q]


def test_tree_compares_ranks_of_the_same_layer_only():
    # 7-rank binary tree in BFS order: layers {0}, {1,2}, {3,4,5,6}
    topo = tg.make_topology(7, [list(range(7))], algo=[tg.ALGO_TREE], tree_parent=[[-1, 0, 0, 1, 1, 2, 2]])
    layer_counts = {0: (20, 4), 1: (12, 12), 2: (12, 12), 3: (6, 2), 4: (6, 2), 5: (6, 2), 6: (6, 2)}
    # layers differ from each other but agree inside: a finished tree operation, not hung
    r = locate(topo, snap_rows(topo, 8, 1, lambda s, c, q, ch: (3, *layer_counts[q])), 8, 1, stall_snapshots=3)
    assert r.comm["hung"][0] == 0 and roots(r) == []
    # rank 5 is behind its layer
    bad = dict(layer_counts); bad[5] = (3, 1)
    r = locate(topo, snap_rows(topo, 8, 1, lambda s, c, q, ch: (3, *bad[q])), 8, 1, stall_snapshots=3)
    assert r.comm["hung"][0] == 1 and r.comm["class"][0] == 3 and roots(r) == [(5, 0, 3)]
    # the same counts on a ring would compare everybody with everybody
    ring = ring_topology(7)
    r = locate(ring, snap_rows(ring, 8, 1, lambda s, c, q, ch: (3, *layer_counts[q])), 8, 1, stall_snapshots=3)
    assert r.comm["hung"][0] == 1


def test_too_few_snapshots_cannot_call_a_stall():
    topo = ring_topology(3)
    cols = snap_rows(topo, 4, 1, lambda s, c, q, ch: (1, q, 0))
    assert roots(locate(topo, cols, 4, 1, stall_snapshots=3)) != []
    r = locate(topo, cols, 4, 1, stall_snapshots=4)
    assert r.pair["stalled"].sum() == 0 and roots(r) == []


def test_statuses():
    topo = ring_topology(4, comms=[[0, 1], [2, 3]])
    cols = snap_rows(topo, 3, 2, lambda s, c, q, ch: (1, 1, 1))
    assert locate(topo, cols, 3, 2).status == "OK"
    cut = {k: v[:-1] for k, v in cols.items()}
    assert locate(topo, cut, 3, 2).status == "E_SNAPSHOT_GAP"
    dup = {k: np.concatenate([v[:-1], v[:1]]) for k, v in cols.items()}
    assert locate(topo, dup, 3, 2).status == "E_DUPLICATE_KEY"
    bad = {k: v.copy() for k, v in cols.items()}; bad["comm"][0] = 9
    assert locate(topo, bad, 3, 2).status == "E_UNKNOWN_COMM"
    bad = {k: v.copy() for k, v in cols.items()}; bad["rank"][0] = 3
    assert locate(topo, bad, 3, 2).status == "E_RANK_NOT_MEMBER"
    bad = {k: v.copy() for k, v in cols.items()}; bad["channel"][0] = 2
    assert locate(topo, bad, 3, 2).status == "E_RANGE"
    bad = {k: v.copy() for k, v in cols.items()}; bad["snap"][0] = 3
    assert locate(topo, bad, 3, 2).status == "E_RANGE"
    # a non-member outranks a range error
    bad = {k: v.copy() for k, v in cols.items()}; bad["channel"][0] = 2; bad["rank"][5] = 3
    assert locate(topo, bad, 3, 2).status == "E_RANK_NOT_MEMBER"


def test_the_operation_counter_of_a_member_is_the_largest_over_its_channels():
    """Channels advance one after the other: a member whose first channel already shows operation 8 has entered
    it, even though its second channel still shows 7; its peer, at 7 on both, has not."""
    topo = ring_topology(2)
    state = lambda s, c, q, ch: (8 if (q == 0 and ch == 0) else 7, 4, 4)
    r = locate(topo, snap_rows(topo, 6, 2, state), 6, 2, stall_snapshots=3)
    assert list(r.pair["seq"]) == [8, 7] and list(r.pair["entered"]) == [1, 0]
    assert roots(r) == [(1, 0, 1)]                                    # H1: not entered


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_cluster_hang_names_exactly_the_injected_rank(seed):
    """The frozen rank is the only root: its ring is a hardware-type hang, every other hung
    communicator only contains victims that are blocked inside the ring."""
    lay = tg.Layout3D(tp=4, pp=2, dp=8, world=True)
    ht = tg.generate_hang(tg.config4(layout=lay, seed=seed, n_channels=4))
    r = orc.Oracle(ht.topo).locate_hang(ht.cols, 64, 4)
    assert roots(r) == [(ht.root_rank, ht.root_comm, 3)]
    hung = r.comm["hung"] == 1
    assert hung.sum() > 3 and (r.comm["class"][hung & (r.comm["comm"] != ht.root_comm)] == 1).all()
    assert r.comm["root_by_count"][ht.root_comm] == ht.root_rank
    # order of the rows does not matter
    p = np.random.default_rng(seed).permutation(ht.n)
    r2 = orc.Oracle(ht.topo).locate_hang({k: v[p] for k, v in ht.cols.items()}, 64, 4)
    for name in ("root", "pair", "comm"):
        for k in getattr(r, name):
            assert np.array_equal(getattr(r, name)[k], getattr(r2, name)[k])
    healthy = tg.generate_hang(tg.config4(layout=lay, seed=seed, n_channels=4, healthy=True))
    rh = orc.Oracle(healthy.topo).locate_hang(healthy.cols, 64, 4)
    assert roots(rh) == [] and rh.comm["hung"].sum() == 0


# --------------------------------------------------------------------------
# the rules of the hardware branch and of the per-member pass, one at a time (expected values
# written out by hand from the definitions)
# --------------------------------------------------------------------------
def test_fewest_counts_tie_goes_to_fewer_received_then_smaller_rank():
    """Fewest SendCount + RecvCount; among equals the rank that received less; then the smaller rank."""
    topo = ring_topology(4)
    # sums: 8, 8, 12, 12; rank 1 received 3, rank 0 received 5 -> rank 1 although rank 0 is smaller
    sr = {0: (3, 5), 1: (5, 3), 2: (6, 6), 3: (6, 6)}
    r = locate(topo, snap_rows(topo, 8, 1, lambda s, c, q, ch: (9, *sr[q])), 8, 1, stall_snapshots=3, fifo_depth=8)
    assert r.comm["hung"][0] == 1 and r.comm["root_by_count"][0] == 1
    # equal sums and equal received counts: the smaller rank
    sr = {0: (6, 6), 1: (4, 4), 2: (4, 4), 3: (6, 6)}
    r = locate(topo, snap_rows(topo, 8, 1, lambda s, c, q, ch: (9, *sr[q])), 8, 1, stall_snapshots=3, fifo_depth=8)
    assert r.comm["root_by_count"][0] == 1
    # a smaller sum beats a smaller received count
    sr = {0: (7, 0), 1: (6, 6), 2: (3, 3), 3: (6, 6)}
    r = locate(topo, snap_rows(topo, 8, 1, lambda s, c, q, ch: (9, *sr[q])), 8, 1, stall_snapshots=3, fifo_depth=8)
    assert r.comm["root_by_count"][0] == 2


def test_back_pressure_starts_at_exactly_fifo_depth_unconsumed_chunks():
    """A rank waits on its successor once the successor holds fifo_depth chunks it has not consumed
    (sent - received_by_successor >= depth), not one chunk later."""
    topo = ring_topology(3)
    # rank 0 sent 12, rank 1 received 4: exactly 8 unconsumed.  rank 0 is not starved (received 2 < 9 sent by rank 2).
    # rank 1: received 4 < 12, sent 4, rank 2 received 4: 0 unconsumed -> waits on nobody: the root.
    # rank 2: received 4 >= 4 sent by rank 1 -> starved, waits on rank 1.
    sr = {0: (12, 2), 1: (4, 4), 2: (9, 4)}
    r = locate(topo, snap_rows(topo, 8, 1, lambda s, c, q, ch: (9, *sr[q])), 8, 1, stall_snapshots=3, fifo_depth=8)
    assert r.comm["class"][0] == 3
    assert list(r.pair["waits_on"]) == [1, NO_RANK, 1]
    assert roots(r) == [(1, 0, 3)] and list(r.pair["hops"]) == [1, 0, 1]
    # one chunk fewer in flight: rank 0 waits on nobody either
    sr[0] = (11, 2)
    r = locate(topo, snap_rows(topo, 8, 1, lambda s, c, q, ch: (9, *sr[q])), 8, 1, stall_snapshots=3, fifo_depth=8)
    assert list(r.pair["waits_on"]) == [NO_RANK, NO_RANK, 1]
    assert roots(r) == [(0, 0, 3), (1, 0, 3)]
    # starvation has precedence over back-pressure: rank 0 with both conditions waits on its predecessor
    sr = {0: (12, 9), 1: (4, 4), 2: (9, 4)}
    r = locate(topo, snap_rows(topo, 8, 1, lambda s, c, q, ch: (9, *sr[q])), 8, 1, stall_snapshots=3, fifo_depth=8)
    assert list(r.pair["waits_on"]) == [2, NO_RANK, 1]


def test_onset_is_the_latest_channel_and_a_stall_needs_every_channel():
    topo = ring_topology(2)

    def st(s, c, q, ch):
        if q == 0:                                  # channel 0 freezes at snapshot 2, channel 1 at snapshot 5
            return (7, min(s, 2) if ch == 0 else min(s, 5), 0)
        if ch == 0:                                 # rank 1: channel 0 frozen from the start ...
            return (7, 1, 1)
        return (7, s, 0)                            # ... channel 1 still moving
    r = locate(topo, snap_rows(topo, 12, 2, st), 12, 2, stall_snapshots=4)
    assert list(r.pair["onset"]) == [5, 11]
    assert list(r.pair["stalled"]) == [1, 0]
    assert list(r.pair["sent"]) == [2 + 5, 1 + 11] and list(r.pair["recv"]) == [0, 1]
    # all entered, rank 1 not stalled -> inconsistent hang with the moving rank as root
    assert roots(r) == [(1, 0, 2)]
    # the other channel moving instead: same verdict
    r = locate(topo, snap_rows(topo, 12, 2, lambda s, c, q, ch: st(s, c, q, 1 - ch)), 12, 2, stall_snapshots=4)
    assert list(r.pair["onset"]) == [5, 11] and list(r.pair["stalled"]) == [1, 0]
    # frozen exactly stall_snapshots before the last snapshot counts as stalled, one later does not
    r = locate(topo, snap_rows(topo, 12, 1, lambda s, c, q, ch: (7, min(s, 7) if q == 0 else min(s, 8), 0)), 12, 1,
               stall_snapshots=4)
    assert list(r.pair["onset"]) == [7, 8] and list(r.pair["stalled"]) == [1, 0]


def test_tree_root_is_only_the_rank_furthest_behind_its_layer():
    # root + four children in one layer, BFS order; sums of the layer: 20, 17, 14, 20 -> deficits 0, 3, 6, 0
    topo = tg.make_topology(5, [list(range(5))], algo=[tg.ALGO_TREE], tree_parent=[[-1, 0, 0, 0, 0]])
    sr = {0: (30, 30), 1: (10, 10), 2: (9, 8), 3: (7, 7), 4: (10, 10)}
    r = locate(topo, snap_rows(topo, 8, 1, lambda s, c, q, ch: (3, *sr[q])), 8, 1, stall_snapshots=3)
    assert r.comm["class"][0] == 3 and roots(r) == [(3, 0, 3)] and r.comm["n_cand"][0] == 1
    # two ranks equally far behind are both roots
    sr[2] = (7, 7)
    r = locate(topo, snap_rows(topo, 8, 1, lambda s, c, q, ch: (3, *sr[q])), 8, 1, stall_snapshots=3)
    assert roots(r) == [(2, 0, 3), (3, 0, 3)]
    # the deficit is measured inside the layer: the root rank's own large counts do not matter
    sr = {0: (1, 1), 1: (10, 10), 2: (10, 10), 3: (10, 9), 4: (10, 10)}
    r = locate(topo, snap_rows(topo, 8, 1, lambda s, c, q, ch: (3, *sr[q])), 8, 1, stall_snapshots=3)
    assert roots(r) == [(3, 0, 3)]


def test_victim_filter_needs_the_rank_inside_the_other_hung_communicator():
    """A rank that has not entered communicator 0 is dropped as a victim only if it HAS entered
    another hung communicator; membership of a hung communicator that it has not entered either
    leaves it a root of both."""
    # communicator 0 = {0, 1, 2}, communicator 1 = {2, 3, 4}
    topo = ring_topology(5, comms=[[0, 1, 2], [2, 3, 4]])

    def st(entered_in_1):
        def f(s, c, q, ch):
            r = topo.members_of(c)[q]
            if c == 0:
                return (50, 9, 9) if r == 2 else (51, 1, 0)         # rank 2 never posts operation 51 on communicator 0
            if r == 2:
                return (71, 2, 1) if entered_in_1 else (70, 9, 9)
            return (71, 1, 0)
        return f
    # rank 2 is blocked inside communicator 1 (entered operation 71 there, everyone stalled, counts differ):
    # communicator 1 is a hardware-type hang, rank 2's absence from communicator 0 is a consequence
    r = locate(topo, snap_rows(topo, 8, 1, st(True)), 8, 1, stall_snapshots=3)
    assert list(r.comm["hung"]) == [1, 1] and list(r.comm["class"]) == [1, 3]
    assert all(c == 1 for _, c, _ in roots(r)) and r.comm["n_cand"][0] == 0
    # rank 2 has entered neither: it is the not-entered root of both
    r = locate(topo, snap_rows(topo, 8, 1, st(False)), 8, 1, stall_snapshots=3)
    assert list(r.comm["class"]) == [1, 1]
    assert roots(r) == [(2, 0, 1), (2, 1, 1)]


def test_a_rank_that_has_not_entered_comes_before_ranks_that_still_progress():
    """First question of the decision tree first: rank 3 never posted the operation, rank 0 still moves data,
    ranks 1 and 2 are stuck.  Not-Entered-Hang with rank 3, not Inconsistent-Hang with rank 0."""
    topo = ring_topology(4)

    def st(s, c, q, ch):
        if q == 3:
            return (6, 5, 5)
        if q == 0:
            return (7, 10 + s, 10 + s)
        return (7, 2, 1)
    r = locate(topo, snap_rows(topo, 8, 1, st), 8, 1, stall_snapshots=3)
    assert list(r.pair["stalled"]) == [0, 1, 1, 1] and list(r.pair["entered"]) == [1, 1, 1, 0]
    assert r.comm["class"][0] == 1 and roots(r) == [(3, 0, 1)]


def test_healthy_communicator_reports_no_rank_by_count():
    topo = ring_topology(3)
    r = locate(topo, snap_rows(topo, 8, 1, lambda s, c, q, ch: (100 + s, 3 + q, 3)), 8, 1, stall_snapshots=3)
    assert r.comm["hung"][0] == 0 and r.comm["root_by_count"][0] == orc.NO_RANK and r.comm["n_cand"][0] == 0


def test_victim_filter_applies_to_not_entered_candidates_of_hung_communicators_only():
    # communicator 0 = ring {0, 1}: all entered, all stuck, rank 0 waits on nobody -> hardware root rank 0.
    # communicator 1 = ring {0, 2, 3}: rank 3 never posted operation 9 -> not-entered root rank 3.
    # Rank 0 has entered the hung communicator 1, but it is a hardware root, not a not-entered candidate: it stays.
    topo = ring_topology(4, comms=[[0, 1], [0, 2, 3]])

    def st(s, c, q, ch):
        if c == 0:
            return (5, 3, 2) if q == 0 else (5, 5, 3)
        return (8, 4, 4) if q == 2 else (9, 1, 1)
    r = locate(topo, snap_rows(topo, 8, 1, st), 8, 1, stall_snapshots=3)
    assert list(r.comm["class"]) == [3, 1]
    assert roots(r) == [(0, 0, 3), (3, 1, 1)]
    # communicator 0 = ring {0, 1}: rank 1 never posted operation 5.  Communicator 1 = ring {1, 2} is finished and
    # idle (equal counts): rank 1 counts as entered there, but an idle communicator blocks nobody: rank 1 stays.
    topo = ring_topology(3, comms=[[0, 1], [1, 2]])

    def st2(s, c, q, ch):
        if c == 0:
            return (5, 1, 0) if q == 0 else (4, 6, 6)
        return (7, 2, 2)
    r = locate(topo, snap_rows(topo, 8, 1, st2), 8, 1, stall_snapshots=3)
    assert list(r.comm["hung"]) == [1, 0] and roots(r) == [(1, 0, 1)]
