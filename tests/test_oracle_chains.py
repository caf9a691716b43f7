"""Pins of the oracle's separation of root-cause and secondary late entries (Section 4.2.2: anomalies
propagate across ranks; the location step tells the rank that triggered one from those that pass it
on): hand-built causal chains with the expected parents written out, tie rules, and a dependent schedule
from the generator in which every link must be causal and the injected ranks cause the most late entries."""
import numpy as np

from oracle import ccld_oracle as orc
from paper_2605_04478_amd import tracegen as tg
from tests.chain_check import chains_by_definition
from tests.helpers import T0, toy_cols

MS = 1_000_000
DUR = 400_000          # every collective runs 0.4 ms after its last member has entered
GAP = 50_000           # compute time between leaving one collective and entering the next


def _chain_case():
    """A = rank 0 is slow of its own.  communicator 0 = {0, 1, 2, 3}, 1 = {1, 4, 5, 6}, 2 = {4, 7, 8, 9}.
    Round 0 of communicator 0: A enters 2 ms late, so B = rank 1 leaves it 2 ms late and enters round 0 of
    communicator 1 late; C = rank 4 leaves that one late and enters round 0 of communicator 2 late."""
    topo = tg.make_topology(10, [[0, 1, 2, 3], [1, 4, 5, 6], [4, 7, 8, 9]])
    rows = []

    def collective(comm, seq, enters):           # enters: {rank: t_enter}; all leave DUR after the last entry
        end = max(enters.values()) + DUR
        for r, t in enters.items():
            rows.append((r, comm, seq, tg.OP_ALLREDUCE, 1 << 20, t, end))
        return end

    e0 = collective(0, 0, {0: T0 + 2 * MS, 1: T0, 2: T0, 3: T0})
    assert e0 == T0 + 2 * MS + DUR
    # communicator 1: ranks 4, 5, 6 were ready at T0 + GAP already; rank 1 comes out of communicator 0 first
    e1 = collective(1, 0, {1: e0 + GAP, 4: T0 + GAP, 5: T0 + GAP, 6: T0 + GAP})
    e2 = collective(2, 0, {4: e1 + GAP, 7: T0 + GAP, 8: T0 + GAP, 9: T0 + GAP})
    # rank 0 is late again in its next operation, of its own (its peers wait for it once more)
    collective(0, 1, {0: e0 + GAP + 1 * MS, 1: e1 + GAP, 2: e0 + GAP, 3: e0 + GAP})
    return topo, rows, e2


def _run(topo, rows, shuffle=None):
    cols = toy_cols(rows)
    if shuffle is not None:
        p = np.random.default_rng(shuffle).permutation(len(rows))
        cols = {k: v[p] for k, v in cols.items()}
    o = orc.Oracle(topo)
    r = o.analyze_window(cols, T0 + 10**12)
    assert r.status == "OK"
    chain, per_rank = o.flag_chains(cols, r)
    return r, chain, per_rank


def test_chain_of_three_ranks_has_one_root():
    topo, rows, _ = _chain_case()
    r, chain, per_rank = _run(topo, rows)
    flags = list(zip(r.flag["comm"].tolist(), r.flag["seq"].tolist(), r.flag["rank"].tolist(), r.flag["kind"].tolist()))
    # (communicator 0, round 1) holds two late entries: rank 0 by 1 ms of its own, rank 1 because it came out of
    # communicator 1 late
    assert flags == [(0, 0, 0, 1), (0, 1, 0, 1), (0, 1, 1, 1), (1, 0, 1, 1), (2, 0, 4, 1)]
    k = {f[:3]: i for i, f in enumerate(flags)}
    # rank 0's second late entry follows its own first one (the operation before it was ended late by rank 0);
    # rank 1 enters (1, 0) late because of rank 0 and (0, 1) late because of its own late entry into (1, 0);
    # rank 4 enters (2, 0) late because rank 1 ended (1, 0) late
    assert list(chain["parent"]) == [-1, k[(0, 0, 0)], k[(1, 0, 1)], k[(0, 0, 0)], k[(1, 0, 1)]]
    assert list(chain["root"]) == [0, 0, 0, 0, 0]
    assert list(chain["root_rank"]) == [0, 0, 0, 0, 0]
    assert list(chain["depth"]) == [0, 1, 2, 1, 2]
    assert list(per_rank["root_entries"]) == [1, 0, 0, 0, 0, 0, 0, 0, 0, 0]
    assert list(per_rank["secondary_entries"]) == [1, 2, 0, 0, 1, 0, 0, 0, 0, 0]
    assert list(per_rank["caused"]) == [5, 0, 0, 0, 0, 0, 0, 0, 0, 0]
    # the order of the records does not matter
    for seed in range(3):
        r2, chain2, per2 = _run(topo, rows, shuffle=seed)
        for name in chain:
            assert np.array_equal(chain[name], chain2[name])
        for name in per_rank:
            assert np.array_equal(per_rank[name], per2[name])


def test_previous_operation_and_latest_member_rules():
    # communicator 0 = {0, 1, 2, 3}, 1 = {0, 4, 5, 6}, 2 = {0, 7, 8, 9}
    topo = tg.make_topology(10, [[0, 1, 2, 3], [0, 4, 5, 6], [0, 7, 8, 9]])
    rows = []

    def collective(comm, seq, enters, end=None):
        end = max(enters.values()) + DUR if end is None else end
        for r, t in enters.items():
            rows.append((r, comm, seq, tg.OP_ALLREDUCE, 1 << 20, t, end))
        return end

    # communicator 0, round 0: ranks 1 and 2 are both late, rank 2 by more; rank 3 equally late as rank 2
    e0 = collective(0, 0, {0: T0, 1: T0 + 1 * MS, 2: T0 + 3 * MS, 3: T0 + 3 * MS})
    # rank 0 then runs communicator 1 (late: caused by the latest member of communicator 0, ranks 2 and 3 tie -> rank 2)
    e1 = collective(1, 0, {0: e0 + GAP, 4: T0 + GAP, 5: T0 + GAP, 6: T0 + GAP})
    # an operation of rank 0 on communicator 2 that ends before communicator 0's does is not its previous one
    collective(2, 0, {0: T0 - 5 * MS, 7: T0 - 5 * MS, 8: T0 - 5 * MS, 9: T0 - 5 * MS})
    # rank 5 leaves communicator 1 late as well, but enters nothing afterwards; rank 4 enters communicator 1's
    # next round late of its own (its previous operation, round 0, was ended late by rank 0, another rank: secondary)
    collective(1, 1, {0: e1 + GAP, 4: e1 + GAP + 2 * MS, 5: e1 + GAP, 6: e1 + GAP})
    cols = toy_cols(rows)
    o = orc.Oracle(topo)
    r = o.analyze_window(cols, T0 + 10**12)
    chain, per_rank = o.flag_chains(cols, r)
    flags = list(zip(r.flag["comm"].tolist(), r.flag["seq"].tolist(), r.flag["rank"].tolist()))
    # in (0, 0) the median arrival is 1 ms (values 0, 1, 3, 3 ms), MAD 1 ms: ranks 2 and 3 (lag 2 ms) are not
    # beyond 4.5 MAD, nobody is flagged there, so rank 0's late entry into communicator 1 is a root flag
    assert (0, 0, 2) not in flags and (1, 0, 0) in flags
    k = {f: i for i, f in enumerate(flags)}
    assert chain["parent"][k[(1, 0, 0)]] == -1
    # rank 4 in (1, 1): its previous operation (1, 0) was ended late by rank 0 -> secondary to that flag
    assert chain["parent"][k[(1, 1, 4)]] == k[(1, 0, 0)] and chain["root_rank"][k[(1, 1, 4)]] == 0
    assert per_rank["root_entries"][0] == 1 and per_rank["secondary_entries"][4] == 1
    # with a tighter spread in (0, 0) ranks 2 and 3 are flagged with equal lags: the smaller rank is the parent
    rows2 = [(rk, c, s, op, nb, (T0 if (c == 0 and s == 0 and rk == 1) else te), tx) for rk, c, s, op, nb, te, tx in rows]
    cols2 = toy_cols(rows2)
    o2 = orc.Oracle(topo)
    r2 = o2.analyze_window(cols2, T0 + 10**12)
    chain2, _ = o2.flag_chains(cols2, r2)
    flags2 = list(zip(r2.flag["comm"].tolist(), r2.flag["seq"].tolist(), r2.flag["rank"].tolist()))
    k2 = {f: i for i, f in enumerate(flags2)}
    assert (0, 0, 2) in k2 and (0, 0, 3) in k2
    assert chain2["parent"][k2[(1, 0, 0)]] == k2[(0, 0, 2)]
    assert chain2["depth"][k2[(1, 1, 4)]] == 2 and chain2["root_rank"][k2[(1, 1, 4)]] == 2


def test_late_exits_have_no_parent_and_clean_traces_have_no_chains():
    topo = tg.make_topology(4, [[0, 1, 2, 3]])
    rows = []
    for s in range(5):
        t = T0 + s * 10 * MS
        for rk in range(4):
            rows.append((rk, 0, s, tg.OP_ALLREDUCE, 1 << 20, t, t + DUR + (2 * MS if (rk == 3 and s == 2) else 0)))
    cols = toy_cols(rows)
    o = orc.Oracle(topo)
    r = o.analyze_window(cols, T0 + 10**12)
    chain, per_rank = o.flag_chains(cols, r)
    assert list(r.flag["kind"]) == [orc.FLAG_LATE_EXIT] and list(chain["parent"]) == [-1]
    assert per_rank["root_entries"].sum() == 0 and per_rank["secondary_entries"].sum() == 0 and per_rank["caused"].sum() == 0


def test_dependent_schedule_chains_are_causal_and_lead_to_the_injected_ranks():
    spec = tg.config2(n_cycles=20)
    spec.same_size_per_kind = True
    tr = tg.propagate(tg.generate(spec), gap_ns=2_000_000)
    c = tr.cols
    o = orc.Oracle(tr.topo)
    r = o.analyze_window(c, int(c["t_exit"].max()) + 1)
    chain, per_rank = o.flag_chains(c, r)
    # the injected slow ranks, and the two ends of the slow link (they leave late and so enter late of their own)
    faulty = sorted([s.rank for s in spec.slow_ranks] + [x for g in spec.slow_groups for x in g.ranks])
    late = (r.flag["kind"] & orc.FLAG_LATE_ENTER) != 0
    has_parent = chain["parent"] >= 0
    assert late.sum() > 1000 and has_parent.sum() > 300 and not has_parent[~late].any()
    # every link is causal: the child's rank took part in the parent's collective, which ended (on the child's own
    # clock) before the child entered its collective; the parent is a late entry itself
    rec = {(int(a), int(b), int(d)): i for i, (a, b, d) in enumerate(zip(c["comm"], c["seq"], c["rank"]))}
    for k in np.nonzero(has_parent)[0][:400]:
        p = int(chain["parent"][k])
        assert r.flag["kind"][p] & orc.FLAG_LATE_ENTER
        child = rec[(int(r.flag["comm"][k]), int(r.flag["seq"][k]), int(r.flag["rank"][k]))]
        via = rec[(int(r.flag["comm"][p]), int(r.flag["seq"][p]), int(r.flag["rank"][k]))]      # the child's rank in the parent's round
        assert c["t_exit"][via] <= c["t_enter"][child]
    # depth and root follow the parents
    for k in np.nonzero(has_parent)[0][:400]:
        p = int(chain["parent"][k])
        assert chain["depth"][k] == chain["depth"][p] + 1 and chain["root"][k] == chain["root"][p]
    roots = ~has_parent
    assert np.array_equal(chain["root"][roots], np.nonzero(roots)[0]) and (chain["depth"][roots] == 0).all()
    assert per_rank["caused"].sum() == late.sum()
    assert (per_rank["secondary_entries"].sum() + per_rank["root_entries"].sum()) == late.sum()
    # the ranks that cause the most late entries are injected ranks; by plain flag counts they do not stand out as far
    top = np.argsort(-per_rank["caused"], kind="stable")[:4]
    assert set(top.tolist()) <= set(faulty), (top, faulty)
    other = np.setdiff1d(np.arange(tr.topo.n_ranks), faulty)
    assert per_rank["caused"][top[3]] > per_rank["caused"][other].max()


def _two_open_rows(enter0, enter1):
    """Rank 0 has two operations open at once (two streams): round 0 of communicator 0 = {0, 1, 2, 3}, made late
    by rank 1, and round 0 of communicator 1 = {0, 4, 5, 6}, made late by rank 4; both end at the same instant.
    Rank 0 then enters communicator 2 = {0, 7, 8, 9} late."""
    topo = tg.make_topology(10, [[0, 1, 2, 3], [0, 4, 5, 6], [0, 7, 8, 9]])
    end = T0 + 2 * MS + DUR
    rows = [(0, 0, 0, tg.OP_ALLREDUCE, 1 << 20, enter0, end), (1, 0, 0, tg.OP_ALLREDUCE, 1 << 20, T0 + 2 * MS, end),
            (2, 0, 0, tg.OP_ALLREDUCE, 1 << 20, T0, end), (3, 0, 0, tg.OP_ALLREDUCE, 1 << 20, T0, end),
            (0, 1, 0, tg.OP_ALLREDUCE, 1 << 20, enter1, end), (4, 1, 0, tg.OP_ALLREDUCE, 1 << 20, T0 + 2 * MS, end),
            (5, 1, 0, tg.OP_ALLREDUCE, 1 << 20, T0, end), (6, 1, 0, tg.OP_ALLREDUCE, 1 << 20, T0, end)]
    rows += [(0, 2, 0, tg.OP_ALLREDUCE, 1 << 20, end + GAP, end + GAP + DUR)]
    rows += [(r, 2, 0, tg.OP_ALLREDUCE, 1 << 20, T0 + GAP, end + GAP + DUR) for r in (7, 8, 9)]
    return topo, rows


def _two_open_operations(enter0, enter1):
    """-> the parent of rank 0's late entry into communicator 2, as (comm, seq, rank)"""
    topo, rows = _two_open_rows(enter0, enter1)
    r, chain, _ = _run(topo, rows)
    flags = list(zip(r.flag["comm"].tolist(), r.flag["seq"].tolist(), r.flag["rank"].tolist()))
    assert flags == [(0, 0, 1), (1, 0, 4), (2, 0, 0)]
    p = int(chain["parent"][2])
    return flags[p] if p >= 0 else None


def test_equal_exit_times_go_to_the_later_entry_then_the_larger_communicator():
    assert _two_open_operations(T0, T0 + 100_000) == (1, 0, 4)          # communicator 1 was entered later
    assert _two_open_operations(T0 + 100_000, T0) == (0, 0, 1)          # communicator 0 was entered later
    assert _two_open_operations(T0, T0) == (1, 0, 4)                    # entered together: the larger communicator


def _chain_case_without_gaps():
    global GAP
    keep, GAP = GAP, 0
    try:
        topo, rows, _ = _chain_case()
    finally:
        GAP = keep
    return topo, rows


def test_an_operation_that_ends_at_the_instant_of_entry_is_the_previous_one():
    # the chain of three ranks with no compute time between operations: t_exit of the previous one == t_enter
    topo, rows = _chain_case_without_gaps()
    r, chain, _ = _run(topo, rows)
    flags = list(zip(r.flag["comm"].tolist(), r.flag["seq"].tolist(), r.flag["rank"].tolist()))
    k = {f: i for i, f in enumerate(flags)}
    rec = {(c, s, rk): (te, tx) for rk, c, s, _, _, te, tx in rows}
    assert rec[(1, 0, 1)][0] == rec[(0, 0, 1)][1]                       # rank 1 enters (1, 0) when it leaves (0, 0)
    assert chain["parent"][k[(1, 0, 1)]] == k[(0, 0, 0)] and chain["parent"][k[(2, 0, 4)]] == k[(1, 0, 1)]


def test_a_late_exit_after_a_late_round_still_has_no_parent():
    topo, rows, _ = _chain_case()
    # rank 2 leaves round 1 of communicator 0 two milliseconds after its peers; round 0, its previous operation,
    # holds rank 0's late entry
    rows = [(rk, c, s, op, nb, te, tx + (2 * MS if (rk, c, s) == (2, 0, 1) else 0)) for rk, c, s, op, nb, te, tx in rows]
    r, chain, per_rank = _run(topo, rows)
    i = [j for j in range(len(r.flag["rank"])) if (r.flag["comm"][j], r.flag["seq"][j], r.flag["rank"][j]) == (0, 1, 2)]
    assert len(i) == 1 and r.flag["kind"][i[0]] == orc.FLAG_LATE_EXIT
    assert chain["parent"][i[0]] == -1 and chain["depth"][i[0]] == 0 and chain["root"][i[0]] == i[0]
    assert per_rank["root_entries"][2] == 0 and per_rank["secondary_entries"][2] == 0


def test_chains_by_definition_agrees_with_the_oracle_where_both_run():
    """The array form above against the oracle's loops on a propagating trace of 160,000 records."""
    spec = tg.config2(n_cycles=20)
    spec.same_size_per_kind = True
    tr = tg.propagate(tg.generate(spec), gap_ns=2_000_000).shuffled(5)
    o = orc.Oracle(tr.topo)
    ref = o.analyze_window(tr.cols, int(tr.cols["t_exit"].max()) + 1)
    chain, per_rank = o.flag_chains(tr.cols, ref)
    c2, p2 = chains_by_definition(tr.cols, ref.flag, tr.topo.n_ranks)
    assert (chain["parent"] >= 0).sum() > 300
    for k in chain:
        assert np.array_equal(chain[k], c2[k]), k
    for k in per_rank:
        assert np.array_equal(per_rank[k], p2[k]), k
