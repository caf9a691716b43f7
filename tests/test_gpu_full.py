"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times."""
import numpy as np
import pytest

from oracle import ccld_oracle as orc
from paper_2605_04478_amd import tracegen as tg
from tests.chain_check import chains_by_definition
from tests.test_gpu_window import compare

pytestmark = pytest.mark.gpu


def _run(tr, seed, placement=0):
    import torch
    from paper_2605_04478_amd import ccld
    an = ccld.Analyzer(tr.topo, max_window_records=tr.n, placement=placement)
    cols = an.to_device(tr.cols)
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    perm = torch.randperm(tr.n, device="cuda", generator=g)
    cols = {k: v[perm].contiguous() for k, v in cols.items()}
    an.ingest(cols)
    now = int(tr.cols["t_exit"].max()) + 1
    res = an.analyze_window(now, n_records=tr.n, seg_cap=tr.n // 4 + 1024, flag_cap=tr.n // 8 + 1024)
    blame, order = an.rank_blame()
    return an, res, blame, order, now


def _check_chains(an, res, tr, ref, what):
    st, chain, per_rank = an.flag_chains(res)
    assert st == "OK"
    done = tr.cols["t_exit"] != tg.INFLIGHT
    assert (tr.cols["t_exit"][done] > tr.cols["t_enter"][done]).all()
    c2, p2 = chains_by_definition(tr.cols, ref.flag, tr.topo.n_ranks)
    for k in c2:
        assert np.array_equal(chain[k], c2[k]), (what, k, np.nonzero(chain[k] != c2[k])[0][:5])
    for k in p2:
        assert np.array_equal(per_rank[k], p2[k]), (what, k)
    return chain


def test_config2_full_size():
    spec = tg.config2()
    tr = tg.generate(spec)
    assert tr.n == 5_120_000
    an, res, blame, order, now = _run(tr, 2)
    ref = orc.Oracle(tr.topo).analyze_window(tr.cols, now)
    compare(res, ref, blame, order, per_record=False, what="config2-full")
    slow = sorted(s.rank for s in spec.slow_ranks)
    link = sorted(spec.slow_groups[0].ranks)
    assert sorted(np.nonzero(blame["n_late_enter"])[0].tolist()) == slow
    assert sorted(np.nonzero(blame["n_late_exit"])[0].tolist()) == link
    assert set(order[:5].tolist()) == set(slow + link)
    an.close()


def test_config3_full_size_82m_records():
    spec = tg.config3()
    tr = tg.generate(spec)
    assert tr.n == 81_920_000 and tr.topo.n_comms == 1088
    an, res, blame, order, now = _run(tr, 3)
    assert res.status == "OK" and res.n_seg == 8_448_000 and res.path == 0
    ref = orc.Oracle(tr.topo).analyze_window(tr.cols, now)
    compare(res, ref, blame, order, per_record=False, what="config3-full")
    slow = sorted(s.rank for s in spec.slow_ranks)
    nic = sorted(x for g in spec.slow_groups for x in g.ranks)
    assert set(order[:8].tolist()) == set(slow)                     # the 8 slow ranks lead the blame
    assert set(np.nonzero(blame["n_late_exit"] >= 20)[0].tolist()) == set(nic)
    chain = _check_chains(an, res, tr, ref, "config3-full chains")
    print(f"config 3: {res.n_flag} flags, {(chain['parent'] >= 0).sum()} with a parent, depth up to {chain['depth'].max()}", flush=True)
    an.close()
    del an, res
    # the same trace by dense placement (no sort): the same tables
    an, res, blame, order, now = _run(tr, 3, placement=1)
    assert res.status == "OK" and res.path == 1
    compare(res, ref, blame, order, per_record=False, what="config3-full dense placement")
    an.close()


def test_config4_full_size_hang_locate():
    from paper_2605_04478_amd import ccld
    ht = tg.generate_hang(tg.config4())
    assert ht.n == 16_777_216
    an = ccld.Analyzer(ht.topo, max_window_records=1024, max_snapshot_rows=ht.n)
    g = an.locate_hang(an.snapshots_to_device(ht.cols), 64, 16)
    assert g.status == "OK"
    assert list(g.root["rank"]) == [ht.root_rank] and list(g.root["comm"]) == [ht.root_comm]
    assert list(g.root["class"]) == [3]
    o = orc.Oracle(ht.topo).locate_hang(ht.cols, 64, 16)
    for name in ("root", "pair", "comm"):
        gt, ot = getattr(g, name), getattr(o, name)
        for k in ot:
            assert np.array_equal(gt[k], ot[k]), (name, k)
    an.close()


def test_progress_rates_at_4096_ranks():
    from paper_2605_04478_amd import ccld
    spec = tg.RateSpec(layout=tg.Layout3D(tp=8, pp=8, dp=64, world=True), n_snapshots=64, n_channels=16, seed=2)
    tr = tg.generate_rates(spec)
    assert tr.n == 16_777_216
    an = ccld.Analyzer(tr.topo, max_window_records=1024, max_snapshot_rows=tr.n)
    g = an.progress_rates(an.snapshots_to_device(tr.cols), 64, 16)
    assert g.status == "OK"
    o = orc.Oracle(tr.topo).progress_rates(tr.cols, 64, 16)
    for name in ("pair", "comm"):
        gt, ot = getattr(g, name), getattr(o, name)
        for k in ot:
            assert np.array_equal(gt[k], ot[k]), (name, k)
    mine = np.unique(o.pair["comm"][o.pair["rank"] == tr.slow_rank])
    assert len(mine) == 4 and all(g.comm["root"][c] == tr.slow_rank for c in mine)
    an.close()


def test_large_batches_wrap_errors_and_many_ranks():
    """Batches above four million records take the placement that regroups its write-out in LDS:
    with more ranks than the LDS membership table holds, across the wrap of the circular window,
    and with a bad record."""
    from paper_2605_04478_amd import ccld
    lay = tg.Layout3D(tp=8, pp=4, dp=144)                            # 4,608 ranks
    tr = tg.generate(tg.config3(n_cycles=95, layout=lay)).shuffled(7)
    assert tr.n > (1 << 22)
    per = tr.n // 3 // lay.n_ranks * lay.n_ranks
    now = int(tr.cols["t_exit"].max()) + 1
    # one batch, all ranks
    an = ccld.Analyzer(tr.topo, max_window_records=tr.n)
    an.ingest(an.to_device(tr.cols))
    g = an.analyze_window(now, n_records=tr.n, per_record=True)
    o = orc.Oracle(tr.topo)
    ref = o.analyze_window(tr.cols, now)
    blame, order = an.rank_blame()
    compare(g, ref, blame, order, what="large-one-batch")
    # a bad record in the middle of the batch
    bad = {k: v.copy() for k, v in tr.cols.items()}
    bad["comm"][tr.n // 2] = tr.topo.n_comms
    an.reset_window()
    an.ingest(an.to_device(bad))
    g = an.analyze_window(now, n_records=tr.n)
    assert g.status == "E_UNKNOWN_COMM" == orc.Oracle(tr.topo).analyze_window(bad, now).status
    an.close()
    # two-batch window over a circular buffer that is not a multiple of the batch: the third batch wraps
    big = tg.generate(tg.config3(n_cycles=830, layout=tg.Layout3D(tp=8, pp=4, dp=48))).shuffled(8)
    nb = big.n // 3
    assert nb > (1 << 22)
    batches = [{k: v[i * nb:(i + 1) * nb] for k, v in big.cols.items()} for i in range(3)]
    an = ccld.Analyzer(big.topo, max_window_records=2 * nb + 4099, max_batch_records=nb, window_batches=2)
    o = orc.Oracle(big.topo, dict(window_batches=2))
    now = int(big.cols["t_exit"].max()) + 1
    for i, b in enumerate(batches):
        an.ingest(an.to_device(b))
        win = batches[max(0, i - 1): i + 1]
        cols = {k: np.concatenate([w[k] for w in win]) for k in b}
        g = an.analyze_window(now, n_records=2 * nb, per_record=True)
        ref = o.analyze_window(cols, now)
        blame, order = an.rank_blame()
        compare(g, ref, blame, order, what=f"large-wrap{i}")
    an.close()


def test_config5_full_size_streaming_steps():
    """16,384 ranks, one-second batches of about 2M records, window of 10 batches: the steps around the first
    full window (the full sort, then the kept order merged with each new batch, then the first eviction) and
    of the steady state beyond step 20 (a batch evicted and a batch merged every step) against the oracle on the
    concatenated window, with a hang in flight.  The oracle analyses every step as well: the repetition counters
    of Section 4.2.1 depend on which windows were looked at."""
    from paper_2605_04478_amd import ccld
    ss = tg.config5(n_steps=23, hang_step=4)
    topo = ss.layout.topology()
    per = ss.slots_per_step * ss.layout.n_ranks
    W = 10
    assert ss.layout.n_ranks == 16_384 and W * per > 19_000_000
    an = ccld.Analyzer(topo, max_window_records=W * per, max_batch_records=per, window_batches=W,
                       hang_threshold_ns=5_000_000_000)
    o = orc.Oracle(topo, dict(hang_threshold_ns=5_000_000_000))
    batches = []
    for step in range(ss.n_steps):
        b = tg.stream_batch(ss, step)
        batches.append(b.cols)
        an.ingest(an.to_device(b.cols))
        now = ss.now_ns(step)
        res = an.analyze_window(now, n_records=W * per, seg_cap=W * per // 4 + 1024, flag_cap=W * per // 8 + 1024)
        blame, order = an.rank_blame()
        assert res.status == "OK"
        batches[:max(0, step - W + 1)] = [None] * max(0, step - W + 1)      # batches that left the window
        win = batches[max(0, step - W + 1): step + 1]
        cols = {k: np.concatenate([w[k] for w in win]) for k in b.cols}
        ref = o.analyze_window(cols, now)
        compare(res, ref, blame, order, per_record=False, what=f"config5-full step{step}")
        print(f"step {step}: {res.n_records} records, {res.n_seg} collectives, {res.n_flag} flags, "
              f"{res.n_alert} alerts", flush=True)
    an.close()
