"""GPU: error reporting and bookkeeping of the C-ABI entry points (no kernel is asked to misbehave:
every case is rejected by a host-side check)."""
import ctypes

import numpy as np
import pytest

from paper_2605_04478_amd import tracegen as tg
from tests.helpers import T0, ring_topology, rounds_with_durations, toy_cols

pytestmark = pytest.mark.gpu


def test_capacity_blame_order_and_profile_calls():
    from paper_2605_04478_amd import ccld
    topo = ring_topology(4)
    cols = toy_cols(rounds_with_durations([[100, 200, 300, 400]] * 8))        # 32 records
    an = ccld.Analyzer(topo, max_window_records=40, max_batch_records=40, window_batches=4)
    with pytest.raises(ccld.CcldError) as e:                                   # no analysis yet: no blame
        an.rank_blame()
    assert e.value.status == -6
    an.ingest(an.to_device(cols))
    with pytest.raises(ccld.CcldError) as e:                                   # 32 + 32 > 40
        an.ingest(an.to_device(cols))
    assert e.value.status == -8
    big = toy_cols(rounds_with_durations([[100, 200, 300, 400]] * 11))        # 44 > batch capacity
    with pytest.raises(ccld.CcldError) as e:
        an.ingest(an.to_device(big))
    assert e.value.status == -8
    an.profile_enable(True)
    g = an.analyze_window(T0 + 10**12)
    assert g.status == "OK" and g.n_records == 32 and g.n_seg == 8            # the rejected batches left no trace
    prof, passes = an.profile_read()
    assert passes >= 1 and prof["segments"][1] >= 1 and prof["segments"][0] > 0
    blame, order = an.rank_blame()
    assert list(blame["n_records"]) == [8, 8, 8, 8] and sorted(order) == [0, 1, 2, 3]
    # one class only: the others record no event
    an.profile_enable(True, only="segments")
    g2 = an.analyze_window(T0 + 10**12)
    prof, _ = an.profile_read()
    assert g2.status == "OK" and prof["segments"][1] >= 1
    assert all(v[1] == 0 for k, v in prof.items() if k != "segments")
    an.profile_enable(False)
    dev_blame, dev_order = an.rank_blame(to_host=False)
    assert dev_blame.shape == (5, 4) and int(dev_blame[4].sum()) == 32 and sorted(dev_order.tolist()) == [0, 1, 2, 3]
    an.reset_window()
    g = an.analyze_window(T0 + 10**12)
    assert g.status == "OK" and g.n_records == 0 and g.n_seg == 0
    an.close()


def test_create_rejects_bad_arguments():
    from paper_2605_04478_amd import ccld
    L = ccld.lib()
    topo = ring_topology(4)
    with pytest.raises(ccld.CcldError):
        ccld.Analyzer(topo, max_window_records=16, tbase_rounds=0)
    # a member list that names a rank twice
    bad = tg.make_topology(4, [[0, 1, 1, 2]])
    with pytest.raises(ccld.CcldError) as e:
        ccld.Analyzer(bad, max_window_records=16)
    assert e.value.status == -10
    assert L.ccld_ingest(None, None, 0) == -7
    assert L.ccld_analyze_window(None, 0, None) == -7
    assert L.ccld_progress_rates(None, None, 0, None) == -7


def test_blame_of_the_last_analysis_survives_a_hang_location():
    """ccld_rank_blame returns the table and the order of the most recent analysis, also when a hang
    location (which borrows the sort buffers and the scratch of the selections) ran in between; an
    analysis of an empty window then leaves an all-zero table and the ranks in ascending order."""
    from oracle import ccld_oracle as orc
    from paper_2605_04478_amd import ccld
    lay = tg.Layout3D(tp=2, pp=2, dp=4, world=True)
    ht = tg.generate_hang(tg.config4(layout=lay, n_channels=3))
    topo = ht.topo
    R = lay.n_ranks
    rng = np.random.default_rng(3)
    rows = []
    for s in range(300):                          # world communicator (the last one): rank 5 enters late every time
        c = topo.n_comms - 1
        for r in range(R):
            te = T0 + s * 1_000_000 + int(rng.integers(0, 1_000)) + (400_000 if r == 5 else 0)
            rows.append((r, c, s, 0, 1 << 20, te, te + 50_000))
    cols = toy_cols(rows)
    an = ccld.Analyzer(topo, max_window_records=len(rows), max_snapshot_rows=ht.n)
    an.ingest(an.to_device(cols))
    g = an.analyze_window(T0 + 10**12)
    ref = orc.Oracle(topo).analyze_window(cols, T0 + 10**12)
    assert g.status == ref.status == "OK" and int(ref.blame["n_late_enter"][5]) == 300
    h = an.locate_hang(an.snapshots_to_device(ht.cols), ht.spec.n_snapshots, ht.spec.n_channels)
    assert h.status == "OK"
    blame, order = an.rank_blame()
    for k in ref.blame:
        assert np.array_equal(blame[k], ref.blame[k]), k
    assert np.array_equal(order, ref.order) and int(order[0]) == 5
    an.reset_window()
    g = an.analyze_window(T0 + 10**12)
    blame, order = an.rank_blame()
    assert g.n_records == 0 and all(int(v.sum()) == 0 for v in blame.values())
    assert list(order) == list(range(R))
    an.close()
