"""ccld_locate_hang_static (the hang pass on the library's static device array, for callers that cannot
allocate) against ccld_locate_hang through the C ABI: identical tables, on two calls in a row, the second
with a smaller input; host-resident rows; the error paths; a grid beyond the array is refused."""
import numpy as np
import pytest

from paper_2605_04478_amd import tracegen as tg
from tests.helpers import ring_topology
from tests.test_oracle_hang import snap_rows

pytestmark = pytest.mark.gpu


def _same(a, b, what):
    assert a.status == b.status == "OK", (what, a.status, b.status)
    assert (a.n_root, a.n_pair, a.n_hung_comm) == (b.n_root, b.n_pair, b.n_hung_comm), what
    for name in ("root", "pair", "comm"):
        ta, tb = getattr(a, name), getattr(b, name)
        for k in tb:
            assert np.array_equal(ta[k], tb[k]), (what, name, k)


def test_static_scratch_matches_workspace_path_on_two_calls_in_a_row():
    from paper_2605_04478_amd import ccld
    big = tg.generate_hang(tg.config4(layout=tg.Layout3D(tp=8, pp=2, dp=16, world=True), seed=1, n_channels=5,
                                      n_snapshots=70))
    small = tg.generate_hang(tg.config4(layout=tg.Layout3D(tp=2, pp=2, dp=4, world=True), seed=2, n_channels=3))
    healthy = tg.generate_hang(tg.config4(layout=tg.Layout3D(tp=2, pp=2, dp=4, world=True), seed=2, n_channels=3,
                                          healthy=True))
    # contexts without snapshot capacity: only the static entry point can analyse snapshots on them
    an_big = ccld.Analyzer(big.topo, max_window_records=1024, max_snapshot_rows=0)
    an_small = ccld.Analyzer(small.topo, max_window_records=1024, max_snapshot_rows=0)
    ref_big = ccld.Analyzer(big.topo, max_window_records=1024, max_snapshot_rows=big.n)
    ref_small = ccld.Analyzer(small.topo, max_window_records=1024, max_snapshot_rows=small.n)
    with pytest.raises(ccld.CcldError) as e:
        an_big.locate_hang(an_big.snapshots_to_device(big.cols), 70, 5)
    assert e.value.name == "E_CAPACITY"
    g1 = an_big.locate_hang(an_big.snapshots_to_device(big.cols), 70, 5, static=True)
    g2 = an_small.locate_hang(an_small.snapshots_to_device(small.cols), 64, 3, static=True)     # smaller, right after
    g3 = an_small.locate_hang(healthy.cols, 64, 3, static=True)                                  # host rows, no hang
    g4 = an_big.locate_hang(an_big.snapshots_to_device(big.cols), 70, 5, static=True)           # and the large one again
    _same(g1, ref_big.locate_hang(ref_big.snapshots_to_device(big.cols), 70, 5), "big")
    _same(g2, ref_small.locate_hang(ref_small.snapshots_to_device(small.cols), 64, 3), "small")
    _same(g3, ref_small.locate_hang(healthy.cols, 64, 3), "healthy")
    _same(g4, g1, "big again")
    assert list(g1.root["rank"]) == [big.root_rank] and list(g2.root["rank"]) == [small.root_rank]
    assert g3.n_root == 0 and g3.n_hung_comm == 0
    for a in (an_big, an_small, ref_big, ref_small):
        a.close()


def test_static_scratch_error_paths_and_limit():
    from paper_2605_04478_amd import ccld
    topo = ring_topology(4, comms=[[0, 1], [2, 3]])
    cols = snap_rows(topo, 3, 2, lambda s, c, q, ch: (1, 1, 1))
    an = ccld.Analyzer(topo, max_window_records=1024, max_snapshot_rows=0)
    ref = ccld.Analyzer(topo, max_window_records=1024, max_snapshot_rows=64)
    cut = {k: v[:-1] for k, v in cols.items()}
    dup = {k: np.concatenate([v[:-1], v[:1]]) for k, v in cols.items()}
    bad = {k: v.copy() for k, v in cols.items()}
    bad["comm"][0] = 9
    for what, c in (("ok", cols), ("gap", cut), ("dup", dup), ("comm", bad)):
        a = an.locate_hang(c, 3, 2, static=True)
        b = ref.locate_hang(c, 3, 2)
        assert a.status == b.status, (what, a.status, b.status)
    assert an.locate_hang(cut, 3, 2, static=True).status == "E_SNAPSHOT_GAP"
    assert an.locate_hang(cols, 3, 2, static=True).status == "OK"          # a failed call leaves nothing behind
    # 4 member slots x 2 channels x 300,000 snapshots = 2.4M cells of 16 bytes: beyond the 32 MiB array
    with pytest.raises(ccld.CcldError) as e:
        an.locate_hang(cut, 300_000, 2, static=True)
    assert e.value.name == "E_CAPACITY"
    an.close(); ref.close()
