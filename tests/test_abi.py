"""The C-ABI library loads and exports every entry point the header declares
(no compute calls: this runs without a GPU)."""
import ctypes
import os
import re

from paper_2605_04478_amd import ccld

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "ccld.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ccld_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    if not os.path.exists(ccld.LIB_PATH):
        from paper_2605_04478_amd import build
        build.build_lib()
    L = ctypes.CDLL(ccld.LIB_PATH)
    names = _declared()
    assert "ccld_analyze_window" in names and "ccld_ingest" in names and "ccld_rank_blame" in names
    for n in names:
        assert hasattr(L, n), n
    assert set(ccld.EXPORTS) == set(names)


def test_host_only_calls():
    L = ccld.lib()
    for name in ccld.EXPORTS:                       # every entry point is called with declared argument types
        assert getattr(L, name).argtypes is not None, name
    p = ccld.default_params()
    assert p.tbase_rounds == 100 and p.theta_num == 3 and p.alpha_num == 4 and p.beta_num == 6
    assert p.hang_threshold_ns == 300 * 10**9 and p.barrier_bytes == 4
    assert L.ccld_status_str(-4) == b"E_DUPLICATE_KEY"
    # argument errors are reported without touching a GPU
    need = ctypes.c_uint64(0)
    assert L.ccld_query_workspace(None, None, 10, 10, 0, ctypes.addressof(need)) == -7
    bad = ccld.default_params(tbase_rounds=0)
    assert L.ccld_query_workspace(ctypes.addressof(bad), None, 10, 10, 0, ctypes.addressof(need)) == -6


def test_workspace_sizes_of_the_benchmark_configuration():
    """ccld_query_workspace is host arithmetic: the 82M-record window of the 4,096-rank layout needs about 10 GiB
    with the default placement (window 40 B, sort buffers 36 B and per-record scratch 57 B per record; host batches
    are staged inside that scratch) and about 13 GiB with the dense placement's partition buffers."""
    import numpy as np
    from paper_2605_04478_amd import tracegen as tg
    L = ccld.lib()
    topo = tg.Layout3D(tp=8, pp=8, dp=64).topology()
    keep = [np.ascontiguousarray(topo.algo, dtype=np.uint8), np.ascontiguousarray(topo.size, dtype=np.uint32),
            np.ascontiguousarray(topo.member_off, dtype=np.uint32), np.ascontiguousarray(topo.members, dtype=np.uint32)]
    p = lambda a: a.ctypes.data_as(ctypes.c_void_p)
    t = ccld._Topology(int(topo.n_ranks), int(keep[1].shape[0]), p(keep[0]), p(keep[1]), p(keep[2]), p(keep[3]), None)
    n = 81_920_000
    sizes = {}
    for placement in (ccld.PLACEMENT_SORT, ccld.PLACEMENT_DENSE):
        prm = ccld.default_params(placement=placement)
        need = ctypes.c_uint64(0)
        assert L.ccld_query_workspace(ctypes.addressof(prm), ctypes.addressof(t), n, n, 0, ctypes.addressof(need)) == 0
        sizes[placement] = need.value / 2**30
    assert 9.5 < sizes[ccld.PLACEMENT_SORT] < 10.5, sizes
    assert 12.5 < sizes[ccld.PLACEMENT_DENSE] < 13.5, sizes
    # a small batch capacity does not shrink the scratch, a large one does not grow it beyond the analysis' own need
    need2 = ctypes.c_uint64(0)
    prm = ccld.default_params()
    assert L.ccld_query_workspace(ctypes.addressof(prm), ctypes.addressof(t), n, n // 10, 0, ctypes.addressof(need2)) == 0
    assert abs(need2.value / 2**30 - sizes[ccld.PLACEMENT_SORT]) < 0.2
