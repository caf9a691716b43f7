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
