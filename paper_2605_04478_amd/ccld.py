"""Python binding of libccld.so (argument marshalling only).

Every step of the analysis runs in the HIP library; PyTorch is used for device
memory and the stream.  Importing this module does not load the library; the
first call does, and fails loudly if the library has not been built.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libccld.so")

T_INFLIGHT = np.iinfo(np.int64).max
NO_RANK = 0xFFFFFFFF

STATUS = {0: "OK", -1: "E_UNKNOWN_COMM", -2: "E_RANK_NOT_MEMBER", -3: "E_RANGE", -4: "E_DUPLICATE_KEY",
          -5: "E_SNAPSHOT_GAP", -6: "E_BAD_ARG", -7: "E_NULL", -8: "E_CAPACITY", -9: "E_KEY_WIDTH",
          -10: "E_BAD_TOPOLOGY", -11: "E_HIP", -12: "E_WORKSPACE", 1: "W_TRUNCATED"}

SEG_COLS = ("comm", "seq", "n", "inflight", "state", "op", "bytes", "enter_min", "enter_med", "enter_max",
            "enter_mad", "exit_min", "exit_med", "exit_max", "exit_mad", "dur_min", "dur_max", "argmin_rank",
            "argmax_rank", "inflight_enter_min", "first")
FLAG_COLS = ("comm", "seq", "rank", "kind", "lag_enter", "lag_exit")
GROUP_COLS = ("comm", "op", "cls", "n_usable", "rstar_seq", "tmax", "tmin", "tbase", "static", "frozen", "m",
              "slow", "class", "root_s1", "root_s2", "repeats", "locate")
ALERT_COLS = ("comm", "seq", "age", "class", "n_cand", "cand_off")
BLAME_COLS = ("n_late_enter", "n_late_exit", "sum_lag_enter", "sum_lag_exit", "n_records")
HANG_ROOT_COLS = ("rank", "comm", "class")
HANG_PAIR_COLS = ("rank", "comm", "stalled", "entered", "seq", "sent", "recv", "waits_on", "hops", "onset")
HANG_COMM_COLS = ("comm", "hung", "class", "seq_max", "root_by_count", "n_cand")


class Params(C.Structure):
    _fields_ = [("hang_threshold_ns", C.c_int64), ("tbase_init_ns", C.c_int64), ("tbase_rounds", C.c_uint32),
                ("repeat_threshold", C.c_uint32), ("tbase_warmup_ns", C.c_int64), ("theta_num", C.c_uint32),
                ("theta_den", C.c_uint32), ("alpha_num", C.c_uint32), ("beta_num", C.c_uint32),
                ("ab_den", C.c_uint32), ("barrier_bytes", C.c_uint32), ("kmad_num", C.c_uint32),
                ("kmad_den", C.c_uint32), ("lag_floor_ns", C.c_int64), ("stall_snapshots", C.c_uint32),
                ("fifo_depth", C.c_uint32), ("window_batches", C.c_uint32), ("placement", C.c_uint32)]


class _Topology(C.Structure):
    _fields_ = [("n_ranks", C.c_uint32), ("n_comms", C.c_uint32), ("algo", C.c_void_p), ("size", C.c_void_p),
                ("member_off", C.c_void_p), ("members", C.c_void_p), ("tree_parent", C.c_void_p)]


class _Records(C.Structure):
    _fields_ = [("rank", C.c_void_p), ("comm", C.c_void_p), ("seq", C.c_void_p), ("op", C.c_void_p),
                ("bytes", C.c_void_p), ("t_enter", C.c_void_p), ("t_exit", C.c_void_p), ("on_device", C.c_int32)]


class _Snapshots(C.Structure):
    _fields_ = [("snap", C.c_void_p), ("rank", C.c_void_p), ("comm", C.c_void_p), ("channel", C.c_void_p),
                ("seq_posted", C.c_void_p), ("chunks_sent", C.c_void_p), ("chunks_recv", C.c_void_p),
                ("on_device", C.c_int32), ("n_snapshots", C.c_uint32), ("n_channels", C.c_uint32)]


class _WindowResult(C.Structure):
    _fields_ = [("seg_cap", C.c_uint64), ("flag_cap", C.c_uint64), ("group_cap", C.c_uint64),
                ("alert_cap", C.c_uint64), ("cand_cap", C.c_uint64),
                ("seg", C.c_void_p), ("flag", C.c_void_p), ("group", C.c_void_p), ("alert", C.c_void_p),
                ("cand", C.c_void_p), ("lag_enter", C.c_void_p), ("lag_exit", C.c_void_p),
                ("rec_flag", C.c_void_p), ("perm", C.c_void_p),
                ("n_records", C.c_uint64), ("n_seg", C.c_uint64), ("n_flag", C.c_uint64), ("n_group", C.c_uint64),
                ("n_alert", C.c_uint64), ("n_cand", C.c_uint64), ("status", C.c_int32), ("path", C.c_int32)]


class _ChainResult(C.Structure):
    _fields_ = [("chain_cap", C.c_uint64), ("chain", C.c_void_p), ("per_rank", C.c_void_p), ("n_chain", C.c_uint64),
                ("status", C.c_int32), ("reserved", C.c_int32)]


CHAIN_COLS = ("parent", "root", "root_rank", "depth")
CHAIN_RANK_COLS = ("root_entries", "secondary_entries", "caused")


class _HangResult(C.Structure):
    _fields_ = [("root_cap", C.c_uint64), ("pair_cap", C.c_uint64), ("comm_cap", C.c_uint64),
                ("root", C.c_void_p), ("pair", C.c_void_p), ("comm", C.c_void_p),
                ("n_root", C.c_uint64), ("n_pair", C.c_uint64), ("n_hung_comm", C.c_uint64),
                ("status", C.c_int32), ("reserved", C.c_int32)]


class _Frames(C.Structure):
    _fields_ = [("frames", C.c_void_p), ("frame_rank", C.c_void_p), ("n_frames", C.c_uint64), ("on_device", C.c_int32),
                ("n_channels", C.c_uint32), ("snapshot", C.c_uint32), ("reserved", C.c_uint32)]


class _SnapshotRows(C.Structure):
    _fields_ = [("snap", C.c_void_p), ("rank", C.c_void_p), ("comm", C.c_void_p), ("channel", C.c_void_p),
                ("seq_posted", C.c_void_p), ("chunks_sent", C.c_void_p), ("chunks_recv", C.c_void_p),
                ("capacity", C.c_uint64)]


class _RateResult(C.Structure):
    _fields_ = [("pair_cap", C.c_uint64), ("comm_cap", C.c_uint64), ("pair", C.c_void_p), ("comm", C.c_void_p),
                ("n_pair", C.c_uint64), ("n_comm", C.c_uint64), ("status", C.c_int32), ("reserved", C.c_int32)]


_lib: Optional[C.CDLL] = None

PROF_CLASSES = ("ingest", "sort_hist", "sort_scan", "sort_scatter", "segments", "flags", "blame", "groups", "alerts",
                "hang", "seg_heads", "dense_partition", "hang_place", "frames")
PLACEMENT_SORT, PLACEMENT_DENSE = 0, 1
PROF_NCLASS = 16

EXPORTS = ("ccld_profile_enable", "ccld_profile_read", "ccld_default_params", "ccld_query_workspace", "ccld_create", "ccld_destroy", "ccld_ingest",
           "ccld_reset_window", "ccld_analyze_window", "ccld_flag_chains", "ccld_rank_blame", "ccld_locate_hang",
           "ccld_locate_hang_static",
           "ccld_progress_rates",
           "ccld_decode_frames", "ccld_reset_frames", "ccld_status_str")


def lib() -> C.CDLL:
    """Load libccld.so; there is no fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2605_04478_amd.build` "
                               "(there is no CPU fallback)")
        L = C.CDLL(LIB_PATH)
        vp, u64 = C.c_void_p, C.c_uint64
        L.ccld_default_params.argtypes = [vp]
        L.ccld_query_workspace.argtypes = [vp, vp, u64, u64, u64, vp]
        L.ccld_create.argtypes = [vp, vp, u64, u64, u64, vp, u64, vp, vp]
        L.ccld_destroy.argtypes = [vp]
        L.ccld_ingest.argtypes = [vp, vp, u64]
        L.ccld_reset_window.argtypes = [vp]
        L.ccld_analyze_window.argtypes = [vp, C.c_int64, vp]
        L.ccld_rank_blame.argtypes = [vp, vp, vp]
        L.ccld_flag_chains.argtypes = [vp, vp, vp]
        L.ccld_locate_hang.argtypes = [vp, vp, u64, vp]
        L.ccld_locate_hang_static.argtypes = [vp, vp, u64, vp]
        L.ccld_progress_rates.argtypes = [vp, vp, u64, vp]
        L.ccld_decode_frames.argtypes = [vp, vp, vp, vp]
        L.ccld_reset_frames.argtypes = [vp]
        L.ccld_profile_enable.argtypes = [vp, C.c_int32]
        L.ccld_profile_read.argtypes = [vp, vp, vp, vp]
        L.ccld_status_str.argtypes = [C.c_int32]
        L.ccld_status_str.restype = C.c_char_p
        for name in EXPORTS:
            if hasattr(L, name) and name != "ccld_status_str":
                getattr(L, name).restype = C.c_int32
        _lib = L
    return _lib


class CcldError(RuntimeError):
    def __init__(self, status: int, where: str):
        super().__init__(f"{where}: {STATUS.get(status, status)}")
        self.status = status
        self.name = STATUS.get(status, str(status))


def default_params(**overrides) -> Params:
    p = Params()
    lib().ccld_default_params(C.addressof(p))
    for k, v in overrides.items():
        if not hasattr(p, k):
            raise KeyError(k)
        setattr(p, k, int(v))
    return p


def _table(t, ncol_names, cap, n) -> Dict[str, np.ndarray]:
    n = min(int(n), int(cap))
    m = t.view(len(ncol_names), cap)[:, :n].cpu().numpy()
    return {nm: np.ascontiguousarray(m[i]) for i, nm in enumerate(ncol_names)}


@dataclass
class WindowResult:
    status: str
    n_records: int
    n_seg: int
    n_flag: int
    n_group: int
    n_alert: int
    n_cand: int
    caps: Dict[str, int]
    dev: Dict[str, "object"] = field(repr=False, default_factory=dict)   # device tensors
    path: int = 0                    # 0: the window was sorted, 1: dense placement
    raw: "object" = field(repr=False, default=None)                     # the C result structure of the call

    @property
    def seg(self): return _table(self.dev["seg"], SEG_COLS, self.caps["seg"], self.n_seg)
    @property
    def flag(self): return _table(self.dev["flag"], FLAG_COLS, self.caps["flag"], self.n_flag)
    @property
    def group(self): return _table(self.dev["group"], GROUP_COLS, self.caps["group"], self.n_group)
    @property
    def alert(self): return _table(self.dev["alert"], ALERT_COLS, self.caps["alert"], self.n_alert)
    @property
    def cand(self): return self.dev["cand"][:min(self.n_cand, self.caps["cand"])].cpu().numpy()

    def per_record(self) -> Dict[str, np.ndarray]:
        out = {}
        for k in ("lag_enter", "lag_exit", "rec_flag", "perm"):
            if k in self.dev:
                out[k] = self.dev[k][:self.n_records].cpu().numpy()
        return out


@dataclass
class HangResult:
    status: str
    n_root: int
    n_pair: int
    n_hung_comm: int
    caps: Dict[str, int]
    dev: Dict[str, "object"] = field(repr=False, default_factory=dict)

    @property
    def root(self): return _table(self.dev["root"], HANG_ROOT_COLS, self.caps["root"], self.n_root)
    @property
    def pair(self): return _table(self.dev["pair"], HANG_PAIR_COLS, self.caps["pair"], self.n_pair)
    @property
    def comm(self): return _table(self.dev["comm"], HANG_COMM_COLS, self.caps["comm"], self.caps["comm"])


RATE_PAIR_COLS = ("rank", "comm", "ops_send", "changes_send", "ops_recv", "changes_recv")
RATE_COMM_COLS = ("comm", "root_send", "root_recv", "root")


@dataclass
class RateResult:
    status: str
    n_pair: int
    n_comm: int
    caps: Dict[str, int]
    dev: Dict[str, "object"] = field(repr=False, default_factory=dict)

    @property
    def pair(self): return _table(self.dev["pair"], RATE_PAIR_COLS, self.caps["pair"], min(self.n_pair, self.caps["pair"]))
    @property
    def comm(self): return _table(self.dev["comm"], RATE_COMM_COLS, self.caps["comm"], min(self.n_comm, self.caps["comm"]))


class Analyzer:
    """One analyzer context on one GPU."""

    def __init__(self, topo, params: Optional[Params] = None, max_window_records: int = 1 << 20,
                 max_batch_records: Optional[int] = None, max_snapshot_rows: int = 0, device: str = "cuda:0",
                 **param_overrides):
        import torch
        self.torch = torch
        self.L = lib()
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the analyzer has no CPU path")
        self.device = torch.device(device)
        self.params = params if params is not None else default_params(**param_overrides)
        self.max_window_records = int(max_window_records)
        self.max_batch_records = int(max_batch_records if max_batch_records is not None else max_window_records)
        self.max_snapshot_rows = int(max_snapshot_rows)
        self._algo = np.ascontiguousarray(topo.algo, dtype=np.uint8)
        self._size = np.ascontiguousarray(topo.size, dtype=np.uint32)
        self._off = np.ascontiguousarray(topo.member_off, dtype=np.uint32)
        self._members = np.ascontiguousarray(topo.members, dtype=np.uint32)
        self._tp = None if topo.tree_parent is None else np.ascontiguousarray(topo.tree_parent, dtype=np.int32)
        p = lambda a: None if a is None else a.ctypes.data_as(C.c_void_p)
        self._topo = _Topology(int(topo.n_ranks), int(self._size.shape[0]), p(self._algo), p(self._size),
                               p(self._off), p(self._members), p(self._tp))
        self.n_ranks = int(topo.n_ranks)
        self.n_comms = int(self._size.shape[0])
        need = C.c_uint64(0)
        self._check(self.L.ccld_query_workspace(C.addressof(self.params), C.addressof(self._topo),
                                                self.max_window_records, self.max_batch_records,
                                                self.max_snapshot_rows, C.addressof(need)), "ccld_query_workspace")
        self.workspace_bytes = int(need.value)
        with torch.cuda.device(self.device):
            self.workspace = torch.empty(self.workspace_bytes + 256, dtype=torch.uint8, device=self.device)
            base = self.workspace.data_ptr()
            self._ws_ptr = (base + 255) & ~255
            self.stream = torch.cuda.current_stream(self.device)
            ctx = C.c_void_p(0)
            self._check(self.L.ccld_create(C.addressof(self.params), C.addressof(self._topo),
                                           self.max_window_records, self.max_batch_records, self.max_snapshot_rows,
                                           self._ws_ptr, self.workspace_bytes, self.stream.cuda_stream,
                                           C.addressof(ctx)), "ccld_create")
        self._ctx = ctx

    def _check(self, status: int, where: str, allow=(0, 1)):
        if status not in allow:
            raise CcldError(status, where)
        return status

    def close(self):
        if getattr(self, "_ctx", None):
            self.L.ccld_destroy(self._ctx)
            self._ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- ingest -------------------------------------------------------------------------
    def to_device(self, cols: Dict[str, np.ndarray]) -> Dict[str, "object"]:
        """numpy record columns -> device tensors (bit patterns preserved)."""
        t = self.torch
        sign = {"rank": np.int32, "comm": np.int32, "seq": np.int64, "op": np.uint8, "bytes": np.int64,
                "t_enter": np.int64, "t_exit": np.int64}
        return {k: t.from_numpy(np.ascontiguousarray(cols[k]).view(sign[k])).to(self.device) for k in sign}

    def ingest(self, cols) -> None:
        """cols: dict of the seven columns, either device tensors or numpy arrays (host)."""
        first = cols["rank"]
        on_device = not isinstance(first, np.ndarray)
        n = int(first.shape[0])
        if on_device:
            ptr = lambda k: C.c_void_p(cols[k].data_ptr())
            keep = cols
        else:
            dt = {"rank": np.uint32, "comm": np.uint32, "seq": np.uint64, "op": np.uint8, "bytes": np.uint64,
                  "t_enter": np.int64, "t_exit": np.int64}
            keep = {k: np.ascontiguousarray(cols[k], dtype=dt[k]) for k in dt}
            ptr = lambda k: keep[k].ctypes.data_as(C.c_void_p)
        rec = _Records(ptr("rank"), ptr("comm"), ptr("seq"), ptr("op"), ptr("bytes"), ptr("t_enter"),
                       ptr("t_exit"), 1 if on_device else 0)
        self._check(self.L.ccld_ingest(self._ctx, C.addressof(rec), n), "ccld_ingest")
        self._last_batch = keep     # device inputs must outlive the asynchronous ingest

    def reset_window(self) -> None:
        self._check(self.L.ccld_reset_window(self._ctx), "ccld_reset_window")

    # ---- analysis -----------------------------------------------------------------------
    def alloc_window_result(self, n_records: int, seg_cap: Optional[int] = None, flag_cap: Optional[int] = None,
                            group_cap: Optional[int] = None, alert_cap: int = 4096, cand_cap: int = 65536,
                            per_record: bool = False):
        t = self.torch
        n = max(int(n_records), 1)
        caps = {"seg": int(seg_cap or n), "flag": int(flag_cap or n),
                "group": int(group_cap or min(n, self.n_comms * 1024)), "alert": int(alert_cap),
                "cand": int(cand_cap)}
        i64 = dict(dtype=t.int64, device=self.device)
        dev = {"seg": t.empty(len(SEG_COLS) * caps["seg"], **i64),
               "flag": t.empty(len(FLAG_COLS) * caps["flag"], **i64),
               "group": t.empty(len(GROUP_COLS) * caps["group"], **i64),
               "alert": t.empty(len(ALERT_COLS) * caps["alert"], **i64),
               "cand": t.empty(caps["cand"], **i64)}
        if per_record:
            dev["lag_enter"] = t.empty(n, **i64)
            dev["lag_exit"] = t.empty(n, **i64)
            dev["rec_flag"] = t.empty(n, dtype=t.uint8, device=self.device)
            dev["perm"] = t.empty(n, dtype=t.int32, device=self.device)
        return caps, dev

    def analyze_window(self, now_ns: int, buffers=None, **alloc_kw) -> WindowResult:
        if buffers is None:
            buffers = self.alloc_window_result(alloc_kw.pop("n_records", self.max_window_records), **alloc_kw)
        caps, dev = buffers
        g = lambda k: C.c_void_p(dev[k].data_ptr()) if k in dev else None
        r = _WindowResult(caps["seg"], caps["flag"], caps["group"], caps["alert"], caps["cand"],
                          g("seg"), g("flag"), g("group"), g("alert"), g("cand"), g("lag_enter"), g("lag_exit"),
                          g("rec_flag"), g("perm"))
        st = self.L.ccld_analyze_window(self._ctx, int(now_ns), C.addressof(r))
        if st in (-7, -11, -6):
            raise CcldError(st, "ccld_analyze_window")
        return WindowResult(STATUS.get(st, str(st)), r.n_records, r.n_seg, r.n_flag, r.n_group, r.n_alert,
                            r.n_cand, caps, dev, int(r.path), r)

    def flag_chains(self, result: WindowResult):
        """Root cause and secondary effects among the late entries of the analysis `result` (which must be
        the context's most recent one): -> (status, {parent, root, root_rank, depth} per flag,
        {root_entries, secondary_entries, caused} per rank)."""
        t = self.torch
        cap = max(int(result.n_flag), 1)
        chain = t.empty(len(CHAIN_COLS) * cap, dtype=t.int64, device=self.device)
        per_rank = t.empty(len(CHAIN_RANK_COLS) * self.n_ranks, dtype=t.int64, device=self.device)
        o = _ChainResult(cap, chain.data_ptr(), per_rank.data_ptr())
        st = self.L.ccld_flag_chains(self._ctx, C.addressof(result.raw), C.addressof(o))
        if st not in (0, 1):
            raise CcldError(st, "ccld_flag_chains")
        n = int(o.n_chain)
        return (STATUS.get(st, str(st)), _table(chain, CHAIN_COLS, cap, n),
                _table(per_rank, CHAIN_RANK_COLS, self.n_ranks, self.n_ranks))

    def rank_blame(self, to_host: bool = True, buffers=None):
        """-> (blame columns, order).  to_host=False leaves both on the device (column-major int64 table
        [len(BLAME_COLS)][n_ranks], int32 order), written into `buffers` = (blame, order) when given."""
        t = self.torch
        if buffers is not None:
            blame, order = buffers
        else:
            blame = t.empty(len(BLAME_COLS) * self.n_ranks, dtype=t.int64, device=self.device)
            order = t.empty(self.n_ranks, dtype=t.int32, device=self.device)
        self._check(self.L.ccld_rank_blame(self._ctx, blame.data_ptr(), order.data_ptr()), "ccld_rank_blame")
        if not to_host:
            return blame.view(len(BLAME_COLS), self.n_ranks), order
        b = blame.view(len(BLAME_COLS), self.n_ranks).cpu().numpy()
        return ({nm: np.ascontiguousarray(b[i]) for i, nm in enumerate(BLAME_COLS)},
                order.cpu().numpy().astype(np.int64))

    # ---- kernel timing ------------------------------------------------------------------
    def profile_enable(self, on: bool = True, only: Optional[str] = None) -> None:
        """Times every kernel class, or (only=<class name>) that one class: each event record costs a few
        microseconds on the stream."""
        mode = 0 if not on else (1 if only is None else 2 + PROF_CLASSES.index(only))
        self._check(self.L.ccld_profile_enable(self._ctx, mode), "ccld_profile_enable")

    def profile_read(self):
        """-> ({class: (milliseconds, launches)}, passes of the last main sort)"""
        ms = (C.c_double * PROF_NCLASS)()
        cnt = (C.c_uint64 * PROF_NCLASS)()
        passes = C.c_uint64(0)
        self._check(self.L.ccld_profile_read(self._ctx, C.addressof(ms), C.addressof(cnt), C.addressof(passes)),
                    "ccld_profile_read")
        return {nm: (ms[i], int(cnt[i])) for i, nm in enumerate(PROF_CLASSES)}, int(passes.value)

    # ---- hang location ----------------------------------------------------------------------
    def snapshots_to_device(self, cols: Dict[str, np.ndarray]) -> Dict[str, "object"]:
        t = self.torch
        sign = {"snap": np.int32, "rank": np.int32, "comm": np.int32, "channel": np.int32, "seq_posted": np.int64,
                "chunks_sent": np.int32, "chunks_recv": np.int32}
        return {k: t.from_numpy(np.ascontiguousarray(cols[k]).view(sign[k])).to(self.device) for k in sign}

    def locate_hang(self, cols, n_snapshots: int, n_channels: int, root_cap: int = 4096,
                    pair_cap: Optional[int] = None, comm_cap: Optional[int] = None, static: bool = False,
                    buffers=None) -> HangResult:
        """static=True calls ccld_locate_hang_static (the pass works in the library's static device array
        instead of the context's workspace); buffers = (caps, dev) reuses result tables."""
        t = self.torch
        first = cols["snap"]
        on_device = not isinstance(first, np.ndarray)
        n = int(first.shape[0])
        if on_device:
            ptr = lambda k: C.c_void_p(cols[k].data_ptr())
        else:
            dt = {"snap": np.uint32, "rank": np.uint32, "comm": np.uint32, "channel": np.uint32,
                  "seq_posted": np.uint64, "chunks_sent": np.uint32, "chunks_recv": np.uint32}
            keep = {k: np.ascontiguousarray(cols[k], dtype=dt[k]) for k in dt}
            ptr = lambda k: keep[k].ctypes.data_as(C.c_void_p)
        sn = _Snapshots(ptr("snap"), ptr("rank"), ptr("comm"), ptr("channel"), ptr("seq_posted"),
                        ptr("chunks_sent"), ptr("chunks_recv"), 1 if on_device else 0, int(n_snapshots),
                        int(n_channels))
        if buffers is not None:
            caps, dev = buffers
        else:
            caps = {"root": int(root_cap), "pair": int(pair_cap or int(self._size.sum())),
                    "comm": int(comm_cap or self.n_comms)}
            i64 = dict(dtype=t.int64, device=self.device)
            dev = {"root": t.empty(len(HANG_ROOT_COLS) * caps["root"], **i64),
                   "pair": t.empty(len(HANG_PAIR_COLS) * caps["pair"], **i64),
                   "comm": t.empty(len(HANG_COMM_COLS) * caps["comm"], **i64)}
        r = _HangResult(caps["root"], caps["pair"], caps["comm"], dev["root"].data_ptr(), dev["pair"].data_ptr(),
                        dev["comm"].data_ptr())
        fn = self.L.ccld_locate_hang_static if static else self.L.ccld_locate_hang
        st = fn(self._ctx, C.addressof(sn), n, C.addressof(r))
        if st in (-7, -11, -6, -8):
            raise CcldError(st, "ccld_locate_hang_static" if static else "ccld_locate_hang")
        return HangResult(STATUS.get(st, str(st)), r.n_root, r.n_pair, r.n_hung_comm, caps, dev)

    def reset_frames(self) -> None:
        self._check(self.L.ccld_reset_frames(self._ctx), "ccld_reset_frames")

    def decode_frames(self, frames, frame_rank, snapshot: int, n_channels: int):
        """One Probing Frame per rank (numpy array of 1184-byte frames on the host, or a device uint8
        tensor) -> (status, the snapshot's rows as device tensors in the snapshot column format)."""
        t = self.torch
        on_device = not isinstance(frames, np.ndarray)
        if on_device:
            n = int(frame_rank.shape[0])
            fptr, rptr = C.c_void_p(frames.data_ptr()), C.c_void_p(frame_rank.data_ptr())
            keep = (frames, frame_rank)
        else:
            buf = np.ascontiguousarray(frames).view(np.uint8).reshape(-1)
            fr = np.ascontiguousarray(frame_rank, dtype=np.uint32)
            n = int(fr.shape[0])
            fptr, rptr = buf.ctypes.data_as(C.c_void_p), fr.ctypes.data_as(C.c_void_p)
            keep = (buf, fr)
        cap = int(self._size.sum()) * int(n_channels)
        i32 = dict(dtype=t.int32, device=self.device)
        out = {k: t.empty(cap, **i32) for k in ("snap", "rank", "comm", "channel", "chunks_sent", "chunks_recv")}
        out["seq_posted"] = t.empty(cap, dtype=t.int64, device=self.device)
        f = _Frames(fptr, rptr, n, 1 if on_device else 0, int(n_channels), int(snapshot), 0)
        r = _SnapshotRows(*[out[k].data_ptr() for k in ("snap", "rank", "comm", "channel", "seq_posted",
                                                        "chunks_sent", "chunks_recv")], cap)
        n_rows = C.c_uint64(0)
        st = self.L.ccld_decode_frames(self._ctx, C.addressof(f), C.addressof(r), C.addressof(n_rows))
        if st in (-7, -11, -6, -8):
            raise CcldError(st, "ccld_decode_frames")
        del keep
        return STATUS.get(st, str(st)), out

    def progress_rates(self, cols, n_snapshots: int, n_channels: int, pair_cap: Optional[int] = None,
                       comm_cap: Optional[int] = None) -> RateResult:
        """SendRate / RecvRate tables from a snapshot series (host numpy columns or device tensors)."""
        t = self.torch
        first = cols["snap"]
        on_device = not isinstance(first, np.ndarray)
        n = int(first.shape[0])
        if on_device:
            ptr = lambda k: C.c_void_p(cols[k].data_ptr())
        else:
            dt = {"snap": np.uint32, "rank": np.uint32, "comm": np.uint32, "channel": np.uint32,
                  "seq_posted": np.uint64, "chunks_sent": np.uint32, "chunks_recv": np.uint32}
            keep = {k: np.ascontiguousarray(cols[k], dtype=dt[k]) for k in dt}
            ptr = lambda k: keep[k].ctypes.data_as(C.c_void_p)
        sn = _Snapshots(ptr("snap"), ptr("rank"), ptr("comm"), ptr("channel"), ptr("seq_posted"),
                        ptr("chunks_sent"), ptr("chunks_recv"), 1 if on_device else 0, int(n_snapshots),
                        int(n_channels))
        caps = {"pair": int(pair_cap or int(self._size.sum())), "comm": int(comm_cap or self.n_comms)}
        i64 = dict(dtype=t.int64, device=self.device)
        dev = {"pair": t.empty(len(RATE_PAIR_COLS) * caps["pair"], **i64),
               "comm": t.empty(len(RATE_COMM_COLS) * caps["comm"], **i64)}
        r = _RateResult(caps["pair"], caps["comm"], dev["pair"].data_ptr(), dev["comm"].data_ptr())
        st = self.L.ccld_progress_rates(self._ctx, C.addressof(sn), n, C.addressof(r))
        if st in (-7, -11, -6, -8):
            raise CcldError(st, "ccld_progress_rates")
        return RateResult(STATUS.get(st, str(st)), r.n_pair, r.n_comm, caps, dev)
