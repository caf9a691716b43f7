"""ctypes wrapper of the CPU oracle (oracle/ccld_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  It never imports the GPU library's binding.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ccld_oracle.c")
_LIB = os.path.join(_HERE, "libccld_oracle.so")

INFLIGHT = np.iinfo(np.int64).max
NO_RANK = 0xFFFFFFFF

STATUS = {0: "OK", -1: "E_UNKNOWN_COMM", -2: "E_RANK_NOT_MEMBER", -3: "E_RANGE", -4: "E_DUPLICATE_KEY",
          -5: "E_SNAPSHOT_GAP", -6: "E_BAD_ARG"}

PARAM_NAMES = ("hang_threshold_ns", "tbase_init_ns", "tbase_rounds", "tbase_warmup_ns", "theta_num", "theta_den",
               "alpha_num", "beta_num", "ab_den", "repeat_threshold", "barrier_bytes", "kmad_num", "kmad_den",
               "lag_floor_ns", "stall_snapshots", "fifo_depth")
DEFAULT_PARAMS: Dict[str, int] = dict(
    hang_threshold_ns=300_000_000_000, tbase_init_ns=(2**63 - 1) // 4, tbase_rounds=100,
    tbase_warmup_ns=120_000_000_000, theta_num=3, theta_den=1, alpha_num=4, beta_num=6, ab_den=10,
    repeat_threshold=2, barrier_bytes=4, kmad_num=9, kmad_den=2, lag_floor_ns=300_000,
    stall_snapshots=30, fifo_depth=8)

SEG_COLS = ("comm", "seq", "n", "inflight", "state", "op", "bytes", "enter_min", "enter_med", "enter_max",
            "enter_mad", "exit_min", "exit_med", "exit_max", "exit_mad", "dur_min", "dur_max", "argmin_rank",
            "argmax_rank", "inflight_enter_min", "first")
FLAG_COLS = ("comm", "seq", "rank", "kind", "lag_enter", "lag_exit")
GROUP_COLS = ("comm", "op", "cls", "n_usable", "rstar_seq", "tmax", "tmin", "tbase", "static", "frozen", "m",
              "slow", "class", "root_s1", "root_s2", "repeats", "locate")
ALERT_COLS = ("comm", "seq", "age", "class", "n_cand", "cand_off")
BLAME_COLS = ("n_late_enter", "n_late_exit", "sum_lag_enter", "sum_lag_exit", "n_records")
REC_COLS = ("lag_enter", "lag_exit", "flag")
CHAIN_COLS = ("parent", "root", "root_rank", "depth")
CHAIN_RANK_COLS = ("root_entries", "secondary_entries", "caused")
SEG_COMPLETE, SEG_CONSISTENT, SEG_BARRIER, SEG_USABLE = 1, 2, 4, 8
FLAG_LATE_ENTER, FLAG_LATE_EXIT = 1, 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, -O2)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-o", _LIB, _SRC])
    return _LIB


class _Topo(C.Structure):
    _fields_ = [("n_ranks", C.c_uint32), ("n_comms", C.c_uint32), ("algo", C.c_void_p), ("size", C.c_void_p),
                ("member_off", C.c_void_p), ("members", C.c_void_p), ("tree_parent", C.c_void_p)]


class _WinRes(C.Structure):
    _fields_ = [("status", C.c_int32), ("n", C.c_uint64), ("n_seg", C.c_uint64), ("n_flag", C.c_uint64),
                ("n_group", C.c_uint64), ("n_alert", C.c_uint64), ("n_cand", C.c_uint64), ("n_ranks", C.c_uint64),
                ("perm", C.c_void_p), ("rec", C.c_void_p), ("seg", C.c_void_p), ("flag", C.c_void_p),
                ("group", C.c_void_p), ("alert", C.c_void_p), ("cand", C.c_void_p), ("blame", C.c_void_p),
                ("order", C.c_void_p)]


class _HangRes(C.Structure):
    _fields_ = [("status", C.c_int32), ("n_root", C.c_uint64), ("n_pair", C.c_uint64), ("n_comm", C.c_uint64),
                ("root", C.c_void_p), ("pair", C.c_void_p), ("comm", C.c_void_p)]


HANG_ROOT_COLS = ("rank", "comm", "class")
HANG_PAIR_COLS = ("rank", "comm", "stalled", "entered", "seq", "sent", "recv", "waits_on", "hops", "onset")
HANG_COMM_COLS = ("comm", "hung", "class", "seq_max", "root_by_count", "n_cand")


@dataclass
class HangResult:
    status: str
    root: Dict[str, np.ndarray]
    pair: Dict[str, np.ndarray]
    comm: Dict[str, np.ndarray]


class _RateRes(C.Structure):
    _fields_ = [("status", C.c_int32), ("n_pair", C.c_uint64), ("n_comm", C.c_uint64),
                ("pair", C.c_void_p), ("comm", C.c_void_p)]


RATE_PAIR_COLS = ("rank", "comm", "ops_send", "changes_send", "ops_recv", "changes_recv")
RATE_COMM_COLS = ("comm", "root_send", "root_recv", "root")


@dataclass
class RateResult:
    status: str
    pair: Dict[str, np.ndarray]
    comm: Dict[str, np.ndarray]


_lib: Optional[C.CDLL] = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        L.orc_state_create.restype = C.c_void_p
        L.orc_state_create.argtypes = [C.c_uint32]
        L.orc_state_destroy.argtypes = [C.c_void_p]
        L.orc_window_result_free.argtypes = [C.c_void_p]
        L.orc_analyze_window.restype = C.c_int
        L.orc_analyze_window.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64] + [C.c_void_p] * 7 + \
            [C.c_int64, C.c_void_p, C.c_void_p]
        L.orc_hang_result_free.argtypes = [C.c_void_p]
        L.orc_locate_hang.restype = C.c_int
        L.orc_locate_hang.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_uint32, C.c_uint32] + \
            [C.c_void_p] * 7 + [C.c_void_p]
        L.orc_frames_create.restype = C.c_void_p
        L.orc_frames_create.argtypes = [C.c_void_p, C.c_uint32]
        L.orc_frames_destroy.argtypes = [C.c_void_p]
        L.orc_decode_frames.restype = C.c_int
        L.orc_decode_frames.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.c_uint32] + \
            [C.c_void_p] * 7
        L.orc_flag_chains.restype = C.c_int
        L.orc_flag_chains.argtypes = [C.c_uint64] + [C.c_void_p] * 5 + [C.c_uint64, C.c_void_p, C.c_uint32,
                                                                         C.c_void_p, C.c_void_p]
        L.orc_rate_result_free.argtypes = [C.c_void_p]
        L.orc_progress_rates.restype = C.c_int
        L.orc_progress_rates.argtypes = [C.c_void_p, C.c_uint64, C.c_uint32, C.c_uint32] + [C.c_void_p] * 7 + \
            [C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _table(ptr, n, ncol) -> np.ndarray:
    if n == 0 or not ptr:
        return np.zeros((0, ncol), dtype=np.int64)
    buf = (C.c_int64 * (n * ncol)).from_address(ptr)
    return np.frombuffer(buf, dtype=np.int64).reshape(n, ncol).copy()


@dataclass
class WindowResult:
    status: str
    perm: np.ndarray                 # [n] input index of the j-th record in (comm, seq, rank) order
    rec: Dict[str, np.ndarray]       # per sorted record
    seg: Dict[str, np.ndarray]
    flag: Dict[str, np.ndarray]
    group: Dict[str, np.ndarray]
    alert: Dict[str, np.ndarray]
    cand: np.ndarray
    blame: Dict[str, np.ndarray]
    order: np.ndarray


def _cols(tab: np.ndarray, names) -> Dict[str, np.ndarray]:
    return {nm: np.ascontiguousarray(tab[:, i]) for i, nm in enumerate(names)}


class Oracle:
    """Holds the topology, the parameters and the per-group detection state
    that persists from one analysed window to the next."""

    def __init__(self, topo, params: Optional[Dict[str, int]] = None):
        self.L = lib()
        self.params = dict(DEFAULT_PARAMS)
        if params:
            self.params.update(params)
        self._p = np.asarray([self.params[k] for k in PARAM_NAMES], dtype=np.int64)
        self._algo = np.ascontiguousarray(topo.algo, dtype=np.uint8)
        self._size = np.ascontiguousarray(topo.size, dtype=np.uint32)
        self._off = np.ascontiguousarray(topo.member_off, dtype=np.uint32)
        self._members = np.ascontiguousarray(topo.members, dtype=np.uint32)
        self._tp = None if topo.tree_parent is None else np.ascontiguousarray(topo.tree_parent, dtype=np.int32)
        self._topo = _Topo(int(topo.n_ranks), int(self._size.shape[0]), _ptr(self._algo), _ptr(self._size),
                           _ptr(self._off), _ptr(self._members), _ptr(self._tp))
        self.n_ranks = int(topo.n_ranks)
        self._state = self.L.orc_state_create(int(self._size.shape[0]))
        if not self._state:
            raise MemoryError("oracle state")

    def close(self):
        if self._state:
            self.L.orc_state_destroy(self._state)
            self._state = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def analyze_window(self, cols: Dict[str, np.ndarray], now_ns: int) -> WindowResult:
        rank = np.ascontiguousarray(cols["rank"], dtype=np.uint32)
        comm = np.ascontiguousarray(cols["comm"], dtype=np.uint32)
        seq = np.ascontiguousarray(cols["seq"], dtype=np.uint64)
        op = np.ascontiguousarray(cols["op"], dtype=np.uint8)
        nbytes = np.ascontiguousarray(cols["bytes"], dtype=np.uint64)
        te = np.ascontiguousarray(cols["t_enter"], dtype=np.int64)
        tx = np.ascontiguousarray(cols["t_exit"], dtype=np.int64)
        n = int(rank.shape[0])
        res = _WinRes()
        self.L.orc_analyze_window(_ptr(self._p), C.addressof(self._topo), n, _ptr(rank), _ptr(comm), _ptr(seq),
                                  _ptr(op), _ptr(nbytes), _ptr(te), _ptr(tx), int(now_ns), self._state,
                                  C.addressof(res))
        try:
            status = STATUS[res.status]
            if res.status != 0:
                z = np.zeros((0,), np.int64)
                e = lambda names: {k: z.copy() for k in names}
                return WindowResult(status, z.astype(np.uint64), e(REC_COLS), e(SEG_COLS), e(FLAG_COLS),
                                    e(GROUP_COLS), e(ALERT_COLS), z, e(BLAME_COLS), z)
            perm = _table(res.perm, n, 1).reshape(-1).astype(np.uint64)
            out = WindowResult(
                status, perm,
                _cols(_table(res.rec, n, len(REC_COLS)), REC_COLS),
                _cols(_table(res.seg, res.n_seg, len(SEG_COLS)), SEG_COLS),
                _cols(_table(res.flag, res.n_flag, len(FLAG_COLS)), FLAG_COLS),
                _cols(_table(res.group, res.n_group, len(GROUP_COLS)), GROUP_COLS),
                _cols(_table(res.alert, res.n_alert, len(ALERT_COLS)), ALERT_COLS),
                _table(res.cand, res.n_cand, 1).reshape(-1),
                _cols(_table(res.blame, self.n_ranks, len(BLAME_COLS)), BLAME_COLS),
                _table(res.order, self.n_ranks, 1).reshape(-1))
            return out
        finally:
            self.L.orc_window_result_free(C.addressof(res))

    def flag_chains(self, cols: Dict[str, np.ndarray], res: WindowResult):
        """Root cause and secondary effects among the late-entry flags of an analysed window:
        -> ({parent, root, root_rank, depth} per flag, {root_entries, secondary_entries, caused} per rank)."""
        rank = np.ascontiguousarray(cols["rank"], dtype=np.uint32)
        comm = np.ascontiguousarray(cols["comm"], dtype=np.uint32)
        seq = np.ascontiguousarray(cols["seq"], dtype=np.uint64)
        te = np.ascontiguousarray(cols["t_enter"], dtype=np.int64)
        tx = np.ascontiguousarray(cols["t_exit"], dtype=np.int64)
        n_flag = int(res.flag["comm"].shape[0])
        flag = np.ascontiguousarray(np.stack([res.flag[k] for k in FLAG_COLS], axis=1), dtype=np.int64) \
            if n_flag else np.zeros((1, len(FLAG_COLS)), np.int64)
        chain = np.zeros((max(n_flag, 1), len(CHAIN_COLS)), np.int64)
        per_rank = np.zeros((max(self.n_ranks, 1), len(CHAIN_RANK_COLS)), np.int64)
        st = self.L.orc_flag_chains(int(rank.shape[0]), _ptr(rank), _ptr(comm), _ptr(seq), _ptr(te), _ptr(tx),
                                    n_flag, _ptr(flag), self.n_ranks, _ptr(chain), _ptr(per_rank))
        if st != 0:
            raise ValueError(STATUS[st])
        return _cols(chain[:n_flag], CHAIN_COLS), _cols(per_rank[:self.n_ranks], CHAIN_RANK_COLS)

    def locate_hang(self, cols: Dict[str, np.ndarray], n_snapshots: int, n_channels: int) -> HangResult:
        dt = {"snap": np.uint32, "rank": np.uint32, "comm": np.uint32, "channel": np.uint32,
              "seq_posted": np.uint64, "chunks_sent": np.uint32, "chunks_recv": np.uint32}
        a = {k: np.ascontiguousarray(cols[k], dtype=dt[k]) for k in dt}
        n = int(a["snap"].shape[0])
        res = _HangRes()
        self.L.orc_locate_hang(_ptr(self._p), C.addressof(self._topo), n, int(n_snapshots), int(n_channels),
                               _ptr(a["snap"]), _ptr(a["rank"]), _ptr(a["comm"]), _ptr(a["channel"]),
                               _ptr(a["seq_posted"]), _ptr(a["chunks_sent"]), _ptr(a["chunks_recv"]),
                               C.addressof(res))
        try:
            status = STATUS[res.status]
            if res.status != 0:
                z = np.zeros((0,), np.int64)
                e = lambda names: {k: z.copy() for k in names}
                return HangResult(status, e(HANG_ROOT_COLS), e(HANG_PAIR_COLS), e(HANG_COMM_COLS))
            return HangResult(status,
                              _cols(_table(res.root, res.n_root, len(HANG_ROOT_COLS)), HANG_ROOT_COLS),
                              _cols(_table(res.pair, res.n_pair, len(HANG_PAIR_COLS)), HANG_PAIR_COLS),
                              _cols(_table(res.comm, res.n_comm, len(HANG_COMM_COLS)), HANG_COMM_COLS))
        finally:
            self.L.orc_hang_result_free(C.addressof(res))

    def progress_rates(self, cols: Dict[str, np.ndarray], n_snapshots: int, n_channels: int) -> RateResult:
        """SendRate / RecvRate of every (communicator, member) from a snapshot series; the
        communicators' minimal-rate ranks stay in the state for the next analyze_window."""
        dt = {"snap": np.uint32, "rank": np.uint32, "comm": np.uint32, "channel": np.uint32,
              "seq_posted": np.uint64, "chunks_sent": np.uint32, "chunks_recv": np.uint32}
        a = {k: np.ascontiguousarray(cols[k], dtype=dt[k]) for k in dt}
        n = int(a["snap"].shape[0])
        res = _RateRes()
        self.L.orc_progress_rates(C.addressof(self._topo), n, int(n_snapshots), int(n_channels),
                                  _ptr(a["snap"]), _ptr(a["rank"]), _ptr(a["comm"]), _ptr(a["channel"]),
                                  _ptr(a["seq_posted"]), _ptr(a["chunks_sent"]), _ptr(a["chunks_recv"]),
                                  self._state, C.addressof(res))
        try:
            status = STATUS[res.status]
            if res.status != 0:
                z = np.zeros((0,), np.int64)
                e = lambda names: {k: z.copy() for k in names}
                return RateResult(status, e(RATE_PAIR_COLS), e(RATE_COMM_COLS))
            return RateResult(status,
                              _cols(_table(res.pair, res.n_pair, len(RATE_PAIR_COLS)), RATE_PAIR_COLS),
                              _cols(_table(res.comm, res.n_comm, len(RATE_COMM_COLS)), RATE_COMM_COLS))
        finally:
            self.L.orc_rate_result_free(C.addressof(res))

    # ---- Probing Frames --------------------------------------------------------------------
    def frames_begin(self, n_channels: int) -> None:
        """Forget every remembered (rank, communicator) state; frames carry `n_channels` channels."""
        self.frames_end()
        self._frames = self.L.orc_frames_create(C.addressof(self._topo), int(n_channels))
        if not self._frames:
            raise ValueError("1 .. 8 channels")
        self._frames_nch = int(n_channels)

    def frames_end(self) -> None:
        if getattr(self, "_frames", None):
            self.L.orc_frames_destroy(self._frames)
        self._frames = None

    def decode_frames(self, frames: np.ndarray, frame_rank: np.ndarray, snap: int):
        """One frame per rank -> (status, the snapshot's rows for every member slot and channel)."""
        buf = np.ascontiguousarray(frames).view(np.uint8).reshape(-1)
        fr = np.ascontiguousarray(frame_rank, dtype=np.uint32)
        n = int(self._size.sum()) * self._frames_nch
        dt = {"snap": np.uint32, "rank": np.uint32, "comm": np.uint32, "channel": np.uint32,
              "seq_posted": np.uint64, "chunks_sent": np.uint32, "chunks_recv": np.uint32}
        out = {k: np.zeros(n, dtype=v) for k, v in dt.items()}
        st = self.L.orc_decode_frames(C.addressof(self._topo), self._frames, _ptr(buf), _ptr(fr), int(fr.shape[0]),
                                      int(snap), *[_ptr(out[k]) for k in dt])
        return STATUS[st], out
