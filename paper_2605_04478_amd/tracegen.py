"""Seeded synthetic inputs: a simulated training cluster that emits per-rank
collective-communication trace records and progress-counter snapshots.

This module only *produces inputs* (and the list of faults it injected).  It
holds none of the analyzer's arithmetic and is the one piece of code that both
the GPU library's tests and the CPU oracle's tests are allowed to share.

Record schema (one row per rank per collective, SoA numpy arrays):
    rank u32, comm u32, seq u64, op u8, bytes u64, t_enter i64 ns, t_exit i64 ns
A collective that has not completed on a rank carries t_exit == INFLIGHT.

All random numbers come from a counter-based generator (a 64-bit mixing hash of
(seed, stream, a, b)), so any slice of a trace can be generated independently
and in parallel, and the same (spec, seed) always yields the same arrays.
Floating point appears only here; every emitted time is an int64 nanosecond.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

INFLIGHT = np.iinfo(np.int64).max
NO_RANK = 0xFFFFFFFF

OP_ALLREDUCE = 0
OP_ALLGATHER = 1
OP_REDUCESCATTER = 2
OP_ALLTOALL = 3
OP_SENDRECV = 4
OP_BROADCAST = 5

ALGO_RING = 0
ALGO_TREE = 1

T_EPOCH_NS = 1_700_000_000 * 1_000_000_000  # traces start at a wall-clock-like origin

_U = np.uint64
_GOLD = _U(0x9E3779B97F4A7C15)
_M1 = _U(0xBF58476D1CE4E5B9)
_M2 = _U(0x94D049BB133111EB)


# --------------------------------------------------------------------------
# counter-based random numbers
# --------------------------------------------------------------------------
def _mix(x: np.ndarray) -> np.ndarray:
    x = (x ^ (x >> _U(30))) * _M1
    x = (x ^ (x >> _U(27))) * _M2
    return x ^ (x >> _U(31))


def rand_u64(seed: int, stream: int, a, b=0) -> np.ndarray:
    """64 random bits for every element of broadcast(a, b)."""
    with np.errstate(over="ignore"):
        a = np.asarray(a).astype(np.uint64, copy=False)
        b = np.asarray(b).astype(np.uint64, copy=False)
        s = _mix(np.asarray([(seed * 0x632BE59BD9B4E019 + stream * 0x9E3779B97F4A7C15 + 1) & (2**64 - 1)],
                            dtype=np.uint64))[0]
        h = _mix((a + s) * _GOLD + _U(0x2545F4914F6CDD1D))
        h = _mix(h ^ ((b + _U(1)) * _M1))
    return h


def rand_unit(seed, stream, a, b=0) -> np.ndarray:
    """Uniform doubles in [0, 1)."""
    return (rand_u64(seed, stream, a, b) >> _U(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


def rand_normal(seed, stream, a, b=0) -> np.ndarray:
    u1 = rand_unit(seed, stream, a, b)
    u2 = rand_unit(seed, stream + 7919, a, b)
    return np.sqrt(-2.0 * np.log1p(-u1)) * np.cos(2.0 * np.pi * u2)


# --------------------------------------------------------------------------
# topology
# --------------------------------------------------------------------------
@dataclass
class Topology:
    """Communicator table: CSR member lists in ring order (successor = next,
    cyclic) or, for tree communicators, in BFS order with a parent slot per
    member (-1 for the root)."""
    n_ranks: int
    algo: np.ndarray          # u8  [n_comms]
    size: np.ndarray          # u32 [n_comms]
    member_off: np.ndarray    # u32 [n_comms]
    members: np.ndarray       # u32 [sum size]
    tree_parent: Optional[np.ndarray] = None   # i32 [sum size], member-slot index within the comm
    names: List[str] = field(default_factory=list)

    @property
    def n_comms(self) -> int:
        return int(self.size.shape[0])

    def members_of(self, c: int) -> np.ndarray:
        o = int(self.member_off[c])
        return self.members[o:o + int(self.size[c])]


def make_topology(n_ranks: int, comms: Sequence[Sequence[int]], algo: Optional[Sequence[int]] = None,
                  tree_parent: Optional[Sequence[Optional[Sequence[int]]]] = None,
                  names: Optional[List[str]] = None) -> Topology:
    size = np.asarray([len(c) for c in comms], dtype=np.uint32)
    off = np.zeros(len(comms), dtype=np.uint32)
    if len(comms) > 1:
        off[1:] = np.cumsum(size[:-1], dtype=np.uint64).astype(np.uint32)
    members = (np.concatenate([np.asarray(c, dtype=np.uint32) for c in comms])
               if len(comms) else np.zeros(0, np.uint32))
    al = np.zeros(len(comms), dtype=np.uint8) if algo is None else np.asarray(algo, dtype=np.uint8)
    tp = None
    if tree_parent is not None:
        tp = np.full(members.shape[0], -1, dtype=np.int32)
        for c, par in enumerate(tree_parent):
            if par is not None:
                tp[int(off[c]):int(off[c]) + int(size[c])] = np.asarray(par, dtype=np.int32)
    return Topology(n_ranks, al, size, off, members, tp, names or [])


@dataclass
class Layout3D:
    """rank = pp*(DP*TP) + dp*TP + tp; a TP group is 8 consecutive ranks (one
    node).  Communicator ids: all TP groups, then all PP groups, then all DP
    groups, then (optionally) one world communicator."""
    tp: int
    pp: int
    dp: int
    world: bool = False

    @property
    def n_ranks(self) -> int:
        return self.tp * self.pp * self.dp

    @property
    def n_tp(self) -> int:
        return self.pp * self.dp

    @property
    def n_pp(self) -> int:
        return self.dp * self.tp

    @property
    def n_dp(self) -> int:
        return self.pp * self.tp

    def coords(self, rank):
        rank = np.asarray(rank)
        return rank // (self.dp * self.tp), (rank // self.tp) % self.dp, rank % self.tp

    def comm_of(self, kind: str, rank) -> np.ndarray:
        p, d, t = self.coords(rank)
        if kind == "tp":
            return p * self.dp + d
        if kind == "pp":
            return self.n_tp + d * self.tp + t
        if kind == "dp":
            return self.n_tp + self.n_pp + p * self.tp + t
        if kind == "world":
            return np.zeros_like(np.asarray(rank)) + (self.n_tp + self.n_pp + self.n_dp)
        raise ValueError(kind)

    def topology(self) -> Topology:
        r = np.arange(self.n_ranks).reshape(self.pp, self.dp, self.tp)
        comms: List[np.ndarray] = []
        names: List[str] = []
        for p in range(self.pp):
            for d in range(self.dp):
                comms.append(r[p, d, :]); names.append("tp")
        for d in range(self.dp):
            for t in range(self.tp):
                comms.append(r[:, d, t]); names.append("pp")
        for p in range(self.pp):
            for t in range(self.tp):
                comms.append(r[p, :, t]); names.append("dp")
        if self.world:
            comms.append(r.reshape(-1)); names.append("world")
        return make_topology(self.n_ranks, comms, names=names)


# --------------------------------------------------------------------------
# trace specification
# --------------------------------------------------------------------------
CYCLE_3D: Tuple[Tuple[str, int], ...] = (
    ("tp", OP_ALLREDUCE), ("tp", OP_ALLREDUCE), ("tp", OP_ALLREDUCE), ("pp", OP_SENDRECV),
    ("tp", OP_ALLREDUCE), ("tp", OP_ALLREDUCE), ("tp", OP_ALLREDUCE), ("pp", OP_SENDRECV),
    ("dp", OP_ALLGATHER), ("dp", OP_ALLREDUCE),
)
CYCLE_WORLD: Tuple[Tuple[str, int], ...] = (("world", OP_ALLREDUCE),)


@dataclass
class SlowRank:
    rank: int
    prob: float                      # probability that an op of this rank is delayed
    dist: Tuple                      # ("const", ns) | ("uniform", lo_ns, hi_ns) | ("exp", mean_ns)


@dataclass
class SlowGroup:
    ranks: Tuple[int, ...]           # ranks whose transfers are stretched
    factor: float                    # multiplier on the transfer time of those ranks
    kind: str                        # communicator kind the fault applies to ("pp", "dp", ...)
    comm: Optional[int] = None       # restrict to one communicator id (slow link); None = all of that kind


@dataclass
class TraceSpec:
    layout: Layout3D
    cycle: Tuple[Tuple[str, int], ...]
    n_slots: int                     # collectives per rank
    bytes_dist: Tuple                # ("pow2", lo_exp, hi_exp) | ("loguniform", lo_exp, hi_exp)
    sigma: float = 0.1               # lognormal jitter of the transfer time, one draw per collective
    skew_ns: int = 50_000            # per-rank clock offset, uniform in [-skew, +skew]
    slot_ns: int = 100_000_000       # spacing of successive collectives on a rank
    bandwidth_b_per_ns: float = 20.0
    enter_jitter_ns: int = 20_000
    exit_jitter_ns: int = 5_000
    slow_ranks: List[SlowRank] = field(default_factory=list)
    slow_groups: List[SlowGroup] = field(default_factory=list)
    same_size_per_kind: bool = False  # one size and jitter draw per (communicator kind, counter): every TP / PP / DP
                                     # group runs the same operation at the same step, as one SPMD program does
    seed: int = 0
    name: str = "trace"

    @property
    def n_records(self) -> int:
        return self.n_slots * self.layout.n_ranks


# streams of the counter-based generator
_S_BYTES, _S_JIT, _S_ENTER, _S_EXIT, _S_SKEW, _S_INJP, _S_INJV, _S_PICK = 11, 12, 13, 14, 15, 16, 17, 18


def _slot_seq_tables(cycle) -> Tuple[np.ndarray, Dict[str, int]]:
    """Ordinal of each cycle position among the positions of its kind, and the
    number of positions of each kind per cycle."""
    cnt: Dict[str, int] = {}
    ordinal = np.zeros(len(cycle), dtype=np.int64)
    for i, (kind, _) in enumerate(cycle):
        ordinal[i] = cnt.get(kind, 0)
        cnt[kind] = cnt.get(kind, 0) + 1
    return ordinal, cnt


def _delay(dist: Tuple, u: np.ndarray) -> np.ndarray:
    if dist[0] == "const":
        return np.full(u.shape, float(dist[1]))
    if dist[0] == "uniform":
        return dist[1] + (dist[2] - dist[1]) * u
    if dist[0] == "exp":
        return -float(dist[1]) * np.log1p(-u)
    raise ValueError(dist)


def _gen_slots(spec: TraceSpec, k0: int, k1: int, out: Dict[str, np.ndarray]) -> None:
    """Fill rows [k0*n_ranks, k1*n_ranks) of the output columns (slot-major)."""
    L = spec.layout
    R = L.n_ranks
    cyc = spec.cycle
    ordinal, per_cycle = _slot_seq_tables(cyc)
    ranks = np.arange(R, dtype=np.int64)
    skew = np.rint((rand_unit(spec.seed, _S_SKEW, ranks) * 2.0 - 1.0) * spec.skew_ns).astype(np.int64)
    view = {k: v.reshape(-1, R) for k, v in out.items()}
    ks_all = np.arange(k0, k1, dtype=np.int64)
    for kind in sorted(per_cycle):
        pos = [i for i, (kd, _) in enumerate(cyc) if kd == kind]
        sel = np.isin(ks_all % len(cyc), pos)
        ks = ks_all[sel]
        if ks.size == 0:
            continue
        m = ks.size
        comm_r = L.comm_of(kind, ranks).astype(np.int64)              # [R]
        seq_k = (ks // len(cyc)) * per_cycle[kind] + ordinal[ks % len(cyc)]   # [m]
        op_k = np.asarray([cyc[int(i)][1] for i in (ks % len(cyc))], dtype=np.uint8)
        # one draw per collective (comm, seq): message size and transfer jitter
        ucomm, inv = np.unique(comm_r, return_inverse=True)
        draw_id = np.full_like(ucomm, 1_000_003 + sorted(per_cycle).index(kind)) if spec.same_size_per_kind else ucomm
        ub = rand_unit(spec.seed, _S_BYTES, draw_id[None, :], seq_k[:, None])
        if spec.bytes_dist[0] == "pow2":
            lo, hi = spec.bytes_dist[1], spec.bytes_dist[2]
            nbytes_c = np.left_shift(np.int64(1), (lo + np.floor(ub * (hi - lo + 1))).astype(np.int64))
        else:
            lo, hi = spec.bytes_dist[1], spec.bytes_dist[2]
            nbytes_c = np.floor(np.exp2(lo + (hi - lo) * ub)).astype(np.int64)
        jit_c = np.exp(spec.sigma * rand_normal(spec.seed, _S_JIT, draw_id[None, :], seq_k[:, None]))
        nbytes = nbytes_c[:, inv]                                    # [m, R]
        jit = jit_c[:, inv]
        # per-record draws
        inject = np.zeros((m, R), dtype=np.float64)
        for sr in spec.slow_ranks:
            hit = rand_unit(spec.seed, _S_INJP, np.int64(sr.rank), ks) < sr.prob
            val = _delay(sr.dist, rand_unit(spec.seed, _S_INJV, np.int64(sr.rank), ks))
            inject[:, sr.rank] += np.where(hit, np.maximum(np.rint(val), 1.0), 0.0)
        enter = (ks[:, None] * spec.slot_ns
                 + np.floor(rand_unit(spec.seed, _S_ENTER, ranks[None, :], ks[:, None]) * spec.enter_jitter_ns)
                 + inject)
        e4 = enter.reshape(m, L.pp, L.dp, L.tp)
        if kind == "tp":
            start = np.broadcast_to(e4.max(axis=3, keepdims=True), e4.shape)
        elif kind == "pp":
            start = np.broadcast_to(e4.max(axis=1, keepdims=True), e4.shape)
        elif kind == "dp":
            start = np.broadcast_to(e4.max(axis=2, keepdims=True), e4.shape)
        else:
            start = np.broadcast_to(e4.max(axis=(1, 2, 3), keepdims=True), e4.shape)
        start = start.reshape(m, R)
        factor = np.ones(R, dtype=np.float64)
        fac2d = None
        for sg in spec.slow_groups:
            if sg.kind != kind:
                continue
            if sg.comm is None:
                factor[list(sg.ranks)] *= sg.factor
            else:
                if fac2d is None:
                    fac2d = np.ones((1, R), dtype=np.float64)
                on = np.zeros(R, dtype=bool)
                on[list(sg.ranks)] = True
                fac2d = fac2d * np.where(on & (comm_r == sg.comm), sg.factor, 1.0)[None, :]
        f = factor[None, :] if fac2d is None else factor[None, :] * fac2d
        dur = np.rint(nbytes.astype(np.float64) / spec.bandwidth_b_per_ns * jit * f)
        exit_ = (start + dur
                 + np.floor(rand_unit(spec.seed, _S_EXIT, ranks[None, :], ks[:, None]) * spec.exit_jitter_ns))
        r0 = ks - k0          # row of each slot inside this chunk's [slots, R] view
        view["rank"][r0, :] = ranks.astype(np.uint32)[None, :]
        view["comm"][r0, :] = comm_r.astype(np.uint32)[None, :]
        view["seq"][r0, :] = seq_k.astype(np.uint64)[:, None]
        view["op"][r0, :] = op_k[:, None]
        view["bytes"][r0, :] = nbytes.astype(np.uint64)
        view["t_enter"][r0, :] = T_EPOCH_NS + enter.astype(np.int64) + skew[None, :]
        view["t_exit"][r0, :] = T_EPOCH_NS + exit_.astype(np.int64) + skew[None, :]
        view["inj_delay"][r0, :] = inject.astype(np.int64)
        view["stretched"][r0, :] = np.broadcast_to(f != 1.0, (m, R))


COLUMNS = ("rank", "comm", "seq", "op", "bytes", "t_enter", "t_exit")
_DTYPES = {"rank": np.uint32, "comm": np.uint32, "seq": np.uint64, "op": np.uint8, "bytes": np.uint64,
           "t_enter": np.int64, "t_exit": np.int64, "inj_delay": np.int64, "stretched": np.bool_}


@dataclass
class Trace:
    spec: TraceSpec
    topo: Topology
    cols: Dict[str, np.ndarray]          # the seven record columns
    inj_delay: np.ndarray                # ns added to this record's entry (0 = none)   [ground truth]
    stretched: np.ndarray                # this record's transfer was stretched          [ground truth]

    @property
    def n(self) -> int:
        return int(self.cols["rank"].shape[0])

    def take(self, index: np.ndarray) -> "Trace":
        return Trace(self.spec, self.topo, {k: v[index] for k, v in self.cols.items()},
                     self.inj_delay[index], self.stretched[index])

    def shuffled(self, seed: int) -> "Trace":
        perm = np.random.Generator(np.random.PCG64(seed)).permutation(self.n)
        return self.take(perm)


def generate(spec: TraceSpec, chunk_slots: int = 0, workers: int = 0) -> Trace:
    R = spec.layout.n_ranks
    n = spec.n_records
    out = {k: np.empty(n, dtype=_DTYPES[k]) for k in _DTYPES}
    if chunk_slots <= 0:
        chunk_slots = max(1, (1 << 20) // R)
    if workers <= 0:
        workers = min(16, os.cpu_count() or 1)
    chunks = [(k, min(k + chunk_slots, spec.n_slots)) for k in range(0, spec.n_slots, chunk_slots)]

    def work(c):
        sub = {k: v[c[0] * R:c[1] * R] for k, v in out.items()}
        _gen_slots(spec, c[0], c[1], sub)

    if workers == 1 or len(chunks) == 1:
        for c in chunks:
            work(c)
    else:
        with ThreadPoolExecutor(max_workers=workers) as ex:
            list(ex.map(work, chunks))
    cols = {k: out[k] for k in COLUMNS}
    return Trace(spec, spec.layout.topology(), cols, out["inj_delay"], out["stretched"])


def propagate(tr: Trace, gap_ns: int) -> Trace:
    """Replays a slot-major trace (as `generate` returns it, not shuffled) as a dependent schedule.

    In the generated trace every collective starts at its slot's fixed time, so a late rank never
    disturbs anybody's later operations.  Here a rank enters its next collective `gap_ns` (its
    compute time) after leaving the previous one, plus the record's own entry jitter and injected
    delay; a collective starts when its last member has entered and every member leaves after the
    record's own transfer time.  A delay therefore travels: the peers of a late rank leave late,
    carry the delay into their next collectives on other communicators, and so on until the whole
    job has absorbed it.  Sizes, jitter draws, injected delays and clock skews are those of the
    input trace; only the two time columns change."""
    spec = tr.spec
    L = spec.layout
    R = L.n_ranks
    cyc = spec.cycle
    ranks = np.arange(R, dtype=np.int64)
    skew = np.rint((rand_unit(spec.seed, _S_SKEW, ranks) * 2.0 - 1.0) * spec.skew_ns).astype(np.int64)
    if not np.array_equal(tr.cols["rank"][:R], ranks.astype(np.uint32)):
        raise ValueError("propagate() needs the slot-major order of generate()")
    te = tr.cols["t_enter"].reshape(-1, R) - T_EPOCH_NS - skew[None, :]
    tx = tr.cols["t_exit"].reshape(-1, R) - T_EPOCH_NS - skew[None, :]
    n_slots = te.shape[0]

    def group_max(v, kind):
        v4 = v.reshape(L.pp, L.dp, L.tp)
        axis = {"tp": 2, "pp": 0, "dp": 1}.get(kind)
        m = v4.max(axis=axis, keepdims=True) if axis is not None else v4.max(keepdims=True)
        return np.broadcast_to(m, v4.shape).reshape(R)

    new_e = np.empty_like(te)
    new_x = np.empty_like(tx)
    ready = np.zeros(R, dtype=np.int64)
    for k in range(n_slots):
        kind = cyc[k % len(cyc)][0]
        own = te[k] - k * spec.slot_ns                      # entry jitter + injected delay of the record
        tail = tx[k] - group_max(te[k], kind)               # transfer time + exit jitter of the record
        ent = ready + gap_ns + own
        ext = group_max(ent, kind) + tail
        new_e[k] = ent
        new_x[k] = ext
        ready = ext
    cols = dict(tr.cols)
    cols["t_enter"] = (new_e + skew[None, :] + T_EPOCH_NS).reshape(-1)
    cols["t_exit"] = (new_x + skew[None, :] + T_EPOCH_NS).reshape(-1)
    return Trace(spec, tr.topo, cols, tr.inj_delay, tr.stretched)


# --------------------------------------------------------------------------
# the benchmark configurations
# --------------------------------------------------------------------------
def _pick_distinct(seed: int, stream: int, n_pick: int, n_total: int, exclude=()) -> List[int]:
    order = np.argsort(rand_u64(seed, stream, np.arange(n_total)), kind="stable")
    ex = set(int(x) for x in exclude)
    outl: List[int] = []
    for r in order:
        if int(r) not in ex:
            outl.append(int(r))
            if len(outl) == n_pick:
                break
    return outl


def config1(n_slots: int = 1000, seed: int = 0, faults: bool = True) -> TraceSpec:
    """16 ranks, one world ring, all-reduce only; rank 5 enters 2 ms late on 5 % of its ops."""
    lay = Layout3D(tp=16, pp=1, dp=1, world=False)
    # a single communicator: use the TP communicator of the 16x1x1 layout as the world ring
    return TraceSpec(layout=lay, cycle=(("tp", OP_ALLREDUCE),), n_slots=n_slots, bytes_dist=("pow2", 20, 28),
                     sigma=0.1, skew_ns=50_000, slot_ns=100_000_000,
                     slow_ranks=[SlowRank(5, 0.05, ("const", 2_000_000))] if faults else [],
                     seed=seed, name="config1")


def config2(n_cycles: int = 1000, seed: int = 0, faults: bool = True) -> TraceSpec:
    """512 ranks = TP8 x PP4 x DP16; 3 slow ranks and one slow pipeline link."""
    lay = Layout3D(tp=8, pp=4, dp=16)
    slow, groups = [], []
    if faults:
        for r in _pick_distinct(seed, _S_PICK, 3, lay.n_ranks):
            slow.append(SlowRank(r, 0.10, ("uniform", 500_000, 5_000_000)))
        # one PP communicator, one adjacent stage pair
        ex = [s.rank for s in slow]
        a = _pick_distinct(seed, _S_PICK + 1, 1, lay.n_ranks - lay.dp * lay.tp, exclude=ex)[0]
        b = a + lay.dp * lay.tp
        groups.append(SlowGroup((a, b), 1.5, "pp", comm=int(lay.comm_of("pp", a))))
    return TraceSpec(layout=lay, cycle=CYCLE_3D, n_slots=10 * n_cycles, bytes_dist=("pow2", 20, 28),
                     sigma=0.1, skew_ns=50_000, slot_ns=100_000_000, slow_ranks=slow, slow_groups=groups,
                     seed=seed, name="config2")


def config3(n_cycles: int = 2000, seed: int = 0, faults: bool = True,
            layout: Optional[Layout3D] = None) -> TraceSpec:
    """4,096 ranks = TP8 x PP8 x DP64; 8 slow ranks (every op, Exp(1 ms)) and two
    nodes whose DP transfers run 1.3x slower."""
    lay = layout or Layout3D(tp=8, pp=8, dp=64)
    slow, groups = [], []
    if faults:
        n_nodes = lay.n_ranks // lay.tp
        nodes = _pick_distinct(seed, _S_PICK + 2, min(2, n_nodes), n_nodes)
        node_ranks = [r for nd in nodes for r in range(nd * lay.tp, (nd + 1) * lay.tp)]
        for r in _pick_distinct(seed, _S_PICK, min(8, lay.n_ranks // 4), lay.n_ranks, exclude=node_ranks):
            slow.append(SlowRank(r, 1.0, ("exp", 1_000_000)))
        for nd in nodes:
            groups.append(SlowGroup(tuple(range(nd * lay.tp, (nd + 1) * lay.tp)), 1.3, "dp"))
    return TraceSpec(layout=lay, cycle=CYCLE_3D, n_slots=10 * n_cycles, bytes_dist=("loguniform", 16.0, 29.0),
                     sigma=0.2, skew_ns=100_000, slot_ns=250_000_000, slow_ranks=slow, slow_groups=groups,
                     seed=seed, name="config3")


# --------------------------------------------------------------------------
# progress-counter snapshots (hang location)
# --------------------------------------------------------------------------
SNAP_COLUMNS = ("snap", "rank", "comm", "channel", "seq_posted", "chunks_sent", "chunks_recv")
_S_HROOT, _S_HC0, _S_HTOT = 31, 32, 33
_S_RSLOW, _S_RPHASE, _S_RK = 41, 42, 43        # _S_RK and _S_RK + 1: send / receive


def ring_steady_state(n: int, frozen: int, c0: np.ndarray, total: int, depth: int):
    """Chunk counters of an n-rank ring in which member slot `frozen` stopped after sending and
    receiving c0 chunks (one value per channel) and everybody else ran until blocked.

    The ring is simulated step by step: a rank may send chunk S when it has received the chunks
    before it (S <= R) and its successor has fewer than `depth` unconsumed chunks (S - R_succ <
    depth); it may receive when its predecessor has sent more than it has received (R < S_pred)
    and it is not already ahead of its own sends (R <= S).  Returns (S, R), each [n, channels]."""
    c0 = np.asarray(c0, dtype=np.int64)
    S = np.zeros((n, c0.shape[0]), dtype=np.int64)
    R = np.zeros_like(S)
    S[frozen] = c0
    R[frozen] = c0
    live = np.ones(n, dtype=bool)
    live[frozen] = False
    for _ in range(4 * (int(c0.max()) + n * (depth + 2)) + 16):
        pred_S = np.roll(S, 1, axis=0)
        succ_R = np.roll(R, -1, axis=0)
        can_recv = (R < pred_S) & (R <= S) & (R < total) & live[:, None]
        R = R + can_recv
        can_send = (S <= R) & (S - succ_R < depth) & (S < total) & live[:, None]
        S2 = S + can_send
        if not can_recv.any() and not can_send.any():
            break
        S = S2
    return S, R


@dataclass
class HangSpec:
    layout: Layout3D
    n_snapshots: int = 64
    n_channels: int = 16
    hang_snapshot: int = 20            # first snapshot that shows the frozen state (None = healthy run)
    hang_seq: int = 12_345
    fifo_depth: int = 8
    seed: int = 0


@dataclass
class HangTrace:
    spec: HangSpec
    topo: Topology
    cols: Dict[str, np.ndarray]
    root_rank: int                     # ground truth (or -1 for a healthy run)
    root_comm: int

    @property
    def n(self) -> int:
        return int(self.cols["snap"].shape[0])


def generate_hang(spec: HangSpec, shuffle: bool = True) -> HangTrace:
    """Snapshots of every (rank, communicator, channel) at 1 s intervals.

    Healthy snapshots show completed operations: every member of a communicator reports the same
    operation counter and S = R = the operation's chunk count per channel, and the counter advances
    from snapshot to snapshot.  From `hang_snapshot` on, one seeded rank of one DP ring is frozen
    in the middle of operation `hang_seq`; the ring's other members run until blocked
    (ring_steady_state); the ring's members post nothing further on their other communicators;
    every other rank posts one more operation on each communicator it shares with a ring member
    (the world communicator included), sends its first chunk and blocks; communicators without a
    ring member stay idle after their last completed operation."""
    L = spec.layout
    topo = L.topology()
    R = L.n_ranks
    nch, nsn = spec.n_channels, spec.n_snapshots
    kinds = ["tp", "pp", "dp"] + (["world"] if L.world else [])
    ranks = np.arange(R, dtype=np.int64)
    seed = spec.seed
    hang = spec.hang_snapshot is not None
    root_rank = root_comm = -1
    ring = np.zeros(0, dtype=np.int64)
    if hang:
        root_rank = int(rand_u64(seed, _S_HROOT, 0) % np.uint64(R))
        root_comm = int(L.comm_of("dp", root_rank))
        ring = topo.members_of(root_comm).astype(np.int64)
    in_ring = np.zeros(R, dtype=bool)
    in_ring[ring] = True
    out = {k: [] for k in SNAP_COLUMNS}
    ch = np.arange(nch, dtype=np.int64)
    Sx = Rx = None
    if hang:
        c0 = 100 + (rand_u64(seed, _S_HC0, ch) % np.uint64(900)).astype(np.int64)
        slot = int(np.nonzero(ring == root_rank)[0][0])
        Sx, Rx = ring_steady_state(len(ring), slot, c0, 1 << 20, spec.fifo_depth)
    for kind in kinds:
        comm_r = L.comm_of(kind, ranks).astype(np.int64)                      # [R]
        # chunks per channel of a completed operation (same for all members) and the counter's pace
        pace = 1 + (rand_u64(seed, _S_HTOT, comm_r, 7) % np.uint64(5)).astype(np.int64)
        base = spec.hang_seq - pace * (spec.hang_snapshot if hang else 0) if kind == "dp" else \
            1000 + (rand_u64(seed, _S_HTOT, comm_r, 8) % np.uint64(9000)).astype(np.int64)
        base = np.broadcast_to(base, (R,)).astype(np.int64)
        touched = np.zeros(R, dtype=bool)          # communicator has a member of the frozen ring
        if hang:
            has = np.zeros(topo.n_comms + 1, dtype=bool)
            has[np.unique(comm_r[ring])] = True
            touched = has[comm_r]
        for s in range(nsn):
            frozen_now = hang and s >= spec.hang_snapshot
            s_eff = min(s, spec.hang_snapshot - 1) if frozen_now else s
            seq = base + pace * s_eff                                           # [R] last completed op
            tot = 64 + (rand_u64(seed, _S_HTOT, comm_r[:, None] * 131071 + seq[:, None], ch[None, :])
                        % np.uint64(1984)).astype(np.int64)                     # [R, ch]
            sent = tot.copy()
            recv = tot.copy()
            seqp = np.broadcast_to(seq[:, None], (R, nch)).copy()
            if frozen_now:
                if kind == "dp":
                    # the frozen ring: mid-operation hang_seq
                    sent[ring] = Sx
                    recv[ring] = Rx
                    seqp[ring] = spec.hang_seq
                else:
                    # everybody outside the ring posted the next operation where a ring member is awaited
                    blocked = touched & ~in_ring
                    seqp[blocked] = seq[blocked, None] + 1
                    sent[blocked] = 1
                    recv[blocked] = 0
            n_rows = R * nch
            out["snap"].append(np.full(n_rows, s, dtype=np.uint32))
            out["rank"].append(np.repeat(ranks, nch).astype(np.uint32))
            out["comm"].append(np.repeat(comm_r, nch).astype(np.uint32))
            out["channel"].append(np.tile(ch, R).astype(np.uint32))
            out["seq_posted"].append(seqp.reshape(-1).astype(np.uint64))
            out["chunks_sent"].append(sent.reshape(-1).astype(np.uint32))
            out["chunks_recv"].append(recv.reshape(-1).astype(np.uint32))
    cols = {k: np.concatenate(v) for k, v in out.items()}
    if shuffle:
        perm = np.random.Generator(np.random.PCG64(seed + 17)).permutation(cols["snap"].shape[0])
        cols = {k: v[perm] for k, v in cols.items()}
    return HangTrace(spec, topo, cols, root_rank, root_comm)


def generate_slots(spec: TraceSpec, k0: int, k1: int) -> Trace:
    """The records of collectives k0 .. k1-1 of every rank (one slice of the trace)."""
    R = spec.layout.n_ranks
    k1 = min(k1, spec.n_slots)
    n = max(k1 - k0, 0) * R
    out = {k: np.empty(n, dtype=_DTYPES[k]) for k in _DTYPES}
    if n:
        _gen_slots(spec, k0, k1, out)
    return Trace(spec, spec.layout.topology(), {k: out[k] for k in COLUMNS}, out["inj_delay"], out["stretched"])


@dataclass
class StreamSpec:
    """A trace delivered in one-second batches, with a slow rank that changes every
    `epoch_steps` batches and (optionally) one rank that stops entering one DP communicator."""
    layout: Layout3D
    n_steps: int = 600
    slots_per_step: int = 122                 # 1 s / 8.192 ms
    slot_ns: int = 8_192_000
    epoch_steps: int = 30
    hang_step: Optional[int] = 300
    seed: int = 0

    def base(self) -> TraceSpec:
        return TraceSpec(layout=self.layout, cycle=CYCLE_3D, n_slots=self.n_steps * self.slots_per_step,
                         bytes_dist=("loguniform", 16.0, 25.0), sigma=0.2, skew_ns=100_000, slot_ns=self.slot_ns,
                         seed=self.seed, name="config5")

    def slow_rank(self, step: int) -> int:
        return int(rand_u64(self.seed, _S_PICK + 5, step // self.epoch_steps) % np.uint64(self.layout.n_ranks))

    def hang_site(self) -> Tuple[int, int, int]:
        """(rank that stops entering, its DP communicator, first operation counter it misses)"""
        r = int(rand_u64(self.seed, _S_PICK + 6, 0) % np.uint64(self.layout.n_ranks))
        comm = int(self.layout.comm_of("dp", r))
        first_slot = self.hang_step * self.slots_per_step
        cyc = len(CYCLE_3D)
        k = first_slot
        while CYCLE_3D[k % cyc][0] != "dp":
            k += 1
        seq = (k // cyc) * 2 + (0 if k % cyc == 8 else 1)
        return r, comm, seq

    def now_ns(self, step: int) -> int:
        return T_EPOCH_NS + (step + 1) * self.slots_per_step * self.slot_ns


def stream_batch(ss: StreamSpec, step: int) -> Trace:
    """Batch `step`: the collectives that start in second `step`.  From the hang on, the hung
    communicator shows its peers in flight on the missed operation and nothing after it; every
    other communicator carries on."""
    spec = ss.base()
    spec.slow_ranks = [SlowRank(ss.slow_rank(step), 1.0, ("exp", 1_000_000))]
    tr = generate_slots(spec, step * ss.slots_per_step, (step + 1) * ss.slots_per_step)
    if ss.hang_step is not None and step >= ss.hang_step:
        r, comm, seq = ss.hang_site()
        c = tr.cols
        on = c["comm"] == comm
        keep = ~(on & ((c["seq"] > seq) | ((c["seq"] == seq) & (c["rank"] == r))))
        c["t_exit"][on & (c["seq"] == seq)] = INFLIGHT
        tr = tr.take(np.nonzero(keep)[0])
    return tr


def config5(n_steps: int = 600, seed: int = 0, layout: Optional[Layout3D] = None, **kw) -> StreamSpec:
    """16,384 ranks = TP8 x PP16 x DP128, about 2M records per one-second batch."""
    return StreamSpec(layout=layout or Layout3D(tp=8, pp=16, dp=128), n_steps=n_steps, seed=seed, **kw)


def config4(seed: int = 0, layout: Optional[Layout3D] = None, healthy: bool = False, **kw) -> HangSpec:
    """4,096 ranks, {TP, PP, DP, world} x 16 channels x 64 snapshots (about 17M rows); one rank of
    one DP ring stops at operation 12,345 from snapshot 20 on."""
    lay = layout or Layout3D(tp=8, pp=8, dp=64, world=True)
    return HangSpec(layout=lay, hang_snapshot=None if healthy else kw.pop("hang_snapshot", 20), seed=seed, **kw)


# --------------------------------------------------------------------------
# progress-rate series: SendCount / RecvCount sampled while operations run
# --------------------------------------------------------------------------
@dataclass
class RateSpec:
    layout: Layout3D
    n_snapshots: int = 64              # samples of every (rank, communicator, channel)
    n_channels: int = 4
    chunks: int = 8                    # chunks one operation moves per channel
    op_samples: int = 10               # samples from one operation's start to the next one's
    normal_changes: Tuple[int, int] = (1, 3)   # samples a healthy rank's count keeps changing, per operation
    slow_changes: Tuple[int, int] = (6, 8)     # the same for the slow rank
    slow_rank: Optional[int] = None    # None = seeded choice; -1 = nobody is slow
    seed: int = 0


@dataclass
class RateTrace:
    spec: RateSpec
    topo: Topology
    cols: Dict[str, np.ndarray]
    slow_rank: int                     # ground truth (-1 = none)

    @property
    def n(self) -> int:
        return int(self.cols["snap"].shape[0])


def generate_rates(spec: RateSpec, shuffle: bool = True) -> RateTrace:
    """SendCount / RecvCount of every (rank, communicator, channel) sampled at a fixed period while
    operations run back to back.

    Communicator c starts an operation every `op_samples` samples (seeded phase).  The sample taken
    at an operation's start shows zero counts; from then on a rank's count rises at every sample
    until the operation's `chunks` chunks are done: after k samples for a healthy rank (k drawn
    from `normal_changes` per rank, operation, channel and direction) and after k drawn from
    `slow_changes` for the slow rank.  Every k is at most `chunks`, so each of those k samples
    shows a new value: an operation is observed with exactly k value changes."""
    L = spec.layout
    topo = L.topology()
    R = L.n_ranks
    nch, nsn = spec.n_channels, spec.n_snapshots
    if max(spec.slow_changes) > spec.chunks or max(spec.slow_changes) >= spec.op_samples:
        raise ValueError("an operation must finish before the next one starts, one chunk or more per sample")
    seed = spec.seed
    slow = spec.slow_rank
    if slow is None:
        slow = int(rand_u64(seed, _S_RSLOW, 0) % np.uint64(R))
    kinds = ["tp", "pp", "dp"] + (["world"] if L.world else [])
    ranks = np.arange(R, dtype=np.int64)
    ch = np.arange(nch, dtype=np.int64)
    out = {k: [] for k in SNAP_COLUMNS}
    is_slow = ranks == slow
    for kind in kinds:
        comm_r = L.comm_of(kind, ranks).astype(np.int64)                          # [R]
        phase = (rand_u64(seed, _S_RPHASE, comm_r) % np.uint64(spec.op_samples)).astype(np.int64)
        seq0 = 1000 + (rand_u64(seed, _S_RPHASE, comm_r, 1) % np.uint64(9000)).astype(np.int64)
        for s in range(nsn):
            j = np.floor_divide(s - phase, spec.op_samples)                       # operation index, -1 before the first
            u = (s - phase) - j * spec.op_samples                                 # samples since its start
            seq = seq0 + j                                                        # [R]
            cnt = []
            for direction in (0, 1):
                lo_n, hi_n = spec.normal_changes
                lo_s, hi_s = spec.slow_changes
                draw = rand_u64(seed, _S_RK + direction, (ranks * 4 + kinds.index(kind))[:, None] * 1000003 + seq[:, None],
                                ch[None, :])                                      # [R, ch]
                k = np.where(is_slow[:, None], lo_s + (draw % np.uint64(hi_s - lo_s + 1)).astype(np.int64),
                             lo_n + (draw % np.uint64(hi_n - lo_n + 1)).astype(np.int64))
                done = np.minimum(u[:, None], k)
                cnt.append(np.where(j[:, None] < 0, spec.chunks, (spec.chunks * done) // k))
            n_rows = R * nch
            out["snap"].append(np.full(n_rows, s, dtype=np.uint32))
            out["rank"].append(np.repeat(ranks, nch).astype(np.uint32))
            out["comm"].append(np.repeat(comm_r, nch).astype(np.uint32))
            out["channel"].append(np.tile(ch, R).astype(np.uint32))
            out["seq_posted"].append(np.repeat(seq, nch).astype(np.uint64))
            out["chunks_sent"].append(cnt[0].reshape(-1).astype(np.uint32))
            out["chunks_recv"].append(cnt[1].reshape(-1).astype(np.uint32))
    cols = {k: np.concatenate(v) for k, v in out.items()}
    if shuffle:
        perm = np.random.Generator(np.random.PCG64(seed + 29)).permutation(cols["snap"].shape[0])
        cols = {k: v[perm] for k, v in cols.items()}
    return RateTrace(spec, topo, cols, slow)


# --------------------------------------------------------------------------
# Probing Frames: the probe's per-rank record of its latest kernels
# --------------------------------------------------------------------------
FRAME_BYTES = 1184                     # 32-byte header + 8 blocks of 144 bytes
FRAME_BLOCKS = 8
FRAME_CHANNELS = 8
FRAME_DTYPE = np.dtype([
    ("counter", "<u8"), ("mode", "<u4"), ("kernel_index", "<u4"), ("n_channels", "<u4"), ("reserved", "<u4", (3,)),
    ("block", [("comm", "<u4"), ("ext", "<u4"), ("counter", "<u8"),
               ("count", "<u8", (FRAME_CHANNELS, 2))], (FRAME_BLOCKS,)),
])
assert FRAME_DTYPE.itemsize == FRAME_BYTES


def encode_frames(topo: Topology, rows: Dict[str, np.ndarray], n_channels: int, keep: Optional[np.ndarray] = None,
                  kernel_counter: int = 0):
    """Packs one snapshot's rows (every (rank, communicator, channel) once) into one frame per rank.

    A rank's communicators take consecutive blocks starting at block `kernel_counter mod 8`, so the
    block positions move from call to call as they do in the probe's cyclic body.  `keep[rank,
    k]` = False leaves the rank's k-th communicator out of its frame (the probe only holds its
    latest kernels: a communicator that was not used lately is not in the frame).  Blocks that are
    not written keep a zero extension field.  Returns (frames as a structured array, ranks)."""
    if n_channels > FRAME_CHANNELS:
        raise ValueError("a frame block has 8 channels")
    R = topo.n_ranks
    frames = np.zeros(R, dtype=FRAME_DTYPE)
    frames["mode"] = 1
    frames["n_channels"] = n_channels
    order = np.lexsort((rows["channel"], rows["comm"], rows["rank"]))
    rk, cm, ch = rows["rank"][order], rows["comm"][order], rows["channel"][order]
    sq, sent, recv = rows["seq_posted"][order], rows["chunks_sent"][order], rows["chunks_recv"][order]
    first = ch == 0
    # ordinal of each (rank, comm) among the rank's communicators
    pair_rank, pair_comm = rk[first], cm[first]
    start = np.r_[True, pair_rank[1:] != pair_rank[:-1]]
    idx = np.arange(len(pair_rank))
    ordinal = idx - np.maximum.accumulate(np.where(start, idx, 0))
    if ordinal.max(initial=0) >= FRAME_BLOCKS:
        raise ValueError("a frame holds 8 kernels: ranks in more than 8 communicators are not supported here")
    on = np.ones(len(pair_rank), dtype=bool) if keep is None else keep[pair_rank, ordinal]
    blk = (kernel_counter + ordinal) % FRAME_BLOCKS
    pr, pb = pair_rank[on], blk[on]
    frames["block"]["comm"][pr, pb] = pair_comm[on]
    frames["block"]["ext"][pr, pb] = 1
    frames["block"]["counter"][pr, pb] = sq[first][on]
    row_on = np.repeat(on, n_channels)
    rr, rb = np.repeat(pair_rank, n_channels)[row_on], np.repeat(blk, n_channels)[row_on]
    frames["block"]["count"][rr, rb, ch[row_on], 0] = sent[row_on]
    frames["block"]["count"][rr, rb, ch[row_on], 1] = recv[row_on]
    frames["counter"] = kernel_counter + FRAME_BLOCKS - 1
    frames["kernel_index"] = frames["counter"] % FRAME_BLOCKS
    return frames, np.arange(R, dtype=np.uint32)
