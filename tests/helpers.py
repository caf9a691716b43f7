"""Small builders shared by the tests (inputs only, no analyzer arithmetic)."""
from __future__ import annotations

from typing import Dict, Iterable, Sequence

import numpy as np

from paper_2605_04478_amd import tracegen as tg

INFLIGHT = tg.INFLIGHT
T0 = tg.T_EPOCH_NS


def toy_cols(rows: Iterable[Sequence[int]]) -> Dict[str, np.ndarray]:
    """rows of (rank, comm, seq, op, bytes, t_enter, t_exit) -> the seven SoA columns."""
    rows = list(rows)
    g = lambda i, dt: np.asarray([r[i] for r in rows], dtype=dt)
    return {"rank": g(0, np.uint32), "comm": g(1, np.uint32), "seq": g(2, np.uint64), "op": g(3, np.uint8),
            "bytes": g(4, np.uint64), "t_enter": g(5, np.int64), "t_exit": g(6, np.int64)}


def ring_topology(n_ranks: int, comms=None) -> tg.Topology:
    if comms is None:
        comms = [list(range(n_ranks))]
    return tg.make_topology(n_ranks, comms)


def rounds_with_durations(durs_per_round, comm=0, op=tg.OP_ALLREDUCE, nbytes=1 << 20, seq0=0,
                          spacing_ns=1_000_000_000, t_start=T0):
    """One record per (round, rank): every rank enters at the round's start and
    leaves after the given duration (ns)."""
    rows = []
    for j, durs in enumerate(durs_per_round):
        t = t_start + j * spacing_ns
        for r, d in enumerate(durs):
            rows.append((r, comm, seq0 + j, op, nbytes, t, t + int(d)))
    return rows


def concat_cols(a: Dict[str, np.ndarray], b: Dict[str, np.ndarray]) -> Dict[str, np.ndarray]:
    return {k: np.concatenate([a[k], b[k]]) for k in a}
