"""Pins of the oracle's Probing Frame decoder: the sizes the paper states, hand-packed frames,
the carry-forward of communicators that left the frame, and the error checks."""
import os
import struct

import numpy as np
import pytest

from oracle import ccld_oracle as orc
from paper_2605_04478_amd import tracegen as tg
from tests.helpers import ring_topology

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "probing_frame_sizes.txt")


def golden():
    out = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if line:
            k, v = [x.strip() for x in line.split("=")]
            out[k] = int(v)
    return out


G = golden()
SLOT = (G["body_bytes"] // G["blocks"] - G["trace_id_bytes"]) // (G["channels"] * G["slots_per_channel"])
BLOCK = G["body_bytes"] // G["blocks"]


def pack_frame(blocks, n_channels=8, counter=0):
    """blocks: list of (block index, comm, written, op counter, [(sent, recv)] * channels)."""
    buf = bytearray(G["frame_bytes"])
    struct.pack_into("<QIII", buf, 0, counter, 1, counter % G["blocks"], n_channels)
    for b, comm, written, cnt, counts in blocks:
        off = G["header_bytes"] + b * BLOCK
        struct.pack_into("<IIQ", buf, off, comm, 1 if written else 0, cnt)
        for ch, (s, r) in enumerate(counts):
            struct.pack_into("<QQ", buf, off + G["trace_id_bytes"] + ch * G["slots_per_channel"] * SLOT, s, r)
    return np.frombuffer(bytes(buf), dtype=np.uint8)


def rows_of(out, rank, comm):
    m = (out["rank"] == rank) & (out["comm"] == comm)
    return list(zip(out["channel"][m].tolist(), out["seq_posted"][m].tolist(), out["chunks_sent"][m].tolist(),
                    out["chunks_recv"][m].tolist()))


def test_sizes_stated_by_the_paper():
    assert G["header_bytes"] + G["body_bytes"] == G["frame_bytes"]
    assert BLOCK == 144 and SLOT == 8
    assert G["trace_id_bytes"] + G["channels"] * G["slots_per_channel"] * SLOT == BLOCK
    assert tg.FRAME_DTYPE.itemsize == G["frame_bytes"] and tg.FRAME_BLOCKS == G["blocks"]


def test_hand_packed_frame_and_carry_forward():
    topo = ring_topology(3, comms=[[0, 1, 2], [2, 0]])
    o = orc.Oracle(topo)
    o.frames_begin(2)
    f0 = pack_frame([(5, 0, True, 40, [(7, 6), (9, 8)]), (6, 1, True, 11, [(1, 2), (3, 4)]),
                     (2, 1, False, 99, [(50, 50), (50, 50)])], n_channels=2)       # block 2 was never written
    st, out = o.decode_frames(np.stack([f0]), np.asarray([0]), 0)
    assert st == "OK" and len(out["rank"]) == 5 * 2
    assert rows_of(out, 0, 0) == [(0, 40, 7, 6), (1, 40, 9, 8)]
    assert rows_of(out, 0, 1) == [(0, 11, 1, 2), (1, 11, 3, 4)]
    assert rows_of(out, 1, 0) == [(0, 0, 0, 0), (1, 0, 0, 0)]                       # no frame of rank 1 yet
    assert list(out["snap"]) == [0] * 10
    # next snapshot: communicator 1 has left rank 0's frame; two blocks carry communicator 0
    f1 = pack_frame([(0, 0, True, 41, [(2, 1), (0, 0)]), (7, 0, True, 42, [(1, 0), (1, 1)])], n_channels=2)
    st, out = o.decode_frames(np.stack([f1]), np.asarray([0]), 1)
    assert st == "OK"
    assert rows_of(out, 0, 0) == [(0, 42, 1, 0), (1, 42, 1, 1)]                     # the later kernel wins
    assert rows_of(out, 0, 1) == [(0, 11, 1, 2), (1, 11, 3, 4)]                     # remembered
    # two written blocks with the same operation counter on one communicator: the block further back in the frame
    # is the later kernel
    o3 = orc.Oracle(topo)
    o3.frames_begin(2)
    f3 = pack_frame([(1, 0, True, 50, [(1, 1), (1, 1)]), (6, 0, True, 50, [(2, 2), (2, 2)]), (3, 0, True, 50, [(3, 3), (3, 3)])],
                    n_channels=2)
    st, out3 = o3.decode_frames(np.stack([f3]), np.asarray([0]), 0)
    assert st == "OK" and rows_of(out3, 0, 0) == [(0, 50, 2, 2), (1, 50, 2, 2)]
    # a stale frame (older operation) does not replace what is remembered
    st, out = o.decode_frames(np.stack([f0]), np.asarray([0]), 2)
    assert rows_of(out, 0, 0) == [(0, 42, 1, 0), (1, 42, 1, 1)]
    # a header with fewer channels than the grid: the missing channels read zero
    f2 = pack_frame([(1, 0, True, 43, [(5, 5), (6, 6)])], n_channels=1)
    st, out = o.decode_frames(np.stack([f2]), np.asarray([0]), 3)
    assert rows_of(out, 0, 0) == [(0, 43, 5, 5), (1, 43, 0, 0)]


def test_error_checks_leave_the_state_alone():
    topo = ring_topology(3, comms=[[0, 1, 2], [2, 0]])
    o = orc.Oracle(topo)
    o.frames_begin(2)
    good = pack_frame([(0, 0, True, 5, [(1, 1), (2, 2)])], n_channels=2)
    assert o.decode_frames(np.stack([good]), np.asarray([1]), 0)[0] == "OK"
    cases = [
        (pack_frame([(0, 9, True, 6, [(1, 1)])], 2), 1, "E_UNKNOWN_COMM"),
        (pack_frame([(0, 1, True, 6, [(1, 1)])], 2), 1, "E_RANK_NOT_MEMBER"),       # rank 1 is not in communicator 1
        (pack_frame([(0, 0, True, 6, [(1, 1)])], 2), 7, "E_RANK_NOT_MEMBER"),       # no such rank
        (pack_frame([(0, 0, True, 6, [(1, 1)])], 9), 1, "E_RANGE"),                 # nine channels
        (pack_frame([(0, 0, True, 6, [(2**32, 1)])], 2), 1, "E_RANGE"),             # a count beyond 32 bits
    ]
    for frame, rank, want in cases:
        st, _ = o.decode_frames(np.stack([frame]), np.asarray([rank]), 1)
        assert st == want, (want, st)
    st, _ = o.decode_frames(np.stack([good, good]), np.asarray([1, 1]), 1)          # two frames of one rank
    assert st == "E_DUPLICATE_KEY"
    # the largest count that fits 32 bits is allowed; a range error outranks two frames of one rank
    edge = pack_frame([(0, 0, True, 5, [(2**32 - 1, 2**32 - 1), (2, 2)])], n_channels=2)
    o2 = orc.Oracle(topo)
    o2.frames_begin(2)
    st, out2 = o2.decode_frames(np.stack([edge]), np.asarray([1]), 0)
    assert st == "OK" and rows_of(out2, 1, 0)[0] == (0, 5, 2**32 - 1, 2**32 - 1)
    nine = pack_frame([(0, 0, True, 6, [(1, 1)])], 9)
    assert o.decode_frames(np.stack([nine, good, good]), np.asarray([0, 1, 1]), 1)[0] == "E_RANGE"
    st, out = o.decode_frames(np.zeros((0, G["frame_bytes"]), np.uint8), np.zeros(0, np.uint32), 2)
    assert st == "OK" and rows_of(out, 1, 0) == [(0, 5, 1, 1), (1, 5, 2, 2)]        # untouched by the failures


def test_frames_of_a_hang_series_locate_the_same_root():
    ht = tg.generate_hang(tg.config4(layout=tg.Layout3D(tp=2, pp=2, dp=4, world=True), n_channels=4, n_snapshots=40,
                                     hang_snapshot=5), shuffle=False)
    o = orc.Oracle(ht.topo)
    direct = o.locate_hang(ht.cols, 40, 4)
    assert list(direct.root["rank"]) == [ht.root_rank]
    o.frames_begin(4)
    rng = np.random.default_rng(2)
    c = ht.cols
    n_comm_of_rank = 4
    prev = None
    decoded = {k: [] for k in c}
    for s in range(40):
        m = c["snap"] == s
        rows = {k: v[m] for k, v in c.items()}
        order = np.lexsort((rows["channel"], rows["comm"], rows["rank"]))
        state = np.stack([rows[k][order].astype(np.int64) for k in ("seq_posted", "chunks_sent", "chunks_recv")])
        state = state.reshape(3, ht.topo.n_ranks, n_comm_of_rank, 4)
        changed = np.ones((ht.topo.n_ranks, n_comm_of_rank), bool) if prev is None else \
            (state != prev).any(axis=(0, 3))
        keep = changed | (rng.random(changed.shape) < 0.5)       # unchanged communicators may be missing
        prev = state
        frames, ranks = tg.encode_frames(ht.topo, rows, 4, keep=keep, kernel_counter=3 * s)
        p = rng.permutation(len(ranks))
        st, out = o.decode_frames(frames[p], ranks[p], s)
        assert st == "OK"
        for k in decoded:
            decoded[k].append(out[k])
    cols = {k: np.concatenate(v) for k, v in decoded.items()}
    via_frames = o.locate_hang(cols, 40, 4)
    assert via_frames.status == "OK" and list(via_frames.root["rank"]) == [ht.root_rank]
    for name in ("root", "pair", "comm"):
        a, b = getattr(direct, name), getattr(via_frames, name)
        for k in a:
            assert np.array_equal(a[k], b[k]), (name, k)
