"""A second derivation of the flag chains for sizes the oracle's loops cannot take (test infrastructure)."""
import numpy as np

from oracle import ccld_oracle as orc
from paper_2605_04478_amd import tracegen as tg


def chains_by_definition(cols, flag, n_ranks):
    """Root-cause / secondary separation of the late entries written out with array primitives (sorts and binary
    searches) straight from its definition, for sizes the oracle's loops cannot take: the previous operation of a
    flag's rank is its completed record with the largest (t_exit, t_enter, communicator, counter) whose t_exit is not
    after the flag's entry; the parent is the late entry with the largest lag (then the smallest rank) in that
    collective.  Assumes every completed record lasts longer than zero (a flag's own record is then never its
    previous operation), which the caller checks."""
    comm, seq, rank = cols["comm"].astype(np.int64), cols["seq"].astype(np.int64), cols["rank"].astype(np.int64)
    te, tx = cols["t_enter"], cols["t_exit"]
    S = int(seq.max()) + 1
    ckey = comm * S + seq                                    # one number per collective
    # every flag's own record -> its entry time
    rkey = ckey * n_ranks + rank
    by_key = np.argsort(rkey, kind="stable")
    fkey = flag["comm"].astype(np.int64) * S + flag["seq"].astype(np.int64)
    at = np.searchsorted(rkey[by_key], fkey * n_ranks + flag["rank"].astype(np.int64))
    own = by_key[at]
    assert np.array_equal(rkey[own], fkey * n_ranks + flag["rank"])
    t_f = te[own]
    late = (flag["kind"] & orc.FLAG_LATE_ENTER) != 0
    # completed records per rank in ascending (t_exit, t_enter, communicator, counter)
    done = np.nonzero(tx != tg.INFLIGHT)[0]
    t0 = int(min(te.min(), tx[done].min()))
    span = int(max(tx[done].max(), te.max())) - t0 + 2
    assert span * n_ranks < 2**62
    o = done[np.lexsort((seq[done], comm[done], te[done], tx[done], rank[done]))]
    okey = rank[o] * span + (tx[o] - t0)
    pos = np.searchsorted(okey, flag["rank"].astype(np.int64) * span + (t_f - t0), side="right") - 1
    has_prev = late & (pos >= 0)
    has_prev[has_prev] &= rank[o[pos[has_prev]]] == flag["rank"][has_prev]
    prev_c = np.where(has_prev, ckey[o[np.maximum(pos, 0)]], -1)
    # per collective the late entry with the largest lag, then the smallest rank
    lf = np.nonzero(late)[0]
    best = lf[np.lexsort((flag["rank"][lf], -flag["lag_enter"][lf], fkey[lf]))]
    ukey, first = np.unique(fkey[best], return_index=True)
    j = np.searchsorted(ukey, prev_c)
    j = np.minimum(j, len(ukey) - 1)
    hit = has_prev & (ukey[j] == prev_c)
    parent = np.where(hit, best[first[j]], -1).astype(np.int64)
    # roots and depths by pointer jumping
    n = len(parent)
    anc = np.where(parent >= 0, parent, np.arange(n))
    depth = (parent >= 0).astype(np.int64)
    while True:
        nxt = anc[anc]
        if np.array_equal(nxt, anc):
            break
        depth = depth + np.where(nxt != anc, depth[anc], 0)
        anc = nxt
    per = {"root_entries": np.bincount(flag["rank"][late & (parent < 0)], minlength=n_ranks),
           "secondary_entries": np.bincount(flag["rank"][late & (parent >= 0)], minlength=n_ranks),
           "caused": np.bincount(flag["rank"][anc[late]], minlength=n_ranks)}
    return {"parent": parent, "root": anc, "root_rank": flag["rank"][anc].astype(np.int64), "depth": depth}, per
