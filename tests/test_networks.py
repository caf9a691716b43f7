"""Host-side check of the compare-exchange schedules that the statistics kernels run in a wavefront's lanes
(csrc/segments.hip: sort_groups, merge_groups).  The schedules are restated here as lists of lane masks and run
on numpy arrays: the sort must order any input (zero-one principle, exhaustive up to 16 lanes), and the merge
must order the absolute deviations of a sorted sequence from its lower median, with the empty lanes' largest
value at the end, which is what the kernels feed it (Section 4.2.2: robust dispersion of arrival and completion)."""
import itertools

import numpy as np
import pytest

SORT_MASKS = {2: [1], 4: [1, 3, 1], 8: [1, 3, 1, 7, 2, 1], 16: [1, 3, 1, 7, 2, 1, 15, 4, 2, 1],
              32: [1, 3, 1, 7, 2, 1, 15, 4, 2, 1, 31, 8, 4, 2, 1],
              64: [1, 3, 1, 7, 2, 1, 15, 4, 2, 1, 31, 8, 4, 2, 1, 63, 16, 8, 4, 2, 1]}
MERGE_MASKS = {g: [g >> s for s in range(1, g.bit_length())] for g in (2, 4, 8, 16, 32, 64)}


def high_bit(m):
    b = 1
    while b * 2 <= m:
        b *= 2
    return b


def run(values, masks):
    """values: (..., G); lane l exchanges with lane l ^ M and keeps the smaller value unless its high bit of M is set"""
    v = np.array(values, copy=True)
    lanes = np.arange(v.shape[-1])
    for m in masks:
        p = v[..., lanes ^ m]
        upper = (lanes & high_bit(m)) != 0
        v = np.where(upper, np.maximum(v, p), np.minimum(v, p))
    return v


@pytest.mark.parametrize("g", [2, 4, 8, 16])
def test_sort_schedule_orders_every_zero_one_input(g):
    x = np.array(list(itertools.product([0, 1], repeat=g)), dtype=np.int64)
    assert np.array_equal(run(x, SORT_MASKS[g]), np.sort(x, axis=-1))


@pytest.mark.parametrize("g", [32, 64])
def test_sort_schedule_orders_random_inputs_with_ties(g):
    rng = np.random.default_rng(g)
    x = rng.integers(0, 50, size=(20000, g))
    assert np.array_equal(run(x, SORT_MASKS[g]), np.sort(x, axis=-1))
    z = (rng.random((20000, g)) < rng.random((20000, 1))).astype(np.int64)        # zero-one inputs of every density
    assert np.array_equal(run(z, SORT_MASKS[g]), np.sort(z, axis=-1))


@pytest.mark.parametrize("g", [2, 4, 8, 16, 32, 64])
def test_merge_schedule_orders_the_deviations_of_a_sorted_group(g):
    rng = np.random.default_rng(100 + g)
    none = np.iinfo(np.int64).max
    for nd in range(0, g + 1):                       # finished records in the group; the other lanes are empty
        x = np.sort(rng.integers(0, 40 if nd % 2 else 10**9, size=(300, nd)), axis=-1)
        dev = np.full((300, g), none, dtype=np.int64)
        if nd:
            med = x[:, (nd - 1) // 2][:, None]
            dev[:, :nd] = np.abs(x - med)
        out = run(dev, MERGE_MASKS[g])
        assert np.array_equal(out, np.sort(dev, axis=-1)), (g, nd)
        if nd:                                       # the MAD is the same order statistic of the sorted deviations
            assert np.array_equal(out[:, (nd - 1) // 2], np.sort(np.abs(x - med), axis=-1)[:, (nd - 1) // 2])


def _kernel_schedule(fn, ty="i64", cx="cmpx"):
    """the cmpx<M> masks of `fn` in csrc/segments.hip, per group width G"""
    import os
    import re
    src = open(os.path.join(os.path.dirname(__file__), "..", "paper_2605_04478_amd", "csrc", "segments.hip")).read()
    body = src[src.index(f" {fn}({ty} v, u32 lane)"):]
    body = body[:body.index("return v;")]
    steps = []                                   # (smallest G that runs the step, mask) in program order
    for m in re.finditer(r"if constexpr \(G >= (\d+)\)([^\n]*(?:\n(?!\s*if constexpr)[^\n]*)*)", body):
        for c in re.findall(cx + r"<(\d+)>", m.group(2)):
            steps.append((int(m.group(1)), int(c)))
    return {g: [mask for need, mask in steps if need <= g] for g in (2, 4, 8, 16, 32, 64)}


def test_the_schedules_checked_here_are_the_kernels():
    assert _kernel_schedule("sort_groups") == SORT_MASKS
    assert _kernel_schedule("merge_groups") == MERGE_MASKS
    assert _kernel_schedule("sort_groups32", "i32", "cmpx32") == SORT_MASKS           # the passes on 32-bit offsets
    assert _kernel_schedule("merge_groups32", "i32", "cmpx32") == MERGE_MASKS
