"""The contract of the plan's optional grouping (include/bagpipe.h, bp_plan.grouped_* / item_* / split_*), as a
checker and as a small host-side builder.  Test code only; it knows nothing of how the planner or the backward
kernels work, only what the header promises a caller:

  * inside a batch the grouped lookups are a permutation of the batch's positions, ordered by id ascending and,
    for one id, by position ascending; grouped_slots[p] is the slot of the lookup at grouped_lookups[p];
  * a work item is a maximal run of grouped lookups of one row that does not cross a multiple of BP_BWD_CHUNK
    (counted from the batch's first grouped lookup); item_starts lists the first grouped lookup of every item,
    ascending, with bit 31 set exactly when that lookup is the first of its row;
  * split_starts lists, ascending, the first grouped lookup of exactly those rows whose lookups reach the second
    multiple of BP_BWD_CHUNK after the row's first lookup (three work items or more).
"""
import numpy as np

HEAD = np.uint32(0x80000000)
POS = np.uint32(0x7FFFFFFF)


def check_batch(ids, slots, gs, gl, items, splits, chunk):
    """One batch: ids / slots in lookup order [n]; gs / gl the grouped arrays [n]; items / splits the batch's
    records (uint32).  Raises AssertionError naming the clause that fails."""
    n = len(ids)
    assert len(gs) == n and len(gl) == n
    if n == 0:
        assert len(items) == 0 and len(splits) == 0
        return
    gl64 = gl.astype(np.int64)
    assert gl64.min() >= 0 and gl64.max() < n, "grouped position out of the batch"
    seen = np.zeros(n, dtype=bool)
    seen[gl64] = True
    assert seen.all(), "grouped_lookups is not a permutation of the batch's positions"
    gid = ids[gl64]
    step = np.diff(gid)
    assert (step >= 0).all(), "ids not ascending in the grouped order"
    assert (np.diff(gl64)[step == 0] > 0).all(), "positions of one id not ascending"
    assert np.array_equal(gs, slots[gl64]), "grouped_slots is not the slot of the grouped lookup"
    first = np.ones(n, dtype=bool)                      # first grouped lookup of its row
    first[1:] = step != 0
    p = np.arange(n, dtype=np.int64)
    want_start = first | (p % chunk == 0)               # maximal runs: a new item exactly at these places
    pos = (items & POS).astype(np.int64)
    assert np.array_equal(pos, np.flatnonzero(want_start)), "item starts are not the maximal single-row runs"
    assert np.array_equal((items & HEAD) != 0, first[pos]), "head bit does not mark the first lookup of a row"
    # rows that reach the second cut after their first lookup
    row_start = np.flatnonzero(first)
    row_end = np.append(row_start[1:], n)               # one past the row's last grouped lookup
    second_cut = (row_start // chunk + 2) * chunk
    want_split = row_start[second_cut < row_end]
    assert np.array_equal(splits.astype(np.int64), want_split), "split list is not the rows spanning three items"


def check_grouping(ids, off, lookup_slots, gs, gl, item_starts, item_off, split_starts, split_off, chunk=32,
                   n_batches=None):
    """All batches of a plan.  off: lookup offsets [T+1]; item_off / split_off: the plan's host offsets into
    item_starts / split_starts (they need not start at 0).  Arrays may be numpy or anything np.asarray takes."""
    T = (len(off) - 1) if n_batches is None else n_batches
    item_starts = np.asarray(item_starts).view(np.uint32)
    split_starts = np.asarray(split_starts).view(np.uint32)
    for i in range(T):
        a, b = int(off[i]), int(off[i + 1])
        check_batch(ids[a:b], lookup_slots[a:b], gs[a:b], gl[a:b], item_starts[int(item_off[i]):int(item_off[i + 1])],
                    split_starts[int(split_off[i]):int(split_off[i + 1])], chunk)


def build_grouping(ids, off, lookup_slots, chunk=32):
    """A grouping that satisfies the contract, built on the host with a stable sort per batch, for tests that feed
    the grouped backward pass without running the planner.
    Returns (grouped_slots, grouped_lookups, item_starts, item_off, split_starts, split_off)."""
    ids = np.asarray(ids, dtype=np.int64)
    lookup_slots = np.asarray(lookup_slots, dtype=np.int32)
    T = len(off) - 1
    gs = np.empty(len(ids), np.int32)
    gl = np.empty(len(ids), np.int32)
    items, splits, ioff, soff = [], [], [0], [0]
    for i in range(T):
        a, b = int(off[i]), int(off[i + 1])
        n = b - a
        order = np.argsort(ids[a:b], kind="stable")
        gl[a:b] = order
        gs[a:b] = lookup_slots[a:b][order]
        if n:
            gid = ids[a:b][order]
            first = np.ones(n, dtype=bool)
            first[1:] = gid[1:] != gid[:-1]
            p = np.arange(n, dtype=np.int64)
            pos = np.flatnonzero(first | (p % chunk == 0))
            items.append(pos.astype(np.uint32) | np.where(first[pos], HEAD, np.uint32(0)))
            row_start = np.flatnonzero(first)
            row_end = np.append(row_start[1:], n)
            splits.append(row_start[(row_start // chunk + 2) * chunk < row_end].astype(np.uint32))
        ioff.append(ioff[-1] + (len(items[-1]) if n else 0))
        soff.append(soff[-1] + (len(splits[-1]) if n else 0))
    cat = lambda parts: np.concatenate(parts) if parts else np.zeros(0, np.uint32)
    return gs, gl, cat(items), np.array(ioff, np.int64), cat(splits), np.array(soff, np.int64)
