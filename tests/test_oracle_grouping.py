"""Pins for the oracle's grouping of a batch's lookups (orc_group_lookups): the optional by-product of the plan
that the grouped backward pass consumes.  The definition is this build's (an interface, not part of Algorithm 1):
lookups of a batch ordered by id, then by position; a work item starts where the id changes and at every multiple
of `chunk` grouped positions counted from the batch's first lookup; an id is "split" when its lookups span three
items or more.  Pinned by a hand-worked example, by a replay written with Python lists and dicts, and by the
properties that follow from the definition."""
import numpy as np
import pytest

import oracle

HEAD = 0x80000000


def replay(ids, off, slots, chunk):
    """The definition, batch by batch, with Python containers only."""
    gs, gl, st, ioff, sp, soff = [], [], [], [0], [], [0]
    for i in range(len(off) - 1):
        a, b = int(off[i]), int(off[i + 1])
        by_id = {}
        for k in range(a, b):
            by_id.setdefault(int(ids[k]), []).append(k - a)          # positions arrive in ascending order
        order = [(g, pos) for g in sorted(by_id) for pos in by_id[g]]
        starts = []
        for p, (g, pos) in enumerate(order):
            gl.append(pos)
            gs.append(int(slots[a + pos]))
            first = p == 0 or order[p - 1][0] != g
            if first or p % chunk == 0:
                starts.append(p | (HEAD if first else 0))
        # items of every id: count the item starts inside its stretch
        p = 0
        for g in sorted(by_id):
            n = len(by_id[g])
            n_items = sum(1 for s in starts if p <= (s & ~HEAD) < p + n)
            if n_items >= 3:
                sp.append(p)
            p += n
        st += starts
        ioff.append(len(st))
        soff.append(len(sp))
    return (np.array(gs, np.int32), np.array(gl, np.int32), np.array(st, np.uint32), np.array(ioff, np.int64),
            np.array(sp, np.uint32), np.array(soff, np.int64))


def test_hand_worked_example():
    # one batch, chunk 2: ids 5 3 5 5 3 5 at positions 0..5, slot = 10 * id
    ids = np.array([5, 3, 5, 5, 3, 5], dtype=np.int64)
    off = np.array([0, 6], dtype=np.int64)
    slots = (ids * 10).astype(np.int32)
    gs, gl, st, ioff, sp, soff = oracle.group_lookups(ids, off, slots, chunk=2)
    # id 3 at positions 1, 4; id 5 at positions 0, 2, 3, 5
    assert gl.tolist() == [1, 4, 0, 2, 3, 5]
    assert gs.tolist() == [30, 30, 50, 50, 50, 50]
    # grouped position 0 starts id 3; position 2 starts id 5 (and is a multiple of 2); position 4 is a cut inside id 5
    assert st.tolist() == [0 | HEAD, 2 | HEAD, 4]
    assert ioff.tolist() == [0, 3]
    # id 5 spans two items only: nothing is split
    assert sp.tolist() == [] and soff.tolist() == [0, 0]
    # with chunk 1 every lookup is an item; id 3 spans 2 items, id 5 spans 4: only id 5 is split, it starts at position 2
    gs1, gl1, st1, ioff1, sp1, soff1 = oracle.group_lookups(ids, off, slots, chunk=1)
    assert st1.tolist() == [0 | HEAD, 1, 2 | HEAD, 3, 4, 5]
    assert sp1.tolist() == [2] and soff1.tolist() == [0, 1]


def test_two_batches_offsets_are_per_batch():
    ids = np.array([7, 7, 7, 2, 9, 9], dtype=np.int64)
    off = np.array([0, 3, 6], dtype=np.int64)
    slots = np.array([4, 4, 4, 1, 8, 8], dtype=np.int32)
    gs, gl, st, ioff, sp, soff = oracle.group_lookups(ids, off, slots, chunk=1)
    assert gl.tolist() == [0, 1, 2, 0, 1, 2]                 # positions are relative to their batch
    assert gs.tolist() == [4, 4, 4, 1, 8, 8]
    assert st.tolist() == [0 | HEAD, 1, 2, 0 | HEAD, 1 | HEAD, 2]
    assert ioff.tolist() == [0, 3, 6]
    assert sp.tolist() == [0] and soff.tolist() == [0, 1, 1]  # batch 0: id 7 spans three items; batch 1: none does


@pytest.mark.parametrize("seed", range(8))
def test_against_replay_and_properties(seed):
    rng = np.random.default_rng(900 + seed)
    T = int(rng.integers(1, 7))
    lens = rng.integers(0, 200, size=T)
    lens[rng.integers(0, T)] = 0                             # an empty batch
    off = np.zeros(T + 1, dtype=np.int64)
    off[1:] = np.cumsum(lens)
    R = int(rng.integers(2, 40))
    ids = np.minimum(rng.zipf(1.3, size=int(off[-1])) - 1, R - 1).astype(np.int64)
    slot_of = rng.permutation(1000)[:R].astype(np.int32)     # any map from id to slot, one slot per id
    slots = slot_of[ids]
    for chunk in (1, 3, 32):
        got = oracle.group_lookups(ids, off, slots, chunk=chunk)
        want = replay(ids, off, slots, chunk)
        for g, w, name in zip(got, want, ("grouped_slots", "grouped_lookups", "item_starts", "item_off", "split_starts",
                                          "split_off")):
            assert np.array_equal(g, w), (name, chunk)
        gs, gl, st, ioff, sp, soff = got
        for i in range(T):
            a, b = int(off[i]), int(off[i + 1])
            # a permutation of the batch's positions, ids ascending, positions ascending inside an id
            assert sorted(gl[a:b].tolist()) == list(range(b - a))
            gid = ids[a:b][gl[a:b]]
            assert np.all(np.diff(gid) >= 0)
            same = np.diff(gid) == 0
            assert np.all(np.diff(gl[a:b])[same] > 0)
            assert np.array_equal(gs[a:b], slots[a:b][gl[a:b]])
            items = st[ioff[i]:ioff[i + 1]]
            pos = (items & np.uint32(~HEAD & 0xFFFFFFFF)).astype(np.int64)
            if b > a:
                assert pos[0] == 0 and items[0] & HEAD
            assert np.all(np.diff(pos) > 0)
            ends = np.append(pos[1:], b - a)
            assert np.all(ends - pos <= chunk)                # no item is longer than a chunk
            for s, e in zip(pos, ends):                       # and none mixes ids
                assert len(set(gid[s:e].tolist())) == 1
            # the head bit is set exactly where the id changes
            change = np.ones(b - a, dtype=bool)
            change[1:] = gid[1:] != gid[:-1]
            assert np.array_equal((items & HEAD) != 0, change[pos])
