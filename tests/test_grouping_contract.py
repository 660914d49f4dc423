"""The checker of the plan's optional grouping (tests/grouping.py) tested on the CPU: it accepts groupings written
out by hand and by a replay with Python lists and dicts, and it rejects every kind of planted damage.  The grouping
is an interface of this build (bookkeeping for the backward pass), not part of the paper's Algorithm 1; GPU tests
hold the planner's output to this contract instead of comparing it with a second implementation."""
import numpy as np
import pytest

import grouping
from grouping import HEAD

H = int(HEAD)


def replay(ids, off, slots, chunk):
    """The contract, batch by batch, with Python containers only."""
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
                starts.append(p | (H if first else 0))
        p = 0
        for g in sorted(by_id):                                       # items of every id: starts inside its stretch
            n = len(by_id[g])
            if sum(1 for s in starts if p <= (s & ~H) < p + n) >= 3:
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
    # id 3 at positions 1, 4; id 5 at positions 0, 2, 3, 5; grouped position 0 starts id 3, position 2 starts id 5
    # (and is a multiple of 2), position 4 is a cut inside id 5, which spans two items only: nothing is split
    gl = np.array([1, 4, 0, 2, 3, 5], np.int32)
    gs = np.array([30, 30, 50, 50, 50, 50], np.int32)
    st = np.array([0 | H, 2 | H, 4], np.uint32)
    none = np.zeros(0, np.uint32)
    grouping.check_grouping(ids, off, slots, gs, gl, st, [0, 3], none, [0, 0], chunk=2)
    got = grouping.build_grouping(ids, off, slots, chunk=2)
    assert got[0].tolist() == gs.tolist() and got[1].tolist() == gl.tolist() and got[2].tolist() == st.tolist()
    assert got[3].tolist() == [0, 3] and got[4].tolist() == [] and got[5].tolist() == [0, 0]
    # with chunk 1 every lookup is an item; id 3 spans 2 items, id 5 spans 4: only id 5 is split, it starts at 2
    st1 = np.array([0 | H, 1, 2 | H, 3, 4, 5], np.uint32)
    grouping.check_grouping(ids, off, slots, gs, gl, st1, [0, 6], np.array([2], np.uint32), [0, 1], chunk=1)
    with pytest.raises(AssertionError):                               # the split row left out
        grouping.check_grouping(ids, off, slots, gs, gl, st1, [0, 6], none, [0, 0], chunk=1)


def test_two_batches_offsets_are_per_batch():
    ids = np.array([7, 7, 7, 2, 9, 9], dtype=np.int64)
    off = np.array([0, 3, 6], dtype=np.int64)
    slots = np.array([4, 4, 4, 1, 8, 8], dtype=np.int32)
    gl = np.array([0, 1, 2, 0, 1, 2], np.int32)                       # positions are relative to their batch
    st = np.array([0 | H, 1, 2, 0 | H, 1 | H, 2], np.uint32)
    # batch 0: id 7 spans three items; batch 1: none does
    grouping.check_grouping(ids, off, slots, slots, gl, st, [0, 3, 6], np.array([0], np.uint32), [0, 1, 1], chunk=1)
    got = grouping.build_grouping(ids, off, slots, chunk=1)
    assert got[2].tolist() == st.tolist() and got[3].tolist() == [0, 3, 6]
    assert got[4].tolist() == [0] and got[5].tolist() == [0, 1, 1]


def random_case(seed):
    rng = np.random.default_rng(900 + seed)
    T = int(rng.integers(1, 7))
    lens = rng.integers(0, 200, size=T)
    lens[rng.integers(0, T)] = 0                             # an empty batch
    off = np.zeros(T + 1, dtype=np.int64)
    off[1:] = np.cumsum(lens)
    R = int(rng.integers(2, 40))
    ids = np.minimum(rng.zipf(1.3, size=int(off[-1])) - 1, R - 1).astype(np.int64)
    slot_of = rng.permutation(1000)[:R].astype(np.int32)     # any map from id to slot, one slot per id
    return ids, off, slot_of[ids], rng


@pytest.mark.parametrize("seed", range(8))
def test_checker_accepts_replay_and_builder(seed):
    ids, off, slots, _ = random_case(seed)
    for chunk in (1, 3, 32):
        want = replay(ids, off, slots, chunk)
        grouping.check_grouping(ids, off, slots, *want, chunk=chunk)
        got = grouping.build_grouping(ids, off, slots, chunk=chunk)
        for g, w, name in zip(got, want, ("grouped_slots", "grouped_lookups", "item_starts", "item_off", "split_starts",
                                          "split_off")):
            assert np.array_equal(g, w), (name, chunk)


@pytest.mark.parametrize("seed", range(4))
def test_checker_rejects_planted_damage(seed):
    """Every clause of the contract, broken once."""
    ids, off, slots, rng = random_case(seed)
    chunk = 3
    gs, gl, st, ioff, sp, soff = replay(ids, off, slots, chunk)
    i = int(np.argmax(np.diff(off)))                         # the largest batch
    a, b = int(off[i]), int(off[i + 1])
    assert b - a >= 20 and ioff[i + 1] - ioff[i] >= 4

    def rejected(gs=gs, gl=gl, st=st, ioff=ioff, sp=sp, soff=soff):
        with pytest.raises(AssertionError):
            grouping.check_grouping(ids, off, slots, gs, gl, st, ioff, sp, soff, chunk=chunk)

    bad = gl.copy(); bad[a] = bad[a + 1]                     # not a permutation
    rejected(gl=bad)
    gid = ids[a:b][gl[a:b]]
    j = int(np.flatnonzero(np.diff(gid) > 0)[0])             # two neighbours of different ids swapped: order broken
    bad, bad_s = gl.copy(), gs.copy()
    bad[[a + j, a + j + 1]] = bad[[a + j + 1, a + j]]
    bad_s[[a + j, a + j + 1]] = bad_s[[a + j + 1, a + j]]
    rejected(gl=bad, gs=bad_s)
    same = np.flatnonzero(np.diff(gid) == 0)
    if len(same):                                            # two lookups of one id swapped: positions not ascending
        j = int(same[0])
        bad = gl.copy(); bad[[a + j, a + j + 1]] = bad[[a + j + 1, a + j]]
        rejected(gl=bad)
    bad = gs.copy(); bad[a + 5] += 1                         # a wrong slot
    rejected(gs=bad)
    k = int(ioff[i]) + 2
    bad = st.copy(); bad[k] ^= H                             # head bit flipped
    rejected(st=bad)
    bad = np.delete(st, k); bo = ioff.copy(); bo[i + 1:] -= 1    # an item missing (its neighbour grows past a cut or row)
    rejected(st=bad, ioff=bo)
    bad = st.copy(); bad[k] = (bad[k] & H) | ((bad[k] & ~HEAD) + 1 if (bad[k] & ~HEAD) + 1 < (st[k + 1] & ~HEAD) else (bad[k] & ~HEAD) - 1)
    if not np.array_equal(bad, st):
        rejected(st=bad)                                     # an item start moved off its place
    extra = np.insert(sp, int(soff[i]), np.uint32(0)) if not (soff[i + 1] > soff[i] and sp[soff[i]] == 0) else None
    if extra is not None:                                    # a row listed as split that is not (or listed twice)
        so = soff.copy(); so[i + 1:] += 1
        first_row_len = int(np.flatnonzero(np.append(np.diff(gid) != 0, True))[0]) + 1
        if first_row_len <= 2 * chunk:
            rejected(sp=extra, soff=so)
    if soff[i + 1] > soff[i]:                                # a split row dropped
        so = soff.copy(); so[i + 1:] -= 1
        rejected(sp=np.delete(sp, int(soff[i])), soff=so)
