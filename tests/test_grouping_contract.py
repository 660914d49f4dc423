"""The checker of the plan's optional grouping (tests/grouping.py) tested on the CPU: it accepts groupings written
out by hand and by a replay with Python lists and dicts, and it rejects every kind of planted damage.  The grouping
is an interface of this build (bookkeeping for the backward pass), not part of the paper's Algorithm 1; GPU tests
hold the planner's output to this contract instead of comparing it with a second implementation."""
import numpy as np
import pytest

import grouping

L = 0x80000000


def replay(ids, off, slots, row_max, piece):
    """The contract, batch by batch, with Python containers only."""
    gl, rows, roff, pieces, poff = [], [], [0], [], [0]
    for i in range(len(off) - 1):
        a, b = int(off[i]), int(off[i + 1])
        by_id = {}
        for k in range(a, b):
            by_id.setdefault(int(ids[k]), []).append(k - a)          # positions arrive in ascending order
        p = 0
        multi = 0
        for g in sorted(by_id):
            pos = by_id[g]
            m = len(pos)
            gl += pos
            slot = int(slots[a + pos[0]])
            rows.append([p | (L if m > row_max else 0), m, slot, pos[0]])
            if m > row_max:
                P = (m + piece - 1) // piece
                for j in range(P):
                    pieces.append([p + j * piece, min(piece, m - j * piece), slot, j, P, multi if P > 1 else 0, 0, 0])
                if P > 1:
                    multi += P
            p += m
        roff.append(len(rows))
        poff.append(len(pieces))
    return (np.array(gl, np.int32), np.array(rows, np.uint32).reshape(-1, 4), np.array(roff, np.int64),
            np.array(pieces, np.uint32).reshape(-1, 8), np.array(poff, np.int64))


def test_hand_worked_example():
    # one batch, rows longer than 1 lookup are long, pieces of 2: ids 5 3 5 5 3 5 5 at positions 0..6, slot = 10 * id
    ids = np.array([5, 3, 5, 5, 3, 5, 5], dtype=np.int64)
    off = np.array([0, 7], dtype=np.int64)
    slots = (ids * 10).astype(np.int32)
    # id 3 at positions 1, 4 (grouped 0..1); id 5 at positions 0, 2, 3, 5, 6 (grouped 2..6)
    gl = np.array([1, 4, 0, 2, 3, 5, 6], np.int32)
    rows = np.array([[0 | L, 2, 30, 1], [2 | L, 5, 50, 0]], np.uint32)
    # id 3: one piece of 2 (no partial number); id 5: pieces of 2, 2, 1 lookups, the batch's first row of several
    # pieces, so its pieces are numbered from 0
    pieces = np.array([[0, 2, 30, 0, 1, 0, 0, 0],
                       [2, 2, 50, 0, 3, 0, 0, 0], [4, 2, 50, 1, 3, 0, 0, 0], [6, 1, 50, 2, 3, 0, 0, 0]], np.uint32)
    grouping.check_grouping(ids, off, slots, gl, rows, [0, 2], pieces, [0, 4], row_max=1, piece=2)
    got = grouping.build_grouping(ids, off, slots, row_max=1, piece=2)
    assert got[0].tolist() == gl.tolist() and got[1].view(np.uint32).tolist() == rows.tolist()
    assert got[2].tolist() == [0, 2] and got[3].view(np.uint32).tolist() == pieces.tolist() and got[4].tolist() == [0, 4]
    # with rows of up to 2 lookups taken whole, only id 5 is long; pieces of 4: 4 + 1 lookups
    rows2 = np.array([[0, 2, 30, 1], [2 | L, 5, 50, 0]], np.uint32)
    pieces2 = np.array([[2, 4, 50, 0, 2, 0, 0, 0], [6, 1, 50, 1, 2, 0, 0, 0]], np.uint32)
    grouping.check_grouping(ids, off, slots, gl, rows2, [0, 2], pieces2, [0, 2], row_max=2, piece=4)
    with pytest.raises(AssertionError):                               # the long row's pieces left out
        grouping.check_grouping(ids, off, slots, gl, rows2, [0, 2], pieces2[:0], [0, 0], row_max=2, piece=4)


def test_two_batches_partial_numbers_are_per_batch():
    ids = np.array([7, 7, 7, 2, 9, 9, 9, 9], dtype=np.int64)
    off = np.array([0, 3, 8], dtype=np.int64)
    slots = np.array([4, 4, 4, 1, 8, 8, 8, 8], dtype=np.int32)
    gl = np.array([0, 1, 2, 0, 1, 2, 3, 4], np.int32)                 # positions are relative to their batch
    rows = np.array([[0 | L, 3, 4, 0], [0, 1, 1, 0], [1 | L, 4, 8, 1]], np.uint32)
    pieces = np.array([[0, 2, 4, 0, 2, 0, 0, 0], [2, 1, 4, 1, 2, 0, 0, 0],       # batch 0: id 7 in pieces 2 + 1
                       [1, 2, 8, 0, 2, 0, 0, 0], [3, 2, 8, 1, 2, 0, 0, 0]], np.uint32)   # batch 1 counts from 0 again
    grouping.check_grouping(ids, off, slots, gl, rows, [0, 1, 3], pieces, [0, 2, 4], row_max=1, piece=2)
    got = grouping.build_grouping(ids, off, slots, row_max=1, piece=2)
    assert got[1].view(np.uint32).tolist() == rows.tolist() and got[3].view(np.uint32).tolist() == pieces.tolist()
    assert got[2].tolist() == [0, 1, 3] and got[4].tolist() == [0, 2, 4]


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
    for row_max, piece in ((1, 1), (2, 3), (4, 16), (32, 256)):
        want = replay(ids, off, slots, row_max, piece)
        grouping.check_grouping(ids, off, slots, *want, row_max=row_max, piece=piece)
        got = grouping.build_grouping(ids, off, slots, row_max=row_max, piece=piece)
        for g, w, name in zip(got, want, ("grouped_lookups", "row_recs", "row_off", "piece_recs", "piece_off")):
            assert np.array_equal(np.asarray(g).view(np.uint32) if g.dtype == np.int32 and g.ndim == 2 else g, w), (name, row_max)


@pytest.mark.parametrize("seed", range(4))
def test_checker_rejects_planted_damage(seed):
    """Every clause of the contract, broken once."""
    ids, off, slots, rng = random_case(seed)
    row_max, piece = 2, 3
    gl, rows, roff, pieces, poff = replay(ids, off, slots, row_max, piece)
    i = int(np.argmax(np.diff(off)))                         # the largest batch
    a, b = int(off[i]), int(off[i + 1])
    ra, pa, pb = int(roff[i]), int(poff[i]), int(poff[i + 1])
    assert b - a >= 20 and roff[i + 1] - ra >= 3 and pb - pa >= 3

    def rejected(gl=gl, rows=rows, roff=roff, pieces=pieces, poff=poff):
        with pytest.raises(AssertionError):
            grouping.check_grouping(ids, off, slots, gl, rows, roff, pieces, poff, row_max=row_max, piece=piece)

    bad = gl.copy(); bad[a] = bad[a + 1]                     # not a permutation
    rejected(gl=bad)
    gid = ids[a:b][gl[a:b]]
    j = int(np.flatnonzero(np.diff(gid) > 0)[0])             # two neighbours of different ids swapped: order broken
    bad = gl.copy(); bad[[a + j, a + j + 1]] = bad[[a + j + 1, a + j]]
    rejected(gl=bad)
    same = np.flatnonzero(np.diff(gid) == 0)
    j = int(same[0])                                         # two lookups of one id swapped: positions not ascending
    bad = gl.copy(); bad[[a + j, a + j + 1]] = bad[[a + j + 1, a + j]]
    rejected(gl=bad)
    for col in range(4):                                     # every field of a row record
        bad = rows.copy(); bad[ra + 1, col] += 1
        rejected(rows=bad)
    bad = rows.copy(); bad[ra + 1, 0] ^= L                   # long flag flipped
    rejected(rows=bad)
    bad = np.delete(rows, ra + 1, axis=0); bo = roff.copy(); bo[i + 1:] -= 1     # a row record missing
    rejected(rows=bad, roff=bo)
    multi_piece = pa + int(np.flatnonzero(pieces[pa:pb, 4] > 1)[0])
    for col in range(8):                                     # every field of a piece record of a row of several pieces
        bad = pieces.copy(); bad[multi_piece, col] += 1
        rejected(pieces=bad)
    bad = np.delete(pieces, multi_piece, axis=0); bo = poff.copy(); bo[i + 1:] -= 1      # a piece missing
    rejected(pieces=bad, poff=bo)
    last_multi = pa + int(np.flatnonzero(pieces[pa:pb, 4] > 1)[-1])
    if pieces[last_multi, 5] > 0:                            # partial numbers must count the earlier rows' pieces
        bad = pieces.copy(); bad[pa:pb, 5] = 0
        rejected(pieces=bad)
