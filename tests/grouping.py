"""The contract of the plan's optional grouping (include/bagpipe.h: bp_plan.grouped_lookups, row_recs, piece_recs,
piece_offsets), as a checker and as a small host-side builder.  Test code only; it knows nothing of how the planner
or the backward kernels work, only what the header promises a caller:

  * inside a batch the grouped lookups are a permutation of the batch's positions, ordered by id ascending and,
    for one id, by position ascending;
  * the batch's distinct rows, in that order, are its keep-list entries, and row record k describes the row of
    keep-list entry k: start = grouped position of its first lookup (bit 31 set iff it has more than BP_BWD_ROW_MAX
    lookups), count = its lookups, slot = its cache slot, first = the lookup position of its first lookup;
  * every long row, in order, owns ceil(count / BP_BWD_PIECE) consecutive piece records: piece j covers the grouped
    lookups [start + j * PIECE, ...) of the row, BP_BWD_PIECE of them except the last; it names the row's slot, j,
    the number of pieces, and, for rows of two or more pieces, the number of the row's first piece when the pieces
    of such rows are counted through the batch from 0; the two reserved words are 0.
"""
import numpy as np

ROW_MAX, PIECE = 16, 256          # BP_BWD_ROW_MAX, BP_BWD_PIECE
LONG = np.uint32(0x80000000)
POS = np.uint32(0x7FFFFFFF)


def _expected_pieces(row_start, row_count, row_slot, row_max, piece):
    """Piece records [P, 8] (uint32) the contract asks for, from the rows of one batch."""
    lr = np.flatnonzero(row_count > row_max)                    # the long rows, in order
    m, s0 = row_count[lr].astype(np.int64), row_start[lr].astype(np.int64)
    P = -(-m // piece)
    total = int(P.sum())
    out = np.zeros((total, 8), dtype=np.uint32)
    if total == 0:
        return out
    first_piece = np.cumsum(P) - P
    r = np.repeat(np.arange(len(lr)), P)                        # row of every piece
    j = np.arange(total, dtype=np.int64) - first_piece[r]       # its number inside the row
    multi = np.where(P > 1, P, 0)
    multi_base = np.cumsum(multi) - multi                       # pieces of rows of several pieces before this row
    out[:, 0] = s0[r] + j * piece
    out[:, 1] = np.minimum(piece, m[r] - j * piece)
    out[:, 2] = row_slot[lr][r].astype(np.int32).view(np.uint32)
    out[:, 3] = j
    out[:, 4] = P[r]
    out[:, 5] = np.where(P[r] > 1, multi_base[r], 0)
    return out


def check_batch(ids, slots, gl, rows, pieces, row_max=ROW_MAX, piece=PIECE):
    """One batch: ids / slots in lookup order [n]; gl the grouped positions [n]; rows [u, 4] and pieces [P, 8] the
    batch's records.  Raises AssertionError naming the clause that fails."""
    n = len(ids)
    rows = np.asarray(rows).view(np.uint32).reshape(-1, 4)
    pieces = np.asarray(pieces).view(np.uint32).reshape(-1, 8)
    assert len(gl) == n
    if n == 0:
        assert len(rows) == 0 and len(pieces) == 0
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
    first = np.ones(n, dtype=bool)                      # first grouped lookup of its row
    first[1:] = step != 0
    row_start = np.flatnonzero(first)
    row_count = np.diff(np.append(row_start, n))
    assert len(rows) == len(row_start), "one row record per distinct row"
    assert np.array_equal((rows[:, 0] & POS).astype(np.int64), row_start), "row starts"
    assert np.array_equal(rows[:, 1].astype(np.int64), row_count), "row counts"
    assert np.array_equal((rows[:, 0] & LONG) != 0, row_count > row_max), "long flag is not `more than ROW_MAX lookups`"
    row_slot = slots[gl64[row_start]]
    assert np.array_equal(rows[:, 2].view(np.int32), row_slot), "row slot is not the slot of the row's lookups"
    assert np.array_equal(slots[gl64], np.repeat(row_slot, row_count)), "a row's lookups do not share one slot"
    assert np.array_equal(rows[:, 3].astype(np.int64), gl64[row_start]), "first is not the row's first lookup position"
    want = _expected_pieces(row_start, row_count, row_slot, row_max, piece)
    assert pieces.shape == want.shape, f"{len(pieces)} piece records, the long rows need {len(want)}"
    multi = want[:, 4] > 1
    for col, name in enumerate(("start", "count", "slot", "index", "pieces", "partial", "reserved0", "reserved1")):
        sel = multi if name == "partial" else slice(None)
        assert np.array_equal(pieces[sel, col], want[sel, col]), f"piece records: {name}"


def check_grouping(ids, off, lookup_slots, gl, row_recs, row_off, piece_recs, piece_off, row_max=ROW_MAX, piece=PIECE,
                   n_batches=None):
    """All batches of a plan.  off: lookup offsets [T+1]; row_off (the plan's keep_offsets) / piece_off: host offsets
    into row_recs / piece_recs (they need not start at 0)."""
    T = (len(off) - 1) if n_batches is None else n_batches
    row_recs = np.asarray(row_recs).reshape(-1, 4)
    piece_recs = np.asarray(piece_recs).reshape(-1, 8)
    for i in range(T):
        a, b = int(off[i]), int(off[i + 1])
        check_batch(ids[a:b], lookup_slots[a:b], gl[a:b], row_recs[int(row_off[i]):int(row_off[i + 1])],
                    piece_recs[int(piece_off[i]):int(piece_off[i + 1])], row_max, piece)


def build_grouping(ids, off, lookup_slots, row_max=ROW_MAX, piece=PIECE):
    """A grouping that satisfies the contract, built on the host with a stable sort per batch, for tests that feed
    the grouped backward pass without running the planner.
    Returns (grouped_lookups int32 [N], row_recs int32 [rows, 4], row_off, piece_recs int32 [pieces, 8], piece_off)."""
    ids = np.asarray(ids, dtype=np.int64)
    lookup_slots = np.asarray(lookup_slots, dtype=np.int32)
    T = len(off) - 1
    gl = np.empty(len(ids), np.int32)
    rows, pieces, roff, poff = [], [], [0], [0]
    for i in range(T):
        a, b = int(off[i]), int(off[i + 1])
        n = b - a
        order = np.argsort(ids[a:b], kind="stable")
        gl[a:b] = order
        nr = npc = 0
        if n:
            gid = ids[a:b][order]
            first = np.ones(n, dtype=bool)
            first[1:] = gid[1:] != gid[:-1]
            row_start = np.flatnonzero(first)
            row_count = np.diff(np.append(row_start, n))
            row_slot = lookup_slots[a:b][order[row_start]]
            rec = np.empty((len(row_start), 4), np.uint32)
            rec[:, 0] = row_start.astype(np.uint32) | np.where(row_count > row_max, LONG, np.uint32(0))
            rec[:, 1] = row_count
            rec[:, 2] = row_slot.view(np.uint32)
            rec[:, 3] = order[row_start]
            rows.append(rec)
            pieces.append(_expected_pieces(row_start, row_count, row_slot, row_max, piece))
            nr, npc = len(rec), len(pieces[-1])
        roff.append(roff[-1] + nr)
        poff.append(poff[-1] + npc)
    cat = lambda parts, w: (np.concatenate(parts) if parts else np.zeros((0, w), np.uint32)).view(np.int32)
    return gl, cat(rows, 4), np.array(roff, np.int64), cat(pieces, 8), np.array(poff, np.int64)
