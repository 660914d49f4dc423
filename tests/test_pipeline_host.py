"""Host logic of the overlapped schedule (no GPU): which prefetches may be fetched while the previous batch
trains, and the capacity policy with reserved slots.  Checked against a slot-by-slot replay of oracle plans."""
import numpy as np
import pytest

import oracle
import workloads


def resident_slots_during(plan, T):
    """For every batch i: the set of slots holding a row while batch i trains (after its inserts, before its
    evictions), replayed from the plan's lists."""
    held, during = set(), []
    for i in range(T):
        ps = plan.prefetch_slots[plan.prefetch_off[i]:plan.prefetch_off[i + 1]]
        assert not (held & set(ps.tolist())), "a prefetch lands in a slot that is in use"
        held |= set(ps.tolist())
        during.append(set(held))
        held -= set(plan.evict_slots[plan.evict_off[i]:plan.evict_off[i + 1]].tolist())
    assert not held
    return during


def brute_early(plan, T):
    """Entry k of batch j's prefetch list is early-safe iff its slot holds no row while batch j-1 trains and its id
    is not written back after batch j-1 (so its backing row is final before batch j-1 starts)."""
    during = resident_slots_during(plan, T)
    safe = []
    for j in range(T):
        a, b = int(plan.prefetch_off[j]), int(plan.prefetch_off[j + 1])
        if j == 0:
            safe.append(np.zeros(b - a, dtype=bool))
            continue
        ev_prev = set(plan.evict_ids[plan.evict_off[j - 1]:plan.evict_off[j]].tolist())
        used_prev = set(plan.keep_ids[plan.keep_off[j - 1]:plan.keep_off[j]].tolist())
        s = np.array([int(plan.prefetch_slots[k]) not in during[j - 1] and int(plan.prefetch_ids[k]) not in ev_prev
                      and int(plan.prefetch_ids[k]) not in used_prev for k in range(a, b)], dtype=bool)
        safe.append(s)
    return safe


def random_trace(seed):
    rng = np.random.default_rng(seed)
    R = int(rng.integers(20, 300))
    T = int(rng.integers(3, 30))
    lens = rng.integers(0, 120, size=T)
    off = np.zeros(T + 1, dtype=np.int64)
    off[1:] = np.cumsum(lens)
    ids = np.minimum(rng.zipf(1.25, size=int(off[-1])) - 1, R - 1).astype(np.int64)
    return ids, off, R, T


@pytest.mark.parametrize("seed", range(12))
def test_early_counts_are_the_safe_prefix(seed):
    import paper_2202_12429_amd as bp
    ids, off, R, T = random_trace(seed)
    if len(ids) == 0:
        return
    umax = max(len(np.unique(ids[off[i]:off[i + 1]])) for i in range(T))
    for L, C, reserve in ((5, umax + 3, 0), (5, 2 * umax, umax // 2), (T, 3 * umax, umax), (2, umax + 1, 0),
                          (3, umax + 2, 1), (1, umax, 0)):
        if C - reserve < umax:
            continue
        plan = oracle.plan(ids, off, R, L, C, reserve=reserve)
        early = bp.bp_pipeline_early_counts(plan.prefetch_off, plan.evict_off, C, plan.L_eff)
        safe = brute_early(plan, T)
        for j in range(T):
            n = len(safe[j])
            assert 0 <= early[j] <= n
            if plan.L_eff >= 2:
                # exactly the safe entries, and they are a prefix of the list
                assert safe[j][:early[j]].all() and not safe[j][early[j]:].any(), (seed, L, C, reserve, j)
            else:
                assert early[j] == 0
        if plan.L_eff >= 2 and reserve >= np.diff(plan.prefetch_off).max():
            assert np.array_equal(early[1:], np.diff(plan.prefetch_off)[1:]), "a full reserve makes every prefetch early"


def test_early_counts_formula_by_hand():
    """Four batches, capacity 4: misses 3, 2, 2, 1; evictions 1, 2, 1, 3.  Ring positions 0..3 are the initial slots,
    position 4 + e is the slot of the e-th eviction.  Batch 1 pops positions 3 and 4: 3 is an initial slot (free
    while batch 0 trains), 4 is freed only after batch 0 -> one early.  Batch 2 pops 5 and 6, freed after batch 1
    -> none.  Batch 3 pops 7, the slot of the last eviction of batch 2 -> none.  With capacity 6 two more initial
    slots shift everything: 2, 2 and 1 early.  With L_eff 1 nothing is early."""
    import paper_2202_12429_amd as bp
    po = np.array([0, 3, 5, 7, 8]); eo = np.array([0, 1, 3, 4, 7])
    assert bp.bp_pipeline_early_counts(po, eo, 4, 3).tolist() == [0, 1, 0, 0]
    assert bp.bp_pipeline_early_counts(po, eo, 6, 3).tolist() == [0, 2, 2, 1]
    assert bp.bp_pipeline_early_counts(po, eo, 6, 1).tolist() == [0, 0, 0, 0]


@pytest.mark.parametrize("seed", range(6))
def test_reserve_is_the_policy_of_a_smaller_cache_on_the_full_ring(seed):
    ids, off, R, T = random_trace(100 + seed)
    if len(ids) == 0:
        return
    umax = max(len(np.unique(ids[off[i]:off[i + 1]])) for i in range(T))
    C, reserve, L = 2 * umax + 4, umax // 2 + 1, 6
    with_reserve = oracle.plan(ids, off, R, L, C, reserve=reserve)
    smaller = oracle.plan(ids, off, R, L, C - reserve)
    assert with_reserve.L_eff == smaller.L_eff and with_reserve.peak == smaller.peak <= C - reserve
    # same residency decisions (ids fetched / written back per batch), slots from the larger ring
    assert np.array_equal(with_reserve.prefetch_ids, smaller.prefetch_ids)
    assert np.array_equal(with_reserve.evict_ids, smaller.evict_ids)
    full = oracle.plan(ids, off, R, L, C, L_eff=with_reserve.L_eff)
    assert np.array_equal(with_reserve.prefetch_slots, full.prefetch_slots)
    assert np.array_equal(with_reserve.lookup_slots, full.lookup_slots)
    with pytest.raises(oracle.OracleError):
        oracle.plan(ids, off, R, L, umax + 3, reserve=4)


@pytest.mark.parametrize("seed", range(8))
def test_late_prefetches_take_the_evicted_slots_in_order(seed):
    """What bp_cache_apply_handoff relies on: of the prefetch list of batch i, the entries after the early ones take
    the slots of batch i-1's evictions, entry by entry in the evictions' order."""
    import paper_2202_12429_amd as bp
    ids, off, R, T = random_trace(200 + seed)
    if len(ids) == 0:
        return
    umax = max(len(np.unique(ids[off[i]:off[i + 1]])) for i in range(T))
    for L, C in ((4, umax + 2), (6, 2 * umax), (3, umax), (T, 4 * umax)):
        plan = oracle.plan(ids, off, R, L, C)
        if plan.L_eff < 2:
            continue
        early = bp.bp_pipeline_early_counts(plan.prefetch_off, plan.evict_off, C, plan.L_eff)
        for i in range(1, T):
            p = plan.prefetch_slots[plan.prefetch_off[i]:plan.prefetch_off[i + 1]]
            e = plan.evict_slots[plan.evict_off[i - 1]:plan.evict_off[i]]
            n_late = len(p) - int(early[i])
            assert 0 <= n_late <= len(e)
            assert np.array_equal(p[int(early[i]):], e[:n_late]), (seed, L, C, i)
            assert not set(p[:int(early[i])].tolist()) & set(e.tolist())


def stationary_trace(seed):
    """Batches of 100 uniform draws from a few thousand rows: the occupancy stays near its peak all along, so with a
    reserve of about one batch's misses the ring is tight and slots change hands every other batch."""
    rng = np.random.default_rng(400 + seed)
    T, B, R = 40, 100, int(rng.integers(600, 3000))
    off = np.arange(T + 1, dtype=np.int64) * B
    return rng.integers(0, R, size=T * B).astype(np.int64), off, R, T


@pytest.mark.parametrize("seed", range(6))
def test_early_prefetches_two_batches_on_take_the_evicted_slots_in_order(seed):
    """What the overlapped schedule's one-launch step relies on: when batch i+1 has no late prefetches, the early
    prefetches of batch i+2 are, in list order, first those whose slot has been free since before batch i ended
    (capacity + evictions before batch i - misses before batch i+2 of them, never negative), then entries that take
    the slots of batch i's evictions from the first one on, one by one; and none of the rows fetched is one of the
    rows written back."""
    import paper_2202_12429_amd as bp
    paired_total = 0
    for make in (stationary_trace, lambda s: random_trace(300 + s)):
        ids, off, R, T = make(seed)
        if len(ids) == 0:
            continue
        umax = max(len(np.unique(ids[off[i]:off[i + 1]])) for i in range(T))
        for C, f in ((4 * umax, 1.2), (5 * umax, 1.6), (3 * umax, 1.0), (3 * umax, 0.0)):
            base = oracle.plan(ids, off, R, T, C)
            reserve = int(f * np.median(np.diff(base.prefetch_off)[2:])) if T > 3 else 0
            try:
                plan = oracle.plan(ids, off, R, T, C, reserve=reserve)
            except oracle.OracleError:
                continue
            if plan.L_eff < 3:
                continue
            early = bp.bp_pipeline_early_counts(plan.prefetch_off, plan.evict_off, C, plan.L_eff)
            misses = np.diff(plan.prefetch_off)
            for i in range(0, T - 2):
                if misses[i + 1] - early[i + 1] != 0:
                    continue                                     # batch i+1 has late prefetches: the staged path
                a = int(plan.prefetch_off[i + 2])
                p_slots = plan.prefetch_slots[a:a + int(early[i + 2])]
                p_ids = plan.prefetch_ids[a:a + int(early[i + 2])]
                e_slots = plan.evict_slots[plan.evict_off[i]:plan.evict_off[i + 1]]
                e_ids = plan.evict_ids[plan.evict_off[i]:plan.evict_off[i + 1]]
                n_free = C + int(plan.evict_off[i]) - a
                assert n_free >= 0, (seed, C, i)
                n_free = min(n_free, len(p_slots))
                paired = len(p_slots) - n_free
                assert paired <= len(e_slots)
                assert np.array_equal(p_slots[n_free:], e_slots[:paired]), (seed, C, i)
                assert not set(p_slots[:n_free].tolist()) & set(e_slots.tolist())
                assert not set(p_ids.tolist()) & set(e_ids.tolist())
                paired_total += paired
    assert paired_total > 100          # the stationary traces do hand slots over two batches on
