"""Pins for the oracle's planner (oracle part A) that do not come from the oracle itself:
the paper's worked example, a brute-force planner written from the plain definitions (next use, residency
recursion), closed-form special cases and the invariants the paper fixes."""
import collections
import itertools
import os

import numpy as np
import pytest

import oracle
import workloads


# --------------------------------------------------------------------------------------------------
# helpers
# --------------------------------------------------------------------------------------------------
def trace_from_batches(batches):
    ids = np.array([g for b in batches for g in b], dtype=np.int64)
    off = np.zeros(len(batches) + 1, dtype=np.int64)
    off[1:] = np.cumsum([len(b) for b in batches])
    return ids, off


def lists(plan, which, i):
    off = getattr(plan, which + "_off")
    a, b = int(off[i]), int(off[i + 1])
    ids = getattr(plan, which + "_ids")[a:b]
    second = getattr(plan, "keep_ttl" if which == "keep" else which + "_slots")[a:b]
    return ids, second


def brute_force_plan(batches, L, C):
    """Planner from the definitions, not from Algorithm 1's data structures.

    next_use(g, i)  = min{ j > i : g in U_j }                     (inf if none)
    kept(g, i, L')  = next_use(g, i) <= i + L' - 1                 (g in U_i stays cached after batch i)
    resident before i = g was in some U_j, j < i, and kept at every use since the last fetch, and the uses chain
    ttl(g, i, L')   = max{ j in [i, min(i+L'-1, T-1)] : g in U_j }
    """
    T = len(batches)
    U = [sorted(set(b)) for b in batches]

    def next_use(g, i):
        for j in range(i + 1, T):
            if g in U[j]:
                return j
        return None

    def simulate(Lp):
        resident = set()
        occ, P, E, K = [], [], [], []
        for i in range(T):
            P.append([g for g in U[i] if g not in resident])
            resident |= set(U[i])
            occ.append(len(resident))
            K.append([(g, max(j for j in range(i, min(i + Lp - 1, T - 1) + 1) if g in U[j])) for g in U[i]])
            ev = []
            for g in U[i]:
                nu = next_use(g, i)
                if nu is None or nu > i + Lp - 1:
                    ev.append(g)
            E.append(ev)
            resident -= set(ev)
        assert not resident
        return occ, P, E, K

    best = None
    for Lp in range(1, L + 1):            # plain definition: largest feasible L'
        occ, P, E, K = simulate(Lp)
        if max(occ, default=0) <= C:
            best = Lp
    if best is None:
        return None
    occ, P, E, K = simulate(best)
    ring = collections.deque(range(C))
    slot = {}
    Ps, Es, S = [], [], []
    for i in range(T):
        for g in P[i]:
            slot[g] = ring.popleft()
        Ps.append([(g, slot[g]) for g in P[i]])
        S.extend(slot[g] for g in batches[i])
        Es.append([(g, slot[g]) for g in E[i]])
        for g in E[i]:
            ring.append(slot.pop(g))
    return dict(L_eff=best, occ=occ, P=Ps, E=Es, K=K, S=S)


def assert_plan_equals_brute(batches, R, L, C):
    ids, off = trace_from_batches(batches)
    ref = brute_force_plan(batches, L, C)
    if ref is None:
        with pytest.raises(oracle.OracleError) as e:
            oracle.plan(ids, off, R, L, C, exhaustive=True)
        assert e.value.code == oracle.ERR_CAPACITY
        return
    for exhaustive in (True, False):
        p = oracle.plan(ids, off, R, L, C, exhaustive=exhaustive)
        assert p.L_eff == ref["L_eff"], (batches, L, C, exhaustive)
        assert p.occ.tolist() == ref["occ"]
        assert p.lookup_slots.tolist() == ref["S"]
        for i in range(len(batches)):
            g, s = lists(p, "prefetch", i)
            assert list(zip(g.tolist(), s.tolist())) == ref["P"][i]
            g, s = lists(p, "evict", i)
            assert list(zip(g.tolist(), s.tolist())) == ref["E"][i]
            g, t = lists(p, "keep", i)
            assert list(zip(g.tolist(), t.tolist())) == ref["K"][i]


# --------------------------------------------------------------------------------------------------
# the paper's worked example
# --------------------------------------------------------------------------------------------------
def parse_golden(path):
    facts = {"batch": {}, "prefetch": {}, "ttl": {}, "evict_after": {}, "cf_batch": {}, "cf_ttl": {},
             "cf_not_evicted": {}}
    L = None
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        cf = line.startswith("counterfactual ")
        if cf:
            line = line[len("counterfactual "):]
        head, _, rest = line.partition(":")
        parts = head.split()
        if parts[0] == "lookahead":
            L = int(parts[1])
            continue
        kind, num = parts[0], int(parts[1])
        if kind == "ttl":
            val = {int(a): int(b) for a, b in (x.split("=") for x in rest.split())}
        else:
            val = [int(x) for x in rest.split()]
        key = {"batch": "cf_batch", "ttl": "cf_ttl", "not_evicted_after": "cf_not_evicted"}[kind] if cf else kind
        facts[key][num] = val
    return L, facts


def check_example(batches, L, prefetch, ttl, evict_after, not_evicted):
    ids, off = trace_from_batches(batches)
    p = oracle.plan(ids, off, total_rows=16, L=L, C=8)
    assert p.L_eff == L
    for b1, want in prefetch.items():                    # 1-based batch numbers in the paper
        g, _ = lists(p, "prefetch", b1 - 1)
        assert sorted(g.tolist()) == sorted(want), f"prefetch at batch {b1}"
    for b1, want in ttl.items():
        g, t = lists(p, "keep", b1 - 1)
        got = dict(zip(g.tolist(), (t + 1).tolist()))
        for emb, last in want.items():
            assert got[emb] == last, f"TTL of {emb} at batch {b1}"
    for b1, want in evict_after.items():
        g, _ = lists(p, "evict", b1 - 1)
        for emb in want:
            assert emb in g.tolist(), f"{emb} evicted after batch {b1}"
    for b1, embs in not_evicted.items():
        g, _ = lists(p, "evict", b1 - 1)
        for emb in embs:
            assert emb not in g.tolist()
    return p


def test_worked_example_from_paper(golden_dir):
    L, f = parse_golden(os.path.join(golden_dir, "lookahead_worked_example.txt"))
    batches = [f["batch"][k] for k in sorted(f["batch"])]
    p = check_example(batches, L, f["prefetch"], f["ttl"], f["evict_after"], {})
    # 3 is fetched once and lives in one slot from batch 1 to batch 3
    assert p.prefetch_ids.tolist().count(3) == 1
    # an embedding that is in the cache is not fetched again (batch 2 does not fetch 3)
    g, _ = lists(p, "prefetch", 1)
    assert 3 not in g.tolist()


def test_worked_example_counterfactual(golden_dir):
    L, f = parse_golden(os.path.join(golden_dir, "lookahead_worked_example.txt"))
    b = dict(f["batch"])
    b.update(f["cf_batch"])
    batches = [b[k] for k in sorted(b)]
    check_example(batches, L, {}, f["cf_ttl"], {}, f["cf_not_evicted"])


def test_window_counts_current_batch():
    """The window holds L batches *including* the current one: with L = 2 an id used at batches 1 and 3 only
    is evicted after batch 1 and fetched again at batch 3 (the reading the worked example forces)."""
    ids, off = trace_from_batches([[5], [6], [5]])
    p = oracle.plan(ids, off, 8, L=2, C=4)
    assert p.prefetch_ids.tolist() == [5, 6, 5]
    p = oracle.plan(ids, off, 8, L=3, C=4)
    assert p.prefetch_ids.tolist() == [5, 6]
    assert p.keep_ttl.tolist() == [2, 1, 2]


# --------------------------------------------------------------------------------------------------
# brute force
# --------------------------------------------------------------------------------------------------
def test_brute_force_exhaustive_tiny():
    """All traces over 3 ids, 4 iterations, batch size <= 2 (lookup order b >= a inside a batch, duplicates
    allowed), L in 1..4 and every capacity from 1 to 3."""
    ids = [0, 1, 2]
    batch_choices = [(a,) for a in ids] + [(b, a) for a in ids for b in ids if b >= a]
    n = 0
    for batches in itertools.product(batch_choices, repeat=4):
        for L in (1, 2, 3, 4):
            for C in (1, 2, 3):
                assert_plan_equals_brute([list(b) for b in batches], 3, L, C)
                n += 1
    assert n == 9 ** 4 * 12


@pytest.mark.parametrize("seed", range(40))
def test_brute_force_random(seed):
    rng = np.random.default_rng(seed)
    R = int(rng.integers(2, 40))
    T = int(rng.integers(1, 14))
    batches = []
    for _ in range(T):
        n = int(rng.integers(0, 12))                      # empty batches allowed
        # skewed ids so that reuse happens
        batches.append((rng.integers(0, R, size=n) * rng.integers(0, 2, size=n)
                        + rng.integers(0, min(R, 4), size=n)).clip(0, R - 1).tolist())
    L = int(rng.integers(1, T + 4))
    umax = max((len(set(b)) for b in batches), default=0)
    for C in sorted({max(1, umax - 1), max(1, umax), umax + 2, umax + 6, 3 * R}):
        assert_plan_equals_brute(batches, R, L, C)


# --------------------------------------------------------------------------------------------------
# closed-form special cases
# --------------------------------------------------------------------------------------------------
def small_trace(seed, R=300, T=30, n=64):
    rng = np.random.default_rng(seed)
    ids = np.minimum(rng.zipf(1.3, size=T * n) - 1, R - 1).astype(np.int64)
    off = np.arange(T + 1, dtype=np.int64) * n
    return ids, off


def test_lookahead_one_fetches_every_iteration():
    ids, off = small_trace(1)
    p = oracle.plan(ids, off, 300, L=1, C=64)
    for i in range(len(off) - 1):
        u = np.unique(ids[off[i]:off[i + 1]])
        assert np.array_equal(lists(p, "prefetch", i)[0], u)
        assert np.array_equal(lists(p, "evict", i)[0], u)
        assert np.array_equal(lists(p, "keep", i)[1], np.full(u.shape, i))


def test_unbounded_window_fetches_each_id_once():
    ids, off = small_trace(2)
    T = len(off) - 1
    nuniq = len(np.unique(ids))
    p = oracle.plan(ids, off, 300, L=T + 5, C=nuniq)
    assert p.L_eff == T + 5
    assert len(p.prefetch_ids) == nuniq and len(np.unique(p.prefetch_ids)) == nuniq
    assert len(p.evict_ids) == nuniq and len(np.unique(p.evict_ids)) == nuniq
    first = {}
    last = {}
    for i in range(T):
        for g in ids[off[i]:off[i + 1]].tolist():
            first.setdefault(g, i)
            last[g] = i
    for i in range(T):
        assert sorted(g for g in first if first[g] == i) == lists(p, "prefetch", i)[0].tolist()
        assert sorted(g for g in last if last[g] == i) == lists(p, "evict", i)[0].tolist()
    # the first C fetches take slots 0..C-1 in order (fresh FIFO ring)
    assert p.prefetch_slots.tolist() == list(range(nuniq))


def test_all_distinct_ids_never_cached():
    T, n = 7, 5
    ids = np.arange(T * n, dtype=np.int64)
    off = np.arange(T + 1, dtype=np.int64) * n
    p = oracle.plan(ids, off, T * n, L=4, C=n)
    assert p.L_eff == 4 and p.occ.tolist() == [n] * T
    assert p.keep_ttl.tolist() == np.repeat(np.arange(T), n).tolist()
    # FIFO: iteration i pops the slots pushed by iteration i-1, which were popped in order 0..n-1
    assert p.lookup_slots.tolist() == list(range(n)) * T


def test_capacity_error_reports_minimum():
    ids, off = small_trace(3)
    umax = max(len(np.unique(ids[off[i]:off[i + 1]])) for i in range(len(off) - 1))
    with pytest.raises(oracle.OracleError) as e:
        oracle.plan(ids, off, 300, L=4, C=umax - 1)
    assert e.value.code == oracle.ERR_CAPACITY and e.value.info["min_capacity"] == umax
    assert oracle.plan(ids, off, 300, L=4, C=umax).L_eff >= 1


def test_id_out_of_range():
    ids, off = trace_from_batches([[0, 5], [7]])
    with pytest.raises(oracle.OracleError) as e:
        oracle.plan(ids, off, 7, L=2, C=4)
    assert e.value.code == oracle.ERR_ID_RANGE


# --------------------------------------------------------------------------------------------------
# invariants fixed by the paper (Section 3.2, "Consistency with the Lookahead algorithm")
# --------------------------------------------------------------------------------------------------
def check_invariants(ids, off, R, L, C):
    p = oracle.plan(ids, off, R, L, C)
    T = len(off) - 1
    Le = p.L_eff
    U = [np.unique(ids[off[i]:off[i + 1]]) for i in range(T)]
    resident = {}                      # g -> slot
    free = set(range(C))
    last_evicted_at = {}
    for i in range(T):
        pg, ps = lists(p, "prefetch", i)
        # prefetch list == ids of the batch that are not resident (I6), ascending
        assert pg.tolist() == [g for g in U[i].tolist() if g not in resident]
        for g, s in zip(pg.tolist(), ps.tolist()):
            assert s in free                      # popped slots were free (I4)
            free.remove(s)
            resident[g] = s
            # no stale fetch (I7): g was not used by any of the previous L_eff-1 batches
            if g in last_evicted_at:
                assert i - last_evicted_at[g] >= Le
        assert len(set(resident.values())) == len(resident)           # injective (I4)
        assert len(resident) + len(free) == C                         # I5
        assert len(resident) == p.occ[i] <= C                         # I3
        for g in U[i].tolist():
            assert g in resident                                      # I1: every id used at i is resident
        seg = ids[off[i]:off[i + 1]]
        assert p.lookup_slots[off[i]:off[i + 1]].tolist() == [resident[g] for g in seg.tolist()]
        kg, kt = lists(p, "keep", i)
        assert np.array_equal(kg, U[i])
        eg, es = lists(p, "evict", i)
        assert eg.tolist() == [g for g, t in zip(kg.tolist(), kt.tolist()) if t == i]
        for g, t in zip(kg.tolist(), kt.tolist()):
            hi = min(i + Le - 1, T - 1)
            uses = [j for j in range(i, hi + 1) if g in U[j]]
            assert t == uses[-1]                                      # TTL = last use inside the window
        for g, s in zip(eg.tolist(), es.tolist()):
            # nothing is evicted before its last use inside the window (I2)
            for j in range(i + 1, min(i + Le - 1, T - 1) + 1):
                assert g not in U[j]
            assert resident.pop(g) == s
            free.add(s)
            last_evicted_at[g] = i
    assert not resident                                               # I9: cache drains
    return p


@pytest.mark.parametrize("seed,L,C", [(0, 5, 64), (1, 8, 90), (2, 30, 80), (3, 3, 200), (4, 40, 1000)])
def test_invariants_random(seed, L, C):
    ids, off = small_trace(seed, R=300, T=30, n=64)
    check_invariants(ids, off, 300, L, C)


def test_peak_occupancy_monotone_in_lookahead():
    ids, off = small_trace(7, R=500, T=40, n=96)
    uniq, uoff = oracle.unique_per_iter(ids, off, 500)
    peaks = [oracle.peak_occupancy(uniq, uoff, 500, Lp)[0] for Lp in range(1, 45)]
    assert all(a <= b for a, b in zip(peaks, peaks[1:]))              # I10
    assert peaks[39] == peaks[43]                                     # windows >= T are all alike
    # required cache grows sub-linearly with the lookahead (Table "Effect of increasing lookahead")
    assert peaks[19] < 2 * peaks[9] and peaks[9] < 2 * peaks[4]
    for C in (peaks[0], peaks[5], peaks[5] + 1, peaks[20], peaks[-1] + 10):
        assert oracle.choose_lookahead(uniq, uoff, 500, 44, C, exhaustive=True) == \
            oracle.choose_lookahead(uniq, uoff, 500, 44, C, exhaustive=False)


def test_tiny_config_plan_invariants():
    cfg = workloads.CONFIGS[0]
    tr = workloads.make_trace(cfg)
    p = check_invariants(tr.ids, tr.iter_offsets, cfg.total_rows, cfg.lookahead, cfg.capacity)
    assert p.L_eff == cfg.lookahead          # capacity does not bind in the tiny configuration
    # capacity binding: L_eff shrinks, occupancy still fits
    p2 = check_invariants(tr.ids, tr.iter_offsets, cfg.total_rows, cfg.lookahead, 1500)
    assert 1 <= p2.L_eff < cfg.lookahead and p2.peak <= 1500


# ---------------------------------------------------------------------------------------------------
# lookahead when none is configured (Section 4, "Automatically Calculating Lookahead")
# ---------------------------------------------------------------------------------------------------
def _auto_by_sets(ids, off, C):
    """Batches prefetched at start-up until the cache is full, with Python sets."""
    held, k = set(), 0
    for i in range(len(off) - 1):
        held |= set(ids[off[i]:off[i + 1]].tolist())
        if len(held) > C:
            break
        k = i + 1
    return k


@pytest.mark.parametrize("seed", range(8))
def test_auto_lookahead_against_sets(seed):
    rng = np.random.default_rng(900 + seed)
    R, T = int(rng.integers(10, 200)), int(rng.integers(1, 25))
    lens = rng.integers(0, 40, size=T)
    off = np.zeros(T + 1, dtype=np.int64)
    off[1:] = np.cumsum(lens)
    ids = rng.integers(0, R, size=int(off[-1])).astype(np.int64)
    uniq, uoff = oracle.unique_per_iter(ids, off, R)
    for C in (1, 3, 10, 40, R, 10 * R):
        assert oracle.auto_lookahead(uniq, uoff, R, C) == _auto_by_sets(ids, off, C), (seed, C)


def test_auto_lookahead_closed_forms():
    # all ids distinct, m per batch: floor(C / m) batches fit
    m, T = 7, 12
    ids = np.arange(m * T, dtype=np.int64)
    off = np.arange(0, m * T + 1, m, dtype=np.int64)
    uniq, uoff = oracle.unique_per_iter(ids, off, m * T)
    for C in (6, 7, 13, 14, 50, 1000):
        assert oracle.auto_lookahead(uniq, uoff, m * T, C) == min(C // m, T)
    # the same batch again and again: everything fits as soon as one batch does
    ids = np.tile(np.arange(5, dtype=np.int64), 9)
    off = np.arange(0, 46, 5, dtype=np.int64)
    uniq, uoff = oracle.unique_per_iter(ids, off, 5)
    assert oracle.auto_lookahead(uniq, uoff, 5, 5) == 9 and oracle.auto_lookahead(uniq, uoff, 5, 4) == 0


def test_plan_without_configured_lookahead():
    """L = 0: the start-up rule picks the lookahead, then the capacity policy may still lower it."""
    rng = np.random.default_rng(5)
    R, T = 120, 30
    off = np.arange(0, 20 * T + 1, 20, dtype=np.int64)
    ids = np.minimum(rng.zipf(1.3, size=20 * T) - 1, R - 1).astype(np.int64)
    uniq, uoff = oracle.unique_per_iter(ids, off, R)
    for C in (25, 40, 80, 400):
        La = oracle.auto_lookahead(uniq, uoff, R, C)
        assert La >= 1
        p = oracle.plan(ids, off, R, 0, C)
        q = oracle.plan(ids, off, R, La, C)
        assert p.L_eff == q.L_eff <= La and np.array_equal(p.lookup_slots, q.lookup_slots)
        assert p.peak <= C
    with pytest.raises(oracle.OracleError):
        oracle.plan(ids, off, R, 0, 3)                   # the first batch alone does not fit


# ---------------------------------------------------------------------------------------------------
# a lookahead that changes from batch to batch; planning a stream chunk by chunk
# ---------------------------------------------------------------------------------------------------
def _plan_varying_by_sets(ids, off, L_of, C):
    """Algorithm 1 with the window of batch i = [i, i + L_of[i] - 1], with Python sets and a deque."""
    from collections import deque
    T = len(off) - 1
    batches = [sorted(set(ids[off[i]:off[i + 1]].tolist())) for i in range(T)]
    free, slot = deque(range(C)), {}
    pre, ev, keep, occ = [], [], [], []
    for i in range(T):
        window = range(i + 1, min(T, i + L_of[i]))
        ttl = {g: max([b for b in window if g in set(batches[b])], default=i) for g in batches[i]}
        keep.append([(g, ttl[g]) for g in batches[i]])
        pre.append([])
        for g in batches[i]:
            if g not in slot:
                slot[g] = free.popleft()
                pre[-1].append((g, slot[g]))
        occ.append(len(slot))
        ev.append([])
        for g in batches[i]:
            if ttl[g] == i:
                ev[-1].append((g, slot[g]))
                free.append(slot.pop(g))
    return pre, ev, keep, occ


def _lists(plan, which, second):
    off = getattr(plan, which + "_off")
    a, b = getattr(plan, which + "_ids"), getattr(plan, second)
    return [list(zip(a[off[i]:off[i + 1]].tolist(), b[off[i]:off[i + 1]].tolist())) for i in range(len(off) - 1)]


@pytest.mark.parametrize("seed", range(6))
def test_plan_varying_against_sets(seed):
    rng = np.random.default_rng(300 + seed)
    R, T = int(rng.integers(8, 60)), int(rng.integers(2, 16))
    lens = rng.integers(0, 25, size=T)
    off = np.zeros(T + 1, dtype=np.int64)
    off[1:] = np.cumsum(lens)
    ids = np.minimum(rng.zipf(1.4, size=int(off[-1])) - 1, R - 1).astype(np.int64)
    L_of = rng.integers(1, 7, size=T).astype(np.int32)
    C = R                                                    # never dry
    p = oracle.plan_varying(ids, off, R, L_of, C)
    pre, ev, keep, occ = _plan_varying_by_sets(ids, off, L_of, C)
    assert _lists(p, "prefetch", "prefetch_slots") == pre
    assert _lists(p, "evict", "evict_slots") == ev
    assert _lists(p, "keep", "keep_ttl") == keep
    assert p.occ.tolist() == occ
    # a constant lookahead is the plan of part A
    q = oracle.plan(ids, off, R, 4, C, L_eff=4)
    r = oracle.plan_varying(ids, off, R, np.full(T, 4, np.int32), C)
    for name in ("lookup_slots", "prefetch_ids", "prefetch_slots", "evict_ids", "evict_slots", "keep_ids", "keep_ttl", "occ"):
        assert np.array_equal(getattr(q, name), getattr(r, name)), name


def test_plan_chunked_policy_small():
    """Chunks of 3 batches, capacity tight: every chunk gets the largest lookahead that fits its own batches and
    leaves the batches its decisions reach plannable; any stream whose batches fit one by one can be planned."""
    rng = np.random.default_rng(11)
    R, T, L = 80, 12, 5
    off = np.arange(0, 15 * T + 1, 15, dtype=np.int64)
    ids = np.minimum(rng.zipf(1.3, size=15 * T) - 1, R - 1).astype(np.int64)
    umax = max(len(np.unique(ids[off[i]:off[i + 1]])) for i in range(T))
    for C in (umax + 1, umax):
        p, L_of = oracle.plan_chunked(ids, off, R, L, C, 3)
        assert p.occ.max() <= C and L_of.min() >= 1 and L_of.max() <= L
        assert len(set(L_of.tolist())) > 1                         # the capacity binds somewhere
        for a in range(0, T, 3):
            assert len(set(L_of[a:a + 3].tolist())) == 1            # one lookahead per chunk
            if L_of[a] < L:                                          # one more would overflow a batch it reaches
                bigger = L_of.copy()
                bigger[a:a + 3] = L_of[a] + 1
                bigger[a + 3:] = 1
                q = oracle.plan_varying(ids, off, R, bigger, R + 1)
                assert q.occ[a:min(T, a + 3 + L - 1)].max() > C
    with pytest.raises(oracle.OracleError):                         # a batch that does not fit by itself
        oracle.plan_chunked(ids, off, R, L, umax - 1, 3)
    # ample capacity: the configured lookahead everywhere, i.e. the plan of part A
    p2, L2 = oracle.plan_chunked(ids, off, R, L, R, 3)
    assert (L2 == L).all() and np.array_equal(p2.lookup_slots, oracle.plan(ids, off, R, L, R, L_eff=L).lookup_slots)


# ---------------------------------------------------------------------------------------------------
# which logical trainer uses a row (single-trainer marking, critical / deferred shared rows)
# ---------------------------------------------------------------------------------------------------
def test_keep_owners_by_hand_and_against_sets():
    # batch 0: positions 0..5 hold ids 7 7 3 7 9 3, trainers own [0,2) [2,4) [4,6); batch 1: ids 3 3 5 5, cuts 0 2 2 4
    ids = np.array([7, 7, 3, 7, 9, 3, 3, 3, 5, 5], dtype=np.int64)
    off = np.array([0, 6, 10], dtype=np.int64)
    cuts = np.array([[0, 2, 4, 6], [0, 2, 2, 4]], dtype=np.int64)
    # keep list order: batch 0 ids 3, 7, 9; batch 1 ids 3, 5
    # id 3 in batch 0: trainers 1 and 2, used again by batch 1 -> -2; id 7: trainers 0 and 1, not in batch 1 -> -1;
    # id 9: trainer 2 alone; batch 1: id 3 trainer 0 alone, id 5 trainer 2 alone (trainer 1 owns nothing)
    assert oracle.keep_owners(ids, off, 10, cuts).tolist() == [-2, -1, 2, 0, 2]
    rng = np.random.default_rng(3)
    for _ in range(5):
        R, T, P = int(rng.integers(5, 40)), int(rng.integers(1, 8)), int(rng.integers(1, 6))
        lens = rng.integers(0, 30, size=T)
        off = np.zeros(T + 1, dtype=np.int64)
        off[1:] = np.cumsum(lens)
        ids = rng.integers(0, R, size=int(off[-1])).astype(np.int64)
        cuts = np.stack([np.concatenate([[0], np.sort(rng.integers(0, n + 1, size=P - 1)), [n]]) for n in lens]).astype(np.int64)
        got = oracle.keep_owners(ids, off, R, cuts).tolist()
        want = []
        for i in range(T):
            b = ids[off[i]:off[i + 1]]
            nxt = set(ids[off[i + 1]:off[i + 2]].tolist()) if i + 1 < T else set()
            for g in sorted(set(b.tolist())):
                ts = {int(np.searchsorted(cuts[i], p, side="right") - 1) for p in np.nonzero(b == g)[0]}
                want.append(ts.pop() if len(ts) == 1 else (-2 if g in nxt else -1))
        assert got == want
