"""ctypes front end of the CPU oracle (oracle/bagpipe_oracle.c).

TEST INFRASTRUCTURE ONLY: the product path (paper_2202_12429_amd) never imports this package; only tests,
the smoke check and the benchmark's CPU-baseline leg do.  Nothing here does arithmetic of its own:
every function allocates numpy buffers and calls the C routine of the same name.
"""
from __future__ import annotations

import ctypes
import dataclasses
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bagpipe_oracle.c")
_LIB = os.path.join(_HERE, "libbagpipe_oracle.so")

OK, ERR_ARG, ERR_CAPACITY, ERR_ID_RANGE, ERR_NOMEM, ERR_INTERNAL = 0, -1, -2, -3, -4, -5
F32, BF16 = 0, 1
SGD, ADAGRAD, ADAGRAD_ROWWISE = 0, 1, 2
DTYPES = {"f32": F32, "bf16": BF16}
OPTIMIZERS = {"sgd": SGD, "adagrad": ADAGRAD, "adagrad_rowwise": ADAGRAD_ROWWISE}


class OracleError(RuntimeError):
    def __init__(self, code, what, **info):
        super().__init__(f"oracle: {what} failed with code {code} {info if info else ''}")
        self.code = code
        self.info = info


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fused multiply-add contraction, so every operation rounds once)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
               "-Wall", "-Wextra", "-pthread", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        i64, i32, p = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
        _lib.orc_unique_per_iter.restype = i64
        _lib.orc_unique_per_iter.argtypes = [p, p, i64, i64, p, p]
        _lib.orc_peak_occupancy.restype = i64
        _lib.orc_peak_occupancy.argtypes = [p, p, i64, i64, i64, p]
        _lib.orc_plan_stream.restype = i64
        _lib.orc_plan_stream.argtypes = [p] * 4 + [i64, i64, p, i64] + [p] * 11
        _lib.orc_keep_owners.restype = i64
        _lib.orc_keep_owners.argtypes = [p, p, p, p, i64, i64, p, p]
        _lib.orc_auto_lookahead.restype = i64
        _lib.orc_auto_lookahead.argtypes = [p, p, i64, i64, i64]
        _lib.orc_choose_lookahead.restype = i64
        _lib.orc_choose_lookahead.argtypes = [p, p, i64, i64, i64, i64, i32, p]
        _lib.orc_plan.restype = i64
        _lib.orc_plan.argtypes = [p, p, p, p, i64, i64, i64, i64] + [p] * 11
        _lib.orc_train_iter.restype = i32
        _lib.orc_train_iter.argtypes = [p, p, i64, i64, i32, i32, ctypes.c_float, ctypes.c_float, p, i64, p, i64, p, p]
        _lib.orc_train_iter_mt.restype = i32
        _lib.orc_train_iter_mt.argtypes = _lib.orc_train_iter.argtypes + [i32]
        _lib.orc_cache_apply.restype = i32
        _lib.orc_cache_apply.argtypes = [p, p, p, p, i64, i64, i64, i32, i32, p, p, i64, p, p, i64]
    return _lib


def _ptr(a):
    return None if a is None else ctypes.c_void_p(a.ctypes.data)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


@dataclasses.dataclass
class Plan:
    L_eff: int
    peak: int
    occ: np.ndarray              # [T] int64, occupancy while iteration i trains
    lookup_slots: np.ndarray     # [N] int32
    prefetch_off: np.ndarray     # [T+1] int64
    prefetch_ids: np.ndarray     # int64
    prefetch_slots: np.ndarray   # int32
    evict_off: np.ndarray
    evict_ids: np.ndarray
    evict_slots: np.ndarray
    keep_off: np.ndarray
    keep_ids: np.ndarray
    keep_ttl: np.ndarray         # int32


def unique_per_iter(ids, iter_off, total_rows):
    lib = _load()
    ids, iter_off = _c(ids, np.int64), _c(iter_off, np.int64)
    T = iter_off.shape[0] - 1
    uniq = np.empty(max(1, ids.shape[0]), dtype=np.int64)
    uoff = np.empty(T + 1, dtype=np.int64)
    m = lib.orc_unique_per_iter(_ptr(ids), _ptr(iter_off), T, total_rows, _ptr(uniq), _ptr(uoff))
    if m < 0:
        raise OracleError(m, "unique_per_iter")
    return uniq[:m].copy(), uoff


def peak_occupancy(uniq, uoff, total_rows, Lp):
    lib = _load()
    T = uoff.shape[0] - 1
    occ = np.zeros(T, dtype=np.int64)
    p = lib.orc_peak_occupancy(_ptr(uniq), _ptr(uoff), T, total_rows, int(Lp), _ptr(occ))
    if p < 0:
        raise OracleError(p, "peak_occupancy")
    return int(p), occ


def choose_lookahead(uniq, uoff, total_rows, L, C, exhaustive=False):
    lib = _load()
    T = uoff.shape[0] - 1
    minc = ctypes.c_int64(0)
    r = lib.orc_choose_lookahead(_ptr(uniq), _ptr(uoff), T, total_rows, int(L), int(C), int(bool(exhaustive)),
                                 ctypes.byref(minc))
    if r < 0:
        raise OracleError(r, "choose_lookahead", min_capacity=int(minc.value))
    return int(r)


def auto_lookahead(uniq, uoff, total_rows, C) -> int:
    """Lookahead when none is configured: batches prefetched at start-up until the cache of C slots is full."""
    lib = _load()
    r = lib.orc_auto_lookahead(_ptr(uniq), _ptr(uoff), uoff.shape[0] - 1, total_rows, int(C))
    if r < 0:
        raise OracleError(r, "auto_lookahead")
    return int(r)


def plan(ids, iter_off, total_rows, L, C, exhaustive=False, L_eff=None, reserve=0) -> Plan:
    """Whole-trace lookahead plan (part A).  L_eff=None applies the capacity policy: the largest lookahead whose
    peak occupancy fits C - reserve slots (reserve > 0 keeps that many slots free, so that a batch's prefetches can
    land while the previous batch trains, Section 3.2); slots always come from the ring over all C slots."""
    lib = _load()
    ids, iter_off = _c(ids, np.int64), _c(iter_off, np.int64)
    T = iter_off.shape[0] - 1
    N = ids.shape[0]
    uniq, uoff = unique_per_iter(ids, iter_off, total_rows)
    if L_eff is None:
        if L == 0:      # no lookahead configured: the start-up rule gives it, then the capacity policy applies
            L = auto_lookahead(uniq, uoff, total_rows, C - reserve)
            if L == 0:
                raise OracleError(-2, "auto_lookahead", min_capacity=int(np.diff(uoff).max()))
        L_eff = choose_lookahead(uniq, uoff, total_rows, L, C - reserve, exhaustive)
    M = max(1, uniq.shape[0])
    occ = np.zeros(T, dtype=np.int64)
    slots = np.empty(max(1, N), dtype=np.int32)
    poff, eoff, koff = (np.zeros(T + 1, dtype=np.int64) for _ in range(3))
    pid, eid, kid = (np.empty(M, dtype=np.int64) for _ in range(3))
    ps, es, kt = (np.empty(M, dtype=np.int32) for _ in range(3))
    r = lib.orc_plan(_ptr(ids), _ptr(iter_off), _ptr(uniq), _ptr(uoff), T, total_rows, int(L_eff), int(C),
                     _ptr(occ), _ptr(slots), _ptr(poff), _ptr(pid), _ptr(ps), _ptr(eoff), _ptr(eid), _ptr(es),
                     _ptr(koff), _ptr(kid), _ptr(kt))
    if r < 0:
        raise OracleError(r, "plan")
    nk = int(koff[-1])
    return Plan(L_eff=int(L_eff), peak=int(occ.max()) if T else 0, occ=occ, lookup_slots=slots[:N],
                prefetch_off=poff, prefetch_ids=pid[:r].copy(), prefetch_slots=ps[:r].copy(),
                evict_off=eoff, evict_ids=eid[:r].copy(), evict_slots=es[:r].copy(),
                keep_off=koff, keep_ids=kid[:nk].copy(), keep_ttl=kt[:nk].copy())


def keep_owners(ids, iter_off, total_rows, cuts) -> np.ndarray:
    """Per keep-list entry: the one logical trainer that uses the row in that batch, -1 (several, not needed by the
    next batch) or -2 (several, and the next batch uses it).  cuts: int64 [T, P+1] lookup positions inside a batch."""
    lib = _load()
    ids, iter_off = _c(ids, np.int64), _c(iter_off, np.int64)
    cuts = _c(cuts, np.int64)
    T = iter_off.shape[0] - 1
    assert cuts.shape[0] == T
    uniq, uoff = unique_per_iter(ids, iter_off, total_rows)
    owner = np.empty(max(1, uniq.shape[0]), dtype=np.int32)
    r = lib.orc_keep_owners(_ptr(ids), _ptr(iter_off), _ptr(uniq), _ptr(uoff), T, cuts.shape[1] - 1, _ptr(cuts),
                            _ptr(owner))
    if r < 0:
        raise OracleError(r, "keep_owners")
    return owner[:uniq.shape[0]]


def plan_varying(ids, iter_off, total_rows, L_of, C) -> Plan:
    """Algorithm 1 with a lookahead per batch: the window of batch i is [i, i + L_of[i] - 1].  Slow, small inputs."""
    lib = _load()
    ids, iter_off = _c(ids, np.int64), _c(iter_off, np.int64)
    L_of = _c(L_of, np.int32)
    T = iter_off.shape[0] - 1
    N = ids.shape[0]
    assert L_of.shape[0] == T
    uniq, uoff = unique_per_iter(ids, iter_off, total_rows)
    M = max(1, uniq.shape[0])
    occ = np.zeros(T, dtype=np.int64)
    slots = np.empty(max(1, N), dtype=np.int32)
    poff, eoff, koff = (np.zeros(T + 1, dtype=np.int64) for _ in range(3))
    pid, eid, kid = (np.empty(M, dtype=np.int64) for _ in range(3))
    ps, es, kt = (np.empty(M, dtype=np.int32) for _ in range(3))
    r = lib.orc_plan_stream(_ptr(ids), _ptr(iter_off), _ptr(uniq), _ptr(uoff), T, total_rows, _ptr(L_of), int(C),
                            _ptr(occ), _ptr(slots), _ptr(poff), _ptr(pid), _ptr(ps), _ptr(eoff), _ptr(eid), _ptr(es),
                            _ptr(koff), _ptr(kid), _ptr(kt))
    if r < 0:
        raise OracleError(r, "plan_varying")
    nk = int(koff[-1])
    return Plan(L_eff=int(L_of.max()) if T else 0, peak=int(occ.max()) if T else 0, occ=occ, lookup_slots=slots[:N],
                prefetch_off=poff, prefetch_ids=pid[:r].copy(), prefetch_slots=ps[:r].copy(),
                evict_off=eoff, evict_ids=eid[:r].copy(), evict_slots=es[:r].copy(),
                keep_off=koff, keep_ids=kid[:nk].copy(), keep_ttl=kt[:nk].copy())


def plan_chunked(ids, iter_off, total_rows, L, C, n_emit, reserve=0):
    """The stream planned chunk by chunk (n_emit batches at a time).  Each chunk takes the largest lookahead <= L
    such that, with the earlier chunks keeping theirs and every later batch planned with a lookahead of one, no
    batch from the chunk's first to the last one its decisions can reach (L - 1 batches past the chunk) holds more
    than C - reserve rows.  So a chunk never leaves the next one a cache it cannot plan.  Returns (plan, L_of).
    Exhaustive and slow: every candidate is planned from the start of the stream."""
    iter_off = _c(iter_off, np.int64)
    T = iter_off.shape[0] - 1
    L_of = np.full(T, L, dtype=np.int32)
    for a in range(0, T, n_emit):
        b = min(T, a + n_emit)
        reach = min(T, b + L - 1)
        chosen = None
        for cand in range(L, 0, -1):
            L_of[a:b] = cand
            L_of[b:] = 1
            # occupancy does not depend on how many slots there are: count it with a ring that cannot run dry
            p = plan_varying(ids, iter_off, total_rows, L_of, total_rows + 1)
            if p.occ[a:reach].max(initial=0) <= C - reserve:
                chosen = cand
                break
        if chosen is None:
            raise OracleError(-2, "plan_chunked", chunk_start=a)
        L_of[a:b] = chosen
    return plan_varying(ids, iter_off, total_rows, L_of, C), L_of


def state_shape(rows, D, optimizer):
    if optimizer == ADAGRAD:
        return (rows, D)
    if optimizer == ADAGRAD_ROWWISE:
        return (rows,)
    return (0,)


def host_threads(limit=16) -> int:
    """Host threads the multi-threaded leg may use: the cores this process may run on, at most `limit`."""
    try:
        n = len(os.sched_getaffinity(0))
    except (AttributeError, OSError):
        n = os.cpu_count() or 1
    return max(1, min(limit, n))


def train_iter(table, state, D, dtype, optimizer, lr, eps, row_idx, bag_off, grad_out, want_out=True, threads=1):
    """One iteration of forward / backward / update on `table` in place (parts B and C).  Returns out or None.
    table: fp32 [rows, D] or uint16 (bf16 bits) [rows, D]; state: fp32 per state_shape().
    threads > 1 runs orc_train_iter_mt (same result bit for bit, see its comment); 1 is the serial routine
    that the pins run."""
    lib = _load()
    rows = table.shape[0]
    assert table.flags.c_contiguous and table.dtype == (np.float32 if dtype == F32 else np.uint16)
    assert state is None or (state.flags.c_contiguous and state.dtype == np.float32)
    row_idx, bag_off = _c(row_idx, np.int64), _c(bag_off, np.int64)
    bags = bag_off.shape[0] - 1
    out = np.empty((bags, D), dtype=np.float32) if want_out else None
    if grad_out is not None:
        grad_out = _c(grad_out, np.float32)
        assert grad_out.shape == (bags, D)
    args = (_ptr(table), _ptr(state), rows, D, dtype, optimizer, lr, eps, _ptr(row_idx), row_idx.shape[0],
            _ptr(bag_off), bags, _ptr(grad_out), _ptr(out))
    r = lib.orc_train_iter(*args) if threads <= 1 else lib.orc_train_iter_mt(*args, int(threads))
    if r != OK:
        raise OracleError(r, "train_iter")
    return out


def cache_apply(cache_w, cache_state, host_w, host_state, D, dtype, optimizer, evict_ids, evict_slots,
                prefetch_ids, prefetch_slots):
    lib = _load()
    ei, es = _c(evict_ids, np.int64), _c(evict_slots, np.int32)
    pi, ps = _c(prefetch_ids, np.int64), _c(prefetch_slots, np.int32)
    r = lib.orc_cache_apply(_ptr(cache_w), _ptr(cache_state), _ptr(host_w), _ptr(host_state), cache_w.shape[0],
                            host_w.shape[0], D, dtype, optimizer, _ptr(ei), _ptr(es), ei.shape[0], _ptr(pi),
                            _ptr(ps), pi.shape[0])
    if r != OK:
        raise OracleError(r, "cache_apply")
