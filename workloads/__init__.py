"""Seeded synthetic workloads for the embedding-access hot path.

This module only *produces inputs*: table shapes, lookup ids, bag offsets,
initial weights and upstream gradients.  It contains none of the method's
arithmetic (no planning, no pooling, no optimizer) and is the one module that
both the CPU oracle's tests and the HIP path's tests / bench may import.

The five workloads take the shapes of the paper's recommendation datasets
(Table "Dataset and their embedding tables": 26 categorical features, tens of
millions of rows, D=16 or 48; Section 2.3 "Embedding Access Patterns": ~1 % of
rows serve > 92 % of accesses, batch 16,384) and of its own skew-sensitivity
generators (Section 5.3, "Effect of Access Pattern Skew": Zipf-distributed ids, and a hot 1 % with an exponential
law over a uniform tail).
No dataset record is reproduced; every value below comes from a seeded
generator.
"""
from __future__ import annotations

import dataclasses
import math
import os
from concurrent.futures import ThreadPoolExecutor
from typing import List, Optional

import numpy as np

__all__ = [
    "Config", "Trace", "CONFIGS", "get_config", "make_trace", "table_offsets",
    "zipf_cdf", "hot_exp_cdf", "rank_cdf", "skew_config", "top_fraction_mass", "tune_zipf_exponent",
    "init_weights", "init_weights_rows", "upstream_grad", "upstream_grad_bags", "hash_u32",
]


# --------------------------------------------------------------------------
# configuration table
# --------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class Config:
    name: str
    index: int
    seed: int
    table_rows: tuple            # rows per table
    dim: int                     # D
    weight_dtype: str            # "f32" | "bf16"
    batch: int                   # samples per iteration
    iterations: int              # T
    lookahead: int               # requested lookahead (number of batches, current one included)
    capacity: int                # cache slots C
    optimizer: str               # "sgd" | "adagrad" | "adagrad_rowwise"
    lr: float
    eps: float
    zipf_s: float
    bag_min: int = 1             # bag length ~ U{bag_min..bag_max}; 1,1 = one-hot
    bag_max: int = 1
    drift_every: int = 0         # re-draw the rank->row permutation every this many iterations (0 = never)
    id_law: str = "zipf"         # "zipf": P(rank r) ~ r**-zipf_s;  "hot_exp": the skew-sensitivity law (hot_exp_cdf)
    hot_skew: float = 0.0        # "hot_exp": access probability carried by the hottest 1 % of every table's rows

    @property
    def num_tables(self) -> int:
        return len(self.table_rows)

    @property
    def total_rows(self) -> int:
        return int(sum(self.table_rows))

    @property
    def bags(self) -> int:
        return self.batch * self.num_tables

    @property
    def one_hot(self) -> bool:
        return self.bag_min == 1 and self.bag_max == 1


def table_offsets(cfg: Config) -> np.ndarray:
    """[num_tables+1] int64 prefix sum of table cardinalities: global row id = offset[t] + local row."""
    off = np.zeros(cfg.num_tables + 1, dtype=np.int64)
    np.cumsum(np.asarray(cfg.table_rows, dtype=np.int64), out=off[1:])
    return off


def _cardinalities_log_uniform(seed: int, n: int, lo: float, hi: float, total: int) -> tuple:
    """n cardinalities drawn log-uniformly in [lo, hi], rescaled so that they sum to about `total`."""
    rng = np.random.default_rng([seed, 101])
    raw = np.exp(rng.uniform(math.log(lo), math.log(hi), size=n))
    scaled = raw * (total / raw.sum())
    rows = np.clip(np.floor(scaled), lo, hi).astype(np.int64)
    return tuple(int(x) for x in rows)


def _cardinalities_log_spaced(n: int, lo: int, hi: int, total: int) -> tuple:
    """n cardinalities from lo to hi, spaced as lo*(hi/lo)**((k/(n-1))**p); p is found by bisection so that the
    sum is `total`; the rounding remainder goes to the second-largest table so min, max and the sum are exact."""
    def rows_for(p: float) -> np.ndarray:
        k = np.arange(n, dtype=np.float64) / (n - 1)
        return np.floor(lo * (hi / lo) ** (k ** p)).astype(np.int64)
    a, b = 0.05, 5.0
    for _ in range(200):
        m = 0.5 * (a + b)
        if rows_for(m).sum() > total:
            a = m          # a larger p bends the curve down
        else:
            b = m
    rows = rows_for(b)
    rows[0], rows[-1] = lo, hi
    rows[-2] += total - rows.sum()
    assert rows.sum() == total and rows.min() == lo and rows.max() == hi and rows[-2] > 0
    return tuple(int(x) for x in rows)


# Zipf exponents for configs 1 and 2 were found with tune_zipf_exponent() so that the hottest 1 % of all rows
# carry 92 % of the access probability; tests/test_workloads.py re-checks the mass.
_ZIPF_S_CFG1 = 1.1470
_ZIPF_S_CFG2 = 1.0994


def _build_configs() -> List[Config]:
    c0 = Config(name="tiny", index=0, seed=0, table_rows=(10_000,) * 8, dim=16, weight_dtype="f32", batch=256,
                iterations=50, lookahead=20, capacity=4096, optimizer="sgd", lr=0.01, eps=1e-8, zipf_s=1.2)
    rows1 = _cardinalities_log_uniform(1, 26, 10, 1e6, 3_000_000)
    c1 = Config(name="criteo_d16", index=1, seed=1, table_rows=rows1, dim=16, weight_dtype="f32", batch=16_384,
                iterations=100, lookahead=200, capacity=int(sum(rows1)) // 100, optimizer="sgd", lr=0.01,
                eps=1e-8, zipf_s=_ZIPF_S_CFG1)
    rows2 = _cardinalities_log_spaced(26, 3, 10_000_000, 33_800_000)
    c2 = Config(name="criteo_kaggle_d48", index=2, seed=2, table_rows=rows2, dim=48, weight_dtype="f32",
                batch=16_384, iterations=200, lookahead=400, capacity=int(sum(rows2)) // 50,
                optimizer="adagrad", lr=0.01, eps=1e-8, zipf_s=_ZIPF_S_CFG2)
    c3 = Config(name="multihot_d64", index=3, seed=3, table_rows=(5_000_000,) * 20, dim=64, weight_dtype="f32",
                batch=8192, iterations=100, lookahead=300, capacity=4_000_000, optimizer="sgd", lr=0.01,
                eps=1e-8, zipf_s=1.1, bag_min=1, bag_max=50)
    c4 = Config(name="large_bf16_d128", index=4, seed=4, table_rows=(10_000_000,) * 40, dim=128,
                weight_dtype="bf16", batch=32_768, iterations=300, lookahead=500, capacity=16_000_000,
                optimizer="adagrad_rowwise", lr=0.01, eps=1e-8, zipf_s=1.05, drift_every=50)
    return [c0, c1, c2, c3, c4]


CONFIGS: List[Config] = _build_configs()


def get_config(index: int, **overrides) -> Config:
    """The index-th benchmark configuration, optionally with fields replaced (e.g. fewer iterations)."""
    cfg = CONFIGS[index]
    return dataclasses.replace(cfg, **overrides) if overrides else cfg


# --------------------------------------------------------------------------
# Zipf ids
# --------------------------------------------------------------------------
def zipf_cdf(n_rows: int, s: float) -> np.ndarray:
    """float64 CDF of the bounded Zipf law P(rank r) ~ r**-s, r = 1..n_rows."""
    p = np.arange(1, n_rows + 1, dtype=np.float64) ** (-s)
    np.cumsum(p, out=p)
    p /= p[-1]
    return p


# Decay of the exponential law over the hot ranks: the hottest row is e**HOT_EXP_DECAY times as likely as the
# coldest hot row.  The paper gives the shape ("an exponential function") but no rate; this value is this build's.
HOT_EXP_DECAY = 5.0
HOT_FRACTION = 0.01


def hot_exp_cdf(n_rows: int, skew: float) -> np.ndarray:
    """float64 CDF over ranks 0..n_rows-1 of the paper's skew-sensitivity workload (Section 5.3, "Effect of Access
    Pattern Skew"): the hottest 1 % of the rows (at least one) share the probability `skew` through an
    exponentially decaying law over their rank, the other rows share 1 - skew uniformly."""
    h = max(1, int(math.ceil(HOT_FRACTION * n_rows)))
    p = np.empty(n_rows, dtype=np.float64)
    hot = np.exp(-HOT_EXP_DECAY * np.arange(h, dtype=np.float64) / h)
    if h == n_rows:
        p[:] = hot / hot.sum()
    else:
        p[:h] = hot * (skew / hot.sum())
        p[h:] = (1.0 - skew) / (n_rows - h)
    np.cumsum(p, out=p)
    p /= p[-1]
    return p


def rank_cdf(cfg: "Config", n_rows: int) -> np.ndarray:
    """CDF over the popularity ranks of a table of n_rows rows under the workload's id law."""
    if cfg.id_law == "zipf":
        return zipf_cdf(n_rows, cfg.zipf_s)
    if cfg.id_law == "hot_exp":
        return hot_exp_cdf(n_rows, cfg.hot_skew)
    raise ValueError(f"unknown id_law {cfg.id_law!r}")


def skew_config(index: int, skew: float, **overrides) -> "Config":
    """configs[index] with its ids drawn from the skew-sensitivity law instead of Zipf: the hottest 1 % of every
    table's rows take `skew` of the accesses (the paper sweeps 0.01 .. 0.90)."""
    base = CONFIGS[index]
    return dataclasses.replace(base, id_law="hot_exp", hot_skew=float(skew),
                               name=f"{base.name}_skew{int(round(skew * 100))}", **overrides)


def top_fraction_mass(table_rows, s: float, fraction: float = 0.01) -> float:
    """Access probability carried by the globally hottest `fraction` of rows when every table is sampled once per
    example with the same exponent s."""
    probs = []
    for n in table_rows:
        p = np.arange(1, n + 1, dtype=np.float64) ** (-s)
        p /= p.sum() * len(table_rows)
        probs.append(p)
    allp = np.concatenate(probs)
    k = max(1, int(math.ceil(fraction * allp.size)))
    part = np.partition(allp, allp.size - k)[allp.size - k:]
    return float(part.sum())


def tune_zipf_exponent(table_rows, target: float = 0.92, fraction: float = 0.01, tol: float = 5e-4) -> float:
    """Bisection on s so that top_fraction_mass(table_rows, s, fraction) == target (mass grows with s)."""
    lo, hi = 0.5, 3.0
    while hi - lo > 1e-5:
        mid = 0.5 * (lo + hi)
        m = top_fraction_mass(table_rows, mid, fraction)
        if abs(m - target) < tol:
            return mid
        if m < target:
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


@dataclasses.dataclass
class Trace:
    """All lookups of a run.  `ids` holds global row ids in lookup order, iterations concatenated; inside an
    iteration the bags are ordered sample-major (bag = sample * num_tables + table) and the lookups of a bag
    are consecutive.  `bag_offsets[i]` is the [bags+1] CSR of iteration i, relative to iter_offsets[i]."""
    cfg: Config
    ids: np.ndarray              # [N] int64
    iter_offsets: np.ndarray     # [T+1] int64
    bag_offsets: np.ndarray      # [T, bags+1] int64 (one shared row, broadcast, when one-hot)

    @property
    def n_lookups(self) -> int:
        return int(self.ids.shape[0])

    def iter_ids(self, i: int) -> np.ndarray:
        return self.ids[self.iter_offsets[i]:self.iter_offsets[i + 1]]


def make_trace(cfg: Config, iterations: Optional[int] = None) -> Trace:
    """Draw the lookup ids of `iterations` (default cfg.iterations) batches.

    Each (sample, table) bag holds U{bag_min..bag_max} ids; an id is a rank drawn from the workload's id law
    (Zipf(s), or the hot-1 % law of skew_config) over the table's rows,
    mapped to a row through a seeded per-table permutation (re-drawn every `drift_every` iterations to move the
    hot set).  Streams are independent per (seed, purpose, table, epoch)."""
    T = cfg.iterations if iterations is None else int(iterations)
    nt, B = cfg.num_tables, cfg.batch
    toff = table_offsets(cfg)
    bags = cfg.bags

    if cfg.one_hot:
        lens = None
        n_per_iter = np.full(T, bags, dtype=np.int64)
        bag_off = np.broadcast_to(np.arange(bags + 1, dtype=np.int64), (T, bags + 1))
    else:
        rng_len = np.random.default_rng([cfg.seed, 202])
        lens = rng_len.integers(cfg.bag_min, cfg.bag_max + 1, size=(T, B, nt), dtype=np.int64)
        bag_off = np.zeros((T, bags + 1), dtype=np.int64)
        np.cumsum(lens.reshape(T, bags), axis=1, out=bag_off[:, 1:])
        n_per_iter = bag_off[:, -1].copy()

    iter_off = np.zeros(T + 1, dtype=np.int64)
    np.cumsum(n_per_iter, out=iter_off[1:])
    ids = np.empty(int(iter_off[-1]), dtype=np.int64)

    epochs = [(0, T)] if cfg.drift_every <= 0 else [
        (a, min(a + cfg.drift_every, T)) for a in range(0, T, cfg.drift_every)]
    cdfs = {}                               # one CDF per table size (10 M rows = 80 MB), shared by the workers
    for n_rows in sorted(set(cfg.table_rows)):
        cdfs[n_rows] = rank_cdf(cfg, n_rows)

    def fill(job):
        # one (table, epoch): its stream depends on (seed, table, epoch) alone and it writes places no other job does,
        # so the trace does not depend on how the jobs are spread over threads
        t, e, a, b = job
        n_rows = cfg.table_rows[t]
        cdf = cdfs[n_rows]
        rng = np.random.default_rng([cfg.seed, 303, t, e])
        perm = rng.permutation(n_rows).astype(np.int64)
        if cfg.one_hot:
            cnt = (b - a) * B
            ranks = np.searchsorted(cdf, rng.random(cnt), side="right")
            np.minimum(ranks, n_rows - 1, out=ranks)
            g = toff[t] + perm[ranks]
            # lookup position inside iteration i: sample * nt + t
            view = ids[iter_off[a]:iter_off[b]].reshape(b - a, B, nt)
            view[:, :, t] = g.reshape(b - a, B)
        else:
            l_t = lens[a:b, :, t]                                   # [b-a, B]
            cnt = int(l_t.sum())
            ranks = np.searchsorted(cdf, rng.random(cnt), side="right")
            np.minimum(ranks, n_rows - 1, out=ranks)
            g = toff[t] + perm[ranks]
            # destination of each drawn id: start of its bag (global) + position inside the bag
            starts = (iter_off[a:b, None] + bag_off[a:b, :-1].reshape(b - a, B, nt)[:, :, t]).ravel()
            flat_l = l_t.ravel()
            first = np.cumsum(flat_l) - flat_l
            dst = np.repeat(starts - first, flat_l) + np.arange(cnt, dtype=np.int64)
            ids[dst] = g

    jobs = [(t, e, a, b) for t in range(nt) for e, (a, b) in enumerate(epochs)]
    workers = max(1, min(8, os.cpu_count() or 1, len(jobs)))
    if workers == 1 or ids.size < (1 << 22):
        for job in jobs:
            fill(job)
    else:
        with ThreadPoolExecutor(max_workers=workers) as pool:
            list(pool.map(fill, jobs))
    return Trace(cfg=cfg, ids=ids, iter_offsets=iter_off, bag_offsets=bag_off)


# --------------------------------------------------------------------------
# hash-defined weights and upstream gradients (torch ops; same bits on CPU and GPU)
# --------------------------------------------------------------------------
_M32 = 0xFFFFFFFF


def hash_u32(x):
    """32-bit avalanche mixer on the low 32 bits of an int64 torch tensor (values kept in [0, 2**32))."""
    x = x & _M32
    x = x ^ (x >> 16)
    x = (x * 0x7FEB352D) & _M32
    x = x ^ (x >> 15)
    x = (x * 0x846CA68B) & _M32
    x = x ^ (x >> 16)
    return x


def _hash_index(idx, seed: int, stream: int):
    """Hash of a 64-bit element index with a (seed, stream) key."""
    key = (seed * 0x9E3779B1 + stream * 0x85EBCA77 + 0x165667B1) & _M32
    hi = hash_u32((idx >> 32) ^ key)
    return hash_u32((idx & _M32) ^ hi ^ ((key * 0x27D4EB2F) & _M32))


def init_weights(cfg: Config, row_begin: int, row_end: int, device="cpu"):
    """Rows [row_begin, row_end) of the initial table, U(-0.05, 0.05), as a pure function of (seed, row, column).
    fp32 tensor [rows, D]; for bf16 storage the caller converts (round-to-nearest-even)."""
    import torch
    return init_weights_rows(cfg, torch.arange(row_begin, row_end, dtype=torch.int64, device=device))


def init_weights_rows(cfg: Config, rows):
    """The same initial weights for an explicit list of global rows (int64 tensor, on the device the result
    should live on)."""
    import torch
    D = cfg.dim
    device = rows.device
    idx = rows[:, None] * D + torch.arange(D, dtype=torch.int64, device=device)[None, :]
    h = _hash_index(idx, cfg.seed, 1)
    k = (h >> 9) - (1 << 22)                    # integer in [-2**22, 2**22)
    w = (k.to(torch.float32) + 0.5) * float(np.float32(0.1 * 2.0 ** -23))
    return w


def upstream_grad(cfg: Config, iteration: int, bags: int, device="cpu"):
    """Synthetic upstream gradient dOut[bags, D] of one iteration: a centred sum of twelve hashed 16-bit
    uniforms scaled by 2**-16 (unit variance, bell-shaped, every value exact in fp32)."""
    import torch
    return upstream_grad_bags(cfg, iteration, torch.arange(bags, dtype=torch.int64, device=device))


def upstream_grad_bags(cfg: Config, iteration: int, bag_index):
    """The same upstream gradient rows for an explicit list of bags (int64 tensor)."""
    import torch
    D = cfg.dim
    device = bag_index.device
    base = (bag_index[:, None] * D
            + torch.arange(D, dtype=torch.int64, device=device)[None, :])
    idx = base + (int(iteration) << 40)
    acc = torch.zeros_like(idx)
    for j in range(6):
        h = _hash_index(idx, cfg.seed, 16 + j)
        acc += (h & 0xFFFF) + (h >> 16)
    return (acc - 393210).to(torch.float32) * float(2.0 ** -16)
