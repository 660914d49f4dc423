"""Shared test drivers: the oracle's uncached / cached training loops and the GPU loop through the C ABI."""
import numpy as np
import torch

import oracle
import workloads


CAPTURE = None      # pytest's capture manager, set by conftest.py


def say(msg):
    """Progress line of a long test, written past pytest's output capture and flushed at once, so that a run of
    several minutes shows signs of life also without -s."""
    if CAPTURE is not None:
        with CAPTURE.global_and_fixture_disabled():
            print(msg, flush=True)
    else:
        print(msg, flush=True)


def table_to_numpy(cfg, w_f32: torch.Tensor) -> np.ndarray:
    """fp32 tensor -> the oracle's storage array (fp32, or bf16 bit patterns as uint16)."""
    if cfg.weight_dtype == "bf16":
        return w_f32.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy()
    return w_f32.numpy().copy()


def oracle_codes(cfg):
    return oracle.DTYPES[cfg.weight_dtype], oracle.OPTIMIZERS[cfg.optimizer]


def _grad_host(cfg, i, bags):
    """Upstream gradient of batch i as a host array.  The generator is integer-exact, so building it on the GPU
    (when there is one) and copying it back gives the same bits as building it on the CPU, only faster."""
    dev = "cuda:0" if torch.cuda.is_available() else "cpu"
    return workloads.upstream_grad(cfg, i, bags, device=dev).cpu().numpy()


def init_table_host(cfg, chunk_rows=1 << 21):
    """The oracle's full table with the hash-defined initial weights, filled chunk by chunk (on the GPU when there
    is one: the generator is integer-exact, so the bits are the same) so that 100 GB tables never need a second
    copy or 64-bit temporaries of their full size."""
    R, D = cfg.total_rows, cfg.dim
    dev = "cuda:0" if torch.cuda.is_available() else "cpu"
    bf16 = cfg.weight_dtype == "bf16"
    W = np.empty((R, D), dtype=np.uint16 if bf16 else np.float32)
    for a in range(0, R, chunk_rows):
        b = min(R, a + chunk_rows)
        w = workloads.init_weights(cfg, a, b, device=dev)
        if bf16:
            W[a:b] = w.to(torch.bfloat16).view(torch.int16).cpu().numpy().view(np.uint16)
        else:
            W[a:b] = w.cpu().numpy()
    return W


class OracleStepper:
    """Oracle part B one batch at a time, for lockstep comparison with the GPU at sizes where keeping every
    pooled output would not fit in memory."""

    def __init__(self, cfg, trace, threads=None):
        self.cfg, self.trace = cfg, trace
        self.dt, self.op = oracle_codes(cfg)
        self.W = init_table_host(cfg)
        self.S = np.zeros(oracle.state_shape(cfg.total_rows, cfg.dim, self.op), dtype=np.float32)
        self.bags = trace.bag_offsets.shape[1] - 1
        self.threads = oracle.host_threads() if threads is None else threads

    def step(self, i, g=None):
        c = self.cfg
        g = _grad_host(c, i, self.bags) if g is None else g
        return oracle.train_iter(self.W, self.S, c.dim, self.dt, self.op, c.lr, c.eps, self.trace.iter_ids(i),
                                 self.trace.bag_offsets[i], g, threads=self.threads)


def oracle_uncached(cfg, trace, T=None, keep_outputs=True, progress=None, threads=1):
    """Oracle part B: synchronous training on the full table.  Returns (W, S, [out_i]).  threads > 1 takes the
    oracle's multi-threaded leg (bit-identical to the serial routine, tests/test_oracle_training.py)."""
    T = trace.iter_offsets.shape[0] - 1 if T is None else T
    R, D = cfg.total_rows, cfg.dim
    dt, op = oracle_codes(cfg)
    W = init_table_host(cfg)
    S = np.zeros(oracle.state_shape(R, D, op), dtype=np.float32)
    outs = []
    bags = trace.bag_offsets.shape[1] - 1
    for i in range(T):
        g = _grad_host(cfg, i, bags)
        o = oracle.train_iter(W, S, D, dt, op, cfg.lr, cfg.eps, trace.iter_ids(i), trace.bag_offsets[i], g,
                              threads=threads)
        if keep_outputs:
            outs.append(o)
        if progress is not None and (i + 1) % 20 == 0:
            progress(f"  oracle: {i + 1}/{T} batches")
    return W, S, outs


def oracle_cached(cfg, trace, plan, T=None):
    """Oracle part C: the same arithmetic through the plan and a cache array with write-backs."""
    T = trace.iter_offsets.shape[0] - 1 if T is None else T
    R, D, C = cfg.total_rows, cfg.dim, cfg.capacity
    dt, op = oracle_codes(cfg)
    W = table_to_numpy(cfg, workloads.init_weights(cfg, 0, R))
    S = np.zeros(oracle.state_shape(R, D, op), dtype=np.float32)
    cw = np.full((C, D), 0x7FC0 if dt == oracle.BF16 else np.nan, dtype=W.dtype)     # poison unfetched slots
    cs = np.full(oracle.state_shape(C, D, op), np.nan, dtype=np.float32)
    outs = []
    e_ids, e_slots = np.zeros(0, np.int64), np.zeros(0, np.int32)
    bags = trace.bag_offsets.shape[1] - 1
    for i in range(T):
        a, b = plan.prefetch_off[i], plan.prefetch_off[i + 1]
        oracle.cache_apply(cw, cs, W, S, D, dt, op, e_ids, e_slots, plan.prefetch_ids[a:b], plan.prefetch_slots[a:b])
        g = _grad_host(cfg, i, bags)
        sl = plan.lookup_slots[trace.iter_offsets[i]:trace.iter_offsets[i + 1]]
        outs.append(oracle.train_iter(cw, cs, D, dt, op, cfg.lr, cfg.eps, sl, trace.bag_offsets[i], g))
        a, b = plan.evict_off[i], plan.evict_off[i + 1]
        e_ids, e_slots = plan.evict_ids[a:b], plan.evict_slots[a:b]
    oracle.cache_apply(cw, cs, W, S, D, dt, op, e_ids, e_slots, np.zeros(0, np.int64), np.zeros(0, np.int32))
    return W, S, outs


# ---------------------------------------------------------------------------------------------------
# GPU side (imports the product package lazily so that CPU-only test runs never need it)
# ---------------------------------------------------------------------------------------------------
def bp_config_of(cfg, capacity=None, reserve=0):
    import paper_2202_12429_amd as bp
    return bp.make_config(cfg.total_rows, cfg.capacity if capacity is None else capacity, cfg.dim, cfg.weight_dtype,
                          cfg.optimizer, cfg.lookahead, cfg.lr, cfg.eps, reserve=reserve)


def make_backing(cfg, pinned=True, chunk_rows=1 << 20):
    """Backing table (+ optimizer state) filled with the hash-defined initial weights.  Pinned host memory
    stands in for the embedding servers; pinned=False keeps it in HBM."""
    from paper_2202_12429_amd.runner import state_shape
    import paper_2202_12429_amd as bp
    R, D = cfg.total_rows, cfg.dim
    wdt = torch.bfloat16 if cfg.weight_dtype == "bf16" else torch.float32
    kw = dict(pin_memory=True) if pinned else dict(device="cuda:0")
    W = torch.empty((R, D), dtype=wdt, **kw)
    for a in range(0, R, chunk_rows):
        b = min(R, a + chunk_rows)
        W[a:b].copy_(workloads.init_weights(cfg, a, b, device="cuda:0").to(wdt))
    ss = state_shape(R, D, {"sgd": bp.SGD, "adagrad": bp.ADAGRAD, "adagrad_rowwise": bp.ADAGRAD_ROWWISE}[cfg.optimizer])
    S = torch.zeros(ss, dtype=torch.float32, **kw) if ss != (0,) else None
    torch.cuda.synchronize()
    return W, S


def gpu_cached_training(cfg, trace, T=None, pinned=True, capacity=None, check_outputs=None, grouping=True,
                        duplex=None, overlapped=False, reserve=0, handoff=None, pass_grad=False, ids_dev=None,
                        forward_grouped=None, slot_map=True):
    """Runs plan + T iterations of cache_apply / fwd / bwd_update + flush through the C ABI.
    check_outputs(i, out_tensor) is called after every forward (with pass_grad: check_outputs(i, out_tensor,
    grad_tensor), the batch's upstream gradient on the device).  Returns (trainer, plan, W, S).
    overlapped=True: cache maintenance runs on the library's maintenance stream (bp_pipeline_*).
    forward_grouped: the forward pass walks the plan's row records (bp_embbag_fwd_grouped) instead of the slot map;
    None: wherever that entry point applies (a plan with the grouping, bags of one lookup), so that the runs with
    grouping=False and the bags of several lookups keep bp_embbag_fwd's kernels covered.
    slot_map=False: the plan carries no slot per lookup (bags of one lookup, grouping on)."""
    from paper_2202_12429_amd.runner import CachedEmbeddingTrainer
    T = trace.iter_offsets.shape[0] - 1 if T is None else T
    bcfg = bp_config_of(cfg, capacity, reserve)
    W, S = make_backing(cfg, pinned)
    # by default the sorting backward (grouping=False) also takes the older maintenance paths, so both stay covered
    tr = CachedEmbeddingTrainer(bcfg, W, S, grouping=grouping, duplex=True if duplex is None else duplex,
                                handoff=grouping if handoff is None else handoff, slot_map=slot_map)
    if ids_dev is None:
        ids_dev = torch.from_numpy(trace.ids[:trace.iter_offsets[T]]).cuda()
    plan = tr.plan(ids_dev, trace.iter_offsets[:T + 1])
    del ids_dev
    bags = trace.bag_offsets.shape[1] - 1
    if forward_grouped is None:
        forward_grouped = bool(grouping and cfg.one_hot)
    if overlapped:
        tr.begin()
    for i in range(T):
        bo = None if cfg.one_hot else torch.from_numpy(np.ascontiguousarray(trace.bag_offsets[i])).cuda()
        g = workloads.upstream_grad(cfg, i, bags, device="cuda:0")
        if overlapped:
            tr.acquire(i)
        else:
            tr.maintain(i)
        out = tr.forward(i, bo, bags, grouped=forward_grouped)
        if check_outputs is not None and not overlapped:
            check_outputs(i, out, g) if pass_grad else check_outputs(i, out)
        tr.backward_update(i, bo, bags, g)
        if overlapped:
            tr.release(i)
            if check_outputs is not None:       # after release: the host waits here while maintenance runs on
                check_outputs(i, out, g) if pass_grad else check_outputs(i, out)
    if overlapped:
        tr.end()
    else:
        tr.flush()
    torch.cuda.synchronize()
    return tr, plan, W, S


def table_from_torch(cfg, W: torch.Tensor) -> np.ndarray:
    W = W.cpu()
    if cfg.weight_dtype == "bf16":
        return W.view(torch.int16).numpy().view(np.uint16)
    return W.numpy()


def bf16_bits_to_f32(a: np.ndarray) -> np.ndarray:
    return (a.astype(np.uint32) << 16).view(np.float32)


def _row_scale(want: np.ndarray, floor: float) -> np.ndarray:
    """Reference magnitude of every element: its own size, or the largest entry of its row (an embedding vector
    is the unit the error is relative to: an element that cancelled to ~0 inside a row of large entries carries
    the absolute rounding error of those entries), or the floor."""
    a = np.abs(want.astype(np.float64))
    return np.maximum(np.maximum(a, a.max(axis=1, keepdims=True)), floor)


def assert_outputs_close(got: np.ndarray, want: np.ndarray, max_bag: int, wmax: float = 0.05, same_table=True):
    """Pooled outputs: relative error 1e-5, taken per pooled vector: |a-b| <= 1e-5 * max(|b|, max|b_row|, floor),
    floor = wmax * sqrt(max_bag) (the size of a sum of max_bag initial weights).  The fp32 path adds the rows of a
    bag in order, so its distance to the fp64-accumulated oracle is at most max_bag * 2^-24 * sum|x| — far inside
    this bar.  One-hot outputs are row copies and must match bit for bit when both sides read the same table
    (same_table=False: the tables went through earlier updates and already differ by fp32 rounding)."""
    if max_bag == 1 and same_table:
        assert np.array_equal(got, want)
        return
    diff = np.abs(got.astype(np.float64) - want.astype(np.float64))
    tol = 1e-5 * _row_scale(want, wmax * np.sqrt(max_bag))
    bad = diff > tol
    assert not bad.any(), f"{bad.sum()} outputs off, worst {diff.max()}, worst ratio {(diff / tol).max()}"


def weight_errors(got: np.ndarray, want: np.ndarray):
    """Both measures of the distance between two tables, each as a multiple of its 1e-4 bar:
      row   |a-b| / (1e-4 * max(|b|, max|b_row|, 1e-2))   an embedding vector is the unit (see _row_scale)
      elem  |a-b| / (1e-4 * max(|b|, 1e-2))               every element against its own magnitude
    Returns (worst row measure, worst elem measure, index of the worst elem measure)."""
    diff = np.abs(got.astype(np.float64) - want.astype(np.float64))
    row = float((diff / (1e-4 * _row_scale(want, 1e-2))).max())
    e = diff / (1e-4 * np.maximum(np.abs(want.astype(np.float64)), 1e-2))
    k = int(e.argmax())
    return row, float(e.flat[k]), np.unravel_index(k, e.shape)


def assert_weights_close(got: np.ndarray, want: np.ndarray, elementwise=False):
    """Final table: |a-b| <= 1e-4 * max(|b|, max|b_row|, 1e-2) element-wise.  Returns the worst error relative
    to that reference magnitude (so 1e-4 is the bound).  elementwise=True also holds every element to
    |a-b| <= 1e-4 * max(|b|, 1e-2), its own magnitude alone."""
    diff = np.abs(got.astype(np.float64) - want.astype(np.float64))
    ref = _row_scale(want, 1e-2)
    bad = diff > 1e-4 * ref
    assert not bad.any(), f"{bad.sum()} weights off, worst {diff.max()} at {np.unravel_index(diff.argmax(), diff.shape)}"
    if elementwise:
        own = np.maximum(np.abs(want.astype(np.float64)), 1e-2)
        bad = diff > 1e-4 * own
        assert not bad.any(), (f"{bad.sum()} weights off by their own magnitude, worst ratio {(diff / (1e-4 * own)).max()} "
                               f"at {np.unravel_index((diff / own).argmax(), diff.shape)}")
    return float((diff / ref).max())


def state_error(got: np.ndarray, want: np.ndarray) -> float:
    """Worst relative error of an optimizer state (entries are sums of squares, never negative)."""
    w = want.astype(np.float64)
    return float((np.abs(got.astype(np.float64) - w) / np.maximum(w, 1e-30)).max()) if w.size else 0.0
