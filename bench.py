#!/usr/bin/env python3
"""Benchmark of the embedding-access hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2]

Workload: benchmark configs[2] by default — 26 tables / 33.8 M rows, D=48 fp32, one-hot Zipf ids (top 1 % of
rows = 92 % of accesses), batch 16,384 (425,984 lookups per step), lookahead 400 over 200 batches, cache = 2 % of
the rows in HBM, element-wise Adagrad.  All inputs are seeded and synthetic.

A step is one pass of the whole hot path over one batch: cache maintenance (write back the previous batch's
evictions, load this batch's prefetches), forward (bp_embbag_fwd_grouped or bp_embbag_fwd), backward + update
(bp_embbag_bwd_update_grouped), plus the batch's share of the plan (bp_oracle_plan over the whole trace, median of 5,
timed apart).  The K steps run that whole loop, and `ms_per_step` is its time.  `value` is the metric the benchmark spec
names, forward + backward + update lookups/s: n / the median over the timed steps of the stream time between an
event before the forward call and one after the backward call, taken inside that running loop, with every input
(ids, upstream gradients, backing table) resident in HBM before the timed region starts.  Beside it:

  whole_hot_path          lookups/s of the whole step (n / ms_per_step)
  fwd_bwd_update          the details of `value` (spread over the steps, the same by the kernels' own durations)
  plan                    ids/s of bp_oracle_plan
  cache_apply             rows/s and GB/s of the cache maintenance, table in HBM and behind the host link
  pinned_host_end_to_end  the same trace with the backing table in pinned host memory (the workload as stated): whole
                          step, synchronous and overlapped (bp_pipeline_*) schedules
  roofline*               algorithmic bytes / kernel time against the 8 TB/s HBM peak: the dominant kernel, the
                          forward kernel, and forward + backward + update together (the 0.60 target)
  cpu_baseline            the CPU oracle on a bounded sample of the same workload, on the host's cores

Every run executes the same K timed steps several times: with events on every kernel (breakdown), with events on
the dominant kernel only (its duration inside the running loop), with no events (`ms_per_step`: a launch that
carries events costs a few microseconds on the host and on the stream), and with a pair of stream events around
forward + backward of every step (`value`).  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0     # MI355X HBM3E, published peak
TARGET_FRAC = 0.60        # forward + backward + update on configs[2], fraction of the HBM peak aimed at
TRAFFIC_PROFILE = os.path.join("profiles", "hbm_traffic_cfg2_pmc.txt")      # rocprofv3 --pmc summary (configs[2])
KERNEL_OF = {"bwd_reduce_update": "bwd_rows_kernel", "embbag_fwd": "embbag_fwd_onehot_kernel"}


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def algorithmic_bytes(kernel: str, n: float, bags: int, u: float, row_b: int, state_b: int, D: int, one_hot: bool) -> float:
    """Bytes the method itself has to move per launch (n lookups, u distinct rows, row_b bytes per weight row,
    state_b bytes of optimizer state per row)."""
    if kernel == "embbag_fwd":
        # slot per lookup + offsets (none for one-hot) + every distinct row once + pooled output
        return 4 * n + (0 if one_hot else 8 * (bags + 1)) + u * row_b + bags * D * 4
    if kernel == "bwd_reduce_update":
        # grouped position + slot per lookup, every distinct gradient row once (a bag's row serves all its lookups),
        # read-modify-write of every distinct row + state
        return 8 * n + min(n, bags) * D * 4 + 2 * u * (row_b + state_b)
    raise KeyError(kernel)


def cpu_model() -> str:
    """The host CPU's name as /proc/cpuinfo gives it (the oracle's figure means little without it)."""
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed steps (default: all batches after the warm-up)")
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--cpu-baseline-iters", type=int, default=100)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--value-only", action="store_true",
                    help="run only the placement and schedule `value` is quoted on (for kernel profiles: the other "
                         "runs launch the same kernels under different conditions and would blur per-kernel averages)")
    ap.add_argument("--slot-map", action="store_true",
                    help="plan with a slot per lookup and run bp_embbag_fwd on it also where every bag has one lookup "
                         "(default there: no slot map, bp_embbag_fwd_grouped walks the plan's row records)")
    ap.add_argument("--skew", type=float, default=None,
                    help="draw the ids from the skew-sensitivity law instead of Zipf: the hottest 1 %% of every "
                         "table's rows take this share of the accesses (0.01 .. 0.9)")
    ap.add_argument("--lookahead", type=int, default=None,
                    help="plan with this lookahead instead of the configuration's (the paper's sensitivity study: the "
                         "planner's rate does not depend on it, the cache the plan needs does)")
    ap.add_argument("--reserve", type=int, default=-1,
                    help="cache slots the capacity policy keeps free for fetches that overlap training "
                         "(-1: 1.5 x the median per-batch miss count of the plan without reserve)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU by design (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import workloads
    import paper_2202_12429_amd as bp
    from paper_2202_12429_amd.profile_summary import kernel_source_digest, read_traffic
    from paper_2202_12429_amd.runner import CachedEmbeddingTrainer, state_shape

    bp.load_library()                      # fails loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    cfg = workloads.CONFIGS[args.config] if args.skew is None else workloads.skew_config(args.config, args.skew)
    if args.lookahead is not None:
        import dataclasses
        cfg = dataclasses.replace(cfg, lookahead=args.lookahead)
    T = cfg.iterations
    W = max(0, min(args.warmup, T - 1))
    K = args.steps if args.steps > 0 else T - W
    if W + K > T:
        K = T - W
    bags, D = cfg.bags, cfg.dim

    t0 = time.time()
    trace = workloads.make_trace(cfg)
    log(f"trace: {trace.n_lookups} lookups in {T} batches ({time.time() - t0:.1f} s)")
    n_per_iter = np.diff(trace.iter_offsets)

    # ---- capacity: configs whose single-batch working set exceeds the stated cache get the stated cache on top of it
    capacity = cfg.capacity
    ids_dev = torch.from_numpy(trace.ids).to(dev)
    bcfg = bp.make_config(cfg.total_rows, capacity, D, cfg.weight_dtype, cfg.optimizer, cfg.lookahead, cfg.lr, cfg.eps)
    capacity_note = None
    try:
        plan = bp.bp_oracle_plan(bcfg, ids_dev, trace.iter_offsets)
    except bp.BagpipeError as e:
        if e.status != -2:
            raise
        need = int(e.info["min_capacity"])
        capacity = cfg.capacity + ((need + 1023) // 1024) * 1024
        capacity_note = (f"stated cache {cfg.capacity} < {need} unique rows of one batch; ran with "
                         f"{capacity} = stated + the batch working set rounded up to 1024")
        log(capacity_note)
        bcfg = bp.make_config(cfg.total_rows, capacity, D, cfg.weight_dtype, cfg.optimizer, cfg.lookahead, cfg.lr, cfg.eps)
        plan = bp.bp_oracle_plan(bcfg, ids_dev, trace.iter_offsets)
    # ---- reserve: free slots for the fetches that run beside the training step (the overlapped schedule)
    reserve = args.reserve
    if reserve < 0:
        # the cold start fetches far more per batch, but then the cache is far from full; what has to stay free in
        # the steady state is one typical batch's misses
        typical = int(np.median(np.diff(plan.prefetch_offsets)[1:])) if T > 1 else 0
        reserve = min(((typical * 3 // 2 + 1023) // 1024) * 1024, capacity - int(plan.min_capacity))
        reserve = max(reserve, 0)
    bcfg = bp.make_config(cfg.total_rows, capacity, D, cfg.weight_dtype, cfg.optimizer, cfg.lookahead, cfg.lr, cfg.eps,
                          reserve=reserve)
    bcfg_sync = bp.make_config(cfg.total_rows, capacity, D, cfg.weight_dtype, cfg.optimizer, cfg.lookahead, cfg.lr,
                               cfg.eps)
    del plan

    # ---- backing table in pinned host memory (stands in for the embedding servers); when the host cannot pin that
    # much (configs[4]: 102 GB) the table is built in HBM only and the pinned-host figures are left out
    t0 = time.time()
    wdt = torch.bfloat16 if cfg.weight_dtype == "bf16" else torch.float32
    ss = state_shape(cfg.total_rows, D, bcfg.optimizer)
    chunk = 1 << 21

    def fill_table(w):
        for a in range(0, cfg.total_rows, chunk):
            b = min(cfg.total_rows, a + chunk)
            w[a:b].copy_(workloads.init_weights(cfg, a, b, device=dev).to(wdt))

    try:
        backing_w = torch.empty((cfg.total_rows, D), dtype=wdt, pin_memory=True)
        backing_s = torch.zeros(ss, dtype=torch.float32, pin_memory=True) if ss != (0,) else None
        fill_table(backing_w)
        pinned_note = None
    except (RuntimeError, MemoryError) as e:
        backing_w = backing_s = None
        pinned_note = f"pinned host allocation of the backing table failed ({str(e).splitlines()[0]}); HBM placement only"
        log(pinned_note)
    torch.cuda.synchronize()
    if backing_w is not None:
        log(f"backing table: {backing_w.numel() * backing_w.element_size() / 2**30:.2f} GiB pinned"
            f"{'' if backing_s is None else f' + {backing_s.numel() * 4 / 2**30:.2f} GiB state'} ({time.time() - t0:.1f} s)")

    # ---- CPU baseline: the oracle as it stands on the first batches of the same workload.  The planner is one thread
    # by nature (a walk over the batches in order); the training iterations run on one thread and on the host's cores.
    cpu = None
    if not args.no_cpu_baseline and backing_w is not None:
        import oracle
        S_it = min(args.cpu_baseline_iters, T)
        threads = oracle.host_threads()
        dt, op = oracle.DTYPES[cfg.weight_dtype], oracle.OPTIMIZERS[cfg.optimizer]
        grads = [workloads.upstream_grad(cfg, i, bags, device=dev).cpu().numpy() for i in range(S_it)]
        n_s = int(trace.iter_offsets[S_it])

        def train(n_threads):
            Wo = (backing_w.view(torch.int16).numpy().view(np.uint16).copy() if dt == oracle.BF16 else backing_w.numpy().copy())
            So = np.zeros(oracle.state_shape(cfg.total_rows, D, op), dtype=np.float32)
            t1 = time.time()
            for i in range(S_it):
                oracle.train_iter(Wo, So, D, dt, op, cfg.lr, cfg.eps, trace.iter_ids(i), trace.bag_offsets[i], grads[i],
                                  threads=n_threads)
            return time.time() - t1
        t_train_1 = train(1)
        t_train_mt = train(threads) if threads > 1 else t_train_1
        t0 = time.time()
        oracle.plan(trace.ids[:n_s], trace.iter_offsets[:S_it + 1], cfg.total_rows, cfg.lookahead, capacity)
        t_plan = time.time() - t0
        cpu = {"value": n_s / t_train_mt, "unit": "lookups/s", "cores": threads, "kind": "oracle",
               "what": "the metric's part of the oracle: uncached forward + backward + update of the same batches "
                       "(oracle.train_iter on the whole table), on the host's cores",
               "sample": f"first {S_it} of {T} batches ({n_s} lookups): uncached forward/backward/update {t_train_mt:.1f} s on "
                         f"{threads} threads ({t_train_1:.1f} s on one); oracle plan {t_plan:.1f} s (one thread: a walk over "
                         f"the batches in order)",
               "plan_ids_per_s": n_s / t_plan, "plan_cores": 1,
               "whole_hot_path_lookups_per_s": n_s / (t_train_mt + t_plan),
               "single_thread": {"value": n_s / t_train_1, "cores": 1, "train_s": t_train_1,
                                 "whole_hot_path_lookups_per_s": n_s / (t_train_1 + t_plan)},
               "cpu_model": cpu_model(), "host_cores_visible": os.cpu_count()}
        del grads
        log(f"cpu oracle: {cpu['value']:.3g} lookups/s on {threads} threads, {cpu['single_thread']['value']:.3g} on one "
            f"({S_it} batches)")

    # ---- GPU: plan (timed), then the trace.  `value` is measured with everything resident in HBM (backing table
    # included); the same trace against the pinned-host backing table is reported as `pinned_host_end_to_end`.
    row_b = D * (2 if cfg.weight_dtype == "bf16" else 4)
    state_b = D * 4 if cfg.optimizer == "adagrad" else 4 if cfg.optimizer == "adagrad_rowwise" else 0
    backing_bytes = cfg.total_rows * (row_b + state_b)
    hbm_resident = backing_bytes < 120e9
    if backing_w is None and not hbm_resident:
        raise SystemExit("bench.py: the backing table fits neither pinned host memory nor HBM")
    if hbm_resident:
        if backing_w is not None:
            backing_w_dev = backing_w.to(dev)
            backing_s_dev = None if backing_s is None else backing_s.to(dev)
        else:
            backing_w_dev = torch.empty((cfg.total_rows, D), dtype=wdt, device=dev)
            fill_table(backing_w_dev)
            backing_s_dev = torch.zeros(ss, dtype=torch.float32, device=dev) if ss != (0,) else None

    # runs: (placement of the backing table, schedule).  The overlapped runs plan with the reserve, the synchronous ones
    # without.
    # bags of one lookup: forward and backward both walk the plan's row records, so the plan carries no slot per lookup.
    # Not where an output row is a whole number of 128-byte lines: the flat forward kernel's streaming stores are then
    # at their best and leave the L2 to the table rows (configs[4]: 2.10 against 2.07 G lookups/s)
    lean = bool(cfg.one_hot) and (D * 4) % 128 != 0 and not args.slot_map
    KERNEL_OF["embbag_fwd"] = "embbag_fwd_rows_kernel" if lean else "embbag_fwd_onehot_kernel"

    def make_trainer(cfg_, w_, s_):
        return CachedEmbeddingTrainer(cfg_, w_, s_, device=dev, max_lookups=int(n_per_iter.max()), max_bags=bags,
                                      slot_map=not lean)

    trainers = {}
    if hbm_resident:
        trainers["hbm", "overlapped"] = make_trainer(bcfg, backing_w_dev, backing_s_dev)
        trainers["hbm", "synchronous"] = make_trainer(bcfg_sync, backing_w_dev, backing_s_dev)
    if backing_w is not None:
        trainers["pinned_host", "overlapped"] = make_trainer(bcfg, backing_w, backing_s)
        trainers["pinned_host", "synchronous"] = make_trainer(bcfg_sync, backing_w, backing_s)
    main_place = "hbm" if hbm_resident else "pinned_host"
    main_sched = "synchronous" if hbm_resident else "overlapped"
    first = next(iter(trainers.values()))
    ws = torch.empty(bp.bp_oracle_plan_workspace_bytes(bcfg, trace.n_lookups, T, grouping=True), dtype=torch.uint8,
                     device=dev)
    torch.cuda.synchronize()
    plan_times = []
    for rep in range(5):
        t0 = time.perf_counter()
        first.plan(ids_dev, trace.iter_offsets, workspace=ws)       # with the grouping the backward pass consumes
        torch.cuda.synchronize()
        plan_times.append(time.perf_counter() - t0)
    plan = first.plan_
    first_sync = trainers[("pinned_host" if backing_w is not None else "hbm"), "synchronous"]
    first_sync.plan(ids_dev, trace.iter_offsets, workspace=ws)
    for (place, sched), tr_ in trainers.items():                     # one plan per schedule serves both placements
        src = first if sched == "overlapped" else first_sync
        if tr_ is not src:
            tr_.plan_, tr_.iter_offsets, tr_._stage, tr_._early = src.plan_, src.iter_offsets, src._stage, src._early
    t_plan = float(np.median(plan_times))
    t_plan_slot_map = None
    if lean:            # for the record: the same plan with a slot per lookup as well
        times = []
        for rep in range(3):
            t0 = time.perf_counter()
            bp.bp_oracle_plan(bcfg, ids_dev, trace.iter_offsets, workspace=ws, grouping=True)
            torch.cuda.synchronize()
            times.append(time.perf_counter() - t0)
        t_plan_slot_map = float(np.median(times))
    del ws
    early = bp.bp_pipeline_early_counts(plan.prefetch_offsets, plan.evict_offsets, capacity, plan.L_eff)
    log(f"plan: L_eff={plan.L_eff} (without reserve {first_sync.plan_.L_eff}) reserve={reserve} "
        f"peak={plan.peak_occupancy} pairs={plan.n_unique_pairs} prefetches={int(plan.prefetch_offsets[-1])} "
        f"early={int(early.sum())}  {t_plan * 1e3:.1f} ms ({trace.n_lookups / t_plan:.3g} ids/s)")

    # ---- plain copy of known size (1 GiB read + 1 GiB written): counter yardstick and copy ceiling of this GPU
    ca = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
    cb = torch.empty_like(ca)
    bp.bp_copy_calibration(cb, ca)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(5):
        bp.bp_copy_calibration(cb, ca)
    torch.cuda.synchronize()
    copy_gbs = 5 * 2 * ca.numel() * 4 / (time.perf_counter() - t0) / 1e9
    del ca, cb
    log(f"plain copy kernel: {copy_gbs:.0f} GB/s (read + write)")
    bracket_us = bp.bp_profile_bracket_overhead(400)
    log(f"event bracket around an empty kernel: {bracket_us:.2f} us")

    bag_off_dev = None if cfg.one_hot else [torch.from_numpy(np.ascontiguousarray(trace.bag_offsets[i])).to(dev)
                                            for i in range(T)]
    # upstream gradients resident before the timed region; beyond 16 GB the buffers are reused round-robin
    n_grad = min(W + K, max(2, int(16e9 // (bags * D * 4))))
    grads_dev = [workloads.upstream_grad(cfg, i, bags, device=dev) for i in range(n_grad)]
    out = torch.empty((bags, D), dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    # ---- randomly placed rows fetched with nothing else going on: every row of a gradient buffer once, in a random
    # order, four per lane group at a time (a different buffer per launch, so nothing is left in the caches)
    g_rows = torch.randperm(bags, device=dev, generator=torch.Generator(device=dev).manual_seed(7)).to(torch.int32)
    reps = min(40, len(grads_dev))
    bp.bp_gather_calibration(grads_dev[0], g_rows)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for r in range(reps):
        bp.bp_gather_calibration(grads_dev[r], g_rows)
    torch.cuda.synchronize()
    gather_s = (time.perf_counter() - t0) / reps

    def median_us_by_events(launch, n_launches):
        """Median duration of the yardstick's launches by the event brackets that time the kernels of the step."""
        bp.bp_profile_select(["copy_calibration"])
        bp.bp_profile_enable(True)
        for r in range(n_launches):
            launch(r)
        torch.cuda.synchronize()
        bp.bp_profile_collect()
        med = bp.profile_spread("copy_calibration")[1] * 1e3
        bp.bp_profile_enable(False)
        bp.bp_profile_select(None)
        return med
    gather_ev_us = median_us_by_events(lambda r: bp.bp_gather_calibration(grads_dev[r % reps], g_rows), 40)
    gather = {"rows": bags, "row_bytes": D * 4, "us_per_launch_wall": gather_s * 1e6, "us_per_launch_events": gather_ev_us,
              "rows_per_s": bags / gather_s,
              "GBps": bags * D * 4 / gather_s / 1e9,
              "note": "bp_gather_calibration: every row of one upstream-gradient buffer read once in random order, "
                      "us_per_launch_wall: wall clock over back-to-back launches on different buffers; us_per_launch_events: median by the event brackets that time the kernels"}
    log(f"random row gather: {bags} rows of {D * 4} B in {gather_s * 1e6:.1f} us back to back, {gather_ev_us:.1f} us by "
        f"events ({gather['GBps']:.0f} GB/s)")
    # ---- and written: every row of an output-sized buffer once, in the same random order, nothing read but the order
    s_bufs = [torch.empty((bags, D), dtype=torch.float32, device=dev) for _ in range(4)]
    bp.bp_scatter_calibration(s_bufs[0], g_rows)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for r in range(40):
        bp.bp_scatter_calibration(s_bufs[r % 4], g_rows)
    torch.cuda.synchronize()
    scatter_s = (time.perf_counter() - t0) / 40
    scatter_ev_us = median_us_by_events(lambda r: bp.bp_scatter_calibration(s_bufs[r % 4], g_rows), 40)
    del s_bufs
    scatter = {"rows": bags, "row_bytes": D * 4, "us_per_launch_wall": scatter_s * 1e6, "us_per_launch_events": scatter_ev_us,
               "rows_per_s": bags / scatter_s,
               "GBps": bags * D * 4 / scatter_s / 1e9,
               "note": "bp_scatter_calibration: every row of an output-sized buffer written once in random order, nothing "
                       "read but the order; us_per_launch_wall: wall clock over back-to-back launches on four buffers in turn; us_per_launch_events: median by the event brackets that time the kernels"}
    log(f"random row scatter: {bags} rows of {D * 4} B in {scatter_s * 1e6:.1f} us back to back, {scatter_ev_us:.1f} us by "
        f"events ({scatter['GBps']:.0f} GB/s)")
    n_timed = int(n_per_iter[W:W + K].sum())
    n_mean = n_timed / K
    u_mean = float(np.diff(first_sync.plan_.keep_offsets)[W:W + K].mean())

    def rows_moved(pl):
        return int(pl.prefetch_offsets[W + K] - pl.prefetch_offsets[W]) + \
            int(pl.evict_offsets[W + K - 1] - pl.evict_offsets[max(W - 1, 0)])
    sort_scan = ["sort_upsweep", "sort_downsweep", "scan_reduce", "scan_spine", "scan_apply"]

    def measure(trainer, overlapped, wall_events=False):
        def step(i, compute=True, ev=None):
            bo = None if bag_off_dev is None else bag_off_dev[i]
            if overlapped:
                trainer.acquire(i)
            else:
                trainer.maintain(i)
            if compute:
                if ev is not None:
                    ev[0].record()
                trainer.forward(i, bo, bags, out=out)
                trainer.backward_update(i, bo, bags, grads_dev[i % n_grad])
                if ev is not None:
                    ev[1].record()
            if overlapped:
                trainer.release(i)

        def run_pass(profile_kernels, events=None):
            """Warm-up W steps, then K timed steps.  profile_kernels: [] = every kernel carries events, a list = only
            those kernels, None = no events at all.  events: one (start, stop) pair of stream events per timed step,
            recorded around forward + backward."""
            if overlapped:
                trainer.begin()
            for i in range(W):
                step(i)
            torch.cuda.synchronize()
            bp.bp_profile_select(profile_kernels or None)
            bp.bp_profile_enable(profile_kernels is not None)
            t0 = time.perf_counter()
            for i in range(W, W + K):
                step(i, ev=None if events is None else events[i - W])
            torch.cuda.synchronize()
            dt_ = time.perf_counter() - t0
            bp.bp_profile_collect()
            prof = bp.profile_totals()
            if profile_kernels:                  # the spread of the one kernel this pass records
                prof["spread_ms"] = bp.profile_spread(profile_kernels[0])
            bp.bp_profile_enable(False)
            bp.bp_profile_select(None)
            for i in range(W + K, T):        # finish the trace: the cache drains, the next pass starts empty
                step(i, compute=False)
            if overlapped:
                trainer.end()
            else:
                trainer.flush()
            torch.cuda.synchronize()
            return dt_, prof

        # pass A: every kernel bracketed by events -> breakdown, picks the dominant HBM kernel
        _, prof_all = run_pass([])
        hot = {k: v for k, v in prof_all.items() if k in ("embbag_fwd", "bwd_reduce_update")}
        dominant = max(hot, key=lambda k: hot[k][1])
        # pass B: the same K steps with events on the dominant kernel only -> its duration inside the running loop
        t_loop_events, prof_dom = run_pass([dominant])
        # pass C: the same K steps with no events at all -> throughput.  A launch that carries events costs ~10 us more
        # on the host and ~4 us on the stream: 5 % of a configs[2] step, a quarter of a step of the small configs.
        t_loop, _ = run_pass(None)
        # pass D: a pair of stream events around forward + backward/update of every timed step -> their wall time
        fbu_wall_us = None
        if wall_events:
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(K)]
            run_pass(None, events=evs)
            fbu_wall_us = sorted(a.elapsed_time(b) * 1e3 for a, b in evs)

        def per_step(names):
            return sum(prof_all[k][1] for k in names if k in prof_all) / K

        kernel_ms = {
            "cache_apply": per_step(["cache_evict", "cache_prefetch", "cache_stage", "cache_duplex"]),   # own stream when overlapped
            "fwd": per_step(["embbag_fwd"]),
            "bwd_sort_and_records": per_step(["bwd_keys"] + sort_scan),    # zero for one-hot bags with the plan's grouping
            "bwd_reduce_update": per_step(["bwd_reduce_update"]),
        }
        t_total = t_loop + t_plan * K / T                      # the plan's share of these K batches
        return dict(t_loop=t_loop, t_loop_events=t_loop_events, t_total=t_total, dominant=dominant,
                    prof_dom=prof_dom[dominant], spread_ms=prof_dom["spread_ms"], kernel_ms=kernel_ms,
                    fbu_wall_us=fbu_wall_us)

    res = {key: measure(tr_, key[1] == "overlapped", wall_events=(key == (main_place, main_sched)))
           for key, tr_ in trainers.items() if not args.value_only or key == (main_place, main_sched)}
    # With the table in HBM every kernel of the step is HBM-bound, so running the maintenance beside the training
    # kernels moves the same bytes through the same memory and gains nothing: the synchronous schedule is the one
    # `value` reports.  With the table behind the host link the overlapped schedule hides the link time.
    m = res[main_place, main_sched]
    plan_main = first_sync.plan_ if main_sched == "synchronous" else plan
    value = n_timed / m["t_total"]
    dominant = m["dominant"]
    kernel_ms = m["kernel_ms"]

    # ---- rooflines.  Counter traffic comes from the rocprofv3 --pmc summary under profiles/ when that was taken on
    # these very kernel sources (its first line names their digest); otherwise it is null.
    digest_now = kernel_source_digest()
    prof_digest, prof_traffic = read_traffic(os.path.join(ROOT, TRAFFIC_PROFILE))
    traffic_fresh = prof_digest == digest_now and cfg.index == 2 and args.skew is None
    traffic_note = (f"{TRAFFIC_PROFILE}, kernel sources {prof_digest}" if traffic_fresh else
                    f"null: {TRAFFIC_PROFILE} was measured on kernel sources {prof_digest}, this build is {digest_now}"
                    if cfg.index == 2 and args.skew is None else f"null: {TRAFFIC_PROFILE} covers configs[2] only")

    def traffic_of(kernel):
        return prof_traffic.get(KERNEL_OF[kernel]) if traffic_fresh else None

    def roof(kernel, dur_s, extra=None):
        alg = algorithmic_bytes(kernel, n_mean, bags, u_mean, row_b, state_b if kernel != "embbag_fwd" else 0, D,
                                cfg.one_hot)
        achieved = alg / dur_s / 1e9
        traffic = traffic_of(kernel)
        r = {"bound": "hbm", "kernel": kernel, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
             "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
             "traffic_frac": (traffic / dur_s / 1e9 / HBM_PEAK_GBS) if traffic else None, "traffic_source": traffic_note,
             "algorithmic_bytes_per_launch": alg, "avg_launch_us": dur_s * 1e6}
        r.update(extra or {})
        return r

    launches, ms = m["prof_dom"]
    dur_s = ms * 1e-3 / launches
    roofline = roof(dominant, dur_s, {
        "launches": launches, "launch_us_min_median_max": [x * 1e3 for x in m["spread_ms"]],
        "empty_kernel_bracket_us": bracket_us, "measured_copy_GBps": copy_gbs, "random_row_gather": gather})
    roofline["frac_of_measured_copy"] = roofline["achieved"] / copy_gbs
    roofline["frac_of_random_row_gather"] = roofline["achieved"] / gather["GBps"]
    roofline_fwd = roof("embbag_fwd", kernel_ms["fwd"] * 1e-3) if kernel_ms["fwd"] > 0 else None
    if roofline_fwd is not None:
        roofline_fwd["random_row_scatter"] = scatter
        # the forward kernel's own time over the time of its stores alone, both by the same event brackets
        roofline_fwd["kernel_us_over_scatter_us"] = kernel_ms["fwd"] * 1e3 / scatter_ev_us if cfg.one_hot else None
    fbu_ms = kernel_ms["fwd"] + kernel_ms["bwd_sort_and_records"] + kernel_ms["bwd_reduce_update"]
    alg_fbu = (algorithmic_bytes("embbag_fwd", n_mean, bags, u_mean, row_b, 0, D, cfg.one_hot) +
               algorithmic_bytes("bwd_reduce_update", n_mean, bags, u_mean, row_b, state_b, D, cfg.one_hot))
    wall = m["fbu_wall_us"]
    wall_median_us = wall[len(wall) // 2] if wall else None
    tr_f, tr_b = traffic_of("embbag_fwd"), traffic_of("bwd_reduce_update")
    roofline_fbu = {
        "bound": "hbm", "kernels": "embbag_fwd + bwd (records, reduce, update)", "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "algorithmic_bytes_per_step": alg_fbu, "kernel_us_per_step": fbu_ms * 1e3,
        "achieved": alg_fbu / (fbu_ms * 1e-3) / 1e9 if fbu_ms > 0 else None,
        "frac": alg_fbu / (fbu_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if fbu_ms > 0 else None,
        "wall_us_per_step_median": wall_median_us,
        "frac_by_wall": alg_fbu / (wall_median_us * 1e-6) / 1e9 / HBM_PEAK_GBS if wall_median_us else None,
        "traffic": (tr_f + tr_b) if tr_f and tr_b else None,
        "traffic_frac": ((tr_f + tr_b) / (fbu_ms * 1e-3) / 1e9 / HBM_PEAK_GBS) if tr_f and tr_b and fbu_ms > 0 else None,
        "traffic_source": traffic_note, "target_frac": TARGET_FRAC,
        "target_met": bool(fbu_ms > 0 and alg_fbu / (fbu_ms * 1e-3) / 1e9 / HBM_PEAK_GBS >= TARGET_FRAC)}

    pin = res.get(("pinned_host", "overlapped"))
    pin_sync = res.get(("pinned_host", "synchronous"))
    moved = rows_moved(first_sync.plan_)

    def brief(r):
        return {"value": n_timed / r["t_total"], "unit": "lookups/s", "ms_per_step": r["t_total"] / K * 1e3,
                "loop_ms_per_step": r["t_loop"] / K * 1e3, "kernel_ms_per_step": r["kernel_ms"]}

    def apply_rate(r):
        s = r["kernel_ms"]["cache_apply"] * 1e-3 * K
        return {"rows_per_s": moved / s, "GBps": moved * (row_b + state_b) / s / 1e9,
                "us_per_step": r["kernel_ms"]["cache_apply"] * 1e3} if s > 0 else None

    def pinned_object():
        """Backing table in pinned host memory: both schedules measured, the faster one quoted as `value`."""
        over = dict(brief(pin), schedule="overlapped", L_eff=plan.L_eff, reserve=reserve,
                    early_prefetch_fraction=float(early[W:W + K].sum()) /
                    max(1, int(plan.prefetch_offsets[W + K] - plan.prefetch_offsets[W])))
        sync = dict(brief(pin_sync), schedule="synchronous", L_eff=first_sync.plan_.L_eff)
        best, other = (over, sync) if over["value"] >= sync["value"] else (sync, over)
        return dict(best, other_schedule=other, overlapped_over_synchronous=over["value"] / sync["value"],
                    backing_table="pinned host DRAM (the workload as stated; stands in for the embedding servers)")

    fbu_value = n_mean / (wall_median_us * 1e-6) if wall_median_us else None
    place = "HBM" if hbm_resident else "pinned host DRAM"
    result = {
        "metric": "cached EmbeddingBag fwd+bwd+update lookups/s: n / median stream time of forward + backward + update of "
                  "a step, taken inside the running loop over the whole hot path (plan, cache apply, forward, backward + "
                  f"update per batch); backing table resident in {place}",
        "value": fbu_value if fbu_value else value,
        "unit": "lookups/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": m["t_total"] / K * 1e3,
        "ms_per_step_covers": "the whole hot path of a batch: its share of bp_oracle_plan + cache apply + forward + backward "
                              "+ update (the loop the K steps run); `value` divides by the forward + backward + update "
                              "part of it, `whole_hot_path` by all of it",
        "whole_hot_path": {"value": value, "unit": "lookups/s", "ms_per_step": m["t_total"] / K * 1e3,
                           "loop_ms_per_step": m["t_loop"] / K * 1e3, "plan_share_ms_per_step": t_plan / T * 1e3,
                           "backing_table": place},
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if cfg.weight_dtype == "f32" else "bf16 storage, f32 arithmetic",
        "data": "synthetic",
        "backing_table": "HBM" if hbm_resident else "pinned host DRAM",
        "config": {"workload": f"configs[{cfg.index}] {cfg.name}: {cfg.num_tables} tables, {cfg.total_rows} rows, D={D} "
                               f"{cfg.weight_dtype}, batch {cfg.batch} ({int(n_mean)} lookups/step), {T} batches, "
                               f"lookahead {cfg.lookahead}, cache {capacity} rows, {cfg.optimizer}",
                   "backing_table": "HBM-resident for `value` and `whole_hot_path` (every input in HBM before the timed region); pinned host "
                                    "DRAM, as the workload states it, for `pinned_host_end_to_end`" if hbm_resident
                                    else "pinned host DRAM (too large to mirror in HBM)",
                   "schedule": f"`value`: {main_sched}; `pinned_host_end_to_end`: the faster of the synchronous schedule "
                               "and of cache maintenance overlapped with training on a second stream (bp_pipeline_*, "
                               "planned with `reserve` free slots); both are listed there",
                   "L_eff": plan_main.L_eff, "peak_occupancy": plan_main.peak_occupancy,
                   "capacity_note": capacity_note, "unique_rows_per_step": u_mean,
                   "kernel_sources": digest_now},
        "fwd_bwd_update": {
            "value": fbu_value, "unit": "lookups/s",
            "median_wall_us_per_step": wall_median_us,
            "wall_us_min_max": [wall[0], wall[-1]] if wall else None,
            "kernel_us_per_step": fbu_ms * 1e3,
            "by_kernel_time": n_mean / (fbu_ms * 1e-3) if fbu_ms > 0 else None,
            "protocol": "n / median over the timed steps of the stream time between an event recorded before "
                        "bp_embbag_fwd and one recorded after bp_embbag_bwd_update_grouped of the same step (launch "
                        "gaps and the events' own few microseconds included); by_kernel_time divides by the sum of the "
                        "kernels' own durations instead"},
        "plan": {"ms": t_plan * 1e3, "ids_per_s": trace.n_lookups / t_plan, "n_lookups": trace.n_lookups,
                 "slot_map": not lean,
                 "with_slot_map_ms": None if t_plan_slot_map is None else t_plan_slot_map * 1e3,
                 "note": "bp_oracle_plan over the whole trace with the grouping, host synchronisation included, median "
                         "of 5; as the step uses it: without a slot per lookup where both passes walk the row records "
                         "(slot_map false); with_slot_map_ms: the same plan with that output too"},
        "cache_apply": {"rows_moved_per_step": moved / K, "row_bytes_with_state": row_b + state_b,
                        "hbm_table": apply_rate(m),
                        "pinned_host_table": apply_rate(pin_sync) if pin_sync else None},
        "roofline": roofline,
        "roofline_fwd": roofline_fwd,
        "roofline_fwd_bwd_update": roofline_fbu,
        "cpu_baseline": cpu,
        "loop_ms_per_step": m["t_loop"] / K * 1e3,
        "loop_ms_per_step_with_events_on_dominant_kernel": m["t_loop_events"] / K * 1e3,
        "kernel_ms_per_step": kernel_ms,
        "other_schedule": None if args.value_only else dict(
            brief(res[main_place, "overlapped" if main_sched == "synchronous" else "synchronous"]),
            schedule="overlapped" if main_sched == "synchronous" else "synchronous"),
        "pinned_host_end_to_end": None if args.value_only or pin is None else pinned_object(),
        "pinned_note": pinned_note,
    }
    for tr_ in trainers.values():
        tr_.close()
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
