"""Orchestration of the library calls over a planned trace (no arithmetic here).

    trainer = CachedEmbeddingTrainer(cfg, backing_w, backing_state)      # cache + workspaces in HBM
    trainer.plan(ids_dev, iter_offsets)                                  # bp_oracle_plan
    for i in range(T):
        trainer.maintain(i)                                              # bp_cache_apply(E_{i-1}, P_i)
        out = trainer.forward(i, bag_offsets_dev, bags)                  # bp_embbag_fwd
        trainer.backward_update(i, bag_offsets_dev, bags, grad_out)      # bp_embbag_bwd_update[_grouped]
    trainer.flush()                                                      # bp_cache_apply(E_{T-1}, {})

Overlapped schedule (cache maintenance on a stream of its own, beside the training step):
    trainer.begin()                                                      # bp_pipeline_create + begin
    for i in range(T):
        trainer.acquire(i); forward(i); backward_update(i); trainer.release(i)
    trainer.end()                                                        # last write-backs ordered before the caller
It needs free slots to fetch into while a batch trains: plan with cfg.reserve >= the misses of one batch.

Streaming (the trace arrives chunk by chunk; synchronous schedule):
    for every chunk: trainer.plan_chunk(ids_of_chunk_and_window_dev, offsets, n_emit)   # bp_oracle_plan_chunk
                     for k in range(n_emit): maintain(k); forward(k); backward_update(k)
    trainer.flush()

The order of calls in the first loop is the synchronous schedule of Section 3.2: the write-backs of batch i-1 are applied before
the prefetches of batch i, so a row is never fetched while an update to it is still only in the cache.
With a whole-trace plan whose L_eff >= 2, maintain() uses bp_cache_apply_handoff (one launch, no staging: the rows
that leave and the rows that enter a slot go through the same lane group; handoff=True, default); otherwise, with
duplex=True (default) and L_eff >= 2, bp_cache_apply_duplex (staging area, then writes to and reads from the backing
table in one launch); otherwise bp_cache_apply.  With grouping=True (default) the plan also lists every batch's lookups grouped by row and the backward pass
uses bp_embbag_bwd_update_grouped (no sort at run time); with grouping=False it sorts the slots itself.
"""
from __future__ import annotations

from typing import Optional

import numpy as np

from . import binding as B


def state_shape(rows: int, dim: int, optimizer: int):
    if optimizer == B.ADAGRAD:
        return (rows, dim)
    if optimizer == B.ADAGRAD_ROWWISE:
        return (rows,)
    return (0,)


class CachedEmbeddingTrainer:
    def __init__(self, cfg: B.bp_config, backing_w, backing_state=None, device="cuda:0", max_lookups: int = 0,
                 max_bags: int = 0, grouping: bool = True, duplex: bool = True, handoff: bool = True,
                 interleave: Optional[bool] = None, slot_map: bool = True):
        """slot_map=False (with grouping, bags of one lookup): the plan carries no slot per lookup and the forward pass
        walks the row records like the backward pass (bp_embbag_fwd_grouped), which saves the planner a scattering pass.
        interleave: keep a cached row's optimizer state right behind its weights, one record per slot (None: do so
        for the element-wise rule, whose state is as large as the row: a 192-byte row and its state then fill three
        whole 128-byte lines where two arrays touch four).  self.cache_w / self.cache_state are then strided views."""
        import torch
        cfg = B.bp_config.from_buffer_copy(cfg)      # the strides below are this trainer's own
        self.cfg = cfg
        self.device = torch.device(device)
        self.backing_w = backing_w
        self.backing_state = backing_state
        self.grouping = grouping
        self.slot_map = slot_map or not grouping
        self.duplex = duplex           # both link directions at once in maintain(); needs a plan with L_eff >= 2
        self.handoff = handoff         # maintenance in one launch; needs a whole-trace plan with L_eff >= 2
        self._early = None
        self._mismatch = torch.zeros(1, dtype=torch.int32, device=self.device)
        self._stage = None
        wdt = torch.float32 if cfg.weight_dtype == B.F32 else torch.bfloat16
        C, D = int(cfg.capacity), int(cfg.dim)
        ss = state_shape(C, D, cfg.optimizer)
        if interleave is None:
            interleave = cfg.optimizer == B.ADAGRAD
        if interleave and cfg.optimizer == B.ADAGRAD and cfg.weight_dtype == B.F32:
            rec = torch.zeros((C, 2 * D), dtype=torch.float32, device=self.device)      # [weights | state] per slot
            self._cache_buf = rec
            self.cache_w, self.cache_state = rec[:, :D], rec[:, D:]
            self._cw, self._cs = rec.data_ptr(), rec.data_ptr() + 4 * D                  # what the library is given
            cfg.cache_w_stride = cfg.cache_state_stride = 8 * D
        else:
            self.cache_w = torch.zeros((C, D), dtype=wdt, device=self.device)
            self.cache_state = torch.zeros(ss, dtype=torch.float32, device=self.device) if ss != (0,) else None
            self._cw, self._cs = self.cache_w, self.cache_state
        self.plan_: Optional[B.Plan] = None
        self.iter_offsets: Optional[np.ndarray] = None
        self._bwd_ws = None
        self._tickets = None           # counters of the backward pass: zeroed here once, every call leaves them zero
        self._out = None
        self._pipeline = None
        self._plan_state = None        # chunked planning: state of the cache at the last chunk boundary
        self._carried_evict = None     # evictions of the previous chunk's last batch, applied before this chunk's first
        self._n_emit = None
        if max_lookups:
            self._reserve(max_lookups, max_bags or max_lookups)

    def _reserve(self, n: int, bags: int):
        import torch
        need = max(B.bp_embbag_bwd_update_workspace_bytes(self.cfg, n, bags),
                   B.bp_embbag_bwd_update_grouped_workspace_bytes(self.cfg, n, bags, True))
        if self._bwd_ws is None or self._bwd_ws.numel() < need:
            self._bwd_ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        if self._tickets is None or self._tickets.numel() * 4 < B.bp_embbag_bwd_ticket_bytes(n):
            self._tickets = B.bwd_tickets(n, device=self.device)
        if self._out is None or self._out.shape[0] < bags:
            self._out = torch.empty((bags, int(self.cfg.dim)), dtype=torch.float32, device=self.device)

    # ---- (1)
    def plan(self, ids_dev, iter_offsets, list_capacity: Optional[int] = None, workspace=None) -> B.Plan:
        self.iter_offsets = np.ascontiguousarray(iter_offsets, dtype=np.int64)
        self._n_emit, self._plan_state, self._carried_evict = None, None, None
        self.plan_ = B.bp_oracle_plan(self.cfg, ids_dev, self.iter_offsets, list_capacity=list_capacity,
                                      workspace=workspace, grouping=self.grouping, slot_map=self.slot_map)
        self.close()
        self._early = None
        if self.handoff and self.plan_.L_eff >= 2:
            self._early = B.bp_pipeline_early_counts(self.plan_.prefetch_offsets, self.plan_.evict_offsets,
                                                     int(self.cfg.capacity), self.plan_.L_eff)
        if self.plan_.L_eff >= 2:
            import torch
            most = int(np.diff(self.plan_.evict_offsets).max()) if len(self.plan_.evict_offsets) > 1 else 0
            need = B.bp_cache_apply_duplex_workspace_bytes(self.cfg, most)
            if self._stage is None or self._stage.numel() < need:
                self._stage = torch.empty(need, dtype=torch.uint8, device=self.device)
        return self.plan_

    def plan_chunk(self, ids_dev, iter_offsets, n_emit: int) -> B.Plan:
        """Plans the next n_emit batches of a stream (bp_oracle_plan_chunk); the batches after them in `ids_dev` are
        the lookahead window.  Batches are then addressed 0 .. n_emit-1 until the next call.  Synchronous schedule."""
        import torch
        if self.plan_ is not None and self._n_emit:
            e_ids, e_slots = self._slice("evict", self._n_emit - 1)
            self._carried_evict = (e_ids.clone(), e_slots.clone(), int(self.plan_.L_eff))
        self.close()
        self.iter_offsets = np.ascontiguousarray(iter_offsets, dtype=np.int64)
        self.plan_, self._plan_state = B.bp_oracle_plan_chunk(self.cfg, ids_dev, self.iter_offsets, n_emit,
                                                              self._plan_state, grouping=self.grouping)
        self._n_emit = n_emit
        self._early = None
        if self.plan_.L_eff >= 2:
            most = int(np.diff(self.plan_.evict_offsets).max()) if n_emit > 0 else 0
            if self._carried_evict is not None:
                most = max(most, int(self._carried_evict[0].numel()))
            need = B.bp_cache_apply_duplex_workspace_bytes(self.cfg, most)
            if self._stage is None or self._stage.numel() < need:
                self._stage = torch.empty(need, dtype=torch.uint8, device=self.device)
        return self.plan_

    def _slice(self, which: str, i: int):
        p = self.plan_
        off = getattr(p, which + "_offsets")
        a, b = int(off[i]), int(off[i + 1])
        return getattr(p, which + "_ids")[a:b], getattr(p, which + "_slots")[a:b]

    def slots(self, i: int):
        a, b = int(self.iter_offsets[i]), int(self.iter_offsets[i + 1])
        return self.plan_.lookup_slots[a:b]

    # ---- (2)
    def maintain(self, i: int, stream=None) -> None:
        e_ids, e_slots = self._slice("evict", i - 1) if i > 0 else (None, None)
        disjoint = self.plan_.L_eff >= 2          # a row evicted after batch i-1 is then not fetched for batch i
        if i == 0 and self._carried_evict is not None:
            e_ids, e_slots, l_prev = self._carried_evict
            disjoint = disjoint and l_prev >= 2    # ... under the lookahead the eviction was decided with
            self._carried_evict = None
        p_ids, p_slots = self._slice("prefetch", i)
        if self._early is not None and disjoint and not self._n_emit:
            n_early = int(self._early[i]) if i > 0 else int(p_ids.numel())
            B.bp_cache_apply_handoff(self.cfg, self._cw, self._cs, self.backing_w, self.backing_state, e_ids,
                                     e_slots, p_ids, p_slots, n_early, self._mismatch, stream=stream)
        elif self.duplex and disjoint:
            B.bp_cache_apply_duplex(self.cfg, self._cw, self._cs, self.backing_w, self.backing_state, e_ids,
                                    e_slots, p_ids, p_slots, self._stage, stream=stream)
        else:
            B.bp_cache_apply(self.cfg, self._cw, self._cs, self.backing_w, self.backing_state, e_ids,
                             e_slots, p_ids, p_slots, stream=stream)

    # ---- (2b) the same maintenance, overlapped with training
    def begin(self, stream=None) -> None:
        if self._n_emit:
            raise RuntimeError("the overlapped schedule takes whole-trace plans (plan()), not chunks (plan_chunk())")
        if self._pipeline is None:
            self._pipeline = B.bp_pipeline_create(self.cfg, self._cw, self._cs, self.backing_w,
                                                  self.backing_state, self.plan_, self._stage)
        B.bp_pipeline_begin(self._pipeline, stream)

    def acquire(self, i: int, stream=None) -> None:
        B.bp_pipeline_acquire(self._pipeline, i, stream)

    def release(self, i: int, stream=None) -> None:
        B.bp_pipeline_release(self._pipeline, i, stream)

    def end(self, stream=None) -> None:
        B.bp_pipeline_end(self._pipeline, stream)

    def close(self) -> None:
        if self._pipeline is not None:
            B.bp_pipeline_destroy(self._pipeline)
            self._pipeline = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def flush(self, stream=None) -> None:
        T = self._n_emit if self._n_emit else self.iter_offsets.shape[0] - 1
        e_ids, e_slots = self._slice("evict", T - 1)
        B.bp_cache_apply(self.cfg, self._cw, self._cs, self.backing_w, self.backing_state, e_ids, e_slots,
                         None, None, stream=stream)
        if self._early is not None and int(self._mismatch.item()) != 0:       # synchronises
            raise RuntimeError("bp_cache_apply_handoff met a slot pairing that is not the plan's: the cache is corrupt")

    # ---- (3)
    def forward(self, i: int, bag_offsets_dev, bags: int, out=None, stream=None, grouped: Optional[bool] = None):
        """grouped: walk the plan's row records instead of a slot per lookup (bags of one lookup only); None: do so
        when the plan carries no slot map."""
        p = self.plan_
        a, b = int(self.iter_offsets[i]), int(self.iter_offsets[i + 1])
        self._reserve(b - a, bags)
        out = self._out[:bags] if out is None else out
        if (p.lookup_slots is None) if grouped is None else grouped:
            if bag_offsets_dev is not None:
                raise ValueError("the forward pass over the row records takes bags of one lookup; plan with slot_map=True")
            ka, kb = int(p.keep_offsets[i]), int(p.keep_offsets[i + 1])
            pa, pb = int(p.piece_offsets[i]), int(p.piece_offsets[i + 1])
            B.bp_embbag_fwd_grouped(self.cfg, self._cw, p.grouped_lookups[a:b], p.row_recs[ka:kb], p.piece_recs[pa:pb],
                                    bags, out, stream=stream)
        else:
            B.bp_embbag_fwd(self.cfg, self._cw, p.lookup_slots[a:b], bag_offsets_dev, bags, out, stream=stream)
        return out

    # ---- (4)
    def backward_update(self, i: int, bag_offsets_dev, bags: int, grad_out, stream=None, grouped: Optional[bool] = None) -> None:
        p = self.plan_
        a, b = int(self.iter_offsets[i]), int(self.iter_offsets[i + 1])
        self._reserve(b - a, bags)
        use_grouped = (p.grouped_lookups is not None) if grouped is None else grouped
        if use_grouped:
            if b == a:
                return
            ka, kb = int(p.keep_offsets[i]), int(p.keep_offsets[i + 1])       # a batch's rows are its keep-list entries
            pa, pb = int(p.piece_offsets[i]), int(p.piece_offsets[i + 1])
            B.bp_embbag_bwd_update_grouped(self.cfg, self._cw, self._cs, p.grouped_lookups[a:b],
                                           p.row_recs[ka:kb], p.piece_recs[pa:pb], bag_offsets_dev, bags, grad_out,
                                           self._bwd_ws, self._tickets, stream=stream)
        else:
            B.bp_embbag_bwd_update(self.cfg, self._cw, self._cs, p.lookup_slots[a:b], bag_offsets_dev,
                                   bags, grad_out, self._bwd_ws, self._tickets, stream=stream)
