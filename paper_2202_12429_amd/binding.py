"""ctypes marshalling for libbagpipe_hip.so.  One Python function per C entry point, same name."""
from __future__ import annotations

import ctypes
import dataclasses
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libbagpipe_hip.so")

F32, BF16 = 0, 1
SGD, ADAGRAD, ADAGRAD_ROWWISE = 0, 1, 2
_DTYPES = {"f32": F32, "bf16": BF16}
_OPTIMIZERS = {"sgd": SGD, "adagrad": ADAGRAD, "adagrad_rowwise": ADAGRAD_ROWWISE}


class BagpipeError(RuntimeError):
    def __init__(self, status: int, message: str, **info):
        super().__init__(f"bagpipe status {status}: {message}")
        self.status = status
        self.info = info


class bp_config(ctypes.Structure):
    _fields_ = [("total_rows", ctypes.c_int64), ("capacity", ctypes.c_int64), ("dim", ctypes.c_int32),
                ("weight_dtype", ctypes.c_int32), ("optimizer", ctypes.c_int32), ("lookahead", ctypes.c_int32),
                ("lr", ctypes.c_float), ("eps", ctypes.c_float), ("reserve", ctypes.c_int64),
                ("cache_w_stride", ctypes.c_int64), ("cache_state_stride", ctypes.c_int64)]


class _bp_plan_state(ctypes.Structure):
    _fields_ = [("n_resident", ctypes.c_int64), ("resident_ids", ctypes.c_void_p), ("ring", ctypes.c_void_p)]


class _bp_plan(ctypes.Structure):
    _fields_ = [("lookup_slots", ctypes.c_void_p), ("prefetch_ids", ctypes.c_void_p),
                ("prefetch_slots", ctypes.c_void_p), ("evict_ids", ctypes.c_void_p), ("evict_slots", ctypes.c_void_p),
                ("keep_ids", ctypes.c_void_p), ("keep_ttl", ctypes.c_void_p), ("list_capacity", ctypes.c_int64),
                ("prefetch_offsets", ctypes.c_void_p), ("evict_offsets", ctypes.c_void_p),
                ("keep_offsets", ctypes.c_void_p), ("occupancy", ctypes.c_void_p),
                ("grouped_lookups", ctypes.c_void_p), ("row_recs", ctypes.c_void_p),
                ("piece_recs", ctypes.c_void_p), ("piece_offsets", ctypes.c_void_p),
                ("trainer_cuts", ctypes.c_void_p), ("n_trainers", ctypes.c_int32), ("keep_owner", ctypes.c_void_p),
                ("L_eff", ctypes.c_int32),
                ("L_requested", ctypes.c_int32), ("peak_occupancy", ctypes.c_int64), ("min_capacity", ctypes.c_int64),
                ("n_unique_pairs", ctypes.c_int64)]


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads libbagpipe_hip.so.  torch is imported first so that the HIP runtime it ships is the one the
    library binds to (one runtime per process)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise BagpipeError(-5, f"{_LIB_PATH} is missing: build it with `python -m paper_2202_12429_amd.build` "
                               "(there is no CPU fallback)")
    import torch  # noqa: F401
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_size_t
    cfgp = ctypes.POINTER(bp_config)
    lib.bp_oracle_plan_workspace_bytes.argtypes = [cfgp, i64, i32, i32, ctypes.POINTER(sz)]
    lib.bp_oracle_plan.argtypes = [cfgp, vp, vp, i32, ctypes.POINTER(_bp_plan), vp, sz, vp]
    lib.bp_oracle_plan_chunk_workspace_bytes.argtypes = [cfgp, i64, i32, i32, ctypes.POINTER(sz)]
    lib.bp_oracle_plan_chunk.argtypes = [cfgp, vp, vp, i32, i32, ctypes.POINTER(_bp_plan_state),
                                         ctypes.POINTER(_bp_plan_state), ctypes.POINTER(_bp_plan), vp, sz, vp]
    lib.bp_cache_apply.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, i64, vp, vp, i64, vp]
    lib.bp_cache_apply_duplex_workspace_bytes.argtypes = [cfgp, i64, ctypes.POINTER(sz)]
    lib.bp_cache_apply_duplex.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, i64, vp, vp, i64, vp, sz, vp]
    lib.bp_cache_apply_handoff.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, i64, vp, vp, i64, i64, vp, vp]
    lib.bp_cache_stage.argtypes = [cfgp, vp, vp, vp, i64, vp, sz, vp]
    lib.bp_cache_apply_staged.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, i64, vp, sz, vp, vp, i64, vp]
    lib.bp_pipeline_early_counts.argtypes = [vp, vp, i32, i64, i32, vp]
    lib.bp_pipeline_create.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, sz,
                                       ctypes.POINTER(vp)]
    lib.bp_pipeline_destroy.argtypes = [vp]
    lib.bp_pipeline_early.argtypes = [vp, i32, ctypes.POINTER(i64)]
    lib.bp_pipeline_begin.argtypes = [vp, vp]
    lib.bp_pipeline_acquire.argtypes = [vp, i32, vp]
    lib.bp_pipeline_release.argtypes = [vp, i32, vp]
    lib.bp_pipeline_end.argtypes = [vp, vp]
    lib.bp_embbag_fwd.argtypes = [cfgp, vp, vp, vp, i64, i64, vp, vp]
    lib.bp_embbag_fwd_grouped.argtypes = [cfgp, vp, vp, vp, i64, vp, i64, i64, vp, vp]
    lib.bp_embbag_fwd_grouped.restype = ctypes.c_int
    lib.bp_embbag_bwd_update_workspace_bytes.argtypes = [cfgp, i64, i64, ctypes.POINTER(sz)]
    lib.bp_embbag_bwd_update.argtypes = [cfgp, vp, vp, vp, vp, i64, i64, vp, vp, sz, vp, vp]
    lib.bp_embbag_bwd_update_grouped_static.argtypes = [cfgp, vp, vp, vp, vp, i64, vp, i64, vp, i64, i64, vp, vp]
    lib.bp_embbag_bwd_update_grouped_static.restype = ctypes.c_int
    lib.bp_embbag_bwd_update_grouped_static_bytes.argtypes = [cfgp, i64, i64, i32, ctypes.POINTER(sz)]
    lib.bp_embbag_bwd_update_grouped_static_bytes.restype = ctypes.c_int
    lib.bp_embbag_bwd_update_grouped_static_max_bytes.argtypes = []
    lib.bp_embbag_bwd_update_grouped_static_max_bytes.restype = sz
    lib.bp_embbag_bwd_ticket_bytes.argtypes = [i64]
    lib.bp_embbag_bwd_ticket_bytes.restype = sz
    lib.bp_embbag_bwd_update_grouped_workspace_bytes.argtypes = [cfgp, i64, i64, i32, ctypes.POINTER(sz)]
    lib.bp_embbag_bwd_update_grouped.argtypes = [cfgp, vp, vp, vp, vp, i64, vp, i64, vp, i64, i64, vp, vp, sz, vp, vp]
    lib.bp_error_string.argtypes = [ctypes.c_int]
    lib.bp_error_string.restype = ctypes.c_char_p
    lib.bp_last_error_message.restype = ctypes.c_char_p
    lib.bp_profile_kernel_name.argtypes = [ctypes.c_int]
    lib.bp_profile_kernel_name.restype = ctypes.c_char_p
    lib.bp_profile_get.argtypes = [ctypes.c_int, ctypes.POINTER(i64), ctypes.POINTER(ctypes.c_double)]
    lib.bp_copy_calibration.argtypes = [vp, vp, sz, vp]
    lib.bp_copy_calibration.restype = ctypes.c_int
    lib.bp_gather_calibration.argtypes = [vp, vp, i64, i32, vp, i64, i32, vp]
    lib.bp_gather_calibration.restype = ctypes.c_int
    lib.bp_scatter_calibration.argtypes = [vp, i64, i32, vp, i64, i32, vp]
    lib.bp_scatter_calibration.restype = ctypes.c_int
    lib.bp_profile_bracket_overhead.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_double)]
    lib.bp_profile_bracket_overhead.restype = ctypes.c_int
    lib.bp_profile_select.argtypes = [ctypes.c_uint64]
    lib.bp_profile_select.restype = ctypes.c_int
    for name in ("bp_oracle_plan_workspace_bytes", "bp_oracle_plan", "bp_cache_apply", "bp_embbag_fwd",
                 "bp_embbag_bwd_update_workspace_bytes", "bp_embbag_bwd_update", "bp_version",
                 "bp_embbag_bwd_update_grouped_workspace_bytes", "bp_embbag_bwd_update_grouped",
                 "bp_cache_apply_duplex_workspace_bytes", "bp_cache_apply_duplex", "bp_cache_stage",
                 "bp_cache_apply_handoff",
                 "bp_cache_apply_staged", "bp_profile_enable", "bp_oracle_plan_chunk_workspace_bytes",
                 "bp_oracle_plan_chunk", "bp_pipeline_early_counts", "bp_pipeline_create",
                 "bp_pipeline_destroy", "bp_pipeline_early", "bp_pipeline_begin", "bp_pipeline_acquire",
                 "bp_pipeline_release", "bp_pipeline_end",
                 "bp_profile_collect", "bp_profile_num_kernels", "bp_profile_get"):
        getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def _check(status: int, **info):
    if status != 0:
        lib = load_library()
        msg = lib.bp_last_error_message().decode() or lib.bp_error_string(status).decode()
        raise BagpipeError(status, msg, **info)


def make_config(total_rows: int, capacity: int, dim: int, weight_dtype="f32", optimizer="sgd", lookahead: int = 1,
                lr: float = 0.01, eps: float = 1e-8, reserve: int = 0, cache_w_stride: int = 0,
                cache_state_stride: int = 0) -> bp_config:
    """cache_w_stride / cache_state_stride: bytes between consecutive rows of the cache arrays (0 = rows back to back)."""
    wd = _DTYPES[weight_dtype] if isinstance(weight_dtype, str) else int(weight_dtype)
    op = _OPTIMIZERS[optimizer] if isinstance(optimizer, str) else int(optimizer)
    return bp_config(int(total_rows), int(capacity), int(dim), wd, op, int(lookahead), float(lr), float(eps), int(reserve),
                     int(cache_w_stride), int(cache_state_stride))


def _ptr(t) -> Optional[int]:
    """Device (or pinned-host) address of a torch tensor, a raw integer address, or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_contiguous(), "tensors passed to the library must be contiguous"
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def bp_error_string(status: int) -> str:
    return load_library().bp_error_string(status).decode()


def bp_last_error_message() -> str:
    return load_library().bp_last_error_message().decode()


def bp_version() -> int:
    return load_library().bp_version()


# ---------------------------------------------------------------------------------------------------
# (1) planner
# ---------------------------------------------------------------------------------------------------
@dataclasses.dataclass
class Plan:
    """Result of bp_oracle_plan: device tensors for the lists and the slot map, host arrays for the CSR
    offsets and the occupancy curve."""
    L_eff: int
    peak_occupancy: int
    min_capacity: int
    n_unique_pairs: int
    lookup_slots: "object"       # int32 [N] device
    prefetch_ids: "object"       # int64 device
    prefetch_slots: "object"     # int32 device
    evict_ids: "object"
    evict_slots: "object"
    keep_ids: "object"
    keep_ttl: "object"
    prefetch_offsets: np.ndarray  # int64 [T+1] host
    evict_offsets: np.ndarray
    keep_offsets: np.ndarray
    occupancy: np.ndarray         # int64 [T] host
    grouped_lookups: "object" = None    # int32 [N] device (optional grouping)
    row_recs: "object" = None           # int32 [pairs, 4] device: bp_row_rec of every keep-list entry (start | long
                                        # flag, count, slot, first), CSR offsets = keep_offsets
    piece_recs: "object" = None         # int32 [pieces, 8] device: bp_piece_rec (start, count, slot, index, pieces,
                                        # partial, 0, 0), trimmed to the piece count
    piece_offsets: Optional[np.ndarray] = None  # int64 [T+1] host
    L_requested: int = 0                # configured lookahead, or the start-up rule's value when none was configured
    keep_owner: "object" = None         # int32 device, parallel to keep_ids (optional trainer marking)


BWD_ROW_MAX, BWD_PIECE = 16, 256      # BP_BWD_ROW_MAX, BP_BWD_PIECE of the C header


def piece_capacity(n_lookups: int) -> int:
    """Entries bp_plan.piece_recs must hold for n_lookups lookups (the bound the C header states)."""
    return n_lookups // (BWD_ROW_MAX + 1) + n_lookups // BWD_PIECE + 2


def bp_oracle_plan_workspace_bytes(cfg: bp_config, n_lookups: int, n_iters: int, grouping: bool = False) -> int:
    out = ctypes.c_size_t(0)
    _check(load_library().bp_oracle_plan_workspace_bytes(ctypes.byref(cfg), int(n_lookups), int(n_iters),
                                                         int(bool(grouping)), ctypes.byref(out)))
    return int(out.value)


def bp_oracle_plan(cfg: bp_config, ids, iter_offsets, list_capacity: Optional[int] = None, workspace=None,
                   stream=None, grouping: bool = False, trainer_cuts=None, slot_map: bool = True) -> Plan:
    """ids: int64 device tensor [N]; iter_offsets: int64 host array [T+1].  Output and workspace tensors are
    allocated here with torch (the library itself allocates nothing); list tensors are trimmed views.
    slot_map=False (with grouping only): no lookup_slots, for callers that walk the row records."""
    import torch
    lib = load_library()
    iter_offsets = np.ascontiguousarray(iter_offsets, dtype=np.int64)
    T = iter_offsets.shape[0] - 1
    N = int(iter_offsets[-1])
    assert ids.dtype == torch.int64 and ids.numel() == N
    dev = ids.device
    cap = N if list_capacity is None else int(list_capacity)
    if workspace is None:
        workspace = torch.empty(bp_oracle_plan_workspace_bytes(cfg, N, T, grouping), dtype=torch.uint8, device=dev)
    i32 = dict(dtype=torch.int32, device=dev)
    i64 = dict(dtype=torch.int64, device=dev)
    assert slot_map or grouping, "a plan without a slot map needs the grouping"
    t = dict(prefetch_ids=torch.empty(max(cap, 1), **i64), prefetch_slots=torch.empty(max(cap, 1), **i32),
             evict_ids=torch.empty(max(cap, 1), **i64), evict_slots=torch.empty(max(cap, 1), **i32),
             keep_ids=torch.empty(max(cap, 1), **i64), keep_ttl=torch.empty(max(cap, 1), **i32))
    if slot_map:
        t.update(lookup_slots=torch.empty(max(N, 1), **i32))
    h = dict(prefetch_offsets=np.zeros(T + 1, np.int64), evict_offsets=np.zeros(T + 1, np.int64),
             keep_offsets=np.zeros(T + 1, np.int64), occupancy=np.zeros(max(T, 1), np.int64))
    if grouping:
        t.update(grouped_lookups=torch.empty(max(N, 1), **i32), row_recs=torch.empty((max(cap, 1), 4), **i32),
                 piece_recs=torch.empty((piece_capacity(N), 8), **i32))
        h.update(piece_offsets=np.zeros(T + 1, np.int64))
    if trainer_cuts is not None:          # int64 [T, P+1]: which logical trainer owns which lookups of a batch
        trainer_cuts = np.ascontiguousarray(trainer_cuts, dtype=np.int64)
        assert trainer_cuts.shape[0] == T
        t.update(keep_owner=torch.empty(max(cap, 1), **i32))
    p = _bp_plan()
    for k, v in t.items():
        setattr(p, k, v.data_ptr())
    for k, v in h.items():
        setattr(p, k, v.ctypes.data)
    p.list_capacity = cap
    if trainer_cuts is not None:
        p.trainer_cuts = trainer_cuts.ctypes.data
        p.n_trainers = trainer_cuts.shape[1] - 1
    st = lib.bp_oracle_plan(ctypes.byref(cfg), _ptr(ids), iter_offsets.ctypes.data, T, ctypes.byref(p),
                            _ptr(workspace), workspace.numel(), _stream(stream))
    _check(st, min_capacity=int(p.min_capacity), n_unique_pairs=int(p.n_unique_pairs))
    n_pf, n_k = int(h["prefetch_offsets"][-1]), int(h["keep_offsets"][-1])
    return Plan(L_eff=int(p.L_eff), L_requested=int(p.L_requested), peak_occupancy=int(p.peak_occupancy), min_capacity=int(p.min_capacity),
                n_unique_pairs=int(p.n_unique_pairs), lookup_slots=t["lookup_slots"][:N] if slot_map else None,
                prefetch_ids=t["prefetch_ids"][:n_pf], prefetch_slots=t["prefetch_slots"][:n_pf],
                evict_ids=t["evict_ids"][:n_pf], evict_slots=t["evict_slots"][:n_pf],
                keep_ids=t["keep_ids"][:n_k], keep_ttl=t["keep_ttl"][:n_k],
                prefetch_offsets=h["prefetch_offsets"], evict_offsets=h["evict_offsets"],
                keep_offsets=h["keep_offsets"], occupancy=h["occupancy"][:T],
                grouped_lookups=t["grouped_lookups"][:N] if grouping else None,
                row_recs=t["row_recs"][:n_k] if grouping else None,
                piece_recs=t["piece_recs"][:int(h["piece_offsets"][-1])] if grouping else None,
                piece_offsets=h["piece_offsets"] if grouping else None,
                keep_owner=t["keep_owner"][:n_k] if trainer_cuts is not None else None)


@dataclasses.dataclass
class PlanState:
    """State of the cache at a chunk boundary (bp_plan_state): device tensors of `capacity` entries."""
    n_resident: int
    resident_ids: "object"       # int64 [C] device, the first n_resident valid, ascending
    ring: "object"               # int32 [C] device: the residents' slots, then the free slots in hand-out order


def bp_oracle_plan_chunk_workspace_bytes(cfg: bp_config, n_lookups: int, n_iters: int, grouping: bool = False) -> int:
    out = ctypes.c_size_t(0)
    _check(load_library().bp_oracle_plan_chunk_workspace_bytes(ctypes.byref(cfg), int(n_lookups), int(n_iters),
                                                               int(bool(grouping)), ctypes.byref(out)))
    return int(out.value)


def bp_oracle_plan_chunk(cfg: bp_config, ids, iter_offsets, n_emit: int, state: Optional[PlanState] = None,
                         stream=None, grouping: bool = False):
    """Plans the first n_emit of the batches given (the rest is the lookahead window) from the carried `state`
    (None: empty cache).  Returns (Plan, PlanState after the last emitted batch).  The Plan's offsets have
    n_emit + 1 entries and index the list tensors, which are left untrimmed at the front."""
    import torch
    lib = load_library()
    iter_offsets = np.ascontiguousarray(iter_offsets, dtype=np.int64)
    T = iter_offsets.shape[0] - 1
    N = int(iter_offsets[-1])
    C = int(cfg.capacity)
    assert ids.dtype == torch.int64 and ids.numel() == N
    dev = ids.device
    cap = N + C
    workspace = torch.empty(bp_oracle_plan_chunk_workspace_bytes(cfg, N, T, grouping), dtype=torch.uint8, device=dev)
    i32 = dict(dtype=torch.int32, device=dev)
    i64 = dict(dtype=torch.int64, device=dev)
    t = dict(lookup_slots=torch.empty(max(N, 1), **i32),
             prefetch_ids=torch.empty(cap, **i64), prefetch_slots=torch.empty(cap, **i32),
             evict_ids=torch.empty(cap, **i64), evict_slots=torch.empty(cap, **i32),
             keep_ids=torch.empty(cap, **i64), keep_ttl=torch.empty(cap, **i32))
    h = dict(prefetch_offsets=np.zeros(n_emit + 1, np.int64), evict_offsets=np.zeros(n_emit + 1, np.int64),
             keep_offsets=np.zeros(n_emit + 1, np.int64), occupancy=np.zeros(max(n_emit, 1), np.int64))
    if grouping:
        t.update(grouped_lookups=torch.empty(max(N, 1), **i32), row_recs=torch.empty((cap, 4), **i32),
                 piece_recs=torch.empty((piece_capacity(N), 8), **i32))
        h.update(piece_offsets=np.zeros(n_emit + 1, np.int64))
    p = _bp_plan()
    for k, v in t.items():
        setattr(p, k, v.data_ptr())
    for k, v in h.items():
        setattr(p, k, v.ctypes.data)
    p.list_capacity = cap
    out = PlanState(0, torch.empty(C, **i64), torch.empty(C, **i32))
    s_out = _bp_plan_state(0, out.resident_ids.data_ptr(), out.ring.data_ptr())
    s_in = None
    if state is not None:
        s_in = ctypes.byref(_bp_plan_state(int(state.n_resident), state.resident_ids.data_ptr(), state.ring.data_ptr()))
    st = lib.bp_oracle_plan_chunk(ctypes.byref(cfg), _ptr(ids) if N else None, iter_offsets.ctypes.data, T, int(n_emit),
                                  s_in, ctypes.byref(s_out), ctypes.byref(p), _ptr(workspace), workspace.numel(),
                                  _stream(stream))
    _check(st, min_capacity=int(p.min_capacity), n_unique_pairs=int(p.n_unique_pairs))
    out.n_resident = int(s_out.n_resident)
    plan = Plan(L_eff=int(p.L_eff), L_requested=int(p.L_requested), peak_occupancy=int(p.peak_occupancy),
                min_capacity=int(p.min_capacity), n_unique_pairs=int(p.n_unique_pairs), lookup_slots=t["lookup_slots"][:N],
                prefetch_ids=t["prefetch_ids"], prefetch_slots=t["prefetch_slots"], evict_ids=t["evict_ids"],
                evict_slots=t["evict_slots"], keep_ids=t["keep_ids"], keep_ttl=t["keep_ttl"],
                prefetch_offsets=h["prefetch_offsets"], evict_offsets=h["evict_offsets"],
                keep_offsets=h["keep_offsets"], occupancy=h["occupancy"][:n_emit],
                grouped_lookups=t["grouped_lookups"][:N] if grouping else None,
                row_recs=t["row_recs"] if grouping else None,
                piece_recs=t["piece_recs"] if grouping else None,
                piece_offsets=h["piece_offsets"] if grouping else None)
    return plan, out


# ---------------------------------------------------------------------------------------------------
# (2) cache maintenance
# ---------------------------------------------------------------------------------------------------
def bp_cache_apply(cfg: bp_config, cache_w, cache_state, backing_w, backing_state, evict_ids, evict_slots,
                   prefetch_ids, prefetch_slots, stream=None) -> None:
    """Lists are device tensors (slices of a Plan); a None or empty list means nothing to do.  backing_* may be
    pinned host tensors (device-visible) or device tensors."""
    n_e = 0 if evict_ids is None else int(evict_ids.numel())
    n_p = 0 if prefetch_ids is None else int(prefetch_ids.numel())
    _check(load_library().bp_cache_apply(
        ctypes.byref(cfg), _ptr(cache_w), _ptr(cache_state), _ptr(backing_w), _ptr(backing_state),
        _ptr(evict_ids) if n_e else None, _ptr(evict_slots) if n_e else None, n_e,
        _ptr(prefetch_ids) if n_p else None, _ptr(prefetch_slots) if n_p else None, n_p, _stream(stream)))


def bp_cache_apply_duplex_workspace_bytes(cfg: bp_config, n_evict: int) -> int:
    out = ctypes.c_size_t(0)
    _check(load_library().bp_cache_apply_duplex_workspace_bytes(ctypes.byref(cfg), int(n_evict), ctypes.byref(out)))
    return int(out.value)


def bp_cache_apply_duplex(cfg: bp_config, cache_w, cache_state, backing_w, backing_state, evict_ids, evict_slots,
                          prefetch_ids, prefetch_slots, workspace, stream=None) -> None:
    """bp_cache_apply with both link directions busy at once; needs id-disjoint lists (any plan with L_eff >= 2)."""
    n_e = 0 if evict_ids is None else int(evict_ids.numel())
    n_p = 0 if prefetch_ids is None else int(prefetch_ids.numel())
    _check(load_library().bp_cache_apply_duplex(
        ctypes.byref(cfg), _ptr(cache_w), _ptr(cache_state), _ptr(backing_w), _ptr(backing_state),
        _ptr(evict_ids) if n_e else None, _ptr(evict_slots) if n_e else None, n_e,
        _ptr(prefetch_ids) if n_p else None, _ptr(prefetch_slots) if n_p else None, n_p,
        _ptr(workspace), 0 if workspace is None else int(workspace.numel()), _stream(stream)))


def bp_cache_apply_handoff(cfg: bp_config, cache_w, cache_state, backing_w, backing_state, evict_ids, evict_slots,
                           prefetch_ids, prefetch_slots, n_early: int, mismatch_flag=None, stream=None) -> None:
    """Maintenance in one launch for lists of a FIFO plan: the last n_prefetch - n_early prefetches take the slots of
    the first evictions, in order.  mismatch_flag: uint32/int32 device tensor of one element, set to 1 on a bad pair."""
    n_e = 0 if evict_ids is None else int(evict_ids.numel())
    n_p = 0 if prefetch_ids is None else int(prefetch_ids.numel())
    _check(load_library().bp_cache_apply_handoff(
        ctypes.byref(cfg), _ptr(cache_w), _ptr(cache_state), _ptr(backing_w), _ptr(backing_state),
        _ptr(evict_ids) if n_e else None, _ptr(evict_slots) if n_e else None, n_e,
        _ptr(prefetch_ids) if n_p else None, _ptr(prefetch_slots) if n_p else None, n_p, int(n_early),
        _ptr(mismatch_flag), _stream(stream)))


def bp_cache_stage(cfg: bp_config, cache_w, cache_state, evict_slots, staging, stream=None) -> None:
    """First half of bp_cache_apply_duplex: evicted rows -> staging area (their slots may then be refilled)."""
    n_e = 0 if evict_slots is None else int(evict_slots.numel())
    _check(load_library().bp_cache_stage(ctypes.byref(cfg), _ptr(cache_w), _ptr(cache_state),
                                         _ptr(evict_slots) if n_e else None, n_e, _ptr(staging),
                                         0 if staging is None else int(staging.numel()), _stream(stream)))


def bp_cache_apply_staged(cfg: bp_config, cache_w, cache_state, backing_w, backing_state, evict_ids, evict_slots,
                          staging, prefetch_ids, prefetch_slots, stream=None) -> None:
    """Second half: staged rows -> backing table and prefetched rows -> cache in one launch (id-disjoint lists)."""
    n_e = 0 if evict_ids is None else int(evict_ids.numel())
    n_p = 0 if prefetch_ids is None else int(prefetch_ids.numel())
    _check(load_library().bp_cache_apply_staged(
        ctypes.byref(cfg), _ptr(cache_w), _ptr(cache_state), _ptr(backing_w), _ptr(backing_state),
        _ptr(evict_ids) if n_e else None, _ptr(evict_slots) if n_e else None, n_e, _ptr(staging),
        0 if staging is None else int(staging.numel()), _ptr(prefetch_ids) if n_p else None,
        _ptr(prefetch_slots) if n_p else None, n_p, _stream(stream)))


# ---------------------------------------------------------------------------------------------------
# (2b) maintenance overlapped with training
# ---------------------------------------------------------------------------------------------------
def bp_pipeline_early_counts(prefetch_offsets, evict_offsets, capacity: int, L_eff: int) -> np.ndarray:
    """Per batch, how many leading prefetch entries may be fetched while the previous batch trains (host only)."""
    po = np.ascontiguousarray(prefetch_offsets, dtype=np.int64)
    eo = np.ascontiguousarray(evict_offsets, dtype=np.int64)
    T = po.shape[0] - 1
    early = np.zeros(T, dtype=np.int64)
    _check(load_library().bp_pipeline_early_counts(po.ctypes.data, eo.ctypes.data, T, int(capacity), int(L_eff),
                                                   early.ctypes.data))
    return early


def bp_pipeline_create(cfg: bp_config, cache_w, cache_state, backing_w, backing_state, plan: "Plan", staging) -> int:
    """Returns the handle of a bp_pipeline over the plan's lists (which, like the tensors, must outlive it)."""
    out = ctypes.c_void_p(0)
    po = np.ascontiguousarray(plan.prefetch_offsets, dtype=np.int64)
    eo = np.ascontiguousarray(plan.evict_offsets, dtype=np.int64)
    _check(load_library().bp_pipeline_create(
        ctypes.byref(cfg), _ptr(cache_w), _ptr(cache_state), _ptr(backing_w), _ptr(backing_state),
        _ptr(plan.prefetch_ids), _ptr(plan.prefetch_slots), po.ctypes.data, _ptr(plan.evict_ids),
        _ptr(plan.evict_slots), eo.ctypes.data, po.shape[0] - 1, int(plan.L_eff), _ptr(staging),
        0 if staging is None else int(staging.numel()), ctypes.byref(out)))
    return int(out.value)


def bp_pipeline_destroy(handle: int) -> None:
    _check(load_library().bp_pipeline_destroy(handle))


def bp_pipeline_early(handle: int, batch: int) -> int:
    out = ctypes.c_int64(0)
    _check(load_library().bp_pipeline_early(handle, int(batch), ctypes.byref(out)))
    return int(out.value)


def bp_pipeline_begin(handle: int, stream=None) -> None:
    _check(load_library().bp_pipeline_begin(handle, _stream(stream)))


def bp_pipeline_acquire(handle: int, batch: int, stream=None) -> None:
    _check(load_library().bp_pipeline_acquire(handle, int(batch), _stream(stream)))


def bp_pipeline_release(handle: int, batch: int, stream=None) -> None:
    _check(load_library().bp_pipeline_release(handle, int(batch), _stream(stream)))


def bp_pipeline_end(handle: int, stream=None) -> None:
    _check(load_library().bp_pipeline_end(handle, _stream(stream)))


# ---------------------------------------------------------------------------------------------------
# (3) forward
# ---------------------------------------------------------------------------------------------------
def bp_embbag_fwd(cfg: bp_config, cache_w, lookup_slots, bag_offsets, bags: int, out, stream=None) -> None:
    """bag_offsets None = one lookup per bag.  out: fp32 device tensor [bags, dim], written in place."""
    n = int(lookup_slots.numel())
    _check(load_library().bp_embbag_fwd(ctypes.byref(cfg), _ptr(cache_w), _ptr(lookup_slots), _ptr(bag_offsets), n,
                                        int(bags), _ptr(out), _stream(stream)))


def bp_embbag_fwd_grouped(cfg: bp_config, cache_w, grouped_lookups, row_recs, piece_recs, bags: int, out,
                          stream=None) -> None:
    """One lookup per bag.  grouped_lookups / row_recs / piece_recs: one batch's slices of the plan's grouping arrays
    (piece_recs may be None or empty).  out: fp32 device tensor [bags, dim], written in place."""
    assert int(grouped_lookups.numel()) == int(bags)
    n_pieces = 0 if piece_recs is None else int(piece_recs.shape[0])
    _check(load_library().bp_embbag_fwd_grouped(ctypes.byref(cfg), _ptr(cache_w), _ptr(grouped_lookups), _ptr(row_recs),
                                                int(row_recs.shape[0]), _ptr(piece_recs) if n_pieces else None, n_pieces,
                                                int(bags), _ptr(out), _stream(stream)))


# ---------------------------------------------------------------------------------------------------
# (4) backward + update
# ---------------------------------------------------------------------------------------------------
def bp_embbag_bwd_update_workspace_bytes(cfg: bp_config, n_lookups: int, bags: int) -> int:
    out = ctypes.c_size_t(0)
    _check(load_library().bp_embbag_bwd_update_workspace_bytes(ctypes.byref(cfg), int(n_lookups), int(bags),
                                                               ctypes.byref(out)))
    return int(out.value)


def bp_embbag_bwd_update(cfg: bp_config, cache_w, cache_state, lookup_slots, bag_offsets, bags: int, grad_out,
                         workspace, tickets, stream=None) -> None:
    """tickets: see bwd_tickets()."""
    n = int(lookup_slots.numel())
    assert tickets.numel() * tickets.element_size() >= bp_embbag_bwd_ticket_bytes(n)
    _check(load_library().bp_embbag_bwd_update(ctypes.byref(cfg), _ptr(cache_w), _ptr(cache_state),
                                               _ptr(lookup_slots), _ptr(bag_offsets), n, int(bags), _ptr(grad_out),
                                               _ptr(workspace), int(workspace.numel()), _ptr(tickets), _stream(stream)))


def bp_embbag_bwd_update_grouped_workspace_bytes(cfg: bp_config, n_lookups: int, bags: int, multi_hot: bool) -> int:
    out = ctypes.c_size_t(0)
    _check(load_library().bp_embbag_bwd_update_grouped_workspace_bytes(ctypes.byref(cfg), int(n_lookups), int(bags),
                                                                       int(bool(multi_hot)), ctypes.byref(out)))
    return int(out.value)


def bp_embbag_bwd_ticket_bytes(n_lookups: int) -> int:
    return int(load_library().bp_embbag_bwd_ticket_bytes(int(n_lookups)))


def bwd_tickets(max_lookups: int, device="cuda"):
    """The counters of the backward entry points for batches of up to max_lookups lookups: they must be zero when a
    call starts and every call leaves them zero, so they are allocated zeroed, once."""
    import torch
    return torch.zeros(bp_embbag_bwd_ticket_bytes(max_lookups) // 4, dtype=torch.int32, device=device)


def bp_embbag_bwd_update_grouped(cfg: bp_config, cache_w, cache_state, grouped_lookups, row_recs, piece_recs,
                                 bag_offsets, bags: int, grad_out, workspace, tickets, stream=None) -> None:
    """grouped_lookups / row_recs / piece_recs: one batch's slices of the plan's grouping arrays (piece_recs may be
    None or empty).  tickets: see bwd_tickets()."""
    n = int(grouped_lookups.numel())
    n_pieces = 0 if piece_recs is None else int(piece_recs.shape[0])
    assert tickets.numel() * tickets.element_size() >= bp_embbag_bwd_ticket_bytes(n)
    _check(load_library().bp_embbag_bwd_update_grouped(
        ctypes.byref(cfg), _ptr(cache_w), _ptr(cache_state), _ptr(grouped_lookups), _ptr(row_recs),
        int(row_recs.shape[0]), _ptr(piece_recs) if n_pieces else None, n_pieces,
        _ptr(bag_offsets), n, int(bags), _ptr(grad_out), _ptr(workspace), int(workspace.numel()), _ptr(tickets),
        _stream(stream)))


def bp_embbag_bwd_update_grouped_static_max_bytes() -> int:
    return int(load_library().bp_embbag_bwd_update_grouped_static_max_bytes())


def bp_embbag_bwd_update_grouped_static_bytes(cfg: bp_config, n_lookups: int, bags: int, multi_hot: bool) -> int:
    out = ctypes.c_size_t(0)
    _check(load_library().bp_embbag_bwd_update_grouped_static_bytes(ctypes.byref(cfg), int(n_lookups), int(bags),
                                                                    int(bool(multi_hot)), ctypes.byref(out)))
    return int(out.value)


def bp_embbag_bwd_update_grouped_static(cfg: bp_config, cache_w, cache_state, grouped_lookups, row_recs, piece_recs,
                                        bag_offsets, bags: int, grad_out, stream=None) -> None:
    """bp_embbag_bwd_update_grouped without workspace and tickets: the library's own fixed scratch array serves."""
    n = int(grouped_lookups.numel())
    n_pieces = 0 if piece_recs is None else int(piece_recs.shape[0])
    _check(load_library().bp_embbag_bwd_update_grouped_static(
        ctypes.byref(cfg), _ptr(cache_w), _ptr(cache_state), _ptr(grouped_lookups), _ptr(row_recs),
        int(row_recs.shape[0]), _ptr(piece_recs) if n_pieces else None, n_pieces,
        _ptr(bag_offsets), n, int(bags), _ptr(grad_out), _stream(stream)))


# ---------------------------------------------------------------------------------------------------
# profiling
# ---------------------------------------------------------------------------------------------------
def bp_copy_calibration(dst, src, stream=None) -> None:
    """dst <- src by the library's plain copy kernel (tensors of equal byte size)."""
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    _check(load_library().bp_copy_calibration(_ptr(dst), _ptr(src), nbytes, _stream(stream)))


def bp_gather_calibration(table, rows, stream=None, rows_in_flight: int = 4, sink=None):
    """Reads table[rows[k]] for every k (table: 2-D device tensor with rows of a multiple of 16 bytes, rows: int32
    device tensor holding uint32 row numbers) rows_in_flight rows per lane group at a time; returns the sink tensor."""
    import torch
    row_bytes = table.shape[1] * table.element_size()
    n = int(rows.numel())
    if sink is None:
        sink = torch.empty((-(-n // rows_in_flight) + 256) * 4, dtype=torch.int32, device=table.device)
    _check(load_library().bp_gather_calibration(_ptr(sink), _ptr(table), int(table.shape[0]), int(row_bytes), _ptr(rows), n,
                                                int(rows_in_flight), _stream(stream)))
    return sink


def bp_scatter_calibration(table, rows, stream=None, rows_in_flight: int = 4) -> None:
    """Writes table[rows[k]] for every k (table: 2-D device tensor with rows of a multiple of 16 bytes, rows: int32
    device tensor holding uint32 row numbers), rows_in_flight list entries per lane group; piece c of row r written for
    entry k holds the int32 words {r, c, k, 0x5ca77e25}."""
    row_bytes = table.shape[1] * table.element_size()
    _check(load_library().bp_scatter_calibration(_ptr(table), int(table.shape[0]), int(row_bytes), _ptr(rows),
                                                 int(rows.numel()), int(rows_in_flight), _stream(stream)))


def bp_profile_enable(on: bool) -> None:
    _check(load_library().bp_profile_enable(int(bool(on))))


def bp_profile_bracket_overhead(reps: int = 200, stream=None) -> float:
    """Microseconds the profiler's event bracket reads around an empty kernel (median of `reps`)."""
    out = ctypes.c_double(0.0)
    _check(load_library().bp_profile_bracket_overhead(_stream(stream), int(reps), ctypes.byref(out)))
    return float(out.value)


def bp_profile_select(kernel_names=None) -> None:
    """Record only the named kernels (None = all)."""
    lib = load_library()
    if kernel_names is None:
        mask = (1 << 64) - 1
    else:
        ids = {lib.bp_profile_kernel_name(k).decode(): k for k in range(lib.bp_profile_num_kernels())}
        mask = 0
        for n in kernel_names:
            mask |= 1 << ids[n]
    _check(lib.bp_profile_select(ctypes.c_uint64(mask)))


def bp_profile_collect() -> None:
    _check(load_library().bp_profile_collect())


def bp_profile_get(kernel_id: int):
    n, ms = ctypes.c_int64(0), ctypes.c_double(0.0)
    _check(load_library().bp_profile_get(int(kernel_id), ctypes.byref(n), ctypes.byref(ms)))
    return int(n.value), float(ms.value)


def profile_spread(name: str):
    """(min, median, max) launch duration in ms of the kernel called `name`, over the launches collected."""
    lib = load_library()
    lib.bp_profile_spread.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double),
                                      ctypes.POINTER(ctypes.c_double)]
    lib.bp_profile_spread.restype = ctypes.c_int
    for k in range(lib.bp_profile_num_kernels()):
        if lib.bp_profile_kernel_name(k).decode() == name:
            lo, med, hi = ctypes.c_double(0), ctypes.c_double(0), ctypes.c_double(0)
            _check(lib.bp_profile_spread(k, ctypes.byref(lo), ctypes.byref(med), ctypes.byref(hi)))
            return float(lo.value), float(med.value), float(hi.value)
    raise KeyError(name)


def profile_totals() -> dict:
    """{kernel name: (launches, total_ms)} for every kernel with at least one recorded launch."""
    lib = load_library()
    out = {}
    for k in range(lib.bp_profile_num_kernels()):
        n, ms = bp_profile_get(k)
        if n:
            out[lib.bp_profile_kernel_name(k).decode()] = (n, ms)
    return out
