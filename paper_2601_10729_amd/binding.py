"""ctypes binding of liborbit.so: argument marshalling only.

Every step of the path runs inside the library's HIP kernels; this module converts torch
tensors / numpy arrays to raw pointers and raises on error codes.  PyTorch is used for device
memory, pinned host memory and stream handles, nothing else.  If the library has not been built
the import of this module fails loudly: there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

from . import build as _build

ORBIT_OK = 0
ORBIT_E_INVAL, ORBIT_E_CAPACITY, ORBIT_E_HOST_CAPACITY = -1, -2, -3
ORBIT_E_NOT_FOUND, ORBIT_E_STATE, ORBIT_E_HIP, ORBIT_E_NOMEM = -4, -5, -6, -7
ORBIT_MAX_LAYERS, ORBIT_MAX_REQUESTS = 128, 256
ORBIT_FLAG_HOST_ONLY = 1
ORBIT_FLAG_ZERO_COPY = 2
ORBIT_FLAG_POISON_STAGING = 4

_ERR_NAMES = {-1: "ORBIT_E_INVAL", -2: "ORBIT_E_CAPACITY", -3: "ORBIT_E_HOST_CAPACITY",
              -4: "ORBIT_E_NOT_FOUND", -5: "ORBIT_E_STATE", -6: "ORBIT_E_HIP", -7: "ORBIT_E_NOMEM"}


class OrbitError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{_ERR_NAMES.get(code, code)}: {msg}")
        self.code = code


class orbit_config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("page_tokens", C.c_int32), ("max_requests", C.c_int32),
                ("max_tokens_per_request", C.c_int64), ("softmax_scale", C.c_float),
                ("prefetch_slots", C.c_int32), ("chunk_tokens", C.c_int32), ("decode_window", C.c_int32),
                ("flags", C.c_int32), ("hbm_arena", C.c_void_p), ("hbm_arena_bytes", C.c_int64),
                ("host_arena", C.c_void_p), ("host_arena_bytes", C.c_int64),
                ("compute_stream", C.c_void_p), ("copy_stream", C.c_void_p)]


class orbit_step_stats(C.Structure):
    _fields_ = [("step_ms", C.c_float), ("attn_ms_total", C.c_float), ("copy_ms_total", C.c_float),
                ("stall_ms_total", C.c_float), ("hbm_kv_bytes", C.c_int64), ("link_kv_bytes", C.c_int64),
                ("hbm_blocks_reserved", C.c_int64), ("hbm_blocks_budget", C.c_int64),
                ("attn_ms", C.c_float * ORBIT_MAX_LAYERS), ("combine_ms", C.c_float * ORBIT_MAX_LAYERS),
                ("copy_ms", C.c_float * ORBIT_MAX_LAYERS), ("stall_ms", C.c_float * ORBIT_MAX_LAYERS),
                ("link_bytes", C.c_int64 * ORBIT_MAX_LAYERS)]


class orbit_plan_info(C.Structure):
    _fields_ = [("page_bytes", C.c_int64), ("budget_blocks", C.c_int64), ("resident_blocks", C.c_int64),
                ("buffer_blocks", C.c_int64), ("staging_first_page", C.c_int64), ("staging_blocks", C.c_int64),
                ("host_blocks", C.c_int64), ("moved_to_host_blocks", C.c_int64),
                ("moved_to_hbm_blocks", C.c_int64), ("relocated_blocks", C.c_int64),
                ("n_requests", C.c_int32), ("chunk_tokens", C.c_int32), ("evicted_blocks", C.c_int64),
                ("paused_resident_blocks", C.c_int64), ("paused_requests", C.c_int32), ("reserved_", C.c_int32),
                ("deferred_to_host_blocks", C.c_int64), ("in_place_blocks", C.c_int64),
                ("reclaimed_blocks", C.c_int64), ("still_in_place_blocks", C.c_int64),
                ("waited_for_deferred", C.c_int64)]

    def as_dict(self):
        return {f: getattr(self, f) for f, _ in self._fields_}


class orbit_slo_report(C.Structure):
    _fields_ = [("tokens", C.c_int64), ("backend_violations", C.c_int64), ("visible_violations", C.c_int64),
                ("max_deposit", C.c_int64), ("tpot", C.c_double), ("max_visible_gap", C.c_double),
                ("tpot_violated", C.c_int32), ("reserved_", C.c_int32)]


EXPORTS = ["orbit_create", "orbit_destroy", "orbit_last_error", "orbit_plan_check", "orbit_plan_load",
           "orbit_get_plan_info", "orbit_request_pause", "orbit_request_drop", "orbit_kv_fill", "orbit_kv_read", "orbit_kv_append", "orbit_kv_append_batch", "orbit_kv_prefetch",
           "orbit_decode_attention", "orbit_decode_layer", "orbit_decode_attention_static", "orbit_step", "orbit_get_pages", "orbit_get_work_items",
           "orbit_get_copy_schedule", "orbit_distance_options", "orbit_distance_pattern", "orbit_model_latency",
           "orbit_plan_search", "orbit_plan_search_staggered", "orbit_plan_search_or_pause", "orbit_planner_create", "orbit_planner_destroy", "orbit_planner_submit",
           "orbit_planner_poll", "orbit_deposit_create", "orbit_deposit_destroy", "orbit_deposit_push",
           "orbit_deposit_finish", "orbit_deposit_release", "orbit_deposit_stats", "orbit_slo_replay", "orbit_profile_mismatch",
           "orbit_profile_ewma"]

_lib = None


def lib() -> C.CDLL:
    """Loads liborbit.so (building it only if no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    path = _build.LIB
    if not os.path.exists(path):
        path = _build.build(True)
    L = C.CDLL(path)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    i32p, i64p, u8p = C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.POINTER(C.c_uint8)
    L.orbit_create.argtypes = [C.POINTER(orbit_config), C.POINTER(vp)]
    L.orbit_destroy.argtypes = [vp]
    L.orbit_last_error.argtypes = [vp]
    L.orbit_last_error.restype = C.c_char_p
    L.orbit_plan_check.argtypes = [i32, i32, i32, i32p, u8p, i32, i32, i64p]
    L.orbit_plan_load.argtypes = [vp, i32, i64p, i32p, u8p, i64]
    L.orbit_get_plan_info.argtypes = [vp, C.POINTER(orbit_plan_info)]
    L.orbit_request_pause.argtypes = [vp, i64]
    L.orbit_request_drop.argtypes = [vp, i64]
    L.orbit_kv_fill.argtypes = [vp, i64, i32, i64, i64, vp, vp]
    L.orbit_kv_read.argtypes = [vp, i64, i32, i64, i64, vp, vp]
    L.orbit_kv_append.argtypes = [vp, i64, i32, vp, vp]
    L.orbit_kv_append_batch.argtypes = [vp, i32, vp, vp]
    L.orbit_kv_prefetch.argtypes = [vp, i32]
    L.orbit_decode_attention.argtypes = [vp, i32, vp, vp, vp]
    L.orbit_decode_attention_static.argtypes = [vp, i32, vp, vp, vp]
    L.orbit_decode_layer.argtypes = [vp, i32, vp, vp, vp, vp, vp]
    L.orbit_step.argtypes = [vp, vp, vp, vp, vp, C.POINTER(orbit_step_stats)]
    L.orbit_get_pages.argtypes = [vp, i64, i32, i32p, i64p, i32p, i32p, i64]
    L.orbit_get_pages.restype = i64
    L.orbit_get_work_items.argtypes = [vp, i32, i32p, i64]
    L.orbit_get_work_items.restype = i64
    L.orbit_get_copy_schedule.argtypes = [vp, i32p, i64]
    L.orbit_get_copy_schedule.restype = i64
    f64p = C.POINTER(C.c_double)
    L.orbit_distance_options.argtypes = [i32, i32p, i32]
    L.orbit_distance_pattern.argtypes = [i32, i32, u8p]
    L.orbit_model_latency.argtypes = [i32, i32, i64p, u8p, C.c_double, f64p, f64p, f64p]
    L.orbit_plan_search.argtypes = [i32, i32, i64p, i64, i32, C.c_double, f64p, i64, u8p, f64p, i64p]
    L.orbit_plan_search_staggered.argtypes = L.orbit_plan_search.argtypes
    L.orbit_plan_search_or_pause.argtypes = [i32, i32, i64p, i64p, i64, i32, C.c_double, f64p, i64, i32, u8p, u8p, f64p]
    L.orbit_planner_create.argtypes = [C.POINTER(vp)]
    L.orbit_planner_destroy.argtypes = [vp]
    L.orbit_planner_submit.argtypes = [vp, i32, i32, i64p, i64, i32, C.c_double, f64p, i64, i32]
    L.orbit_planner_submit.restype = i64
    L.orbit_planner_poll.argtypes = [vp, i32, i64p, u8p, i64, f64p, i64p]
    L.orbit_deposit_create.argtypes = [C.c_double, C.POINTER(vp)]
    L.orbit_deposit_destroy.argtypes = [vp]
    L.orbit_deposit_push.argtypes = [vp, i32, C.c_double]
    L.orbit_deposit_finish.argtypes = [vp, C.c_double]
    L.orbit_deposit_release.argtypes = [vp, C.c_double, i32p, f64p, i64]
    L.orbit_deposit_release.restype = i64
    L.orbit_deposit_stats.argtypes = [vp, i64p]
    L.orbit_slo_replay.argtypes = [f64p, i64, C.c_double, i32, C.POINTER(orbit_slo_report)]
    L.orbit_profile_mismatch.argtypes = [C.c_double, C.c_double, C.c_double]
    L.orbit_profile_ewma.argtypes = [f64p, f64p, i64, C.c_double]
    for name in EXPORTS:
        fn = getattr(L, name)
        if fn.restype is C.c_int:
            fn.restype = C.c_int
    _lib = L
    return L


def _ptr(x) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _np(a, dtype):
    return np.ascontiguousarray(np.asarray(a, dtype=dtype))


def orbit_plan_check(ctx_len: Sequence[int], placement: np.ndarray, page_tokens: int = 16,
                     prefetch_slots: int = 1, decode_window: int = 0):
    """Eq. (1) pieces: (resident blocks, B_buf, resident + slots*B_buf, host blocks)."""
    pl = np.asarray(placement, dtype=np.uint8)
    n_req, n_layers = pl.shape
    bm = _np(np.packbits(pl, axis=1, bitorder="little"), np.uint8)
    n = _np(ctx_len, np.int32)
    out = np.zeros(4, dtype=np.int64)
    rc = lib().orbit_plan_check(n_req, n_layers, page_tokens, n.ctypes.data_as(C.POINTER(C.c_int32)),
                                bm.ctypes.data_as(C.POINTER(C.c_uint8)), prefetch_slots, decode_window,
                                out.ctypes.data_as(C.POINTER(C.c_int64)))
    if rc != 0:
        raise OrbitError(rc, "orbit_plan_check")
    return tuple(int(v) for v in out)


def _bitmap(placement) -> np.ndarray:
    return _np(np.packbits(np.asarray(placement, dtype=np.uint8), axis=1, bitorder="little"), np.uint8)


def _unbitmap(bm: np.ndarray, n_layers: int) -> np.ndarray:
    return np.unpackbits(bm, axis=1, bitorder="little")[:, :n_layers].astype(np.uint8)


def orbit_distance_options(n_layers: int):
    """The D(L) distance-driven offload counts, descending."""
    out = np.zeros(ORBIT_MAX_LAYERS, dtype=np.int32)
    n = lib().orbit_distance_options(n_layers, out.ctypes.data_as(C.POINTER(C.c_int32)), len(out))
    if n < 0:
        raise OrbitError(n, "orbit_distance_options")
    return [int(v) for v in out[:n]]


def orbit_distance_pattern(n_layers: int, offload_count: int) -> np.ndarray:
    row = np.zeros((1, (n_layers + 7) // 8), dtype=np.uint8)
    rc = lib().orbit_distance_pattern(n_layers, offload_count, row.ctypes.data_as(C.POINTER(C.c_uint8)))
    if rc != 0:
        raise OrbitError(rc, "orbit_distance_pattern")
    return _unbitmap(row, n_layers)[0]


def orbit_model_latency(blocks, placement, blocks_per_time: float, comp):
    """(T_batch, stall time per layer) of a placement under the library's prefetch model."""
    pl = np.asarray(placement, dtype=np.uint8)
    n_req, n_layers = pl.shape
    b, cp, bm = _np(blocks, np.int64), _np(comp, np.float64), _bitmap(pl)
    stall, t = np.zeros(n_layers, dtype=np.float64), C.c_double()
    rc = lib().orbit_model_latency(n_req, n_layers, b.ctypes.data_as(C.POINTER(C.c_int64)),
                                   bm.ctypes.data_as(C.POINTER(C.c_uint8)), float(blocks_per_time),
                                   cp.ctypes.data_as(C.POINTER(C.c_double)),
                                   stall.ctypes.data_as(C.POINTER(C.c_double)), C.byref(t))
    if rc != 0:
        raise OrbitError(rc, "orbit_model_latency")
    return t.value, stall


def orbit_plan_search(blocks, n_layers: int, gpu_blocks: int, blocks_per_time: float, comp,
                      prefetch_slots: int = 1, max_evals: int = 100000, stagger: bool = False):
    """(T_batch, placement [B][L], evaluations) of the best plan in the pruned space; ``stagger``
    selects orbit_plan_search_staggered (request r's pattern rotated by r layers)."""
    b, cp = _np(blocks, np.int64), _np(comp, np.float64)
    bm = np.zeros((len(b), (n_layers + 7) // 8), dtype=np.uint8)
    t, ev = C.c_double(), C.c_int64()
    fn = lib().orbit_plan_search_staggered if stagger else lib().orbit_plan_search
    rc = fn(len(b), n_layers, b.ctypes.data_as(C.POINTER(C.c_int64)), int(gpu_blocks),
                                 prefetch_slots, float(blocks_per_time), cp.ctypes.data_as(C.POINTER(C.c_double)),
                                 int(max_evals), bm.ctypes.data_as(C.POINTER(C.c_uint8)), C.byref(t), C.byref(ev))
    if rc != 0:
        raise OrbitError(rc, "orbit_plan_search: no feasible placement" if rc == ORBIT_E_CAPACITY else "orbit_plan_search")
    return t.value, _unbitmap(bm, n_layers), ev.value


def orbit_plan_search_or_pause(blocks, deposited_tokens, n_layers: int, gpu_blocks: int, blocks_per_time: float, comp,
                               prefetch_slots: int = 1, max_evals: int = 100000, stagger: bool = False):
    """Pause-Resume fallback: (T_batch, placement [B][L], paused [B] of 0/1).  Requests are paused,
    largest blocks + deposited tokens first, until the rest has a feasible plan."""
    b, dep, cp = _np(blocks, np.int64), _np(deposited_tokens, np.int64), _np(comp, np.float64)
    assert len(b) == len(dep)
    bm = np.zeros((len(b), (n_layers + 7) // 8), dtype=np.uint8)
    paused = np.zeros(max(len(b), 1), dtype=np.uint8)
    t = C.c_double()
    rc = lib().orbit_plan_search_or_pause(len(b), n_layers, b.ctypes.data_as(C.POINTER(C.c_int64)),
                                          dep.ctypes.data_as(C.POINTER(C.c_int64)), int(gpu_blocks), prefetch_slots,
                                          float(blocks_per_time), cp.ctypes.data_as(C.POINTER(C.c_double)), int(max_evals),
                                          1 if stagger else 0, bm.ctypes.data_as(C.POINTER(C.c_uint8)),
                                          paused.ctypes.data_as(C.POINTER(C.c_uint8)), C.byref(t))
    if rc < 0:
        raise OrbitError(rc, "orbit_plan_search_or_pause")
    return t.value, _unbitmap(bm, n_layers), paused[:len(b)].copy()


class BackgroundPlanner:
    """The planner in its own thread (orbit_planner_* calls): submit the next iteration's problem,
    collect the finished plan one iteration later."""

    def __init__(self):
        self._L = lib()
        h = C.c_void_p()
        rc = self._L.orbit_planner_create(C.byref(h))
        if rc != 0:
            raise OrbitError(rc, "orbit_planner_create")
        self._h = h
        self._shape = {}          # ticket -> (n_req, n_layers), to size the bitmap buffer

    def submit(self, blocks, n_layers: int, gpu_blocks: int, blocks_per_time: float, comp,
               prefetch_slots: int = 1, max_evals: int = 100000, stagger: bool = False) -> int:
        b, cp = _np(blocks, np.int64), _np(comp, np.float64)
        t = self._L.orbit_planner_submit(self._h, len(b), n_layers, b.ctypes.data_as(C.POINTER(C.c_int64)),
                                         int(gpu_blocks), prefetch_slots, float(blocks_per_time),
                                         cp.ctypes.data_as(C.POINTER(C.c_double)), int(max_evals), 1 if stagger else 0)
        if t <= 0:
            raise OrbitError(int(t), "orbit_planner_submit")
        self._shape[int(t)] = (len(b), n_layers)
        return int(t)

    def poll(self, wait: bool = False):
        """None if no plan is ready; else (ticket, T_batch, placement [B][L], evaluations).  Raises
        OrbitError(ORBIT_E_CAPACITY) if the collected job found nothing feasible."""
        cap = max([n * ((l + 7) // 8) for n, l in self._shape.values()] + [1])
        bm = np.zeros(cap, dtype=np.uint8)
        ticket, t, ev = C.c_int64(), C.c_double(), C.c_int64()
        rc = self._L.orbit_planner_poll(self._h, 1 if wait else 0, C.byref(ticket), bm.ctypes.data_as(C.POINTER(C.c_uint8)),
                                        cap, C.byref(t), C.byref(ev))
        if rc == 0:
            return None
        n, l = self._shape.get(ticket.value, (0, 1))
        self._shape = {k: v for k, v in self._shape.items() if k > ticket.value}
        if rc < 0:
            raise OrbitError(rc, "orbit_planner_poll: no feasible placement" if rc == ORBIT_E_CAPACITY else "orbit_planner_poll")
        bpr = (l + 7) // 8
        return ticket.value, t.value, _unbitmap(bm[:n * bpr].reshape(n, bpr), l), ev.value

    def close(self):
        if self._h is not None:
            self._L.orbit_planner_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class TokenDeposit:
    """One request's Token-Deposit (orbit_deposit_* calls)."""

    def __init__(self, slo_interval: float):
        self._L = lib()
        h = C.c_void_p()
        rc = self._L.orbit_deposit_create(float(slo_interval), C.byref(h))
        if rc != 0:
            raise OrbitError(rc, "orbit_deposit_create")
        self._h = h

    def push(self, token: int, now: float):
        rc = self._L.orbit_deposit_push(self._h, int(token), float(now))
        if rc != 0:
            raise OrbitError(rc, "orbit_deposit_push")

    def finish(self, now: float):
        self._L.orbit_deposit_finish(self._h, float(now))

    def release(self, now: float, cap: int = 4096):
        toks, times = np.zeros(cap, dtype=np.int32), np.zeros(cap, dtype=np.float64)
        n = self._L.orbit_deposit_release(self._h, float(now), toks.ctypes.data_as(C.POINTER(C.c_int32)),
                                          times.ctypes.data_as(C.POINTER(C.c_double)), cap)
        if n < 0:
            raise OrbitError(int(n), "orbit_deposit_release")
        return toks[:n].tolist(), times[:n].tolist()

    def stats(self) -> dict:
        out = np.zeros(4, dtype=np.int64)
        self._L.orbit_deposit_stats(self._h, out.ctypes.data_as(C.POINTER(C.c_int64)))
        return dict(waiting=int(out[0]), delivered=int(out[1]), visible_violations=int(out[2]), max_size=int(out[3]))

    def __del__(self):
        try:
            if self._h:
                self._L.orbit_deposit_destroy(self._h)
                self._h = None
        except Exception:
            pass


def orbit_slo_replay(step_latency, slo_interval: float, finish_at_end: bool = False) -> dict:
    """TBT / TPOT accounting of a run of step latencies behind the Token-Deposit."""
    s = _np(step_latency, np.float64)
    rep = orbit_slo_report()
    rc = lib().orbit_slo_replay(s.ctypes.data_as(C.POINTER(C.c_double)), len(s), float(slo_interval),
                                1 if finish_at_end else 0, C.byref(rep))
    if rc != 0:
        raise OrbitError(rc, "orbit_slo_replay")
    return dict(tokens=rep.tokens, backend_violations=rep.backend_violations, visible_violations=rep.visible_violations,
                max_deposit=rep.max_deposit, tpot=rep.tpot, max_visible_gap=rep.max_visible_gap,
                tpot_violated=bool(rep.tpot_violated))


def orbit_profile_mismatch(predicted: float, observed: float, fraction: float) -> bool:
    return bool(lib().orbit_profile_mismatch(float(predicted), float(observed), float(fraction)))


def orbit_profile_ewma(profile, observed, weight: float) -> np.ndarray:
    p, o = _np(profile, np.float64).copy(), _np(observed, np.float64)
    rc = lib().orbit_profile_ewma(p.ctypes.data_as(C.POINTER(C.c_double)), o.ctypes.data_as(C.POINTER(C.c_double)),
                                  len(p), float(weight))
    if rc != 0:
        raise OrbitError(rc, "orbit_profile_ewma")
    return p


class OrbitContext:
    """One liborbit context.  Method names mirror the C entry points (orbit_ prefix dropped)."""

    def __init__(self, *, n_layers: int, n_q_heads: int, n_kv_heads: int, head_dim: int = 128,
                 page_tokens: int = 16, max_requests: int, max_tokens_per_request: int,
                 softmax_scale: float = 0.0, prefetch_slots: int = 1, chunk_tokens: int = 0,
                 decode_window: int = 0, host_only: bool = False, zero_copy: bool = False, poison_staging: bool = False, hbm_arena=None, hbm_arena_bytes: int = 0,
                 host_arena=None, host_arena_bytes: int = 0, compute_stream=None, copy_stream=None):
        self._L = lib()
        self._keep = (hbm_arena, host_arena, compute_stream, copy_stream)   # keep caller objects alive
        cfg = orbit_config()
        cfg.n_layers, cfg.n_q_heads, cfg.n_kv_heads = n_layers, n_q_heads, n_kv_heads
        cfg.head_dim, cfg.page_tokens = head_dim, page_tokens
        cfg.max_requests, cfg.max_tokens_per_request = max_requests, max_tokens_per_request
        cfg.softmax_scale, cfg.prefetch_slots, cfg.chunk_tokens = softmax_scale, prefetch_slots, chunk_tokens
        cfg.decode_window = decode_window
        cfg.flags = ((ORBIT_FLAG_HOST_ONLY if host_only else 0) | (ORBIT_FLAG_ZERO_COPY if zero_copy else 0) |
                     (ORBIT_FLAG_POISON_STAGING if poison_staging else 0))
        cfg.hbm_arena = _ptr(hbm_arena)
        cfg.hbm_arena_bytes = hbm_arena_bytes if hbm_arena is None else hbm_arena.numel() * hbm_arena.element_size()
        cfg.host_arena = _ptr(host_arena)
        cfg.host_arena_bytes = host_arena_bytes if host_arena is None else host_arena.numel() * host_arena.element_size()
        cfg.compute_stream = None if compute_stream is None else compute_stream.cuda_stream
        cfg.copy_stream = None if copy_stream is None else copy_stream.cuda_stream
        self.cfg = cfg
        self.n_layers, self.n_q_heads, self.n_kv_heads, self.head_dim = n_layers, n_q_heads, n_kv_heads, head_dim
        self.page_tokens = page_tokens
        self.page_bytes = 2 * n_kv_heads * page_tokens * head_dim * 2
        h = C.c_void_p()
        rc = self._L.orbit_create(C.byref(cfg), C.byref(h))
        if rc != 0:
            raise OrbitError(rc, self._L.orbit_last_error(None).decode())
        self._h = h

    # -- plumbing
    def _check(self, rc: int):
        if rc < 0:
            raise OrbitError(int(rc), self._L.orbit_last_error(self._h).decode())
        return rc

    def destroy(self):
        if getattr(self, "_h", None):
            self._L.orbit_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    # -- C entry points
    def plan_load(self, req_ids, ctx_len, placement, hbm_budget_bytes: Optional[int] = None):
        ids = _np(req_ids, np.int64)
        n = _np(ctx_len, np.int32)
        pl = np.asarray(placement, dtype=np.uint8).reshape(len(ids), self.n_layers)
        bm = _np(np.packbits(pl, axis=1, bitorder="little"), np.uint8) if len(ids) else np.zeros((0, 1), np.uint8)
        budget = int(self.cfg.hbm_arena_bytes) if hbm_budget_bytes is None else int(hbm_budget_bytes)
        self._check(self._L.orbit_plan_load(self._h, len(ids), ids.ctypes.data_as(C.POINTER(C.c_int64)),
                                            n.ctypes.data_as(C.POINTER(C.c_int32)),
                                            bm.ctypes.data_as(C.POINTER(C.c_uint8)), budget))

    def get_plan_info(self) -> dict:
        info = orbit_plan_info()
        self._check(self._L.orbit_get_plan_info(self._h, C.byref(info)))
        return info.as_dict()

    def request_pause(self, req_id: int):
        self._check(self._L.orbit_request_pause(self._h, int(req_id)))

    def request_drop(self, req_id: int):
        self._check(self._L.orbit_request_drop(self._h, int(req_id)))

    def kv_fill(self, req_id: int, layer: int, first_token: int, k, v):
        self._check(self._L.orbit_kv_fill(self._h, int(req_id), layer, first_token, k.shape[0], _ptr(k), _ptr(v)))

    def kv_read(self, req_id: int, layer: int, first_token: int, n_tokens: int, k_out, v_out):
        self._check(self._L.orbit_kv_read(self._h, int(req_id), layer, first_token, n_tokens, _ptr(k_out), _ptr(v_out)))

    def kv_append(self, req_id: int, layer: int, k, v):
        self._check(self._L.orbit_kv_append(self._h, int(req_id), layer, _ptr(k), _ptr(v)))

    def kv_append_batch(self, layer: int, k, v):
        self._check(self._L.orbit_kv_append_batch(self._h, layer, _ptr(k), _ptr(v)))

    def kv_prefetch(self, layer: int):
        self._check(self._L.orbit_kv_prefetch(self._h, layer))

    def decode_attention(self, layer: int, q, out, out_f32=None):
        self._check(self._L.orbit_decode_attention(self._h, layer, _ptr(q), _ptr(out), _ptr(out_f32)))

    def decode_layer(self, layer: int, q, k_new, v_new, out, out_f32=None):
        self._check(self._L.orbit_decode_layer(self._h, layer, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out), _ptr(out_f32)))

    def decode_attention_static(self, layer: int, q, out, out_f32=None):
        self._check(self._L.orbit_decode_attention_static(self._h, layer, _ptr(q), _ptr(out), _ptr(out_f32)))

    def step(self, q, k_new, v_new, out, want_stats: bool = False):
        stats = orbit_step_stats() if want_stats else None
        self._check(self._L.orbit_step(self._h, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out),
                                       C.byref(stats) if stats is not None else None))
        return stats

    # -- introspection
    def get_pages(self, req_id: int, layer: int):
        tier, host0, length = C.c_int32(), C.c_int64(), C.c_int32()
        n = self._check(self._L.orbit_get_pages(self._h, int(req_id), layer, C.byref(tier), C.byref(host0),
                                                C.byref(length), None, 0))
        pages = np.zeros(max(int(n), 1), dtype=np.int32)
        self._check(self._L.orbit_get_pages(self._h, int(req_id), layer, None, None, None,
                                            pages.ctypes.data_as(C.POINTER(C.c_int32)), int(n)))
        return dict(tier=tier.value, host_first_page=host0.value, length=length.value, pages=pages[:int(n)])

    def get_work_items(self, layer: int) -> np.ndarray:
        n = self._check(self._L.orbit_get_work_items(self._h, layer, None, 0))
        items = np.zeros((max(int(n), 1), 4), dtype=np.int32)
        self._check(self._L.orbit_get_work_items(self._h, layer, items.ctypes.data_as(C.POINTER(C.c_int32)), int(n)))
        return items[:int(n)]

    def get_copy_schedule(self) -> np.ndarray:
        n = self._check(self._L.orbit_get_copy_schedule(self._h, None, 0))
        rows = np.zeros((max(int(n), 1), 5), dtype=np.int32)
        self._check(self._L.orbit_get_copy_schedule(self._h, rows.ctypes.data_as(C.POINTER(C.c_int32)), int(n)))
        return rows[:int(n)]
