"""Python face of the CPU oracle (test infrastructure; never imported by the product).

* ``PagedStore``        – the oracle's OWN paged KV arena on the host (its own allocator, its
                          own page tables); K/V are written and read through the page layout
                          stated in ``orbit_oracle.c``.
* ``decode_attention``  – float64 two-pass softmax attention over that store (one layer).
* ``blocks`` / ``prefetch_buffer_blocks`` / ``gpu_blocks_needed`` / ``feasible``
                        – the GPU capacity bound, Eq. (1) of Section 3.3.1, written out.

Placement (HBM or host) does not enter the attention values: the result of the method is the
same wherever a block lives, so the oracle keeps a single host arena.
"""
from __future__ import annotations

import ctypes
import math
from typing import Dict, List, Sequence, Tuple

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(_build.build())
        i32p, u16p, f64p = (ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_uint16),
                            ctypes.POINTER(ctypes.c_double))
        i64, ci = ctypes.c_int64, ctypes.c_int
        L.oracle_pack_tokens.argtypes = [u16p, i64, i32p, i64, ci, ci, ci, i64, i64, u16p, u16p]
        L.oracle_unpack_tokens.argtypes = [u16p, i64, i32p, i64, ci, ci, ci, i64, i64, u16p, u16p]
        L.oracle_decode_attention.argtypes = [u16p, i64, ci, ci, ci, ci, ci, i32p, i64, i32p, u16p,
                                              ctypes.c_double, f64p]
        L.oracle_attention_weights.argtypes = [u16p, i64, i32p, i64, ci, ci, ci, ci, ci, u16p,
                                               ctypes.c_double, f64p, f64p]
        L.oracle_num_threads.restype = ci
        L.oracle_set_threads.argtypes = [ci]
        L.oracle_set_threads.restype = None
        _lib = L
    return _lib


def _p(a: np.ndarray, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def as_u16(x) -> np.ndarray:
    """bf16 torch tensor / uint16 array -> contiguous numpy uint16 bit patterns."""
    if isinstance(x, np.ndarray):
        assert x.dtype == np.uint16
        return np.ascontiguousarray(x)
    import torch
    assert x.dtype == torch.bfloat16
    return np.ascontiguousarray(x.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16))


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


# --------------------------------------------------------------------------- capacity, Eq. (1)

def blocks(ctx_len: Sequence[int], page_tokens: int = 16) -> np.ndarray:
    """b_r: KV blocks per layer of each request; a block is added only when a multiple of
    ``page_tokens`` is crossed (Section 2.3)."""
    n = np.asarray(ctx_len, dtype=np.int64)
    return -(-n // page_tokens)


def prefetch_buffer_blocks(b: Sequence[int], x: np.ndarray) -> int:
    """B_buf = max over layers of the offloaded blocks that one layer needs (below Eq. (1))."""
    b = np.asarray(b, dtype=np.int64)
    x = np.asarray(x, dtype=np.int64)
    if x.size == 0:
        return 0
    return int(((1 - x) * b[:, None]).sum(axis=0).max())


def resident_blocks(b: Sequence[int], x: np.ndarray) -> int:
    b = np.asarray(b, dtype=np.int64)
    return int((np.asarray(x, dtype=np.int64) * b[:, None]).sum())


def gpu_blocks_needed(b: Sequence[int], x: np.ndarray, prefetch_slots: int = 1) -> int:
    """Left side of Eq. (1); ``prefetch_slots`` > 1 charges that many staging buffers (the paper
    has exactly one)."""
    return resident_blocks(b, x) + prefetch_slots * prefetch_buffer_blocks(b, x)


def feasible(b: Sequence[int], x: np.ndarray, b_gpu: int, prefetch_slots: int = 1) -> bool:
    return gpu_blocks_needed(b, x, prefetch_slots) <= b_gpu


# --------------------------------------------------------------------------- paged store

class PagedStore:
    """Host arena of ``n_pages`` KV blocks plus a (request, layer) -> page-list table."""

    def __init__(self, n_layers: int, n_kv_heads: int, head_dim: int, page_tokens: int,
                 n_pages: int, seed: int = 0):
        self.L, self.Hkv, self.D, self.P = n_layers, n_kv_heads, head_dim, page_tokens
        self.page_elems = 2 * n_kv_heads * page_tokens * head_dim
        self.n_pages = n_pages
        # poison with a NaN pattern so that reading an unwritten slot is visible
        self.arena = np.full((n_pages, self.page_elems), 0x7FC1, dtype=np.uint16)
        order = np.random.Generator(np.random.PCG64(seed)).permutation(n_pages)
        self._free: List[int] = [int(p) for p in order[::-1]]
        self.pages: Dict[Tuple[int, int], List[int]] = {}
        self.length: Dict[int, int] = {}

    def add_request(self, req_id: int) -> None:
        assert req_id not in self.length
        self.length[req_id] = 0
        for l in range(self.L):
            self.pages[(req_id, l)] = []

    def _ensure(self, req_id: int, layer: int, n_tokens: int) -> None:
        lst = self.pages[(req_id, layer)]
        while len(lst) * self.P < n_tokens:
            lst.append(self._free.pop())

    def write(self, req_id: int, layer: int, tok0: int, k, v) -> None:
        """k, v: [ntok][Hkv][D] bf16 (torch) or uint16 bits."""
        k, v = as_u16(k), as_u16(v)
        ntok = k.shape[0]
        assert k.shape == (ntok, self.Hkv, self.D) and v.shape == k.shape
        self._ensure(req_id, layer, tok0 + ntok)
        pg = np.asarray(self.pages[(req_id, layer)], dtype=np.int32)
        rc = lib().oracle_pack_tokens(_p(self.arena, ctypes.c_uint16), self.n_pages,
                                      _p(pg, ctypes.c_int32), len(pg), self.Hkv, self.D, self.P,
                                      tok0, ntok, _p(k, ctypes.c_uint16), _p(v, ctypes.c_uint16))
        assert rc == 0, rc
        self.length[req_id] = max(self.length[req_id], tok0 + ntok)

    def read(self, req_id: int, layer: int, tok0: int, ntok: int):
        pg = np.asarray(self.pages[(req_id, layer)], dtype=np.int32)
        k = np.empty((ntok, self.Hkv, self.D), dtype=np.uint16)
        v = np.empty_like(k)
        rc = lib().oracle_unpack_tokens(_p(self.arena, ctypes.c_uint16), self.n_pages,
                                        _p(pg, ctypes.c_int32), len(pg), self.Hkv, self.D, self.P,
                                        tok0, ntok, _p(k, ctypes.c_uint16), _p(v, ctypes.c_uint16))
        assert rc == 0, rc
        return k, v

    def table(self, layer: int, req_ids: Sequence[int]):
        stride = max(1, max(len(self.pages[(r, layer)]) for r in req_ids))
        t = np.full((len(req_ids), stride), -1, dtype=np.int32)
        for i, r in enumerate(req_ids):
            lst = self.pages[(r, layer)]
            t[i, :len(lst)] = lst
        n = np.asarray([self.length[r] for r in req_ids], dtype=np.int32)
        return t, n

    def permute_pages(self, seed: int) -> None:
        """Move every block to a new physical page and rewrite the tables accordingly."""
        perm = np.random.Generator(np.random.PCG64(seed)).permutation(self.n_pages)
        new = np.empty_like(self.arena)
        new[perm] = self.arena
        self.arena = new
        for key, lst in self.pages.items():
            self.pages[key] = [int(perm[p]) for p in lst]
        self._free = [int(perm[p]) for p in self._free]


def decode_attention(store: PagedStore, layer: int, req_ids: Sequence[int], q, n_q_heads: int,
                     scale: float = 0.0, ctx_len: Sequence[int] = None) -> np.ndarray:
    """float64 attention output [B][Hq][D] of one layer.  q: [B][Hq][D] bf16.
    ``ctx_len`` overrides the stored lengths (must not exceed them)."""
    qb = as_u16(q)
    table, n = store.table(layer, req_ids)
    if ctx_len is not None:
        n2 = np.asarray(ctx_len, dtype=np.int32)
        assert np.all(n2 <= n)
        n = n2
    assert qb.shape == (len(req_ids), n_q_heads, store.D)
    out = np.empty(qb.shape, dtype=np.float64)
    rc = lib().oracle_decode_attention(_p(store.arena, ctypes.c_uint16), store.n_pages, len(req_ids),
                                       n_q_heads, store.Hkv, store.D, store.P,
                                       _p(table, ctypes.c_int32), table.shape[1],
                                       _p(n, ctypes.c_int32), _p(qb, ctypes.c_uint16),
                                       float(scale), _p(out, ctypes.c_double))
    if rc != 0:
        raise ValueError(f"oracle_decode_attention failed with {rc}")
    return out


def attention_weights(store: PagedStore, layer: int, req_id: int, head: int, q_row, n_q_heads: int,
                      scale: float = 0.0):
    """(weights [n], output [D]) of one (request, query head)."""
    qb = as_u16(q_row)
    pg = np.asarray(store.pages[(req_id, layer)], dtype=np.int32)
    n = store.length[req_id]
    w = np.empty(n, dtype=np.float64)
    o = np.empty(store.D, dtype=np.float64)
    rc = lib().oracle_attention_weights(_p(store.arena, ctypes.c_uint16), store.n_pages,
                                        _p(pg, ctypes.c_int32), n, head, n_q_heads, store.Hkv,
                                        store.D, store.P, _p(qb, ctypes.c_uint16), float(scale),
                                        _p(o, ctypes.c_double), _p(w, ctypes.c_double))
    if rc != 0:
        raise ValueError(f"oracle_attention_weights failed with {rc}")
    return w, o


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def set_threads(n: int) -> None:
    """Size of the OpenMP team the attention call uses from now on (timing runs only)."""
    lib().oracle_set_threads(int(n))


def default_scale(head_dim: int) -> float:
    return 1.0 / math.sqrt(head_dim)
