"""Counter-based synthetic data and the five benchmark workloads.

Values
------
Every K, V and Q element is a pure integer function of
``(seed, tensor, layer, request id, token, head, dim)``: a 64-bit counter is mixed
(splitmix64 finaliser), its top 16 bits index a 65536-entry table holding
``bf16(Phi^-1((i + 1/2) / 65536))``, i.e. a bf16-rounded standard normal.  Only integer
torch ops are used after the table is built, so the same call returns bit-identical data
on the CPU and on the GPU, any slice can be regenerated without copying it from anywhere,
and the content never depends on where a KV block is placed.

Workloads
---------
``make_workload(name, seed)`` returns shapes, context lengths and a placement matrix
(1 = keep in HBM, 0 = hold in pinned host memory) for the five configurations the bench
names.  Lengths and placements come from a numpy PCG64 stream seeded independently of the
value stream.  They are stand-ins with the *shapes* of the paper's workloads (LLaMA3-8B /
70B attention geometry, 16-token blocks, batches of 4 and up, contexts up to 128K); no
request trace is reproduced.
"""
from __future__ import annotations

import dataclasses
import functools
from typing import Optional, Sequence

import numpy as np
import torch

_M64 = (1 << 64) - 1
_GOLD = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB

TENSOR_K, TENSOR_V, TENSOR_Q = 0, 1, 2


def _signed(x: int) -> int:
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


def mix64_int(z: int) -> int:
    """splitmix64 finaliser on a Python int (reference for the torch version)."""
    z &= _M64
    z = ((z ^ (z >> 30)) * _C1) & _M64
    z = ((z ^ (z >> 27)) * _C2) & _M64
    return z ^ (z >> 31)


def stream_key(seed: int, tensor: int, layer: int, req_id: int) -> int:
    """64-bit key of one (seed, tensor, layer, request) value stream."""
    k = mix64_int(seed * _GOLD + 0x1234567)
    k = mix64_int(k + tensor * _GOLD + 1)
    k = mix64_int(k + layer * _GOLD + 2)
    k = mix64_int(k + req_id * _GOLD + 3)
    return k


def _mix64_torch(z: torch.Tensor) -> torch.Tensor:
    # int64 arithmetic wraps; (z >> s) is arithmetic, so mask to get the logical shift.
    z = (z ^ ((z >> 30) & ((1 << 34) - 1))) * _signed(_C1)
    z = (z ^ ((z >> 27) & ((1 << 37) - 1))) * _signed(_C2)
    return z ^ ((z >> 31) & ((1 << 33) - 1))


@functools.lru_cache(maxsize=None)
def _table_cpu() -> torch.Tensor:
    p = (torch.arange(65536, dtype=torch.float64) + 0.5) / 65536.0
    x = torch.special.ndtri(p)
    return x.to(torch.bfloat16).contiguous()


_table_cache = {}


def normal_bf16_table(device="cpu") -> torch.Tensor:
    """The 65536-entry bf16 inverse-normal-CDF table, resident on ``device``."""
    dev = torch.device(device)
    key = (dev.type, dev.index)
    if key not in _table_cache:
        _table_cache[key] = _table_cpu().to(dev)
    return _table_cache[key]


def _draw(key: int, idx: torch.Tensor) -> torch.Tensor:
    """bf16 N(0,1) values for int64 element counters ``idx`` of stream ``key``."""
    z = _mix64_torch(idx * _signed(_GOLD) + _signed(key))
    sel = (z >> 48) & 0xFFFF
    return normal_bf16_table(idx.device)[sel]


def draw_int(key: int, idx: int) -> int:
    """Python-int version of the table index for one element (used by tests)."""
    return mix64_int(idx * _GOLD + key) >> 48


def _elem_index(tok0, ntok, heads, n_heads_total, head_dim, device):
    t = torch.arange(tok0, tok0 + ntok, dtype=torch.int64, device=device).view(-1, 1, 1)
    h = torch.as_tensor(list(heads), dtype=torch.int64, device=device).view(1, -1, 1)
    d = torch.arange(head_dim, dtype=torch.int64, device=device).view(1, 1, -1)
    return (t * n_heads_total + h) * head_dim + d


def gen_kv(seed: int, layer: int, req_id: int, tok0: int, ntok: int, n_kv_heads: int,
           head_dim: int, device="cpu", heads: Optional[Sequence[int]] = None,
           max_elems: int = 1 << 25):
    """K and V of tokens ``[tok0, tok0+ntok)`` of one (layer, request).

    Returns two bf16 tensors ``[ntok][len(heads)][head_dim]`` (token-major).  ``heads``
    defaults to all KV heads.  Work is chunked so temporaries stay below ``max_elems``
    int64 elements.
    """
    heads = range(n_kv_heads) if heads is None else heads
    nh = len(list(heads))
    out = []
    for tensor in (TENSOR_K, TENSOR_V):
        key = stream_key(seed, tensor, layer, req_id)
        dst = torch.empty((ntok, nh, head_dim), dtype=torch.bfloat16, device=device)
        step = max(1, max_elems // (nh * head_dim))
        for a in range(0, ntok, step):
            n = min(step, ntok - a)
            dst[a:a + n] = _draw(key, _elem_index(tok0 + a, n, heads, n_kv_heads, head_dim, device))
        out.append(dst)
    return out[0], out[1]


def gen_kv_new(seed: int, layer: int, req_id: int, token: int, n_kv_heads: int, head_dim: int,
               device="cpu"):
    """K and V ``[n_kv_heads][head_dim]`` of the single token at position ``token``."""
    k, v = gen_kv(seed, layer, req_id, token, 1, n_kv_heads, head_dim, device)
    return k[0], v[0]


def gen_q(seed: int, layer: int, req_id: int, step: int, n_q_heads: int, head_dim: int,
          device="cpu"):
    """Query ``[n_q_heads][head_dim]`` bf16 of decode step ``step`` for (layer, request)."""
    key = stream_key(seed, TENSOR_Q, layer, req_id)
    idx = _elem_index(step, 1, range(n_q_heads), n_q_heads, head_dim, device)
    return _draw(key, idx)[0]


def gen_q_steps(seed: int, layer: int, req_id: int, step0: int, n_steps: int, n_q_heads: int,
                head_dim: int, device="cpu"):
    """Queries ``[n_steps][n_q_heads][head_dim]`` of decode steps ``step0 .. step0+n_steps-1``."""
    key = stream_key(seed, TENSOR_Q, layer, req_id)
    return _draw(key, _elem_index(step0, n_steps, range(n_q_heads), n_q_heads, head_dim, device))


def gen_rising_k(seed: int, layer: int, req_id: int, ntok: int, n_kv_heads: int, head_dim: int,
                 total_rise: float, device="cpu"):
    """Keys whose projection on a fixed +-1 direction grows linearly with the token index, on top
    of quarter-amplitude seeded noise, and the unit-amplitude query along that direction.

    Returns ``(k [ntok][n_kv_heads][head_dim] bf16, q_dir [head_dim] bf16)``: ``q_dir . k_t`` rises
    by about ``total_rise`` from the first to the last token, so a running softmax maximum has to
    move on every tile it visits.  A data recipe only: no softmax, no scaling convention."""
    k, _ = gen_kv(seed, layer, req_id, 0, ntok, n_kv_heads, head_dim, device)
    sign = torch.where(torch.arange(head_dim, device=device) % 3 == 0, -1.0, 1.0)
    ramp = torch.arange(ntok, dtype=torch.float32, device=device) * (total_rise / max(ntok - 1, 1) / head_dim)
    kf = k.float() * 0.25 + ramp.view(-1, 1, 1) * sign.view(1, 1, -1)
    return kf.to(torch.bfloat16).contiguous(), sign.to(torch.bfloat16)


def pack_bitmap(placement: np.ndarray) -> np.ndarray:
    """Placement matrix [B][L] of 0/1 -> row-major bitmap [B][ceil(L/8)], bit l LSB-first."""
    return np.packbits(np.asarray(placement, dtype=np.uint8), axis=1, bitorder="little")


@dataclasses.dataclass
class Workload:
    name: str
    seed: int
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    page_tokens: int
    req_ids: np.ndarray          # int64 [B]
    ctx_len: np.ndarray          # int32 [B], stored tokens before the first step
    placement: np.ndarray        # uint8 [B][L], 1 = HBM, 0 = pinned host
    steps: int = 1               # decode steps (one appended token each)
    hbm_budget_bytes: Optional[int] = None
    note: str = ""

    @property
    def n_req(self) -> int:
        return len(self.req_ids)

    @property
    def kv_bytes_per_token_layer(self) -> int:
        return 2 * self.n_kv_heads * self.head_dim * 2

    @property
    def page_bytes(self) -> int:
        return self.kv_bytes_per_token_layer * self.page_tokens

    def blocks(self, extra_tokens: int = 0) -> np.ndarray:
        return (self.ctx_len.astype(np.int64) + extra_tokens + self.page_tokens - 1) // self.page_tokens

    def with_placement(self, placement: np.ndarray, note: str = "") -> "Workload":
        return dataclasses.replace(self, placement=np.asarray(placement, dtype=np.uint8), note=note)

    def all_resident(self) -> "Workload":
        return self.with_placement(np.ones_like(self.placement), "all layers resident")

    def all_host(self) -> "Workload":
        return self.with_placement(np.zeros_like(self.placement), "all layers on host")

    def complement(self) -> "Workload":
        return self.with_placement(1 - self.placement, "complemented placement")


def _per_request_subsets(rng, n_req, n_layers, n_resident):
    pl = np.zeros((n_req, n_layers), dtype=np.uint8)
    for r in range(n_req):
        keep = rng.permutation(n_layers)[: int(n_resident[r])]
        pl[r, keep] = 1
    return pl


def make_workload(name: str, seed: int = 0, n_req: Optional[int] = None,
                  steps: Optional[int] = None, n_layers: Optional[int] = None) -> Workload:
    """One of: tiny, llama8b_b16, long_ctx, heavy_mixed, llama70b.

    ``n_req`` truncates the batch and ``n_layers`` takes a slice of the layers (both for machines
    that cannot pin enough host memory for the whole workload); ``steps`` overrides the number of
    decode steps the plan must leave room for.  A layer slice keeps every request, so one layer's
    launch and one layer's transfers have the full workload's size: ``heavy_mixed`` keeps the first
    ``n_layers`` columns of the drawn placement and scales the byte budget by ``n_layers / 32``;
    ``llama70b`` keeps, in layer order, the first resident and the first offloaded layers in the
    workload's own 1 : 3 proportion.
    """
    rng = np.random.Generator(np.random.PCG64([seed, sum(map(ord, name))]))
    shape8b = dict(n_layers=32, n_q_heads=32, n_kv_heads=8, head_dim=128, page_tokens=16)
    if name == "tiny":
        ctx = np.array([17, 256, 1000, 2048], dtype=np.int32)
        pl = np.zeros((4, 2), dtype=np.uint8)
        pl[:, 0] = 1                                     # layer 0 in HBM, layer 1 on host
        w = Workload(name, seed, 2, 8, 2, 128, 16, np.arange(4, dtype=np.int64) + 100, ctx, pl)
    elif name == "llama8b_b16":
        b = 16
        ctx = rng.integers(8192, 32768, size=b, endpoint=True).astype(np.int32)
        pl = _per_request_subsets(rng, b, 32, np.full(b, 24))
        w = Workload(name, seed, req_ids=np.arange(b, dtype=np.int64) + 1000, ctx_len=ctx,
                     placement=pl, **shape8b)
    elif name == "long_ctx":
        b = 4
        ctx = rng.integers(65536, 131072, size=b, endpoint=True).astype(np.int32)
        pl = _per_request_subsets(rng, b, 32, np.full(b, 16))
        w = Workload(name, seed, req_ids=np.arange(b, dtype=np.int64) + 2000, ctx_len=ctx,
                     placement=pl, steps=32, **shape8b)
    elif name == "heavy_mixed":
        b = 64
        ctx = np.exp(rng.uniform(np.log(1024.0), np.log(65536.0), size=b)).astype(np.int32)
        frac = rng.uniform(0.0, 1.0, size=b)
        pl = _per_request_subsets(rng, b, 32, np.floor(frac * 32))
        budget = 40 * 10**9
        if n_layers is not None and n_layers < 32:
            pl = pl[:, :n_layers]
            budget = budget * n_layers // 32
            shape8b = dict(shape8b, n_layers=n_layers)
        w = Workload(name, seed, req_ids=np.arange(b, dtype=np.int64) + 3000, ctx_len=ctx,
                     placement=pl, hbm_budget_bytes=budget, **shape8b)
        if n_layers is not None and n_layers < 32:
            w = dataclasses.replace(w, note=f"first {n_layers} of 32 layers, budget scaled to {budget / 1e9:.1f} GB")
    elif name == "llama70b":
        b = 32
        ctx = rng.integers(16384, 131072, size=b, endpoint=True).astype(np.int32)
        keep = rng.permutation(80)[:20]
        pl = np.zeros((b, 80), dtype=np.uint8)
        pl[:, keep] = 1                                  # same 20 of 80 layers for everyone
        w = Workload(name, seed, 80, 64, 8, 128, 16, np.arange(b, dtype=np.int64) + 4000, ctx, pl)
        if n_layers is not None and n_layers < 80:
            n_res = max(1, round(n_layers / 4))
            res = np.nonzero(pl[0] == 1)[0][:n_res]
            off = np.nonzero(pl[0] == 0)[0][:n_layers - n_res]
            cols = np.sort(np.concatenate([res, off]))
            w = dataclasses.replace(w, n_layers=n_layers, placement=pl[:, cols],
                                    note=f"{n_layers} of 80 layers ({n_res} resident, {n_layers - n_res} streamed), all 32 requests")
    else:
        raise ValueError(f"unknown workload {name!r}")
    if n_layers is not None and name in ("llama8b_b16", "long_ctx") and n_layers < w.n_layers:
        w = dataclasses.replace(w, n_layers=n_layers, placement=w.placement[:, :n_layers],
                                note=f"first {n_layers} of 32 layers")
    if n_req is not None and n_req < w.n_req:
        w = dataclasses.replace(w, req_ids=w.req_ids[:n_req], ctx_len=w.ctx_len[:n_req],
                                placement=w.placement[:n_req],
                                note=(w.note + f" truncated to {n_req} requests").strip())
    if steps is not None:
        w = dataclasses.replace(w, steps=steps)
    if w.hbm_budget_bytes is not None:
        w = _clip_to_budget(w)
    return w


def _clip_to_budget(w: Workload, prefetch_slots: int = 1) -> Workload:
    """Demote layers until resident blocks plus the staging reserve fit the byte budget.

    Victim: the request holding the most resident blocks (ties: lower index); its
    highest-numbered resident layer moves to the host.  The result is only an *input*;
    the library and the oracle each re-check feasibility on their own.
    """
    pl = w.placement.copy()
    b = w.blocks(extra_tokens=w.steps).astype(np.int64)
    budget = w.hbm_budget_bytes // w.page_bytes
    while True:
        resident = int((pl.astype(np.int64) * b[:, None]).sum())
        staging = int(((1 - pl.astype(np.int64)) * b[:, None]).sum(axis=0).max())
        if resident + prefetch_slots * staging <= budget:
            break
        per_req = pl.sum(axis=1).astype(np.int64) * b
        r = int(np.argmax(per_req))
        if per_req[r] == 0:
            raise ValueError("budget too small even with everything on the host")
        layer = int(np.nonzero(pl[r])[0].max())
        pl[r, layer] = 0
    return w.with_placement(pl, (w.note + " clipped to the byte budget").strip())
