"""Shared test/bench plumbing: build a liborbit context for a synthetic workload, fill it from
the seeded generator, and build the oracle's own store from the same generator.

The two sides never exchange page tables, arenas or results: both start from
``workloads.gen_kv`` / ``gen_q`` and only their outputs are compared.
"""
from __future__ import annotations

import numpy as np
import torch

from workloads import Workload, gen_kv, gen_q


def errors(got: torch.Tensor, want: np.ndarray):
    """(max abs error, relative L2 error) of a GPU tensor against the float64 oracle."""
    g = got.detach().to(torch.float64).cpu().numpy()
    d = g - want
    return float(np.abs(d).max()), float(np.sqrt((d * d).sum() / max((want * want).sum(), 1e-300)))


def release_pinned_cache():
    """Returns torch's cached (freed) pinned host blocks to the driver."""
    import gc
    gc.collect()
    torch._C._host_emptyCache()


class GpuRun:
    """A liborbit context on cuda:0 holding workload ``w`` under ``placement``."""

    def __init__(self, w: Workload, placement=None, *, prefetch_slots=1, decode_window=None,
                 chunk_tokens=0, budget_pages=None, extra_pages=4, max_tokens=None, host_pages=None,
                 fill=True, layers=None, zero_copy=False, host_tensor=None, streams=None, poison_staging=False):
        from paper_2601_10729_amd import OrbitContext, orbit_plan_check
        self.w = w
        self.dev = torch.device("cuda:0")
        self.placement = np.asarray(w.placement if placement is None else placement, dtype=np.uint8)
        self.window = w.steps if decode_window is None else decode_window
        res, buf, need, host = orbit_plan_check(w.ctx_len, self.placement, w.page_tokens,
                                                0 if zero_copy else prefetch_slots, self.window)
        pages = (need + extra_pages) if budget_pages is None else budget_pages
        # room for any other placement of the same workload in the host arena
        all_host = int(w.blocks(self.window).sum()) * w.n_layers
        hpages = all_host if host_pages is None else host_pages
        self.hbm = torch.empty(pages * w.page_bytes, dtype=torch.uint8, device=self.dev)
        self._host_borrowed = host_tensor is not None
        if host_tensor is None:
            release_pinned_cache()
            self.host = torch.empty(max(hpages, 1) * w.page_bytes, dtype=torch.uint8, pin_memory=True)
        else:                                   # a slice of a pinned arena the caller keeps for several runs
            assert host_tensor.is_pinned() and host_tensor.numel() >= hpages * w.page_bytes
            self.host = host_tensor[:max(hpages, 1) * w.page_bytes]
        self.cs, self.xs = streams if streams else (torch.cuda.Stream(device=self.dev), torch.cuda.Stream(device=self.dev))
        mt = int(w.ctx_len.max()) + self.window + 16 if max_tokens is None else max_tokens
        self.ctx = OrbitContext(n_layers=w.n_layers, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads,
                                head_dim=w.head_dim, page_tokens=w.page_tokens, max_requests=max(w.n_req, 1),
                                max_tokens_per_request=mt, prefetch_slots=prefetch_slots,
                                chunk_tokens=chunk_tokens, decode_window=self.window, zero_copy=zero_copy, poison_staging=poison_staging,
                                hbm_arena=self.hbm, host_arena=self.host,
                                compute_stream=self.cs, copy_stream=self.xs)
        self.ctx.plan_load(w.req_ids, w.ctx_len, self.placement, w.hbm_budget_bytes)
        self.len = w.ctx_len.astype(np.int64).copy()
        if fill:
            self.fill(layers)

    def fill(self, layers=None):
        w = self.w
        for l in (range(w.n_layers) if layers is None else layers):
            for r, rid in enumerate(w.req_ids):
                n = int(w.ctx_len[r])
                if n == 0:
                    continue
                k, v = gen_kv(w.seed, l, int(rid), 0, n, w.n_kv_heads, w.head_dim, self.dev)
                torch.cuda.synchronize()
                self.ctx.kv_fill(int(rid), l, 0, k, v)
                torch.cuda.synchronize()

    def q_layer(self, layer: int, step: int = 0) -> torch.Tensor:
        w = self.w
        return torch.stack([gen_q(w.seed, layer, int(rid), step, w.n_q_heads, w.head_dim, self.dev)
                            for rid in w.req_ids]).contiguous()

    def q_all(self, step: int = 0) -> torch.Tensor:
        return torch.stack([self.q_layer(l, step) for l in range(self.w.n_layers)]).contiguous()

    def kv_new_all(self):
        """k_new, v_new [L][B][Hkv][D] of the token each request appends next."""
        w = self.w
        ks, vs = [], []
        for l in range(w.n_layers):
            kl, vl = [], []
            for r, rid in enumerate(w.req_ids):
                k, v = gen_kv(w.seed, l, int(rid), int(self.len[r]), 1, w.n_kv_heads, w.head_dim, self.dev)
                kl.append(k[0])
                vl.append(v[0])
            ks.append(torch.stack(kl))
            vs.append(torch.stack(vl))
        return torch.stack(ks).contiguous(), torch.stack(vs).contiguous()

    def attention(self, layer: int, step: int = 0, want_f32=True):
        w = self.w
        q = self.q_layer(layer, step)
        out = torch.empty((w.n_req, w.n_q_heads, w.head_dim), dtype=torch.bfloat16, device=self.dev)
        out32 = torch.empty(out.shape, dtype=torch.float32, device=self.dev) if want_f32 else None
        torch.cuda.synchronize()
        self.ctx.decode_attention(layer, q, out, out32)
        self.cs.synchronize()
        return out, out32

    def step(self, step: int = 0, want_stats=False):
        w = self.w
        q = self.q_all(step)
        k_new, v_new = self.kv_new_all()
        out = torch.empty((w.n_layers, w.n_req, w.n_q_heads, w.head_dim), dtype=torch.bfloat16, device=self.dev)
        torch.cuda.synchronize()
        stats = self.ctx.step(q, k_new, v_new, out, want_stats)
        self.cs.synchronize()
        self.xs.synchronize()
        self.len += 1
        return out, stats

    def read_kv(self, r: int, layer: int, tok0: int, ntok: int):
        w = self.w
        k = torch.empty((ntok, w.n_kv_heads, w.head_dim), dtype=torch.bfloat16, device=self.dev)
        v = torch.empty_like(k)
        torch.cuda.synchronize()
        self.ctx.kv_read(int(w.req_ids[r]), layer, tok0, ntok, k, v)
        self.cs.synchronize()
        return k, v

    def close(self):
        torch.cuda.synchronize()
        self.ctx.destroy()
        # torch keeps freed pinned blocks cached, and the boxes refuse pinned memory beyond a total that differs
        # from box to box: hand the arenas back so that the sum over a test session stays small
        owned = not getattr(self, "_host_borrowed", False)
        self.hbm = self.host = None
        if owned:
            release_pinned_cache()


class OracleRun:
    """The oracle's own paged store filled from the same generator (CPU)."""

    def __init__(self, w: Workload, extra_tokens: int = 0, layers=None, seed: int = 7):
        from oracle import reference as ref
        self.ref = ref
        self.w = w
        self.layers = list(range(w.n_layers)) if layers is None else list(layers)
        n_pages = int(w.blocks(extra_tokens).sum()) * w.n_layers + 5
        self.store = ref.PagedStore(w.n_layers, w.n_kv_heads, w.head_dim, w.page_tokens, n_pages, seed=seed)
        for r, rid in enumerate(w.req_ids):
            self.store.add_request(int(rid))
            for l in self.layers:
                n = int(w.ctx_len[r])
                if n:
                    k, v = gen_kv(w.seed, l, int(rid), 0, n, w.n_kv_heads, w.head_dim, "cpu")
                    self.store.write(int(rid), l, 0, k, v)
        self.len = w.ctx_len.astype(np.int64).copy()

    def append_all(self):
        w = self.w
        for r, rid in enumerate(w.req_ids):
            for l in self.layers:
                k, v = gen_kv(w.seed, l, int(rid), int(self.len[r]), 1, w.n_kv_heads, w.head_dim, "cpu")
                self.store.write(int(rid), l, int(self.len[r]), k, v)
        self.len += 1

    def attention(self, layer: int, step: int = 0) -> np.ndarray:
        w = self.w
        q = torch.stack([gen_q(w.seed, layer, int(rid), step, w.n_q_heads, w.head_dim, "cpu") for rid in w.req_ids])
        return self.ref.decode_attention(self.store, layer, [int(x) for x in w.req_ids], q, w.n_q_heads)


def oracle_one_group(w: Workload, r: int, layer: int, g: int, n_tokens: int, step: int = 0) -> np.ndarray:
    """Oracle output [G][D] of the query heads of kv head ``g`` for one request, generating only
    that head's K/V (for full-size sampled checks)."""
    from oracle import reference as ref
    G = w.n_q_heads // w.n_kv_heads
    rid = int(w.req_ids[r])
    st = ref.PagedStore(1, 1, w.head_dim, w.page_tokens, -(-n_tokens // w.page_tokens) + 3, seed=11)
    st.add_request(rid)
    k, v = gen_kv(w.seed, layer, rid, 0, n_tokens, w.n_kv_heads, w.head_dim, "cpu", heads=[g])
    st.write(rid, 0, 0, k, v)
    q = gen_q(w.seed, layer, rid, step, w.n_q_heads, w.head_dim, "cpu")[g * G:(g + 1) * G]
    return ref.decode_attention(st, 0, [rid], q.unsqueeze(0).contiguous(), G)[0]
