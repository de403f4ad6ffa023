"""Oracle for the planner's cost model (test infrastructure; never imported by the product).

Three things, each written from the paper's text:

* ``distance_offload_counts`` / ``distance_pattern`` – the distance-driven placements of
  Section 3.3.2: offloading every N-th layer; the per-request candidates are the distinct
  values of floor(L/k), k = 2..L, whose number D(L) is at most 2*floor(sqrt(L)) - 1.
* ``algorithm1_as_printed`` – Algorithm 1 (Section 3.3.1) step by step, in its own notation
  (All, Pending, Cur, DestL, elapsed, comp_prev, beta = B/n, need = size/beta).
* ``simulate_prefetch`` – the rules that Algorithm 1 is said to model ("Scheduling KV
  Prefetching"): layers run strictly in order; a layer starts only when its KV is on the GPU;
  a request has one stream and at most one layer in flight, and fetches its next offloaded
  layer as soon as the previously fetched one has been executed; active streams share the
  bandwidth evenly and a finished stream's share is redistributed.  Written as an
  event-driven processor-sharing simulation.

The two disagree on the paper's own example (Section 2.3): with 3 blocks per layer-time both
give 9 for placement A at step 1, but at step 16 the printed algorithm gives 11 where the text
says 12; the simulation gives 9 and 12 when stalls are counted in block-transfer units
(stall time x B).  The planner in the library therefore uses the simulation; see the tests.
"""
from __future__ import annotations

import math
from typing import List, Sequence, Tuple

import numpy as np


# ----------------------------------------------------------------------------- pruning (3.3.2)

def distance_offload_counts(n_layers: int) -> List[int]:
    """Distinct floor(L/k) for k = 2..L, descending (16, 10, 8, 6, 5, 4, 3, 2, 1 for L = 32)."""
    return sorted({n_layers // k for k in range(2, n_layers + 1)}, reverse=True)


def distance_of_count(n_layers: int, count: int) -> int:
    """The largest distance N with floor(L/N) == count (the most evenly spread choice)."""
    return max(k for k in range(1, n_layers + 1) if n_layers // k == count)


def distance_pattern(n_layers: int, count: int) -> np.ndarray:
    """x[l] for one request offloading `count` layers: layer l (1-based) is offloaded iff
    l mod N == 0.  count == 0 keeps everything on the GPU, count == L offloads everything."""
    x = np.ones(n_layers, dtype=np.uint8)
    if count <= 0:
        return x
    n = distance_of_count(n_layers, count)
    for l in range(1, n_layers + 1):
        if l % n == 0:
            x[l - 1] = 0
    return x


# ----------------------------------------------------------------------------- Algorithm 1

def _can_start(pending, cur, x, layer):
    """Tasks that may be promoted at the boundary before `layer` (1-based): a request whose
    stream is idle starts its next offloaded layer if the current layer's KV is on the GPU
    (condition 1) or if that next layer IS the current layer (it is needed now)."""
    busy = {r for (r, _l) in cur}
    out = []
    for r in range(x.shape[0]):
        if r in busy:
            continue
        nxt = [l for (rr, l) in pending if rr == r and l >= layer]
        if not nxt:
            continue
        l2 = min(nxt)
        if l2 == layer or x[r, layer - 1] == 1:
            out.append((r, l2))
    return out


def algorithm1_as_printed(x: np.ndarray, b: Sequence[float], bandwidth: float,
                          comp: Sequence[float]) -> Tuple[float, List[float]]:
    """T_batch and per-layer stalls exactly as Algorithm 1 states them."""
    x = np.asarray(x)
    n_req, n_layers = x.shape
    size = {(r, l): float(b[r]) for r in range(n_req) for l in range(1, n_layers + 1) if x[r, l - 1] == 0}
    pending = set(size)
    cur: List[Tuple[int, int]] = []
    stall_tot, comp_tot, comp_prev = 0.0, 0.0, 0.0
    stalls = []
    for layer in range(1, n_layers + 1):
        q = _can_start(pending, cur, x, layer)
        for e in q:
            pending.discard(e)
            cur.append(e)
        dest = {e for e in cur if e[1] == layer}
        cur.sort(key=lambda e: (size[e], e))
        elapsed, n, stall_l = 0.0, len(cur), 0.0
        while dest:
            beta = bandwidth / n
            need = size[cur[0]] / beta
            elapsed += need
            if elapsed > comp_prev:
                stall_l = elapsed - comp_prev
            dest.discard(cur[0])
            cur.pop(0)
            n -= 1
        stall_tot += stall_l
        comp_tot += comp[layer - 1]
        comp_prev = comp[layer - 1]
        stalls.append(stall_l)
    return comp_tot + stall_tot, stalls


# ----------------------------------------------------------------------------- simulation

def simulate_prefetch(x: np.ndarray, b: Sequence[float], bandwidth: float,
                      comp: Sequence[float]) -> Tuple[float, List[float]]:
    """(T_batch, stall time per layer) under the prefetch rules of Section 3.3.1.

    `b[r]` blocks per offloaded layer of request r, `bandwidth` blocks per unit time,
    `comp[l]` compute time of layer l.  Stall in block units is stall time x bandwidth.
    """
    x = np.asarray(x)
    n_req, n_layers = x.shape
    remaining = [0.0] * n_req       # blocks still to move of the request's task in flight
    target = [0] * n_req            # layer (1-based) being fetched or held, 0 = none
    active = [False] * n_req

    def advance(limit: float, need_layer: int) -> float:
        """Share the bandwidth among active streams for `limit` time, or (limit < 0) until
        every transfer for `need_layer` is complete.  Returns the time that passed."""
        passed = 0.0
        while True:
            live = [r for r in range(n_req) if active[r]]
            if limit < 0 and not any(target[r] == need_layer for r in live):
                return passed
            if not live or (limit >= 0 and passed >= limit):
                return passed if limit < 0 else limit
            rate = bandwidth / len(live)
            dt = min(remaining[r] for r in live) / rate
            if limit >= 0 and passed + dt > limit:
                dt = limit - passed
                for r in live:
                    remaining[r] -= rate * dt
                return limit
            for r in live:
                remaining[r] -= rate * dt
            passed += dt
            for r in live:
                if remaining[r] <= 1e-12 * max(1.0, float(b[r])):
                    remaining[r] = 0.0
                    active[r] = False         # data is now held in the request's buffer

    stalls, total = [], 0.0
    for layer in range(1, n_layers + 1):
        for r in range(n_req):                 # boundary before `layer`: greedy launches
            if active[r] or target[r] >= layer:
                continue                       # in flight, or holding a layer not yet executed
            nxt = [l for l in range(layer, n_layers + 1) if x[r, l - 1] == 0]
            if nxt:
                target[r] = nxt[0]
                remaining[r] = float(b[r])
                active[r] = remaining[r] > 0
        stall = advance(-1.0, layer)
        stalls.append(stall)
        advance(float(comp[layer - 1]), layer)
        total += stall + comp[layer - 1]
        for r in range(n_req):
            if target[r] == layer and not active[r]:
                target[r] = 0                  # executed: the buffer may be reused
    return total, stalls


# ----------------------------------------------------------------------------- brute-force search

def candidate_counts(n_layers: int) -> List[int]:
    """Per-request candidates in search order: keep everything, the D(L) distance-driven
    counts ascending, offload everything."""
    return [0] + sorted(distance_offload_counts(n_layers)) + ([n_layers] if n_layers > 1 else [])


def exhaustive_search(b: Sequence[int], n_layers: int, gpu_blocks: int, prefetch_slots: int,
                      bandwidth: float, comp: Sequence[float], stagger: bool = False):
    """Minimum-latency feasible plan over all per-request candidate combinations; ties go to
    the lexicographically first index vector.  Returns (T, placement) or (inf, None).
    ``stagger`` (not in the paper): request r's pattern is rotated right by r layers."""
    import itertools
    from . import reference as ref
    cands = candidate_counts(n_layers)
    pats = [distance_pattern(n_layers, c) for c in cands]
    best_t, best_x = math.inf, None
    for combo in itertools.product(range(len(cands)), repeat=len(b)):
        x = np.stack([np.roll(pats[i], r % n_layers) if stagger else pats[i] for r, i in enumerate(combo)])
        if not ref.feasible(b, x, gpu_blocks, prefetch_slots):
            continue
        t, _ = simulate_prefetch(x, b, bandwidth, comp)
        if t < best_t - 1e-12:
            best_t, best_x = t, x
    return best_t, best_x


def pause_victim(b: Sequence[int], deposited: Sequence[int]) -> int:
    """Section 3.4, "Pause-Resume Fallback": the victim is the request with the largest sum of KV
    blocks and deposited tokens (our tie rule: the later request)."""
    score = [int(x) + int(d) for x, d in zip(b, deposited)]
    best = max(score)
    return max(i for i, v in enumerate(score) if v == best)


def search_or_pause(b: Sequence[int], deposited: Sequence[int], n_layers: int, gpu_blocks: int, prefetch_slots: int,
                    bandwidth: float, comp: Sequence[float], stagger: bool = False):
    """Pause requests, one victim at a time, until the exhaustive search finds a feasible plan for
    the rest.  Returns (T, placement of the kept requests in original order, paused index list)."""
    keep = list(range(len(b)))
    paused = []
    while True:
        if not keep:
            return float(sum(comp)), None, paused
        t, x = exhaustive_search([b[i] for i in keep], n_layers, gpu_blocks, prefetch_slots, bandwidth, comp, stagger)
        if x is not None:
            return t, x, paused
        v = pause_victim([b[i] for i in keep], [deposited[i] for i in keep])
        paused.append(keep.pop(v))
