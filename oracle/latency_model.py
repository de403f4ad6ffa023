"""Oracle for the planner's cost model (test infrastructure; never imported by the product).

Two things, each written from the paper's text:

* ``distance_offload_counts`` / ``distance_pattern`` - the distance-driven placements of
  Section 3.3.2: offloading every N-th layer; the per-request candidates are the distinct
  values of floor(L/k), k = 2..L, whose number D(L) is at most 2*floor(sqrt(L)) - 1.
* ``simulate_prefetch`` - the decode latency of a placement under the prefetch rules of
  Section 3.3.1 ("Scheduling KV Prefetching"), the rules Algorithm 1 is said to apply: exact
  rational arithmetic, even link sharing tracked with one shared service counter and a heap of
  landing marks.  It reproduces the stall totals the paper prints for its example (Section
  2.3: 9 and 12 block-transfer units for the uniform placement, none for the request-wise one).

Pins (tests/test_planner.py): the example's totals, single-request recurrences worked by hand,
the two-stream sharing closed form, the equivalence of a uniform placement with one request of
the summed size, bounds and monotonicity.
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


# ----------------------------------------------------------------------------- latency model

def simulate_prefetch(x: np.ndarray, b: Sequence[float], bandwidth: float,
                      comp: Sequence[float]) -> Tuple[float, List[float]]:
    """(T_batch, stall time in front of each layer) for placement ``x`` under the prefetch rules
    of Section 3.3.1, "Scheduling KV Prefetching", in exact rational arithmetic.

    ``b[r]`` blocks per offloaded layer of request r, ``bandwidth`` blocks per unit time,
    ``comp[l]`` compute time of layer l.  A stall in block units is stall time x bandwidth.

    The rules, as that paragraph gives them:
      * layers execute strictly in order, and layer l starts only when the previous layer has
        finished and every offloaded KV of layer l has arrived; the wait in between is the stall;
      * a request owns one prefetch buffer and one stream, so it has at most one layer in
        flight, and the buffer stays taken until the layer it holds has executed (condition 1);
      * transfers are launched greedily: at the boundary before a layer, every request whose
        buffer is free starts fetching its next offloaded layer, if it has one (condition 2);
      * the streams that are still transferring (condition 3) divide the link evenly, and when
        one finishes its share goes to the others.

    Even sharing is tracked with one shared service counter instead of per-stream remainders:
    ``served`` is the number of blocks every stream in flight has received since time zero, so a
    transfer of ``b`` blocks launched when the counter reads ``s`` lands when it reads ``s + b``,
    and while ``n`` streams are in flight the counter advances by ``bandwidth / n`` per unit time.
    Landing marks are kept in a heap.  All quantities are ``fractions.Fraction`` (a float is an
    exact rational), so there is no tolerance anywhere; results are rounded to float on return.
    """
    import heapq
    from fractions import Fraction

    x = np.asarray(x)
    n_req, n_layers = x.shape
    link = Fraction(float(bandwidth))
    size = [Fraction(float(v)) for v in b]
    work = [Fraction(float(c)) for c in comp]

    served = Fraction(0)
    in_flight: list = []                    # heap of (landing mark, request)
    holds = [0] * n_req                     # 1-based layer sitting in (or travelling to) the request's buffer

    def next_offloaded(r: int, first: int) -> int:
        for l in range(first, n_layers + 1):
            if x[r, l - 1] == 0:
                return l
        return 0

    stalls: List[Fraction] = []
    for layer in range(1, n_layers + 1):
        # boundary before `layer`: greedy launches
        for r in range(n_req):
            if holds[r] == 0:
                holds[r] = next_offloaded(r, layer)
                if holds[r] and size[r] > 0:
                    heapq.heappush(in_flight, (served + size[r], r))
        # stall: the link keeps running until nothing destined for `layer` is in flight
        waited = Fraction(0)
        while any(holds[r] == layer for _, r in in_flight):
            mark, _ = in_flight[0]
            waited += (mark - served) * len(in_flight) / link
            served = mark
            heapq.heappop(in_flight)
        stalls.append(waited)
        # the layer executes; transfers for later layers continue underneath
        left = work[layer - 1]
        while in_flight and left > 0:
            mark, _ = in_flight[0]
            until_landing = (mark - served) * len(in_flight) / link
            if until_landing <= left:
                left -= until_landing
                served = mark
                heapq.heappop(in_flight)
            else:
                served += left * link / len(in_flight)
                left = Fraction(0)
        # executed: buffers that held this layer are free again
        for r in range(n_req):
            if holds[r] == layer:
                holds[r] = 0
    total = sum(work, Fraction(0)) + sum(stalls, Fraction(0))
    return float(total), [float(s) for s in stalls]


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
