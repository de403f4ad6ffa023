"""Planner helpers: pins for the oracle's cost model and pruning enumerator (numbers printed in
the paper), then parity of the library's host implementation against that oracle.  CPU only."""
import json
import math
import os

import numpy as np
import pytest

import paper_2601_10729_amd as orbit
from oracle import latency_model as lm
from oracle import reference as ref

HERE = os.path.dirname(os.path.abspath(__file__))


def _toy():
    with open(os.path.join(HERE, "golden", "toy_example.json")) as f:
        return json.load(f)


def _x(n_layers, offloaded_1based):
    m = np.ones((len(offloaded_1based), n_layers), dtype=np.uint8)
    for r, layers in enumerate(offloaded_1based):
        for l in layers:
            m[r, l - 1] = 0
    return m


# ------------------------------------------------------------------ pins: pruning (Section 3.3.2)

def test_distance_counts_match_the_papers_numbers():
    assert len(lm.distance_offload_counts(32)) == 9                       # D(32) = 9
    assert 9 ** 4 == 6561
    for L in range(2, 129):
        assert len(lm.distance_offload_counts(L)) <= 2 * math.isqrt(L) - 1       # the bound of Section 3.3.2
    # two of six layers offloaded: [1 1 0 1 1 0]  (Section 2.2)
    assert lm.distance_pattern(6, 2).tolist() == [1, 1, 0, 1, 1, 0]
    # every 4th / 5th of 32 layers: 8 / 6 layers offloaded
    assert lm.distance_of_count(32, 8) == 4 and int((lm.distance_pattern(32, 8) == 0).sum()) == 8
    assert lm.distance_of_count(32, 6) == 5 and int((lm.distance_pattern(32, 6) == 0).sum()) == 6
    for c in lm.distance_offload_counts(32):
        assert int((lm.distance_pattern(32, c) == 0).sum()) == c
    assert lm.distance_pattern(32, 0).all() and not lm.distance_pattern(32, 32).any()


# ------------------------------------------------------------------ pins: latency model (Sections 2.3, 3.3.1)

def test_simulation_reproduces_the_stall_totals_of_the_papers_example():
    toy = _toy()
    L, bw = toy["n_layers"], float(toy["link_blocks_per_layer_time"])
    comp = [1.0] * L
    A = _x(L, toy["placement_A"]["offloaded_layers_1based"])
    B = _x(L, [[], [3, 6, 9]])
    for step in ("step1", "step16"):
        b = toy[step]["blocks_per_layer"]
        t, stalls = lm.simulate_prefetch(A, b, bw, comp)
        assert abs(sum(stalls) * bw - toy["placement_A"]["stalls"][step]) < 1e-9    # 9 and 12, in block units
        assert abs(t - (L + sum(stalls))) < 1e-12
        assert [i + 1 for i, s in enumerate(stalls) if s > 0] == [3, 6, 9]
    t, stalls = lm.simulate_prefetch(B, toy["step1"]["blocks_per_layer"], bw, comp)
    assert sum(stalls) == toy["placement_B"]["stalls"]["step1"] == 0


def _single_request_by_hand(offloaded_1based, size, bw, comp):
    """One request, worked the long way: its fetches run one after the other at the full link
    rate.  Fetch k starts at the boundary at which the layer of fetch k-1 has finished executing
    (the first one at time zero) and takes size/bw; a layer starts at the later of "previous
    layer finished" and "its own fetch has landed"."""
    finish_prev, buffer_free_at, stalls = 0.0, 0.0, []
    landed = {}
    todo = sorted(offloaded_1based)
    if todo:
        landed[todo[0]] = size / bw
    for l in range(1, len(comp) + 1):
        start = max(finish_prev, landed.get(l, 0.0))
        stalls.append(start - finish_prev)
        finish_prev = start + comp[l - 1]
        if l in landed:                                   # executed: the next fetch may start now
            later = [k for k in todo if k > l]
            if later:
                landed[later[0]] = finish_prev + size / bw
    return finish_prev, stalls


def test_single_request_matches_the_recurrence_worked_by_hand():
    rng = np.random.default_rng(11)
    for _ in range(60):
        L = int(rng.integers(1, 12))
        off = [l for l in range(1, L + 1) if rng.random() < 0.4]
        size, bw = int(rng.integers(1, 40)), float(rng.integers(1, 8))
        comp = [float(c) for c in rng.integers(1, 6, size=L)]      # small integers: every quantity is exact in binary
        t, st = lm.simulate_prefetch(_x(L, [off]), [size], bw, comp)
        tw, sw = _single_request_by_hand(off, size, bw, comp)
        assert abs(t - tw) < 1e-9 and np.allclose(st, sw, atol=1e-9), (off, size, bw, comp)


def test_uniform_placement_equals_one_request_of_the_summed_size():
    """Streams launched together that block the same layer share the link until the last one lands,
    which is when one stream carrying all their blocks would land (the example's placement A: 3 + 6)."""
    rng = np.random.default_rng(12)
    for _ in range(40):
        L, n_req = int(rng.integers(1, 10)), int(rng.integers(2, 6))
        off = [l for l in range(1, L + 1) if rng.random() < 0.5]
        b = rng.integers(1, 30, size=n_req)
        comp = rng.uniform(0.2, 3.0, size=L)
        bw = float(rng.uniform(0.5, 9.0))
        t, st = lm.simulate_prefetch(_x(L, [off] * n_req), b, bw, comp)
        t1, st1 = lm.simulate_prefetch(_x(L, [off]), [int(b.sum())], bw, comp)
        assert abs(t - t1) < 1e-9 * max(1.0, t1) and np.allclose(st, st1, atol=1e-9)


def test_two_streams_share_the_link_and_the_share_is_redistributed():
    """Request 0 (a blocks) offloads only layer p, request 1 (c blocks) only layer q > p.  Both start
    at time zero and halve the link; when the smaller lands the other gets all of it.  Hence the
    smaller lands at 2*min(a, c)/B and the larger at (a + c)/B, whatever the layer times are."""
    rng = np.random.default_rng(13)
    for _ in range(60):
        L = int(rng.integers(2, 9))
        p = int(rng.integers(1, L))
        q = int(rng.integers(p + 1, L + 1))
        a, c = int(rng.integers(1, 40)), int(rng.integers(1, 40))
        bw = float(rng.integers(1, 6))
        comp = [float(v) for v in rng.integers(1, 5, size=L)]
        land0 = (2 * min(a, c) if a <= c else a + c) / bw
        land1 = (2 * min(a, c) if c < a else a + c) / bw
        before_p = sum(comp[:p - 1])
        stall_p = max(0.0, land0 - before_p)
        before_q = sum(comp[:q - 1]) + stall_p
        stall_q = max(0.0, land1 - before_q)
        t, st = lm.simulate_prefetch(_x(L, [[p], [q]]), [a, c], bw, comp)
        want = [0.0] * L
        want[p - 1], want[q - 1] = stall_p, stall_q
        assert np.allclose(st, want, atol=1e-9) and abs(t - (sum(comp) + stall_p + stall_q)) < 1e-9, (p, q, a, c, bw, comp)


def test_a_busy_buffer_delays_the_next_fetch():
    """Condition (1): while layer l of a request executes out of its prefetch buffer, that request
    cannot fetch.  Layers 1 and 2 offloaded, 4 blocks at 2 blocks per unit, unit layer times: the first
    fetch lands at 2 (stall 2), layer 1 runs 2..3, only then the second fetch starts and lands at 5
    (stall 2 again), layer 2 runs 5..6, layer 3 runs 6..7."""
    t, st = lm.simulate_prefetch(_x(3, [[1, 2]]), [4], 2.0, [1.0, 1.0, 1.0])
    assert st == [2.0, 2.0, 0.0] and t == 7.0
    # with a resident layer in between the second fetch hides behind it: lands at 3 + 2 = 5, layer 2 ends at 4
    t, st = lm.simulate_prefetch(_x(3, [[1, 3]]), [4], 2.0, [1.0, 1.0, 1.0])
    assert st == [2.0, 0.0, 1.0] and t == 6.0


def test_simulation_closed_forms():
    comp = [2.0, 1.0, 3.0, 1.5]
    # nothing offloaded: pure compute
    t, st = lm.simulate_prefetch(np.ones((3, 4), np.uint8), [5, 7, 9], 2.0, comp)
    assert t == sum(comp) and not any(st)
    # one request, only layer 1 offloaded: nothing to overlap with
    t, st = lm.simulate_prefetch(_x(4, [[1]]), [6], 2.0, comp)
    assert st == [3.0, 0, 0, 0] and t == sum(comp) + 3.0
    # one request, every layer offloaded: the buffer is busy while a layer runs, no overlap at all
    t, st = lm.simulate_prefetch(np.zeros((1, 4), np.uint8), [6], 2.0, comp)
    assert st == [3.0] * 4 and t == sum(comp) + 12.0
    # one request, layer 3 offloaded: the fetch overlaps layers 1 and 2 (3 time units)
    t, st = lm.simulate_prefetch(_x(4, [[3]]), [10], 2.0, comp)
    assert st == [0, 0, 2.0, 0]
    # two equal requests sharing the link evenly finish together: same as one request of twice the size
    t2, st2 = lm.simulate_prefetch(_x(4, [[3], [3]]), [5, 5], 2.0, comp)
    assert st2 == st
    # more bandwidth never hurts; the link bound holds
    rng = np.random.default_rng(0)
    for _ in range(30):
        n_req, L = int(rng.integers(1, 5)), int(rng.integers(1, 9))
        x = rng.integers(0, 2, size=(n_req, L)).astype(np.uint8)
        b = rng.integers(1, 20, size=n_req)
        cp = rng.uniform(0.5, 2.0, size=L)
        t1, _ = lm.simulate_prefetch(x, b, 3.0, cp)
        t2, _ = lm.simulate_prefetch(x, b, 6.0, cp)
        assert t2 <= t1 + 1e-9 and t1 >= cp.sum() - 1e-9
        assert t1 >= float(((1 - x.astype(np.int64)) * b[:, None]).sum()) / 3.0 - 1e-9


# ------------------------------------------------------------------ library against the oracle

def test_library_enumerator_matches_oracle():
    for L in (1, 2, 6, 9, 32, 80, 128):
        assert orbit.orbit_distance_options(L) == lm.distance_offload_counts(L)
        for c in [0] + lm.distance_offload_counts(L) + [L]:
            assert orbit.orbit_distance_pattern(L, c).tolist() == lm.distance_pattern(L, c).tolist()
    with pytest.raises(orbit.OrbitError):
        orbit.orbit_distance_pattern(32, 7)                   # 7 is not a floor(32/k)


def test_library_latency_model_matches_oracle():
    rng = np.random.default_rng(1)
    for _ in range(200):
        n_req, L = int(rng.integers(1, 7)), int(rng.integers(1, 13))
        x = rng.integers(0, 2, size=(n_req, L)).astype(np.uint8)
        b = rng.integers(0, 50, size=n_req)
        comp = rng.uniform(0.1, 3.0, size=L)
        bw = float(rng.uniform(0.5, 20.0))
        t, st = orbit.orbit_model_latency(b, x, bw, comp)
        tw, sw = lm.simulate_prefetch(x, b, bw, comp)
        assert abs(t - tw) <= 1e-9 * max(1.0, tw)
        np.testing.assert_allclose(st, sw, rtol=1e-9, atol=1e-9)
    toy = _toy()
    A = _x(9, toy["placement_A"]["offloaded_layers_1based"])
    t, st = orbit.orbit_model_latency([4, 6], A, 3.0, [1.0] * 9)
    assert abs(st.sum() * 3.0 - 12.0) < 1e-9


def test_library_search_matches_brute_force_and_picks_the_papers_plan():
    toy = _toy()
    L, cap, bw, comp = toy["n_layers"], toy["gpu_blocks"], 3.0, [1.0] * toy["n_layers"]
    # step 1: keep the short request resident, offload 3 evenly spaced layers of the long one (placement B)
    t, x, evals = orbit.orbit_plan_search([3, 6], L, cap, bw, comp)
    assert t == 9.0 and x.tolist() == _x(L, [[], [3, 6, 9]]).tolist()
    # step 16: B no longer fits; whatever is chosen is feasible and no slower than uniform placement A
    t16, x16, _ = orbit.orbit_plan_search([4, 6], L, cap, bw, comp)
    assert ref.feasible([4, 6], x16, cap)
    assert t16 <= lm.simulate_prefetch(_x(L, [[3, 6, 9], [3, 6, 9]]), [4, 6], bw, comp)[0] + 1e-9
    rng = np.random.default_rng(2)
    for _ in range(12):
        n_req, L = int(rng.integers(1, 4)), int(rng.integers(2, 9))
        b = rng.integers(1, 30, size=n_req)
        comp = rng.uniform(0.5, 2.0, size=L)
        bw = float(rng.uniform(1.0, 10.0))
        slots = int(rng.integers(1, 3))
        cap = int(b.sum() * L * rng.uniform(0.3, 1.1))
        tw, xw = lm.exhaustive_search(b, L, cap, slots, bw, comp)
        if xw is None:
            with pytest.raises(orbit.OrbitError) as e:
                orbit.orbit_plan_search(b, L, cap, bw, comp, prefetch_slots=slots)
            assert e.value.code == orbit.ORBIT_E_CAPACITY
            continue
        t, x, _ = orbit.orbit_plan_search(b, L, cap, bw, comp, prefetch_slots=slots)
        assert abs(t - tw) <= 1e-9 * tw and x.tolist() == xw.tolist()
        # the staggered space (request r's pattern rotated by r layers), against the same brute force
        ts, xs = lm.exhaustive_search(b, L, cap, slots, bw, comp, stagger=True)
        t2, x2, _ = orbit.orbit_plan_search(b, L, cap, bw, comp, prefetch_slots=slots, stagger=True)
        assert abs(t2 - ts) <= 1e-9 * ts and x2.tolist() == xs.tolist()
        assert sorted((x2 == 0).sum(axis=1).tolist()) != [] and ref.feasible(b, x2, cap, slots)


def test_descent_mode_is_feasible_and_not_worse_than_uniform():
    rng = np.random.default_rng(3)
    L, n_req = 32, 16
    b = rng.integers(512, 2048, size=n_req)
    comp = np.full(L, 0.25)
    bw = 900.0
    cap = int(b.sum() * L * 0.8)
    t, x, evals = orbit.orbit_plan_search(b, L, cap, bw, comp, prefetch_slots=2, max_evals=10000)
    assert ref.feasible(b, x, cap, 2) and evals < 10000
    best_uniform = min(lm.simulate_prefetch(np.tile(lm.distance_pattern(L, c), (n_req, 1)), b, bw, comp)[0]
                       for c in lm.candidate_counts(L)
                       if ref.feasible(b, np.tile(lm.distance_pattern(L, c), (n_req, 1)), cap, 2))
    assert t <= best_uniform + 1e-9
    assert abs(t - lm.simulate_prefetch(x, b, bw, comp)[0]) <= 1e-9 * t


def test_descent_stops_at_the_evaluation_cap():
    """max_evals bounds the descent too: it returns the best plan seen so far (never worse than the best
    uniform plan, which is always tried) and reports how many placements it simulated."""
    rng = np.random.default_rng(4)
    L, n_req = 32, 24
    b = rng.integers(512, 2048, size=n_req)
    comp, bw = np.full(L, 0.25), 900.0
    cap = int(b.sum() * L * 0.8)
    t_free, _, ev_free = orbit.orbit_plan_search(b, L, cap, bw, comp, prefetch_slots=2, max_evals=100000)
    t_cap, x_cap, ev_cap = orbit.orbit_plan_search(b, L, cap, bw, comp, prefetch_slots=2, max_evals=40)
    assert ev_cap <= 40 < ev_free and ref.feasible(b, x_cap, cap, 2)
    assert t_free <= t_cap + 1e-9
    assert abs(t_cap - lm.simulate_prefetch(x_cap, b, bw, comp)[0]) <= 1e-9 * t_cap


# ------------------------------------------------------------------ background planner (Section 4)

def test_background_planner_delivers_the_same_plans_one_iteration_later():
    """The planner thread solves the next iteration's problem while the caller does other work;
    what it delivers equals the synchronous search, tickets grow, a newer result supersedes an
    uncollected one, and an infeasible job surfaces as ORBIT_E_CAPACITY."""
    rng = np.random.default_rng(3)
    L = 8
    comp = rng.uniform(0.5, 1.5, size=L)
    p = orbit.BackgroundPlanner()
    assert p.poll() is None and p.poll(wait=True) is None          # nothing submitted yet
    last = 0
    for it in range(6):
        b = rng.integers(1, 30, size=4)
        budget = int(b.sum() * L * rng.uniform(0.4, 1.0))
        stag = it % 3 == 0
        t = p.submit(b, L, budget, 3.0, comp, prefetch_slots=1 + it % 2, stagger=stag)
        assert t > last
        last = t
        try:
            want = orbit.orbit_plan_search(b, L, budget, 3.0, comp, prefetch_slots=1 + it % 2, stagger=stag)
        except orbit.OrbitError as e:
            assert e.code == orbit.ORBIT_E_CAPACITY
            with pytest.raises(orbit.OrbitError) as e2:
                p.poll(wait=True)
            assert e2.value.code == orbit.ORBIT_E_CAPACITY
            continue
        ticket, tb, x, ev = p.poll(wait=True)
        assert ticket == t and tb == want[0] and ev == want[2] and np.array_equal(x, want[1])
        assert p.poll() is None                                     # collected exactly once
    # two submissions, one collection: the newest finished plan is what comes back
    b1, b2 = np.array([5, 9, 2]), np.array([20, 1, 1])
    p.submit(b1, L, 10 ** 6, 3.0, comp)
    t2 = p.submit(b2, L, 40, 3.0, comp)
    ticket, tb, x, _ = p.poll(wait=True)
    want = orbit.orbit_plan_search(b2, L, 40, 3.0, comp)
    assert ticket == t2 and tb == want[0] and np.array_equal(x, want[1])
    assert p.poll(wait=True) is None
    # infeasible: nothing fits into zero blocks with a prefetch buffer
    p.submit(np.array([4, 4]), L, 0, 3.0, comp)
    with pytest.raises(orbit.OrbitError) as e:
        p.poll(wait=True)
    assert e.value.code == orbit.ORBIT_E_CAPACITY
    with pytest.raises(orbit.OrbitError):
        p.submit(np.array([-1]), L, 10, 3.0, comp)
    p.close()


def test_background_planner_runs_while_the_caller_works():
    """A long search (large pruned space, exhaustive) is in flight while the caller keeps polling
    without blocking; destroying a planner with a job in flight joins cleanly."""
    L = 32
    comp = np.full(L, 1.0)
    b = np.arange(1, 6) * 7
    p = orbit.BackgroundPlanner()
    t = p.submit(b, L, int(b.sum() * L * 0.7), 2.0, comp, max_evals=200000)       # 11^5 = 161051 points
    polls = 0
    while True:
        got = p.poll()
        polls += 1
        if got is not None:
            break
        import time
        time.sleep(0.01)
    assert got[0] == t and got[3] > 1000
    want = orbit.orbit_plan_search(b, L, int(b.sum() * L * 0.7), 2.0, comp, max_evals=200000)
    assert got[1] == want[0] and np.array_equal(got[2], want[1])
    p.submit(b, L, int(b.sum() * L * 0.7), 2.0, comp, max_evals=200000)
    p.close()                                                       # job still running: must not hang or crash


def test_staggered_patterns_need_a_smaller_prefetch_buffer():
    """Same offload counts, rotated per request: Eq. (1)'s B_buf shrinks, so a budget that rejects
    the aligned plan admits the staggered one, and the search exploits it."""
    L, n_req = 32, 8
    b = np.full(n_req, 100)
    row = lm.distance_pattern(L, 8)                                  # every 4th layer offloaded
    aligned = np.tile(row, (n_req, 1))
    rotated = np.stack([np.roll(row, r) for r in range(n_req)])
    assert ref.prefetch_buffer_blocks(b, aligned) == 800 and ref.prefetch_buffer_blocks(b, rotated) == 200
    comp, bw = np.full(L, 1.0), 50.0
    cap = ref.resident_blocks(b, rotated) + 2 * 200                   # fits rotated, not aligned
    assert ref.feasible(b, rotated, cap, 2) and not ref.feasible(b, aligned, cap, 2)
    t_plain, _, _ = orbit.orbit_plan_search(b, L, cap, bw, comp, prefetch_slots=2, max_evals=5000)
    t_stag, x_stag, _ = orbit.orbit_plan_search(b, L, cap, bw, comp, prefetch_slots=2, max_evals=5000, stagger=True)
    assert ref.feasible(b, x_stag, cap, 2)
    assert t_stag < t_plain
    assert abs(t_stag - lm.simulate_prefetch(x_stag, b, bw, comp)[0]) <= 1e-9 * t_stag


# ------------------------------------------------------------------ Pause-Resume fallback (Section 3.4)

def test_pause_victim_rule():
    """Section 3.4: the victim is the request with the largest sum of KV blocks and deposited
    tokens.  Hand-worked: blocks (10, 40, 25) alone pick request 1; 30 deposited tokens on request 2
    make it 55 > 40 and move the choice; a tie goes to the later request (our rule)."""
    assert lm.pause_victim([10, 40, 25], [0, 0, 0]) == 1
    assert lm.pause_victim([10, 40, 25], [0, 0, 30]) == 2
    assert lm.pause_victim([10, 40, 25], [35, 5, 20]) == 2           # 45, 45, 45: the last of the tied
    assert lm.pause_victim([7], [0]) == 0


def test_fallback_pauses_until_the_rest_fits():
    L, comp, bw = 6, [1.0] * 6, 3.0
    # everything fits: nobody is paused and the plan equals the plain search
    t, x, paused = orbit.orbit_plan_search_or_pause([3, 6], [0, 0], L, 70, bw, comp)
    t0, x0, _ = orbit.orbit_plan_search([3, 6], L, 70, bw, comp)
    assert paused.tolist() == [0, 0] and t == t0 and x.tolist() == x0.tolist()
    # 12 blocks, one prefetch buffer: with every layer offloaded Eq. (1) needs B_buf = 3 + 6 = 9 <= 12, so the
    # pair still has a feasible (if slow) plan and nobody is paused
    _, _, paused = orbit.orbit_plan_search_or_pause([3, 6], [0, 0], L, 12, bw, comp)
    assert paused.tolist() == [0, 0]
    # 8 blocks: B_buf = 9 > 8 -> request 1 (6 blocks) is paused; request 0 alone (3 <= 8) stays
    t, x, paused = orbit.orbit_plan_search_or_pause([3, 6], [0, 0], L, 8, bw, comp)
    assert paused.tolist() == [0, 1] and ref.feasible([3], x[:1], 8)
    # deposited tokens move the choice: request 0 now scores 3 + 5 = 8 > 6
    _, _, paused = orbit.orbit_plan_search_or_pause([3, 6], [5, 0], L, 8, bw, comp)
    assert paused.tolist() == [1, 0]
    # nothing fits at all: everyone is paused, the empty batch costs the compute time only
    t, _, paused = orbit.orbit_plan_search_or_pause([3, 6], [0, 0], L, 2, bw, comp)
    assert paused.tolist() == [1, 1] and t == 6.0
    rng = np.random.default_rng(9)
    n_paused_total = 0
    for _ in range(25):
        n_req, L = int(rng.integers(1, 4)), int(rng.integers(2, 7))
        b = rng.integers(1, 30, size=n_req)
        dep = rng.integers(0, 20, size=n_req)
        comp = rng.uniform(0.5, 2.0, size=L)
        bw = float(rng.uniform(1.0, 10.0))
        slots = int(rng.integers(1, 3))
        cap = int(b.sum() * rng.uniform(0.2, 2.0))
        stag = bool(rng.integers(0, 2))
        tw, xw, pw = lm.search_or_pause(b, dep, L, cap, slots, bw, comp, stagger=stag)
        t, x, paused = orbit.orbit_plan_search_or_pause(b, dep, L, cap, bw, comp, prefetch_slots=slots, stagger=stag)
        assert sorted(np.flatnonzero(paused).tolist()) == sorted(pw)
        assert abs(t - tw) <= 1e-9 * tw
        kept = [i for i in range(n_req) if not paused[i]]
        if kept:
            assert x[kept].tolist() == xw.tolist() and ref.feasible(b[kept], x[kept], cap, slots)
        n_paused_total += len(pw)
    assert n_paused_total > 5
