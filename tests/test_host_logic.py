"""CPU-only tests of liborbit's host logic through the C ABI (ORBIT_FLAG_HOST_ONLY contexts make
no GPU call): exported symbols, Eq. (1), block tables, delta migration, staging schedule and
gating rules, split-K work list.  Expected values come from the oracle's capacity functions,
from brute force written here, or from the numbers printed in the paper's example."""
import itertools
import json
import os
import re

import numpy as np
import pytest

import paper_2601_10729_amd as orbit
from paper_2601_10729_amd import OrbitContext, OrbitError, orbit_plan_check
from oracle import reference as ref

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
PAGE = 2 * 8 * 16 * 128 * 2        # bytes of one block for 8 kv heads


def ctx(L=4, Hq=32, Hkv=8, max_req=8, max_tokens=8192, hbm_pages=4096, host_pages=4096, slots=1, window=0,
        chunk=0, zero_copy=False):
    page = 2 * Hkv * 16 * 128 * 2
    return OrbitContext(n_layers=L, n_q_heads=Hq, n_kv_heads=Hkv, max_requests=max_req,
                        max_tokens_per_request=max_tokens, prefetch_slots=slots, decode_window=window,
                        chunk_tokens=chunk, host_only=True, zero_copy=zero_copy, hbm_arena_bytes=hbm_pages * page,
                        host_arena_bytes=host_pages * page)


# ------------------------------------------------------------------ boundary

def test_library_exports_every_declared_symbol():
    with open(os.path.join(ROOT, "include", "orbit.h")) as f:
        declared = re.findall(r"ORBIT_API[^;(]*?\b(orbit_[a-z0-9_]+)\s*\(", f.read())
    assert len(declared) >= 15 and len(set(declared)) == len(declared)
    L = orbit.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert sorted(declared) == sorted(orbit.EXPORTS)


def test_create_rejects_unsupported_shapes():
    for kw in (dict(head_dim=64), dict(page_tokens=32), dict(n_q_heads=30), dict(n_q_heads=136, n_kv_heads=8),
               dict(chunk_tokens=100), dict(prefetch_slots=0), dict(max_requests=0),
               # index ranges: work items beyond 2^31, a page table beyond 2^34 entries
               dict(max_tokens_per_request=1 << 24, chunk_tokens=32, n_kv_heads=128, n_q_heads=128, n_layers=128,
                    max_requests=256),
               dict(max_tokens_per_request=1 << 24, n_layers=128, max_requests=256)):
        args = dict(n_layers=2, n_q_heads=32, n_kv_heads=8, max_requests=4, max_tokens_per_request=1024,
                    host_only=True, hbm_arena_bytes=PAGE * 64, host_arena_bytes=PAGE * 64)
        args.update(kw)
        with pytest.raises(OrbitError) as e:
            OrbitContext(**args)
        assert e.value.code == orbit.ORBIT_E_INVAL


def test_gpu_context_without_arena_is_an_error_not_a_fallback():
    with pytest.raises(OrbitError):
        OrbitContext(n_layers=2, n_q_heads=32, n_kv_heads=8, max_requests=4, max_tokens_per_request=1024)


# ------------------------------------------------------------------ Eq. (1)

def test_plan_check_reproduces_the_papers_example():
    with open(os.path.join(HERE, "golden", "toy_example.json")) as f:
        toy = json.load(f)
    L = toy["n_layers"]

    def x(off):
        m = np.ones((2, L), dtype=np.uint8)
        for r, layers in enumerate(off):
            for l in layers:
                m[r, l - 1] = 0
        return m
    n1 = [b * 16 for b in toy["step1"]["blocks_per_layer"]]
    n16 = [b * 16 for b in toy["step16"]["blocks_per_layer"]]
    A, B, C = x([[3, 6, 9], [3, 6, 9]]), x([[], [3, 6, 9]]), x([[4, 8], [3, 6, 9]])
    assert orbit_plan_check(n1, A)[1:3] == (9, 63)
    assert orbit_plan_check(n16, A)[1:3] == (10, 70)
    assert orbit_plan_check(n1, x([[3, 6], [3, 6]]))[2] == 72
    assert orbit_plan_check(n1, B)[2] == 69
    assert orbit_plan_check(n16, B)[2] == toy["placement_B"]["gpu_blocks_used_step16"]
    assert orbit_plan_check(n16, C)[2] == toy["gpu_blocks"]
    # the same verdicts through orbit_plan_load with a 70-block budget (2 kv heads here)
    page = 2 * 2 * 16 * 128 * 2
    c = OrbitContext(n_layers=L, n_q_heads=8, n_kv_heads=2, max_requests=2, max_tokens_per_request=1024,
                     host_only=True, hbm_arena_bytes=200 * page, host_arena_bytes=200 * page)
    c.plan_load([1, 2], n1, B, hbm_budget_bytes=70 * page)
    assert c.get_plan_info()["resident_blocks"] + c.get_plan_info()["staging_blocks"] == 69
    c2 = OrbitContext(n_layers=L, n_q_heads=8, n_kv_heads=2, max_requests=2, max_tokens_per_request=1024,
                      host_only=True, hbm_arena_bytes=200 * page, host_arena_bytes=200 * page)
    with pytest.raises(OrbitError) as e:
        c2.plan_load([1, 2], n16, B, hbm_budget_bytes=70 * page)
    assert e.value.code == orbit.ORBIT_E_CAPACITY
    c2.plan_load([1, 2], n16, C, hbm_budget_bytes=70 * page)


def test_plan_check_matches_oracle_on_random_plans():
    rng = np.random.default_rng(0)
    for _ in range(50):
        B, L = int(rng.integers(1, 9)), int(rng.integers(1, 12))
        n = rng.integers(0, 5000, size=B)
        x = rng.integers(0, 2, size=(B, L)).astype(np.uint8)
        k, win = int(rng.integers(1, 4)), int(rng.integers(0, 40))
        b = ref.blocks(n + win)
        want = (ref.resident_blocks(b, x), ref.prefetch_buffer_blocks(b, x), ref.gpu_blocks_needed(b, x, k),
                int(((1 - x.astype(np.int64)) * b[:, None]).sum()))
        assert orbit_plan_check(n, x, prefetch_slots=k, decode_window=win) == want


def test_capacity_boundary_and_atomic_failure():
    c = ctx(L=3, hbm_pages=1000)
    n = [100, 900]
    x = np.array([[1, 0, 1], [0, 1, 1]], dtype=np.uint8)
    need = orbit_plan_check(n, x)[2]
    with pytest.raises(OrbitError) as e:
        c.plan_load([7, 8], n, x, hbm_budget_bytes=(need - 1) * PAGE)
    assert e.value.code == orbit.ORBIT_E_CAPACITY
    with pytest.raises(OrbitError):
        c.get_plan_info()                                   # nothing was installed
    c.plan_load([7, 8], n, x, hbm_budget_bytes=need * PAGE)
    before = [c.get_pages(r, l) for r in (7, 8) for l in range(3)]
    for bad in (dict(ids=[7, 7]), dict(n=[101, 900]), dict(budget=(need - 1) * PAGE, x=np.ones((2, 3), np.uint8))):
        with pytest.raises(OrbitError):
            c.plan_load(bad.get("ids", [7, 8]), bad.get("n", n), bad.get("x", x),
                        hbm_budget_bytes=bad.get("budget", need * PAGE))
    after = [c.get_pages(r, l) for r in (7, 8) for l in range(3)]
    for a, b in zip(before, after):
        assert a["tier"] == b["tier"] and a["host_first_page"] == b["host_first_page"]
        assert np.array_equal(a["pages"], b["pages"])


def test_host_arena_capacity():
    c = ctx(L=2, host_pages=10)
    with pytest.raises(OrbitError) as e:
        c.plan_load([1], [16 * 11], np.array([[0, 1]], dtype=np.uint8))
    assert e.value.code == orbit.ORBIT_E_HOST_CAPACITY
    c.plan_load([1], [16 * 10], np.array([[0, 1]], dtype=np.uint8))


# ------------------------------------------------------------------ block tables

def _layout_invariants(c, ids, L):
    info = c.get_plan_info()
    first, nstage = info["staging_first_page"], info["staging_blocks"]
    seen_hbm, host_runs, in_place = set(), [], set()
    per_layer_stage = {l: [] for l in range(L)}
    for r in ids:
        for l in range(L):
            p = c.get_pages(r, l)
            pages = [int(v) for v in p["pages"]]
            if p["tier"] == 1:
                assert all(0 <= q < first for q in pages)
                assert not (seen_hbm & set(pages))
                seen_hbm |= set(pages)
            elif p["tier"] == 2:                # on its way to the host, read in place: pages it no longer owns
                assert all(0 <= q < first for q in pages)
                in_place |= set(pages)
                host_runs.append((p["host_first_page"], p["host_first_page"] + 1))
            else:
                assert pages == list(range(pages[0], pages[0] + len(pages)))       # contiguous staging range
                assert first <= pages[0] and pages[-1] < first + nstage
                per_layer_stage[l].append((pages[0], pages[-1]))
                host_runs.append((p["host_first_page"], p["host_first_page"] + len(pages)))
    assert len(seen_hbm) == info["resident_blocks"]
    assert not (seen_hbm & in_place)                        # nothing this plan owns was handed a page still read in place
    for l, spans in per_layer_stage.items():                # requests of one layer never share staging pages
        spans.sort()
        assert all(a[1] < b[0] for a, b in zip(spans, spans[1:]))
    host_runs.sort()
    assert all(a[1] <= b[0] for a, b in zip(host_runs, host_runs[1:]))
    return info


def test_block_tables_are_consistent_for_random_plans():
    rng = np.random.default_rng(1)
    for trial in range(20):
        B, L = int(rng.integers(1, 7)), int(rng.integers(1, 7))
        c = ctx(L=L, hbm_pages=6000, host_pages=6000, slots=int(rng.integers(1, 3)), window=int(rng.integers(0, 50)))
        ids = [int(v) for v in rng.permutation(100)[:B]]
        n = rng.integers(1, 3000, size=B)
        x = rng.integers(0, 2, size=(B, L)).astype(np.uint8)
        c.plan_load(ids, n, x)
        info = _layout_invariants(c, ids, L)
        assert info["buffer_blocks"] == ref.prefetch_buffer_blocks(ref.blocks(n + c.cfg.decode_window), x)
        assert info["staging_first_page"] + info["staging_blocks"] == info["budget_blocks"]


def test_plan_switch_moves_exactly_the_delta():
    rng = np.random.default_rng(2)
    B, L = 5, 6
    c = ctx(L=L, hbm_pages=5000, host_pages=5000)
    ids = list(range(10, 10 + B))
    n = rng.integers(1, 2000, size=B)
    b = ref.blocks(n)
    x0 = rng.integers(0, 2, size=(B, L)).astype(np.uint8)
    c.plan_load(ids, n, x0)
    assert c.get_plan_info()["moved_to_host_blocks"] == 0 and c.get_plan_info()["moved_to_hbm_blocks"] == 0
    for _ in range(6):
        x1 = rng.integers(0, 2, size=(B, L)).astype(np.uint8)
        c.plan_load(ids, n, x1)
        info = _layout_invariants(c, ids, L)
        assert info["moved_to_host_blocks"] == int((((x0 == 1) & (x1 == 0)) * b[:, None]).sum())
        # a block that left HBM in the previous switch and is still read in place there takes its pages back
        assert info["moved_to_hbm_blocks"] + info["reclaimed_blocks"] == int((((x0 == 0) & (x1 == 1)) * b[:, None]).sum())
        x0 = x1
    c.plan_load(ids, n, x0)                                # identical plan: nothing moves
    info = c.get_plan_info()
    assert (info["moved_to_host_blocks"], info["moved_to_hbm_blocks"], info["relocated_blocks"]) == (0, 0, 0)
    # drop two requests, add one
    keep = ids[:3] + [77]
    c.plan_load(keep, list(n[:3]) + [500], np.ones((4, L), dtype=np.uint8))
    _layout_invariants(c, keep, L)
    with pytest.raises(OrbitError) as e:
        c.get_pages(ids[4], 0)
    assert e.value.code == orbit.ORBIT_E_NOT_FOUND


def test_growing_staging_region_relocates_resident_blocks():
    L = 1
    c = ctx(L=L, hbm_pages=100)
    c.plan_load([1, 2], [16 * 40, 16 * 40], np.ones((2, L), dtype=np.uint8), hbm_budget_bytes=100 * PAGE)
    # a third request, offloaded, needs a 20-block staging region at the top of the budget
    with pytest.raises(OrbitError):
        c.plan_load([1, 2, 3], [640, 640, 16 * 21], np.array([[1], [1], [0]], np.uint8), hbm_budget_bytes=100 * PAGE)
    c.plan_load([1, 2, 3], [640, 640, 16 * 20], np.array([[1], [1], [0]], np.uint8), hbm_budget_bytes=100 * PAGE)
    info = _layout_invariants(c, [1, 2, 3], L)
    assert info["staging_first_page"] == 80 and info["relocated_blocks"] == 0   # the lowest pages were in use
    # shrink the budget: resident blocks above the new staging start must move down
    c2 = ctx(L=1, hbm_pages=100)
    c2.plan_load([1, 2], [16 * 30, 16 * 30], np.ones((2, 1), dtype=np.uint8))
    c2.plan_load([2], [16 * 30], np.ones((1, 1), dtype=np.uint8), hbm_budget_bytes=30 * PAGE)
    info = _layout_invariants(c2, [2], 1)
    assert info["relocated_blocks"] == 30 and max(c2.get_pages(2, 0)["pages"]) < 30


# ------------------------------------------------------------------ appends and the decode window

def test_block_growth_and_window_expiry():
    c = ctx(L=2, window=20)
    c.plan_load([5], [40], np.array([[1, 0]], dtype=np.uint8))       # reserves ceil(60/16) = 4 blocks
    assert len(c.get_pages(5, 0)["pages"]) == 4
    steps = 0
    with pytest.raises(OrbitError) as e:
        for _ in range(100):
            c.step(None, None, None, None)
            steps += 1
    assert e.value.code == orbit.ORBIT_E_STATE and steps == 64 - 40   # 4 blocks hold 64 tokens
    assert c.get_pages(5, 0)["length"] == 64 and c.get_pages(5, 1)["length"] == 64
    c.plan_load([5], [64], np.array([[1, 0]], dtype=np.uint8))        # a new plan opens a new window
    c.step(None, None, None, None)
    assert c.get_pages(5, 1)["length"] == 65
    # per-layer appends through orbit_kv_append
    c.kv_append(5, 0, 1, 1)
    assert c.get_pages(5, 0)["length"] == 66 and c.get_pages(5, 1)["length"] == 65
    with pytest.raises(OrbitError):
        c.step(None, None, None, None) if False else c.plan_load([5], [65], np.array([[1, 0]], dtype=np.uint8))


# ------------------------------------------------------------------ work list

def _expected_chunk(n, Hkv, fixed=0, n_cu=256):
    if fixed:
        return fixed
    if max(n) <= 512 or (max(n) <= 4096 and len(n) * Hkv * 2 >= n_cu):   # short, or whole requests fill half of the machine
        return max(128, 1 << int(max(n) - 1).bit_length())
    for c in (4096, 2048, 1024, 512, 256):
        if sum(-(-int(v) // c) for v in n) * Hkv >= n_cu:
            return c
    return 128


@pytest.mark.parametrize("chunk", [0, 64, 1024])
@pytest.mark.parametrize("lengths", [(1, 64, 65, 191, 777, 5000), (2048,), (100,), (7700, 7700, 2250, 1024),
                                     (30000, 9000, 17, 1, 1, 25000, 33, 8191), (8192,), (32768,),
                                     tuple(500 + 7 * r for r in range(16)), tuple(20000 + 977 * r for r in range(16))])
def test_work_segments_match_brute_force(chunk, lengths):
    L, Hkv = 2, 8
    n = np.array(lengths)
    B = len(n)
    c = ctx(L=L, max_req=16, max_tokens=40000, hbm_pages=80000, chunk=chunk)
    c.plan_load(list(range(B)), n, np.ones((B, L), dtype=np.uint8))
    items = [[int(v) for v in row] for row in c.get_work_items(1)]
    C = _expected_chunk(lengths, Hkv, chunk)
    want = [(r, t, min(C, int(n[r]) - t)) for r in range(B) for t in range(0, int(n[r]), C)]
    assert [tuple(row[:3]) for row in items] == want
    # launch order: a permutation, longest segment first, ties in list order
    rank = [row[3] for row in items]
    assert sorted(rank) == list(range(len(items)))
    by_rank = sorted(range(len(items)), key=lambda i: rank[i])
    assert by_rank == sorted(range(len(items)), key=lambda i: (-items[i][2], i))


def test_chunk_choice_examples():
    """One request of 8K tokens on 8 kv heads: 256-token chunks give all 256 units a workgroup; 16 short requests
    already fill half of the machine and are not cut; a 16 x 20K batch uses the largest chunk."""
    L = 1
    c = ctx(L=L, max_req=16, max_tokens=40000, hbm_pages=50000)
    for k, (n, want) in enumerate([([8192], 256), ([2048], 128), ([300], 512), ([600], 128), ([32768], 1024), ([8192] * 4, 1024),
                                   ([500] * 16, 512), ([2048] * 16, 2048), ([5000] * 16, 4096), ([20000] * 16, 4096)]):
        ids = list(range(100 * k, 100 * k + len(n)))
        c.plan_load(ids, n, np.ones((len(n), L), dtype=np.uint8))
        items = c.get_work_items(0)
        assert int(items[:, 2].max()) == min(want, max(n)), (n, want)
        assert len(items) == sum(-(-v // want) for v in n)


@pytest.mark.parametrize("Hkv", [1, 2, 8, 16, 128])
def test_work_list_always_fits_the_buffers_sized_at_creation(Hkv):
    """The buffers hold max_requests x ceil(max_tokens / 4096) + 2 x (256 / Hkv) + max_requests segments; the
    chunk choice never produces more (a smaller chunk is only taken when the next larger one leaves units idle)."""
    rng = np.random.default_rng(Hkv)
    max_req, max_tokens, L = 12, 20000, 1
    page = 2 * Hkv * 16 * 128 * 2
    c = OrbitContext(n_layers=L, n_q_heads=Hkv, n_kv_heads=Hkv, max_requests=max_req, max_tokens_per_request=max_tokens,
                     host_only=True, hbm_arena_bytes=page * (max_req * (max_tokens // 16 + 2)), host_arena_bytes=page)
    bound = max_req * -(-max_tokens // 4096) + 2 * max(1, 256 // Hkv) + max_req
    nid = 0
    for trial in range(60):
        B = int(rng.integers(1, max_req + 1))
        kind = trial % 3
        n = (rng.integers(1, 600, size=B) if kind == 0 else
             rng.integers(1, max_tokens + 1, size=B) if kind == 1 else
             np.maximum(1, (2.0 ** rng.uniform(0, np.log2(max_tokens), size=B)).astype(np.int64)))
        ids = list(range(nid, nid + B))
        nid += B
        c.plan_load(ids, n, np.ones((B, L), dtype=np.uint8))
        items = c.get_work_items(0)
        assert len(items) <= bound
        C = _expected_chunk([int(v) for v in n], Hkv)
        assert len(items) == sum(-(-int(v) // C) for v in n)


def test_attention_on_an_empty_request_is_an_error():
    c = ctx(L=1)
    c.plan_load([1, 2], [0, 5], np.ones((2, 1), dtype=np.uint8))
    with pytest.raises(OrbitError) as e:
        c.decode_attention(0, None, None)
    assert e.value.code == orbit.ORBIT_E_INVAL


# ------------------------------------------------------------------ staging schedule and gating

def test_copy_schedule_order_and_ring_layout():
    rng = np.random.default_rng(4)
    for slots in (1, 2, 3):
        B, L = 5, 7
        c = ctx(L=L, hbm_pages=8000, host_pages=8000, slots=slots)
        n = rng.integers(1, 3000, size=B)
        b = ref.blocks(n)
        x = rng.integers(0, 2, size=(B, L)).astype(np.uint8)
        c.plan_load(list(range(B)), n, x)
        info = c.get_plan_info()
        rows = c.get_copy_schedule()
        # brute force: layers ascending; inside a layer requests by ascending block count (stable);
        # each layer's range packed round-robin into the staging region, wrapping to 0 when it does not fit
        want, cursor = [], 0
        for l in range(L):
            off = [r for r in range(B) if x[r, l] == 0]
            if not off:
                continue
            off.sort(key=lambda r: b[r])
            tot = int(sum(b[r] for r in off))
            if cursor + tot > info["staging_blocks"]:
                cursor = 0
            at = cursor
            for r in off:
                want.append([l, r, info["staging_first_page"] + at, int(b[r]), cursor])
                at += int(b[r])
            cursor += tot
        assert rows.tolist() == want


def test_staging_range_is_reused_only_after_its_layer_was_attended():
    # single buffer (the paper's B_buf): two offloaded layers share the staging range
    c = ctx(L=3, slots=1)
    c.plan_load([1], [100], np.array([[0, 1, 0]], dtype=np.uint8))
    c.kv_prefetch(0)
    c.kv_prefetch(0)                                        # already prefetched: no-op
    c.kv_prefetch(1)                                        # nothing offloaded: no-op
    with pytest.raises(OrbitError) as e:
        c.kv_prefetch(2)                                    # would overwrite layer 0's data
    assert e.value.code == orbit.ORBIT_E_STATE
    c.decode_attention(0, None, None)
    c.kv_prefetch(2)                                        # layer 0 was attended: its range is free
    with pytest.raises(OrbitError):
        c.step(None, None, None, None)                      # layer 2 prefetched but never attended
    c.decode_attention(2, None, None)
    # two slots: both layers can be in flight at once
    c2 = ctx(L=3, slots=2)
    c2.plan_load([1], [100], np.array([[0, 1, 0]], dtype=np.uint8))
    c2.kv_prefetch(0)
    c2.kv_prefetch(2)
    c2.decode_attention(0, None, None)
    c2.decode_attention(2, None, None)
    for _ in range(3):
        c2.step(None, None, None, None) if c2.cfg.decode_window else None


def test_steps_run_for_every_placement_of_a_small_batch():
    # exhaustive over 2 requests x 3 layers: the schedule never deadlocks, lengths advance
    for bits in itertools.product([0, 1], repeat=6):
        x = np.array(bits, dtype=np.uint8).reshape(2, 3)
        for slots in (1, 2):
            c = ctx(L=3, slots=slots, window=3)
            c.plan_load([1, 2], [30, 70], x)
            for _ in range(3):
                c.step(None, None, None, None)
            assert c.get_pages(2, 2)["length"] == 73


# ------------------------------------------------------------------ pause / resume (removable cache)

def test_pause_keeps_blocks_and_evicts_only_what_is_needed():
    L = 4
    c = ctx(L=L, hbm_pages=200, host_pages=2000)
    ones = lambda b: np.ones((b, L), dtype=np.uint8)
    c.plan_load([1, 2, 3], [160, 240, 320], ones(3))                 # 10 + 15 + 20 blocks per layer
    before = [c.get_pages(3, l)["pages"].copy() for l in range(L)]
    c.request_pause(3)
    info = c.get_plan_info()
    assert (info["n_requests"], info["paused_requests"], info["paused_resident_blocks"]) == (2, 1, 80)
    assert (info["evicted_blocks"], info["moved_to_host_blocks"], info["moved_to_hbm_blocks"]) == (0, 0, 0)
    for l in range(L):
        p = c.get_pages(3, l)
        assert p["tier"] == 1 and np.array_equal(p["pages"], before[l])
    with pytest.raises(OrbitError) as e:
        c.request_pause(3)
    assert e.value.code == orbit.ORBIT_E_STATE
    assert sorted({int(r) for r, _, _, _ in c.get_work_items(0)}) == [0, 1]    # only the two active requests
    # a new request needs 40 blocks: 100 + 40 + 80 paused > 200, so exactly one paused layer (20 blocks) goes
    c.plan_load([1, 2, 4], [160, 240, 160], ones(3))
    info = c.get_plan_info()
    assert (info["evicted_blocks"], info["paused_resident_blocks"], info["paused_requests"]) == (20, 60, 1)
    assert c.get_pages(3, 3)["tier"] == 0                             # highest layer first
    for l in range(3):
        p = c.get_pages(3, l)
        assert p["tier"] == 1 and np.array_equal(p["pages"], before[l])
    _layout_invariants(c, [1, 2, 4], L)
    # resume with the evicted layer left on the host: nothing moves
    x = ones(3)
    x[2, 3] = 0
    c.plan_load([1, 2, 3], [160, 240, 320], x)
    info = c.get_plan_info()
    assert (info["moved_to_hbm_blocks"], info["moved_to_host_blocks"], info["evicted_blocks"]) == (0, 0, 0)
    assert info["paused_requests"] == 0
    with pytest.raises(OrbitError):
        c.get_pages(4, 0)                                             # request 4 was active and not listed: dropped
    _layout_invariants(c, [1, 2, 3], L)
    # pause again, then resume wanting every layer in HBM: only the evicted layer comes back
    c.request_pause(3)
    c.plan_load([1, 2, 3], [160, 240, 320], ones(3))
    assert c.get_plan_info()["moved_to_hbm_blocks"] == 20
    # drop
    c.request_pause(2)
    with pytest.raises(OrbitError):
        c.request_drop(1)                                             # active
    c.request_drop(2)
    with pytest.raises(OrbitError) as e:
        c.request_drop(2)
    assert e.value.code == orbit.ORBIT_E_NOT_FOUND
    c.plan_load([1, 3, 9], [160, 320, 16 * 15], ones(3))              # the freed blocks are usable again
    _layout_invariants(c, [1, 3, 9], L)


def test_paused_blocks_leave_a_growing_staging_region():
    L = 2
    c = ctx(L=L, hbm_pages=100, host_pages=1000)
    c.plan_load([1, 2], [16 * 20, 16 * 25], np.ones((2, L), dtype=np.uint8))    # pages 0..89 in use
    c.request_pause(2)
    # request 3 is offloaded: staging region of 30 blocks = pages 70..99, where paused blocks sit
    c.plan_load([1, 3], [16 * 20, 16 * 30], np.array([[1, 1], [0, 0]], dtype=np.uint8))
    info = c.get_plan_info()
    assert info["staging_first_page"] == 70
    for l in range(L):
        p = c.get_pages(2, l)
        assert p["tier"] == 0 or max(p["pages"]) < 70
    assert info["evicted_blocks"] in (25, 50) and info["evicted_blocks"] + info["paused_resident_blocks"] == 50


def test_empty_batch_and_bad_calls():
    c = ctx(L=2)
    with pytest.raises(OrbitError) as e:
        c.step(None, None, None, None)                                # no plan yet
    assert e.value.code == orbit.ORBIT_E_STATE
    c.plan_load([], [], np.zeros((0, 2), dtype=np.uint8))             # an empty batch is a valid plan
    assert c.get_plan_info()["n_requests"] == 0
    for call in (lambda: c.step(None, None, None, None), lambda: c.decode_attention(0, None, None)):
        with pytest.raises(OrbitError) as e:
            call()
        assert e.value.code == orbit.ORBIT_E_STATE
    with pytest.raises(OrbitError) as e:
        c.kv_prefetch(5)
    assert e.value.code == orbit.ORBIT_E_INVAL
    with pytest.raises(OrbitError) as e:
        c.kv_append(1, 0, 1, 1)
    assert e.value.code == orbit.ORBIT_E_NOT_FOUND
    with pytest.raises(OrbitError) as e:
        c.plan_load(list(range(9)), [1] * 9, np.ones((9, 2), dtype=np.uint8))   # max_requests is 8
    assert e.value.code == orbit.ORBIT_E_INVAL
    with pytest.raises(OrbitError) as e:
        c.plan_load([1], [8193], np.ones((1, 2), dtype=np.uint8))               # beyond max_tokens_per_request
    assert e.value.code == orbit.ORBIT_E_INVAL


def test_zero_copy_mode_charges_no_prefetch_buffer():
    """ORBIT_FLAG_ZERO_COPY drops the B_buf term of Eq. (1): a budget that holds exactly the
    resident blocks is accepted (the staged mode rejects it), nothing is scheduled for copying,
    and offloaded layers have no staging pages."""
    lens = np.array([100, 900, 2000], dtype=np.int32)
    pl = np.array([[1, 1, 0, 0], [1, 0, 1, 0], [0, 0, 1, 1]], dtype=np.uint8)
    ids = np.array([5, 6, 7], dtype=np.int64)
    res, buf, need1, host = orbit_plan_check(lens, pl, 16, 1, 0)
    _, _, need0, _ = orbit_plan_check(lens, pl, 16, 0, 0)
    assert need0 == res == ref.resident_blocks(ref.blocks(lens), pl) and need1 == res + buf and buf > 0
    staged = ctx(slots=1)
    with pytest.raises(OrbitError) as e:
        staged.plan_load(ids, lens, pl, res * PAGE)
    assert e.value.code == orbit.ORBIT_E_CAPACITY
    c = ctx(zero_copy=True, slots=3)
    c.plan_load(ids, lens, pl, res * PAGE)
    info = c.get_plan_info()
    assert info["staging_blocks"] == 0 and info["resident_blocks"] == res and info["host_blocks"] == host
    assert len(c.get_copy_schedule()) == 0
    for r, rid in enumerate(ids):
        for l in range(4):
            pg = c.get_pages(int(rid), l)
            assert pg["tier"] == pl[r, l] and pg["length"] == lens[r]
            if pg["tier"] == 0:
                assert pg["host_first_page"] >= 0 and (pg["pages"] == -1).all()
            else:
                assert (pg["pages"] >= 0).all() and (pg["pages"] < res).all()
    for l in range(4):
        c.kv_prefetch(l)                       # a no-op in this mode
    with pytest.raises(OrbitError) as e:
        c.plan_load(ids, lens, pl, (res - 1) * PAGE)
    assert e.value.code == orbit.ORBIT_E_CAPACITY


def test_batched_append_is_all_or_nothing():
    """orbit_kv_append_batch grows every request of the plan by one token in a layer; when any
    request has used up its reserved blocks nothing changes for anyone."""
    c = ctx(L=2, window=2)
    ids = np.array([1, 2], dtype=np.int64)
    lens = np.array([13, 30], dtype=np.int32)          # reserved: ceil(15/16) = 1 and ceil(32/16) = 2 blocks
    c.plan_load(ids, lens, np.ones((2, 2), dtype=np.uint8), 64 * PAGE)
    for step in range(2):
        for l in range(2):
            c.kv_append_batch(l, None, None)
    assert [c.get_pages(1, l)["length"] for l in range(2)] == [15, 15]
    assert [c.get_pages(2, l)["length"] for l in range(2)] == [32, 32]
    with pytest.raises(OrbitError) as e:
        c.kv_append_batch(0, None, None)                # request 2 would need a third block; request 1 still has room
    assert e.value.code == orbit.ORBIT_E_STATE
    assert c.get_pages(1, 0)["length"] == 15 and c.get_pages(2, 0)["length"] == 32
    c.plan_load(ids, np.array([15, 32], dtype=np.int32), np.ones((2, 2), dtype=np.uint8), 64 * PAGE)
    c.kv_append_batch(0, None, None)
    assert c.get_pages(1, 0)["length"] == 16 and c.get_pages(2, 0)["length"] == 33


# ------------------------------------------------------------------ deferred demotions of a plan switch

def test_demotions_are_deferred_unless_their_pages_are_needed_at_once():
    """A block that leaves HBM in a plan switch may be copied out beside the following steps when the new plan
    needs none of its pages: they lie below the new staging region and no allocation of the switch took them."""
    L, B = 4, 4
    n = [160, 160, 160, 160]                                   # 10 blocks per (request, layer), 160 in all
    ones = np.ones((B, L), dtype=np.uint8)
    # roomy arena: the all-resident plan occupies pages 0..159, the staging region sits at the top of 4096
    c = ctx(L=L, hbm_pages=4096)
    c.plan_load(list(range(B)), n, ones)
    x = ones.copy()
    x[:, 1] = 0                                                # demote layer 1 of every request: 40 blocks
    c.plan_load(list(range(B)), n, x)
    info = c.get_plan_info()
    # a block that stays readable in place sends its last page at once (new tokens go there) and defers the rest
    assert info["moved_to_host_blocks"] == 40 and info["deferred_to_host_blocks"] == 36 and info["in_place_blocks"] == 40
    assert info["relocated_blocks"] == 0
    # back to all-resident, then the same demotion in an arena with no slack: the staging region (40 pages) now
    # covers resident pages 120..159; what lies there must leave or move at once, the rest may still wait
    c = ctx(L=L, hbm_pages=160)
    c.plan_load(list(range(B)), n, ones)
    before = {(r, l): [int(p) for p in c.get_pages(r, l)["pages"]] for r in range(B) for l in range(L)}
    c.plan_load(list(range(B)), n, x)
    info = c.get_plan_info()
    first = info["staging_first_page"]
    assert first == 120 and info["moved_to_host_blocks"] == 40
    in_region = sum(1 for r in range(B) if any(p >= first for p in before[(r, 1)]))
    moved_in = info["relocated_blocks"]
    assert moved_in > 0                                        # residents inside the region moved into freed pages
    assert info["deferred_to_host_blocks"] < 40                # ... so the blocks that freed those pages went at once
    assert info["deferred_to_host_blocks"] % 9 == 0 and info["deferred_to_host_blocks"] <= 36 - 9 * in_region
    assert info["in_place_blocks"] == info["deferred_to_host_blocks"] // 9 * 10
    _layout_invariants(c, list(range(B)), L)
    # zero-copy mode has no staging region: every demotion whose pages nobody takes is deferred and read in place
    c = ctx(L=L, hbm_pages=160, zero_copy=True)
    c.plan_load(list(range(B)), n, ones)
    c.plan_load(list(range(B)), n, x)
    assert c.get_plan_info()["deferred_to_host_blocks"] == 36 and c.get_plan_info()["in_place_blocks"] == 40
    assert c.get_pages(2, 1)["tier"] == 2
    c.decode_attention(1, None, None)                          # no copies in flight in a host-only context: handed over
    assert c.get_pages(2, 1)["tier"] == 0
    # a promotion in the same switch takes pages that were free before it; the pages this switch's own demotions
    # vacate are handed out only when nothing else is left, so those blocks may all wait
    y = x.copy()
    y[:, 1] = 1
    y[:, 2] = 0                                                # layer 1 back in, layer 2 out
    c.plan_load(list(range(B)), n, y)
    info = c.get_plan_info()
    assert info["moved_to_host_blocks"] == 40 and info["moved_to_hbm_blocks"] == 40
    assert info["deferred_to_host_blocks"] == 36 and info["in_place_blocks"] == 40
    # ... and when nothing else is left: a new resident request (30 blocks) arrives while layer 2 comes back (it
    # is still read in place: it takes its 40 pages back, nothing is copied) and layer 3 leaves; the new request can
    # only get pages that layer 3 vacates
    z = y.copy()
    z[:, 2] = 1
    z[:, 3] = 0
    c2 = ctx(L=L, hbm_pages=160, zero_copy=True, max_req=8)
    c2.plan_load(list(range(B)), n, ones)
    c2.plan_load(list(range(B)), n, x)
    c2.plan_load(list(range(B)), n, y)
    c2.plan_load(list(range(B)) + [9], n + [160], np.vstack([z, np.array([[1, 1, 1, 0]], dtype=np.uint8)]))
    info = c2.get_plan_info()
    assert info["moved_to_host_blocks"] == 40 and info["moved_to_hbm_blocks"] == 0 and info["reclaimed_blocks"] == 40
    assert info["deferred_to_host_blocks"] == 9 and info["in_place_blocks"] == 10   # three of the four vacated blocks were taken at once


def test_demoted_blocks_are_read_in_place_until_their_copies_have_landed():
    """Host-only contexts have no copies in flight: the hand-over to the staging schedule happens at the layer's
    first prefetch.  Until then the page list attention reads is the one the block had in HBM."""
    L, B = 3, 3
    n = [160, 100, 47]
    ones = np.ones((B, L), dtype=np.uint8)
    c = ctx(L=L, hbm_pages=2000, window=40)
    ids = [5, 6, 7]
    c.plan_load(ids, n, ones)
    before = {(r, l): [int(p) for p in c.get_pages(r, l)["pages"]] for r in ids for l in range(L)}
    x = ones.copy()
    x[0, 1] = x[2, 1] = x[1, 2] = 0
    c.plan_load(ids, n, x)
    info = _layout_invariants(c, ids, L)
    assert info["in_place_blocks"] == 10 + 3 + 7 and info["deferred_to_host_blocks"] == 9 + 2 + 6
    for r, l in ((5, 1), (7, 1), (6, 2)):
        p = c.get_pages(r, l)
        assert p["tier"] == 2 and [int(v) for v in p["pages"]] == before[(r, l)]   # used and reserved pages alike
    assert c.get_pages(6, 1)["tier"] == 1
    # the copy schedule still has their staging ranges; the first prefetch of a layer switches its blocks over
    c.kv_prefetch(1)
    for r in (5, 7):
        p = c.get_pages(r, 1)
        assert p["tier"] == 0 and int(p["pages"][0]) >= info["staging_first_page"]
    assert c.get_pages(6, 2)["tier"] == 2
    c.decode_attention(1, None, None)
    # a plan load that leaves the block offloaded and its old pages alone leaves it where it is read
    c.plan_load(ids, n, x)
    info = c.get_plan_info()
    p = c.get_pages(6, 2)
    assert p["tier"] == 2 and [int(v) for v in p["pages"]] == before[(6, 2)]
    assert info["in_place_blocks"] == 0 and info["still_in_place_blocks"] == 7 and info["waited_for_deferred"] == 0
    _layout_invariants(c, ids, L)
    # ... one that needs the pages does not: two newcomers that fill the arena up to the staging region
    free_pages = info["staging_first_page"] - info["resident_blocks"]
    rest = (free_pages - 512 * L) // L                   # blocks per layer left beside a request of 512 blocks
    c.plan_load(ids + [8, 9], n + [8192 - 40, 16 * rest - 40], np.vstack([x, np.ones((2, L), dtype=np.uint8)]))
    info = c.get_plan_info()
    assert c.get_pages(6, 2)["tier"] == 0 and info["still_in_place_blocks"] == 0 and info["waited_for_deferred"] == 1
    _layout_invariants(c, ids + [8, 9], L)


def test_a_block_still_read_in_place_takes_its_pages_back():
    """Demote, then promote again before the copies have landed: the block never left its pages, so the second
    switch copies nothing and the page lists are the original ones (grown by the new reservation)."""
    L, B = 3, 3
    n = [160, 100, 47]
    ones = np.ones((B, L), dtype=np.uint8)
    c = ctx(L=L, hbm_pages=2000, window=40)
    ids = [5, 6, 7]
    c.plan_load(ids, n, ones)
    before = {(r, l): [int(p) for p in c.get_pages(r, l)["pages"]] for r in ids for l in range(L)}
    x = ones.copy()
    x[0, 1] = x[2, 1] = x[1, 2] = 0
    c.plan_load(ids, n, x)
    y = ones.copy()
    y[2, 1] = 0                                          # (7, 1) stays out; (5, 1) and (6, 2) come back
    c.plan_load(ids, n, y)
    info = _layout_invariants(c, ids, L)
    assert info["reclaimed_blocks"] == 10 + 7 and info["moved_to_hbm_blocks"] == 0 and info["moved_to_host_blocks"] == 0
    for r, l in ((5, 1), (6, 2)):
        p = c.get_pages(r, l)
        assert p["tier"] == 1 and [int(v) for v in p["pages"]] == before[(r, l)]
    assert c.get_pages(7, 1)["tier"] == 2                # what stays offloaded goes on being read in place
    assert info["still_in_place_blocks"] == 3
    # once a layer has been handed over (in a host-only context: at its first prefetch), coming back is a real copy
    c.plan_load(ids, n, x)
    c.kv_prefetch(1)
    c.decode_attention(1, None, None)
    c.plan_load(ids, n, ones)
    info = c.get_plan_info()
    assert info["reclaimed_blocks"] == 7 and info["moved_to_hbm_blocks"] == 10 + 3


def test_a_single_block_demotion_is_not_read_in_place():
    L = 2
    c = ctx(L=L, hbm_pages=500)
    c.plan_load([1], [9], np.ones((1, L), dtype=np.uint8))
    c.plan_load([1], [9], np.array([[1, 0]], dtype=np.uint8))
    info = c.get_plan_info()
    assert info["moved_to_host_blocks"] == 1 and info["deferred_to_host_blocks"] == 0 and info["in_place_blocks"] == 0
    assert c.get_pages(1, 1)["tier"] == 0


def test_a_plan_load_waits_for_earlier_deferred_copies_only_when_it_touches_their_pages():
    """Blocks of 10 pages are demoted with deferred copies; the next plan loads are judged one by one: whether they
    must wait for those copies follows from the pages they hand out and the blocks they move."""
    L, B = 4, 2
    n = [160, 160]
    ids = [1, 2]
    ones = np.ones((B, L), dtype=np.uint8)

    def fresh(hbm_pages):
        c = ctx(L=L, hbm_pages=hbm_pages, host_pages=4000, window=0, slots=1)
        c.plan_load(ids, n, ones)
        x = ones.copy()
        x[:, 1] = 0                                          # layer 1 leaves: 2 x 9 deferred pages, 2 at once
        c.plan_load(ids, n, x)
        info = c.get_plan_info()
        assert info["deferred_to_host_blocks"] == 18 and info["waited_for_deferred"] == 0
        return c, x

    # the blocks come back while their copies travel: they keep their pages, nobody else's page is touched
    c, x = fresh(2000)
    c.plan_load(ids, n, ones)
    assert c.get_plan_info()["reclaimed_blocks"] == 20 and c.get_plan_info()["waited_for_deferred"] == 0

    # another layer leaves as well, into host pages nobody has used: beside the first copies
    c, x = fresh(2000)
    x2 = x.copy()
    x2[:, 2] = 0
    c.plan_load(ids, n, x2)
    info = c.get_plan_info()
    assert info["deferred_to_host_blocks"] == 18 and info["waited_for_deferred"] == 0
    assert info["still_in_place_blocks"] == 20           # layer 1 goes on being read in place
    # ... and, once layer 1 has been handed over to its host runs (in a host-only context: at its first prefetch),
    # a third plan load that brings it back reads host pages the first copies write
    c.kv_prefetch(1)
    c.decode_attention(1, None, None)
    x3 = x2.copy()
    x3[:, 1] = 1
    c.plan_load(ids, n, x3)
    info = c.get_plan_info()
    assert info["moved_to_hbm_blocks"] == 20 and info["waited_for_deferred"] == 1
    # after that wait nothing is outstanding but the copies of layer 2, which this one leaves alone
    x4 = x3.copy()
    x4[:, 3] = 0
    c.plan_load(ids, n, x4)
    assert c.get_plan_info()["waited_for_deferred"] == 0

    # a new request that needs the vacated HBM pages: the arena has no other page left
    c, x = fresh(hbm_pages=4 * 20 + 20)                      # 80 resident + 20 staging at the start
    c.plan_load(ids + [3], n + [16], np.array([[1, 0, 1, 1], [1, 0, 1, 1], [1, 1, 1, 1]], dtype=np.uint8))
    assert c.get_plan_info()["waited_for_deferred"] == 1

    # the staging region grows down over the vacated pages
    c, x = fresh(2000)
    x5 = np.zeros((B, L), dtype=np.uint8)
    c.plan_load(ids, n, x5, hbm_budget_bytes=60 * PAGE)
    assert c.get_plan_info()["waited_for_deferred"] == 1

    # the request leaves and a newcomer gets its host pages
    c, x = fresh(2000)
    c.plan_load([2], [160], x[1:])
    assert c.get_plan_info()["waited_for_deferred"] == 0    # dropping alone touches nothing
    c.plan_load([2, 9], [160, 100], np.array([[1, 0, 1, 1], [0, 0, 0, 0]], dtype=np.uint8))
    assert c.get_plan_info()["waited_for_deferred"] == 1


def test_decode_layer_moves_one_layers_lengths_and_respects_the_window():
    L = 3
    c = ctx(L=L, hbm_pages=500, window=2)
    ids = [4, 5]
    c.plan_load(ids, [30, 40], np.array([[1, 0, 1], [0, 1, 1]], dtype=np.uint8))
    c.decode_layer(1, None, None, None, None)
    assert [c.get_pages(4, l)["length"] for l in range(L)] == [30, 31, 30]
    assert [c.get_pages(5, l)["length"] for l in range(L)] == [40, 41, 40]
    c.decode_layer(1, None, None, None, None)              # 32 tokens fill the two blocks request 4 has reserved
    with pytest.raises(OrbitError) as e:
        c.decode_layer(1, None, None, None, None)
    assert e.value.code == orbit.ORBIT_E_STATE
    assert c.get_pages(4, 1)["length"] == 32 and c.get_pages(5, 1)["length"] == 42      # nothing moved
    with pytest.raises(OrbitError):
        c.decode_layer(7, None, None, None, None)          # no such layer
