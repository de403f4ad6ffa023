"""GPU parity at the full lengths of the larger benchmark workloads, on two-layer slices (one
launch per layer has the real shape: all requests at their real context lengths), checked on
sampled (request, kv head) groups that the oracle computes one by one."""
import dataclasses

import numpy as np
import pytest
import torch

from workloads import make_workload

pytestmark = pytest.mark.gpu

MAX_ABS, REL_L2, REL_L2_F32 = 1e-2, 5e-3, 3e-3


def _two_layer_slice(name, seed=0, n_req=None, steps=0):
    w = make_workload(name, seed, n_req=n_req)
    pl = np.zeros((w.n_req, 2), dtype=np.uint8)
    pl[0::2] = [1, 0]                      # even requests: layer 0 resident, layer 1 streamed
    pl[1::2] = [0, 1]
    return dataclasses.replace(w, n_layers=2, placement=pl, steps=steps)


def _check_groups(h, w, out, out32, lens, samples, step=0):
    G = w.n_q_heads // w.n_kv_heads
    for layer, r, g in samples:
        want = h.oracle_one_group(w, r, layer, g, int(lens[r]), step)
        got = out[layer][r, g * G:(g + 1) * G]
        ma, rl = h.errors(got, want)
        assert ma <= MAX_ABS and rl <= REL_L2, (layer, r, g, ma, rl)
        if out32 is not None:
            _, rl32 = h.errors(out32[layer][r, g * G:(g + 1) * G], want)
            assert rl32 <= REL_L2_F32, (layer, r, g, rl32)


def test_long_ctx_32_appended_steps():
    """Batch 4, contexts in [64K, 128K], one token appended per step for 32 steps."""
    import harness as h
    w = _two_layer_slice("long_ctx", steps=32)
    g = h.GpuRun(w, prefetch_slots=2)
    out = None
    for s in range(32):
        out, _ = g.step(s)
    assert torch.isfinite(out.float()).all()
    lens = w.ctx_len.astype(np.int64) + 32
    _check_groups(h, w, out, None, lens, [(0, 0, 3), (1, 0, 5), (0, 3, 0), (1, 2, 7)], step=31)
    g.close()


def test_llama70b_shape_group_of_eight():
    """64 query heads over 8 KV heads at the workload's full batch of 32 with contexts in [16K, 128K]: each of the
    two launches reads 9.7 GB of KV (half of the requests resident, half streamed).  Attention over the stored
    cache, then one orbit_step (the append folded into the launch) at the same size."""
    import harness as h
    w = _two_layer_slice("llama70b", steps=1)
    assert w.n_req == 32 and w.n_q_heads // w.n_kv_heads == 8
    host_blocks = int(((1 - w.placement.astype(np.int64)) * w.blocks(1)[:, None]).sum())
    g = h.GpuRun(w, prefetch_slots=1, host_pages=host_blocks + 8)      # pin only what this placement streams
    outs, outs32 = [], []
    for layer in range(2):
        o, o32 = g.attention(layer)
        outs.append(o)
        outs32.append(o32)
    order = np.argsort(w.ctx_len)
    picks = [int(order[0]), int(order[15]), int(order[-1])]
    _check_groups(h, w, outs, outs32, w.ctx_len, [(0, picks[0], 0), (1, picks[0], 6), (0, picks[1], 2), (1, picks[2], 4)])
    out, _ = g.step(0)
    assert torch.isfinite(out.float()).all()
    _check_groups(h, w, out, None, w.ctx_len.astype(np.int64) + 1, [(0, picks[2], 7), (1, picks[1], 3), (1, 31, 5)], step=0)
    g.close()


def test_heavy_mixed_lengths():
    """Batch 64, log-uniform contexts in [1K, 64K]: short and long requests in one launch."""
    import harness as h
    w = _two_layer_slice("heavy_mixed")
    g = h.GpuRun(w, prefetch_slots=1)
    outs, outs32 = [], []
    for layer in range(2):
        o, o32 = g.attention(layer)
        outs.append(o)
        outs32.append(o32)
    order = np.argsort(w.ctx_len)
    picks = [int(order[0]), int(order[len(order) // 2]), int(order[-1])]
    _check_groups(h, w, outs, outs32, w.ctx_len, [(0, picks[0], 1), (1, picks[0], 6), (0, picks[1], 2),
                                                  (1, picks[2], 4), (0, picks[2], 7)])
    g.close()


def test_heavy_mixed_under_its_byte_budget():
    """Batch 64 with the workload's own per-request placement and byte budget (an eight-layer slice: 8/32 of the
    40 GB; the prefetch buffer of Eq. (1) is one layer's worth whatever the number of layers, so a thinner slice
    has no feasible plan), one staging buffer."""
    import harness as h
    w = make_workload("heavy_mixed", 0, n_layers=8, steps=1)
    assert w.n_req == 64 and w.hbm_budget_bytes == 40 * 10**9 * 8 // 32
    host_blocks = int(((1 - w.placement.astype(np.int64)) * w.blocks(1)[:, None]).sum())
    g = h.GpuRun(w, prefetch_slots=1, budget_pages=w.hbm_budget_bytes // w.page_bytes, host_pages=host_blocks + 8)
    info = g.ctx.get_plan_info()
    assert info["resident_blocks"] + info["staging_blocks"] <= info["budget_blocks"] and info["host_blocks"] > 0
    out, stats = g.step(0, want_stats=True)
    assert torch.isfinite(out.float()).all() and stats.link_kv_bytes > 0
    order = np.argsort(w.ctx_len)
    lens = w.ctx_len.astype(np.int64) + 1
    samples = [(l, int(r), int(k)) for l, r, k in ((0, order[0], 1), (7, order[0], 6), (3, order[32], 2), (5, order[-1], 4), (0, order[-1], 7))]
    _check_groups(h, w, out, None, lens, samples, step=0)
    g.close()


def test_bench_configuration_full_step_sampled():
    """The exact configuration bench.py times: all 32 layers of the 8B-shaped batch-16 workload
    with its 75 %-resident placement and two staging ranges; one full orbit_step, then sampled
    (layer, request, kv head) groups of resident and streamed layers against the oracle."""
    import harness as h
    from paper_2601_10729_amd import orbit_plan_check
    w = dataclasses.replace(make_workload("llama8b_b16", 0), steps=1)
    _, _, need, host_blocks = orbit_plan_check(w.ctx_len, w.placement, w.page_tokens, 2, 1)
    g = h.GpuRun(w, prefetch_slots=2, budget_pages=need + 8, host_pages=host_blocks + 8)
    out, stats = g.step(0, want_stats=True)
    assert torch.isfinite(out.float()).all()
    assert stats.link_kv_bytes == int(((1 - w.placement.astype(np.int64)) * w.blocks()[:, None]).sum()) * w.page_bytes
    rng = np.random.default_rng(3)
    lens = w.ctx_len.astype(np.int64) + 1
    samples = []
    for want_tier in (0, 1, 0, 1):
        while True:
            layer, r = int(rng.integers(w.n_layers)), int(rng.integers(w.n_req))
            if w.placement[r, layer] == want_tier:
                samples.append((layer, r, int(rng.integers(w.n_kv_heads))))
                break
    _check_groups(h, w, out, None, lens, samples, step=0)
    g.close()


def test_bench_configuration_every_output_is_placement_invariant():
    """A property checked on EVERY output element at full size: the 8B-shaped batch-16 workload
    attended under its 75 %-resident placement (streamed layers through the staging ranges) and
    again after a plan switch to all-resident gives bit-identical outputs for all 32 layers."""
    import harness as h
    w = make_workload("llama8b_b16", 0)
    all_res = int(w.blocks().sum()) * w.n_layers
    host_blocks = int(((1 - w.placement.astype(np.int64)) * w.blocks()[:, None]).sum())
    g = h.GpuRun(w, prefetch_slots=2, budget_pages=all_res + 8, host_pages=host_blocks + 8)
    qs = [g.q_layer(l) for l in range(w.n_layers)]
    outs = []
    for pl in (None, np.ones_like(w.placement)):
        if pl is not None:
            g.ctx.plan_load(w.req_ids, w.ctx_len, pl)
            info = g.ctx.get_plan_info()
            assert info["moved_to_hbm_blocks"] == host_blocks and info["moved_to_host_blocks"] == 0
        o = torch.empty((w.n_layers, w.n_req, w.n_q_heads, w.head_dim), dtype=torch.bfloat16, device=g.dev)
        torch.cuda.synchronize()
        for l in range(w.n_layers):
            g.ctx.decode_attention(l, qs[l], o[l], None)
        g.cs.synchronize()
        g.xs.synchronize()
        assert torch.isfinite(o.float()).all()
        outs.append(o)
    assert torch.equal(outs[0].view(torch.int16), outs[1].view(torch.int16))
    g.close()


def test_full_size_layer_every_element_against_oracle():
    """One whole launch at the bench workload's real shape (16 requests, 8K-32K tokens each, a mix of
    resident and streamed requests) compared with the oracle on EVERY output element."""
    import harness as h
    w = make_workload("llama8b_b16", 0)
    col = int(np.argmax((w.placement == 0).sum(axis=0)))          # the layer with most streamed requests
    w1 = dataclasses.replace(w, n_layers=1, placement=w.placement[:, col:col + 1].copy())
    assert 0 < int(w1.placement.sum()) < w1.n_req
    g = h.GpuRun(w1, prefetch_slots=2)
    out, out32 = g.attention(0)
    want = h.OracleRun(w1).attention(0)
    ma, rl = h.errors(out, want)
    assert ma <= MAX_ABS and rl <= REL_L2, (ma, rl)
    _, rl32 = h.errors(out32, want)
    assert rl32 <= REL_L2_F32, rl32
    # per (request, head) rows as well: no single short row hides inside the global norm
    d = out.to(torch.float64).cpu().numpy() - want
    row = np.sqrt((d * d).sum(-1) / (want * want).sum(-1))
    assert row.max() <= 2 * REL_L2, float(row.max())
    g.close()


@pytest.mark.parametrize("zero_copy", [False, True])
def test_steps_run_in_place_while_a_large_demotion_is_in_flight(zero_copy):
    """A switch that sends 1 GB of KV to the host, with steps enqueued right behind it and no host-side wait: the
    copies take tens of milliseconds, the steps a fraction of one, so several steps read the demoted blocks where
    they were, append into them and into the host runs, and later steps take the blocks over layer by layer.  Every
    step equals, bit for bit, a run that had the placement from the start; sampled groups are checked against the
    oracle at the end."""
    import time
    import harness as h
    from workloads import gen_q_steps, gen_kv
    L, S = 4, 10
    base = make_workload("llama8b_b16", 0, n_req=4)
    lens = np.array([20000, 17001, 23000, 9000], dtype=base.ctx_len.dtype)
    ones = np.ones((4, L), dtype=np.uint8)
    x = ones.copy()
    x[:, 1:] = 0                                           # three of four layers leave HBM: 0.85 GB
    w = dataclasses.replace(base, n_layers=L, ctx_len=lens, placement=x, steps=S)
    blocks = int(w.blocks(S).sum())
    kw = dict(prefetch_slots=2, budget_pages=blocks * L + 2 * blocks + 64, host_pages=blocks * L + 64, decode_window=S,
              max_tokens=int(lens.max()) + S + 16, zero_copy=zero_copy)

    def inputs(dev):
        B = w.n_req
        q = torch.stack([torch.stack([gen_q_steps(w.seed, l, int(rid), 0, S, w.n_q_heads, w.head_dim, dev)
                                      for rid in w.req_ids], dim=1) for l in range(L)], dim=1).contiguous()
        kv = [[gen_kv(w.seed, l, int(rid), int(lens[r]), S, w.n_kv_heads, w.head_dim, dev)
               for r, rid in enumerate(w.req_ids)] for l in range(L)]
        k_new = torch.stack([torch.stack([kv[l][r][0] for r in range(B)], dim=1) for l in range(L)], dim=1).contiguous()
        v_new = torch.stack([torch.stack([kv[l][r][1] for r in range(B)], dim=1) for l in range(L)], dim=1).contiguous()
        return q, k_new, v_new

    def run(switching: bool):
        g = h.GpuRun(w, placement=ones if switching else x, **kw)
        q, k_new, v_new = inputs(g.dev)
        outs = torch.zeros((S, L, w.n_req, w.n_q_heads, w.head_dim), dtype=torch.bfloat16, device=g.dev)
        torch.cuda.synchronize()
        in_place = []
        for s in range(S):
            if switching and s == 2:
                g.ctx.plan_load(w.req_ids, lens + s, x)
                info = g.ctx.get_plan_info()
                assert info["in_place_blocks"] == info["moved_to_host_blocks"] == 3 * int(np.ceil((lens + s) / 16).sum())
                assert info["deferred_to_host_blocks"] == info["in_place_blocks"] - 12      # one page per block went at once
            if switching and s == 3:                         # the same plan again, one token on: nothing moves, nothing waits
                g.ctx.plan_load(w.req_ids, lens + s, x)
                info = g.ctx.get_plan_info()
                assert info["moved_to_host_blocks"] == info["moved_to_hbm_blocks"] == 0 and info["waited_for_deferred"] == 0
                assert info["still_in_place_blocks"] == sum(
                    int(np.ceil((lens[r] + s) / 16)) for r, rid in enumerate(w.req_ids) for l in range(L)
                    if g.ctx.get_pages(int(rid), l)["tier"] == 2)
            g.ctx.step(q[s], k_new[s], v_new[s], outs[s])
            if switching and s >= 2:
                in_place.append(sum(g.ctx.get_pages(int(rid), l)["tier"] == 2 for rid in w.req_ids for l in range(L)))
            if switching and s == 6:
                time.sleep(0.2)                              # the copies (about 20 ms) have landed by now
        g.cs.synchronize()
        g.xs.synchronize()
        res = outs.cpu()
        lens_end = lens.astype(np.int64) + S
        if switching:
            assert in_place[0] == 12                         # the step right behind the switch read everything in place
            assert in_place[-1] == 0                         # ... and by the end every block has been taken over
            _check_groups(h, w, [outs[S - 1][l] for l in range(L)], None, lens_end, [(1, 0, 3), (2, 2, 7), (3, 3, 0), (0, 1, 5)], step=S - 1)
        g.close()
        return res, in_place

    (a, in_place), (b, _) = run(True), run(False)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16)), in_place


@pytest.mark.parametrize("zero_copy", [False, True])
def test_blocks_demoted_and_wanted_back_at_once_never_move(zero_copy):
    """A plan sends 0.85 GB to the host, one step runs (reading and appending in place), and the next plan wants
    everything resident again while the copies are still travelling: the blocks take their pages back, nothing is
    copied to HBM, and every step equals a run that never switched, bit for bit."""
    import harness as h
    from workloads import gen_q_steps, gen_kv
    L, S = 4, 5
    base = make_workload("llama8b_b16", 0, n_req=4)
    lens = np.array([20000, 17001, 23000, 9000], dtype=base.ctx_len.dtype)
    ones = np.ones((4, L), dtype=np.uint8)
    x = ones.copy()
    x[:, 1:] = 0
    w = dataclasses.replace(base, n_layers=L, ctx_len=lens, placement=ones, steps=S)
    blocks = int(w.blocks(S).sum())
    kw = dict(prefetch_slots=2, budget_pages=blocks * L + 2 * blocks + 64, host_pages=blocks * L + 64, decode_window=S,
              max_tokens=int(lens.max()) + S + 16, zero_copy=zero_copy)

    def run(switching: bool):
        g = h.GpuRun(w, placement=ones, **kw)
        B = w.n_req
        q = torch.stack([torch.stack([gen_q_steps(w.seed, l, int(rid), 0, S, w.n_q_heads, w.head_dim, g.dev)
                                      for rid in w.req_ids], dim=1) for l in range(L)], dim=1).contiguous()
        kv = [[gen_kv(w.seed, l, int(rid), int(lens[r]), S, w.n_kv_heads, w.head_dim, g.dev)
               for r, rid in enumerate(w.req_ids)] for l in range(L)]
        k_new = torch.stack([torch.stack([kv[l][r][0] for r in range(B)], dim=1) for l in range(L)], dim=1).contiguous()
        v_new = torch.stack([torch.stack([kv[l][r][1] for r in range(B)], dim=1) for l in range(L)], dim=1).contiguous()
        outs = torch.zeros((S, L, B, w.n_q_heads, w.head_dim), dtype=torch.bfloat16, device=g.dev)
        torch.cuda.synchronize()
        for s in range(S):
            if switching and s == 1:
                g.ctx.plan_load(w.req_ids, lens + s, x)
                assert g.ctx.get_plan_info()["in_place_blocks"] > 0
            if switching and s == 2:
                g.ctx.plan_load(w.req_ids, lens + s, ones)
                info = g.ctx.get_plan_info()
                assert info["reclaimed_blocks"] == 3 * int(np.ceil((lens + s) / 16).sum()) and info["moved_to_hbm_blocks"] == 0
            g.ctx.step(q[s], k_new[s], v_new[s], outs[s])
        g.cs.synchronize()
        g.xs.synchronize()
        res = outs.cpu()
        if switching:                                       # the KV reads back complete, appended tokens included
            for r, l in ((0, 1), (3, 3)):
                n = int(lens[r]) + S
                k, v = g.read_kv(r, l, n - 40, 40)
                kw_, vw_ = gen_kv(w.seed, l, int(w.req_ids[r]), n - 40, 40, w.n_kv_heads, w.head_dim, g.dev)
                assert torch.equal(k.view(torch.int16), kw_.view(torch.int16))
                assert torch.equal(v.view(torch.int16), vw_.view(torch.int16))
            _check_groups(h, w, [outs[S - 1][l] for l in range(L)], None, lens.astype(np.int64) + S,
                          [(1, 0, 3), (2, 2, 7), (3, 3, 0)], step=S - 1)
        g.close()
        return res

    a, b = run(True), run(False)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


@pytest.mark.parametrize("zero_copy", [False, True])
def test_plan_loads_that_run_beside_the_copies_of_earlier_ones(zero_copy):
    """Four plan loads in five steps, with no host-side wait anywhere: layer 1 leaves HBM (0.28 GB of deferred
    copies), then layer 2 as well, beside the first copies and from a second op list, then layer 3, then layer 1
    is wanted back (a real copy that waits for the first copies, or none at all if the layer is still read in
    place, as earlier plan loads leave it when they do not need its pages).  Every step equals, bit for
    bit, a run that never switched; the KV of a block that went out and came back reads back complete."""
    import harness as h
    from workloads import gen_q_steps, gen_kv
    L, S = 4, 8
    base = make_workload("llama8b_b16", 0, n_req=4)
    lens = np.array([20000, 17001, 23000, 9000], dtype=base.ctx_len.dtype)
    ones = np.ones((4, L), dtype=np.uint8)
    plans = {}
    x = ones.copy()
    for s, (layer, v) in {1: (1, 0), 2: (2, 0), 3: (3, 0), 5: (1, 1)}.items():
        x = x.copy()
        x[:, layer] = v
        plans[s] = x
    w = dataclasses.replace(base, n_layers=L, ctx_len=lens, placement=ones, steps=S)
    blocks = int(w.blocks(S).sum())
    kw = dict(prefetch_slots=2, budget_pages=blocks * L + 2 * blocks + 64, host_pages=blocks * L + 64, decode_window=S,
              max_tokens=int(lens.max()) + S + 16, zero_copy=zero_copy)

    def run(switching: bool):
        g = h.GpuRun(w, placement=ones, **kw)
        B = w.n_req
        q = torch.stack([torch.stack([gen_q_steps(w.seed, l, int(rid), 0, S, w.n_q_heads, w.head_dim, g.dev)
                                      for rid in w.req_ids], dim=1) for l in range(L)], dim=1).contiguous()
        kv = [[gen_kv(w.seed, l, int(rid), int(lens[r]), S, w.n_kv_heads, w.head_dim, g.dev)
               for r, rid in enumerate(w.req_ids)] for l in range(L)]
        k_new = torch.stack([torch.stack([kv[l][r][0] for r in range(B)], dim=1) for l in range(L)], dim=1).contiguous()
        v_new = torch.stack([torch.stack([kv[l][r][1] for r in range(B)], dim=1) for l in range(L)], dim=1).contiguous()
        outs = torch.zeros((S, L, B, w.n_q_heads, w.head_dim), dtype=torch.bfloat16, device=g.dev)
        torch.cuda.synchronize()
        waited = []
        for s in range(S):
            if switching and s in plans:
                g.ctx.plan_load(w.req_ids, lens + s, plans[s])
                info = g.ctx.get_plan_info()
                waited.append(info["waited_for_deferred"])
                if s < 5:
                    assert info["deferred_to_host_blocks"] > 0 and info["moved_to_hbm_blocks"] == 0
                else:                                       # copied back, or never left (if still read in place)
                    assert info["moved_to_hbm_blocks"] + info["reclaimed_blocks"] == int(np.ceil((lens + s) / 16).sum())
            g.ctx.step(q[s], k_new[s], v_new[s], outs[s])
        g.cs.synchronize()
        g.xs.synchronize()
        res = outs.cpu()
        if switching:
            assert waited[0] == 0 and waited[1] == 0, waited   # (the later ones depend on how far the copies have come)
            for r, l in ((0, 1), (2, 3), (1, 2)):
                n = int(lens[r]) + S
                k, v = g.read_kv(r, l, n - 40, 40)
                kw_, vw_ = gen_kv(w.seed, l, int(w.req_ids[r]), n - 40, 40, w.n_kv_heads, w.head_dim, g.dev)
                assert torch.equal(k.view(torch.int16), kw_.view(torch.int16))
                assert torch.equal(v.view(torch.int16), vw_.view(torch.int16))
            _check_groups(h, w, [outs[S - 1][l] for l in range(L)], None, lens.astype(np.int64) + S,
                          [(1, 0, 3), (2, 2, 7), (3, 3, 0), (0, 1, 2)], step=S - 1)
        g.close()
        return res

    a, b = run(True), run(False)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
