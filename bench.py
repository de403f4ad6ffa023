#!/usr/bin/env python3
"""Decode-step benchmark of liborbit on one MI355X.

A "step" is one pass of the whole hot path over the batch: for every layer, append the new
token's K/V, stream that layer's offloaded KV from pinned host memory into the staging region
(copy stream, running ahead), split-K attention over the grown cache, combine.  KV, Q and the
new K/V rows are resident (HBM, or pinned host for offloaded layers) before the clock starts.

Prints ONE JSON line: the whole-step effective KV rate (HBM-resident + host-streamed KV bytes
attended per second), the HBM roofline of the split-K attention kernel measured with HIP events
on the compute stream, the host-link figures, and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth

WORKLOAD_TEXT = {
    "tiny": "Tiny decode step: 2 layers, 4 requests {17,256,1000,2048}, Hq8/Hkv2, layer 0 HBM, layer 1 host",
    "llama8b_b16": "Llama-3-8B-shaped decode: 32 layers, Hq32/Hkv8, D128, bf16, batch 16, ctx U[8K,32K], page 16, "
                   "75% of each request's layers in HBM, 25% streamed from pinned host",
    "long_ctx": "Long-context decode: 8B shape, batch 4, ctx U[64K,128K], 50% of layers offloaded",
    "heavy_mixed": "Heavy mixed load: 8B shape, batch 64, ctx log-uniform [1K,64K], 40 GB budget",
    "llama70b": "70B-shaped attention: 80 layers, Hq64/Hkv8, batch 32, ctx U[16K,128K], 25% resident",
}


def measure_link_peak(torch, sizes=(1 << 20, 16 << 20, 256 << 20, 1 << 30), reps=4):
    """Pinned host -> device copy rate (GB/s) of single transfers of 1 MiB .. 1 GiB: the best one is
    the link roofline.  Returns (peak, {size in MiB: GB/s})."""
    src = torch.empty(max(sizes), dtype=torch.uint8, pin_memory=True)
    src.fill_(1)
    dst = torch.empty(max(sizes), dtype=torch.uint8, device="cuda:0")
    dst.copy_(src, non_blocking=True)
    torch.cuda.synchronize()
    sweep = {}
    for n in sizes:
        best = 0.0
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            dst[:n].copy_(src[:n], non_blocking=True)
            e1.record()
            torch.cuda.synchronize()
            best = max(best, n / (e0.elapsed_time(e1) * 1e-3) / 1e9)
        sweep[str(n >> 20)] = best
    del src, dst
    return max(sweep.values()), sweep


def cpu_baseline(w, n_req_sample=16, n_layers_sample=3):
    """The oracle as it stands, timed on a bounded sample: `n_req_sample` requests x
    `n_layers_sample` layers x all query heads, through its own paged store.  Returns GB/s of KV
    consumed (threads x seconds is about 10-20 core-seconds on the GPU machine's host)."""
    import dataclasses
    import harness
    from oracle import reference as ref
    n_req_sample = min(n_req_sample, w.n_req)
    nl = min(n_layers_sample, w.n_layers)
    ws = dataclasses.replace(w, n_layers=nl, req_ids=w.req_ids[:n_req_sample], ctx_len=w.ctx_len[:n_req_sample],
                             placement=w.placement[:n_req_sample, :nl])
    o = harness.OracleRun(ws)
    t0 = time.perf_counter()
    for layer in range(nl):
        o.attention(layer, 0)
    dt = time.perf_counter() - t0
    nbytes = int(ws.ctx_len.astype("int64").sum()) * ws.kv_bytes_per_token_layer * nl
    cores = ref.num_threads()
    ref.set_threads(1)                      # the same oracle on one core, one layer of the sample
    t1 = time.perf_counter()
    o.attention(0, 0)
    dt1 = time.perf_counter() - t1
    ref.set_threads(cores)
    return {"value": nbytes / dt / 1e9, "unit": "GB/s", "cores": cores, "kind": "oracle",
            "one_core_value": nbytes / nl / dt1 / 1e9,
            "sample": f"{n_req_sample} requests x {nl} layers x {w.n_q_heads} query heads of the same workload "
                      f"({nbytes / 1e6:.0f} MB of KV, {dt:.2f} s)", "seconds": dt}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama8b_b16", choices=sorted(WORKLOAD_TEXT))
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--prefetch-slots", type=int, default=2)
    ap.add_argument("--chunk-tokens", type=int, default=0)
    ap.add_argument("--placement", default="workload", choices=["workload", "resident", "host"])
    ap.add_argument("--n-req", type=int, default=None, help="truncate the batch")
    ap.add_argument("--max-host-gib", type=float, default=60.0,
                    help="largest pinned host arena to ask for; the batch is truncated to fit")
    ap.add_argument("--zero-copy", action="store_true",
                    help="ORBIT_FLAG_ZERO_COPY: the attention kernel reads offloaded blocks in place over the link "
                         "(no staging region, no host->staging copies); a measured alternative, not the default")
    ap.add_argument("--run-ahead", type=int, default=2,
                    help="steps the host may be ahead of the GPU in the timed loop (0 = no bound)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-resident-variant", action="store_true")
    ap.add_argument("--no-searched-variant", action="store_true",
                    help="do not install and time the plan found by the pruned search")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three plain 1 GiB device-to-device copies (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build drives exactly one GPU (no sharding, no collectives); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import dataclasses
    import numpy as np
    import torch
    import harness
    from workloads import make_workload, gen_kv, gen_q_steps

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    K, W = args.steps, args.warmup
    total_steps = W + 2 * K + 8          # warm-up, timed, timed-with-events, searched-plan and all-resident variants
    from paper_2601_10729_amd import orbit_plan_check
    n_req = args.n_req
    while True:
        w = make_workload(args.workload, args.seed, n_req=n_req, steps=total_steps)
        if args.placement == "resident":
            w = w.all_resident()
        elif args.placement == "host":
            w = w.all_host()
        slots = args.prefetch_slots if w.hbm_budget_bytes is None else 1   # the byte budget was clipped for one buffer
        _, _, need, host_blocks = orbit_plan_check(w.ctx_len, w.placement, w.page_tokens,
                                                   0 if args.zero_copy else slots, total_steps)
        if (host_blocks + 8) * w.page_bytes <= args.max_host_gib * (1 << 30) or w.n_req == 1:
            break
        n_req = w.n_req - 1            # this host cannot pin that much: drop the last request and say so

    link_peak, link_sweep = measure_link_peak(torch)
    t_setup = time.perf_counter()
    # the arena is sized so that the all-resident variant of the same workload also fits
    all_res = int(w.blocks(2 * total_steps).sum()) * w.n_layers
    fits_resident = w.hbm_budget_bytes is None and all_res * w.page_bytes < 250e9
    pages = (max(need, all_res) if fits_resident else need) + 8
    if w.hbm_budget_bytes is not None:
        pages = max(pages, w.hbm_budget_bytes // w.page_bytes)
    # head-room in the pinned arena for the switch to the searched plan: its demotions are placed
    # before the promotions release the old runs, so both splits are held for a moment
    host_pages = min(int(host_blocks * 2.2) + 8, int(args.max_host_gib * (1 << 30)) // w.page_bytes)
    host_pages = max(host_pages, host_blocks + 8)
    g = harness.GpuRun(w, prefetch_slots=slots, chunk_tokens=args.chunk_tokens,
                       budget_pages=pages, host_pages=host_pages, zero_copy=args.zero_copy,
                       max_tokens=int(w.ctx_len.max()) + 2 * total_steps + 32)
    B, L = w.n_req, w.n_layers
    # per-step inputs, generated once and resident in HBM: [S][L][B][...]
    q_all = torch.empty((total_steps, L, B, w.n_q_heads, w.head_dim), dtype=torch.bfloat16, device=dev)
    k_all = torch.empty((total_steps, L, B, w.n_kv_heads, w.head_dim), dtype=torch.bfloat16, device=dev)
    v_all = torch.empty_like(k_all)
    for l in range(L):
        for r, rid in enumerate(w.req_ids):
            q_all[:, l, r] = gen_q_steps(w.seed, l, int(rid), 0, total_steps, w.n_q_heads, w.head_dim, dev)
            kk, vv = gen_kv(w.seed, l, int(rid), int(w.ctx_len[r]), total_steps, w.n_kv_heads, w.head_dim, dev)
            k_all[:, l, r], v_all[:, l, r] = kk, vv
    out = torch.empty((L, B, w.n_q_heads, w.head_dim), dtype=torch.bfloat16, device=dev)
    torch.cuda.synchronize()
    setup_s = time.perf_counter() - t_setup

    step_no = [0]

    def run_step(stats=False):
        s = step_no[0]
        st = g.ctx.step(q_all[s], k_all[s], v_all[s], out, stats)
        step_no[0] += 1
        return st

    def drain():
        g.cs.synchronize()
        g.xs.synchronize()
        torch.cuda.synchronize()

    for _ in range(W):
        run_step()
    drain()
    t0 = time.perf_counter()
    host_enqueue = 0.0
    # The host runs at most RUN_AHEAD steps ahead of the GPU, as a serving loop that samples a token per step
    # would (it cannot run ahead at all): hundreds of queued copies and launches otherwise fill the runtime's
    # queues and the enqueue calls themselves start to block at awkward points.
    RUN_AHEAD = args.run_ahead
    done = []
    for _ in range(K):
        if RUN_AHEAD > 0 and len(done) >= RUN_AHEAD:
            done.pop(0).synchronize()
        th = time.perf_counter()
        run_step()
        host_enqueue += time.perf_counter() - th     # host time spent enqueueing the step (no GPU wait inside)
        ev = torch.cuda.Event()
        ev.record(g.cs)
        done.append(ev)
    drain()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / K

    # bytes of KV attended per step at the middle of the timed region (lengths grow by one per step)
    tok_bytes = w.kv_bytes_per_token_layer
    mid_len = w.ctx_len.astype(np.int64) + W + (K + 1) / 2.0
    layer_bytes = float(mid_len.sum()) * tok_bytes
    resident_frac = float((w.placement * mid_len[:, None]).sum() / (mid_len.sum() * L))
    step_bytes = layer_bytes * L
    value = step_bytes / (ms_per_step * 1e-3) / 1e9

    # same K steps again with the library's HIP events (on its compute / copy streams) switched on
    attn_ms, comb_ms, copy_ms, stall_ms, step_ev_ms, link_bytes, hbm_bytes = [], [], [], [], [], 0, 0
    drain()
    t1 = time.perf_counter()
    for _ in range(K):
        st = run_step(True)
        attn_ms += [st.attn_ms[l] for l in range(L)]
        comb_ms += [st.combine_ms[l] for l in range(L)]
        copy_ms.append(st.copy_ms_total)
        stall_ms.append(st.stall_ms_total)
        step_ev_ms.append(st.step_ms)
        link_bytes += st.link_kv_bytes
        hbm_bytes += st.hbm_kv_bytes
    drain()
    ms_per_step_events = (time.perf_counter() - t1) * 1e3 / K
    ev_len = w.ctx_len.astype(np.int64) + W + K + (K + 1) / 2.0
    launch_bytes = float(ev_len.sum()) * tok_bytes               # algorithmic bytes of one attention launch
    avg_attn_ms = float(np.mean(attn_ms))
    achieved = launch_bytes / (avg_attn_ms * 1e-3) / 1e9
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "attention_traffic.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            tj = json.load(f)
        if tj.get("workload") == args.workload and args.placement == "workload" and not args.zero_copy:
            traffic = tj.get("hbm_bytes_per_launch")
    roofline = {"bound": "hbm", "kernel": "attention_kernel (split-K GQA decode attention, one launch per layer)",
                "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                "traffic": traffic, "bytes_per_launch": launch_bytes, "avg_launch_ms": avg_attn_ms,
                "launches_timed": len(attn_ms), "avg_combine_ms": float(np.mean(comb_ms))}
    link = None
    if link_bytes and args.zero_copy:
        # the kernel itself pulls the offloaded blocks over the link: the attention launches are the transfer
        rate = link_bytes / (sum(attn_ms) * 1e-3) / 1e9
        link = {"bytes_per_step": link_bytes / K, "mode": "zero-copy (read in place by attention_kernel)",
                "achieved": rate, "measured_peak": link_peak, "unit": "GB/s", "frac_of_measured_peak": rate / link_peak,
                "attn_ms_per_step": float(np.sum(attn_ms) / K)}
    elif link_bytes:
        rate = link_bytes / (sum(copy_ms) * 1e-3) / 1e9 if sum(copy_ms) > 0 else 0.0
        link = {"bytes_per_step": link_bytes / K, "copy_busy_ms_per_step": float(np.mean(copy_ms)),
                "achieved": rate, "measured_peak": link_peak, "unit": "GB/s",
                "frac_of_measured_peak": rate / link_peak, "stall_ms_per_step": float(np.mean(stall_ms)),
                "attn_ms_per_step": float(np.sum(attn_ms) / K), "peak_sweep_gbs_by_mib": link_sweep,
                "overlap_efficiency": max(float(np.mean(copy_ms)), float(np.sum(attn_ms) / K)) / ms_per_step_events}

    # the planner's cost model fed with what was just measured (per-layer compute time, link rate):
    # its prediction for this placement against the observed step, and the plan its pruned search
    # would pick under the same block budget
    planner = None
    if link_bytes and not args.zero_copy:
        from paper_2601_10729_amd import orbit_model_latency, orbit_plan_search
        per_layer = np.asarray(attn_ms, dtype=np.float64).reshape(K, L).mean(axis=0) + \
            np.asarray(comb_ms, dtype=np.float64).reshape(K, L).mean(axis=0)
        blocks_per_ms = (link_bytes / (sum(copy_ms) * 1e-3) / 1e3) / w.page_bytes
        b_now = -(-(w.ctx_len.astype(np.int64) + W + 2 * K) // w.page_tokens)
        pred, _ = orbit_model_latency(b_now, w.placement, blocks_per_ms, per_layer)
        # profile refresh as the controller would do it: moving average of the per-layer compute times over the
        # timed steps, and the re-planning trigger on the gap between prediction and observation
        from paper_2601_10729_amd import orbit_profile_ewma, orbit_profile_mismatch
        per_step = (np.asarray(attn_ms, dtype=np.float64) + np.asarray(comb_ms, dtype=np.float64)).reshape(K, L)
        profile = per_step[0].copy()
        for row in per_step[1:]:
            profile = orbit_profile_ewma(profile, row, 0.25)
        pred_ewma, _ = orbit_model_latency(b_now, w.placement, blocks_per_ms, profile)
        replan = bool(orbit_profile_mismatch(pred_ewma, ms_per_step_events, 0.05))
        t_s = time.perf_counter()
        try:
            t_paper, x_paper, evals = orbit_plan_search(b_now, L, need, blocks_per_ms,
                                                        per_layer, prefetch_slots=slots, max_evals=20000)
            search_ms = (time.perf_counter() - t_s) * 1e3
            # the same counts and distances with request r's pattern rotated by r layers (ours): installed below
            t_plan, x_plan, _ = orbit_plan_search(b_now, L, need, blocks_per_ms, per_layer, prefetch_slots=slots,
                                                  max_evals=20000, stagger=True)
            planner = {"predicted_ms_for_this_placement": pred, "observed_ms": ms_per_step_events,
                       "relative_gap": abs(pred - ms_per_step_events) / pred,
                       "paper_space_plan_predicted_ms": t_paper, "paper_space_plan_resident_fraction":
                       float((x_paper * b_now[:, None]).sum() / (b_now.sum() * L)),
                       "searched_plan_predicted_ms": t_plan, "searched_plan_resident_fraction":
                       float((x_plan * b_now[:, None]).sum() / (b_now.sum() * L)),
                       "searched_plan_space": "distance-driven counts, staggered by request",
                       "ewma_profile_predicted_ms": pred_ewma, "replan_triggered_at_5_percent": replan,
                       "search_budget_blocks": need, "search_evaluations": evals, "search_ms": search_ms}
        except Exception as e:                                   # infeasible under the pruned space
            planner = {"predicted_ms_for_this_placement": pred, "observed_ms": ms_per_step_events,
                       "relative_gap": abs(pred - ms_per_step_events) / pred, "search": str(e)}

    # closing the loop: install the searched plan (a stream-ordered switch) and time it against its prediction
    if planner and "searched_plan_predicted_ms" in planner and not args.no_searched_variant and fits_resident:
        try:
            drain()
            cur = w.ctx_len.astype(np.int64) + step_no[0]
            g.ctx.plan_load(w.req_ids, cur.astype(np.int32), x_plan)
            run_step()
            drain()
            sts = [run_step(True) for _ in range(3)]
            drain()
            obs = float(np.mean([s.step_ms for s in sts]))
            planner["searched_plan_observed_ms"] = obs
            planner["searched_plan_relative_gap"] = abs(obs - t_plan) / t_plan
        except Exception as e:                                   # e.g. the host arena cannot hold its offloaded blocks
            planner["searched_plan_observed_ms"] = None
            planner["searched_plan_note"] = str(e)

    # all-resident variant of the same workload: the kernel's HBM rate without the link in the way
    resident = None
    if not args.no_resident_variant and args.placement == "workload" and not w.placement.all() and fits_resident:
        drain()
        cur = w.ctx_len.astype(np.int64) + step_no[0]
        g.ctx.plan_load(w.req_ids, cur.astype(np.int32), np.ones_like(w.placement))
        run_step()
        drain()
        t2 = time.perf_counter()
        n_res = 3
        sts = [run_step(True) for _ in range(n_res)]
        drain()
        res_ms = (time.perf_counter() - t2) * 1e3 / n_res
        rl = w.ctx_len.astype(np.int64) + step_no[0] - 1
        res_launch_bytes = float(rl.sum()) * tok_bytes
        res_attn = float(np.mean([s.attn_ms[l] for s in sts for l in range(L)]))
        resident = {"ms_per_step": res_ms, "effective_kv_gbs": res_launch_bytes * L / (res_ms * 1e-3) / 1e9,
                    "attention_gbs": res_launch_bytes / (res_attn * 1e-3) / 1e9,
                    "attention_frac_of_hbm_peak": res_launch_bytes / (res_attn * 1e-3) / 1e9 / HBM_PEAK_GBS,
                    "avg_launch_ms": res_attn}
    g.close()
    if args.calibrate_copy:
        a = torch.ones(1 << 30, dtype=torch.uint8, device=dev)
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        del a, b

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(dataclasses.replace(w, ctx_len=(w.ctx_len + W).astype(np.int32)))
        # the same rate applied to the whole step's KV bytes: an extrapolation from the sample, not a measurement
        cpu["extrapolated_seconds_per_step"] = step_bytes / (cpu["value"] * 1e9)

    line = {
        "metric": "effective KV GB/s per decode step (HBM + host link)",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {WORKLOAD_TEXT[args.workload]}", "seed": args.seed,
                   "placement": args.placement, "n_req": B, "n_layers": L, "tokens_per_layer": float(mid_len.sum()),
                   "kv_bytes_per_step": step_bytes, "resident_fraction": resident_frac,
                   "prefetch_slots": 0 if args.zero_copy else slots, "zero_copy": bool(args.zero_copy), "note": w.note, "hbm_budget_bytes": w.hbm_budget_bytes, "chunk_tokens": args.chunk_tokens or 1024},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "host_link": link,
        "planner_model": planner,
        "all_resident_variant": resident,
        "host_enqueue_ms_per_step": host_enqueue * 1e3 / K,
        "ms_per_step_with_events": ms_per_step_events,
        "step_ms_median": float(np.median(step_ev_ms)), "step_ms_min": float(np.min(step_ev_ms)),
        "setup_seconds": setup_s,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
