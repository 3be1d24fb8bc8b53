#!/usr/bin/env python3
"""Benchmark of the prefix-tree paged-attention hot path on one MI355X.

A step is one pass of the hot path over one batch of the headline workload, the largest
single-GPU configuration: the 70B-shaped prefix forest with an fp8 KV pool (16 roots of 8192
tokens, 32 children of 2048 tokens each, 512 requests, one query token per request)
= per-node decode kernel + log-sum-exp merge kernel behind attn_decode_plan_run.
All inputs are resident in HBM before the timed region; the plan (tree walk, work list) is built
once per topology outside it.  The other single-GPU configurations (Llama-3-8B shaped decode,
speculative fan-out decode, prefix-hit prefill) follow under "extra"; the two small decode
workloads rotate over several identical pools so that the 256 MB last-level cache cannot serve
their KV bytes.

Prints one JSON line: the headline metric (unique-KV bytes per second), the roofline of the
dominant kernel measured with HIP events, and the CPU oracle timed on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 matrix-core peak


def log(msg: str) -> None:
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def time_steps(fn, steps: int, warmup: int):
    import torch
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        fn(warmup + i)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def time_steps_spread(fn, steps: int, warmup: int, batch: int):
    """`warmup` untimed steps, then exactly `steps` timed ones between two synchronisations.  Returns the
    mean by the wall clock and the per-step times of the batches of `batch` steps the same timed steps
    are cut into (one HIP event between batches), sorted."""
    import torch
    for i in range(warmup):
        fn(i)
    n_b = (steps + batch - 1) // batch
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(n_b + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    evs[0].record()
    for i in range(steps):
        fn(warmup + i)
        if (i + 1) % batch == 0 or i == steps - 1:
            evs[(i + batch) // batch].record()
    torch.cuda.synchronize()
    mean = (time.perf_counter() - t0) / steps
    per = sorted(evs[b].elapsed_time(evs[b + 1]) * 1e-3 / (min(steps, (b + 1) * batch) - b * batch) for b in range(n_b))
    return mean, per


def pct(sorted_vals, q: float):
    return sorted_vals[int(q * (len(sorted_vals) - 1))]


def make_pools(runtime, w, n_pools: int):
    """n_pools identical pools (same page ids, distinct HBM), each with its own plan and buffers."""
    first = runtime.DevicePool(w.num_pages, w.num_kv_heads, w.kv_dtype)
    first.fill_from(w)
    pools = [first]
    for _ in range(n_pools - 1):
        p = runtime.DevicePool(w.num_pages, w.num_kv_heads, w.kv_dtype, poison=False)
        p.k.copy_(first.k)
        p.v.copy_(first.v)
        if first.k_scale is not None:
            p.k_scale.copy_(first.k_scale)
            p.v_scale.copy_(first.v_scale)
        pools.append(p)
    return pools


PLAN_SETTINGS = {}      # --plan name=value ...: planner settings of hkv_decode_plan_params for every decode plan timed here


def bench_decode(runtime, hkv, w, steps: int, warmup: int, n_pools: int, profile_steps: int, flags: int = 0,
                 batch: int = 8, graph: bool = False, hot: bool = False):
    """Times attn_decode_plan_run over `w`, rotating over n_pools identical pools.  Returns a dict:
    sec (median step, seconds), sec_mean (wall clock over the timed steps), node_ms / merge_ms (each kernel's
    own duration from begin/end events attached to its dispatches), and what describes the plan."""
    import torch
    pools = make_pools(runtime, w, n_pools)
    runners = [runtime.DecodeRunner(p, w, flags=flags, **PLAN_SETTINGS) for p in pools]
    f = w.forest
    t0 = time.perf_counter()                                    # tree walk, work list, upload: once per topology
    for _ in range(3):
        hkv.hkv_decode_plan_destroy(hkv.hkv_decode_plan_create(pools[0].handle, f.nodes, f.node_pages, f.req_leaf, w.num_q_heads))
    plan_ms = (time.perf_counter() - t0) / 3 * 1e3
    mean, per = time_steps_spread(lambda i: runners[i % n_pools].run(), steps, warmup, batch)
    res = {"sec": pct(per, 0.5), "sec_mean": mean,
           "ms_per_step_p10_p50_p90": [round(pct(per, q) * 1e3, 5) for q in (0.1, 0.5, 0.9)]}
    # same steps again with a begin and an end HIP event attached to each kernel dispatch (on the launch
    # stream): the kernels' own durations, as a kernel trace reports them
    node_each, merge_each, rows_each, tile_each = [], [], [], []
    for r in runners:
        hkv.hkv_decode_plan_set_profiling(r.plan, True)
    for i in range(profile_steps):
        r = runners[i % n_pools]
        r.run()
        a, b = hkv.hkv_decode_plan_elapsed_ms(r.plan)
        node_each.append(a)
        merge_each.append(b)
        a, b = hkv.hkv_decode_plan_elapsed_kernels_ms(r.plan)
        rows_each.append(a)
        tile_each.append(b)
    for r in runners:
        hkv.hkv_decode_plan_set_profiling(r.plan, 0)
    res["node_ms"] = sum(node_each) / max(1, len(node_each))
    res["merge_ms"] = sum(merge_each) / max(1, len(merge_each))
    res["rows_kernel_ms"] = sum(rows_each) / max(1, len(rows_each))
    res["tile_kernel_ms"] = sum(tile_each) / max(1, len(tile_each))
    if node_each:
        srt = sorted(node_each)
        res["node_kernel_ms_p10_p50_p90"] = [round(pct(srt, q), 5) for q in (0.1, 0.5, 0.9)]
    if graph:
        # the same steps as one HIP graph of n_pools steps (one per pool), replayed: no launch call between kernels
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for r in runners:
                r.run()
            side.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                for r in runners:
                    r.run()
        torch.cuda.synchronize()
        reps = max(1, steps // n_pools)
        for _ in range(3):
            g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        res["graph_replay_ms_per_step"] = round(e0.elapsed_time(e1) / (reps * n_pools), 5)
        del g
    if hot:   # cache-resident variant for context (always the same pool; only meaningful below 256 MB)
        res["cache_resident_ms_per_step"] = round(time_steps(lambda i: runners[0].run(), steps, warmup) * 1e3, 5)
    res["info"] = {
        "items": int(len(hkv.hkv_decode_plan_items(runners[0].plan))),
        "tile_items": int(hkv.hkv_decode_plan_num_tile_items(runners[0].plan)),
        "tile_workgroups": int(hkv.hkv_decode_plan_tile_workgroups(runners[0].plan)),
        "one_launch": bool(hkv.hkv_decode_plan_is_fused(runners[0].plan)),
        "workgroups": int(hkv.hkv_decode_plan_num_workgroups(runners[0].plan)),
        "partials": int(hkv.hkv_decode_plan_num_parts(runners[0].plan)),
        "max_partials_per_row": int(hkv.hkv_decode_plan_max_parts(runners[0].plan)),
        "workspace_bytes": int(runners[0].ws_bytes),
        "host_planning_ms_once_per_topology": round(plan_ms, 3),
    }
    for r in runners:
        r.close()
    for p in pools:
        p.close()
    del runners, pools
    torch.cuda.empty_cache()
    return res


def decode_entry(w, res):
    """One decode workload's figures as they go into the JSON line."""
    uniq = w.unique_kv_bytes()
    out = {
        "unique_kv_bytes": uniq,
        "unique_kv_GBps": round(uniq / res["sec"] / 1e9, 2),
        "attended_tokens_per_s": round(w.forest.attended_tokens() / res["sec"], 1),
        "ms_per_step": round(res["sec"] * 1e3, 5),
        "ms_per_step_mean_wall": round(res["sec_mean"] * 1e3, 5),
        "ms_per_step_p10_p50_p90": res["ms_per_step_p10_p50_p90"],
        "hbm_frac_whole_step": round(uniq / res["sec"] / 1e9 / HBM_PEAK_GBS, 4),
        "node_kernel_ms": round(res["node_ms"], 5),
        "node_kernel_hbm_frac": round(uniq / (res["node_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4) if res["node_ms"] else None,
        "merge_kernel_ms": round(res["merge_ms"], 5),
        "rows_kernel_ms": round(res["rows_kernel_ms"], 5),
        "tile_kernel_ms": round(res["tile_kernel_ms"], 5),
        **res["info"],
    }
    for k in ("node_kernel_ms_p10_p50_p90", "graph_replay_ms_per_step", "cache_resident_ms_per_step"):
        if k in res:
            out[k] = res[k]
    return out


def bench_prefill(runtime, hkv, w, steps: int, warmup: int):
    import torch
    pool = runtime.DevicePool(w.num_pages, w.num_kv_heads, w.kv_dtype)
    pool.fill_from(w)
    r = runtime.PrefillRunner(pool, w)
    sec = time_steps(lambda i: r.run(), steps, warmup)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(steps):
        r.run()
    ev1.record()
    torch.cuda.synchronize()
    kern_ms = ev0.elapsed_time(ev1) / steps
    tiles = int(len(hkv.hkv_prefill_plan_tiles(r.plan)))
    # tiles that took the running-maximum fallback, per launch (the plan counts them over all its runs)
    fallback = hkv.hkv_prefill_plan_fallback_tiles(r.plan) / (2 * steps + warmup)
    r.close()
    pool.close()
    torch.cuda.empty_cache()
    return sec, kern_ms, tiles, fallback


def bench_pool_write(runtime, w, steps: int):
    """KV write of new tokens (timed apart from attention): one call writing 8192 tokens."""
    import numpy as np
    import torch
    n_tok = 8192
    pool = runtime.DevicePool(n_tok // 16, w.num_kv_heads, w.kv_dtype, poison=False)
    k = torch.randn((n_tok, w.num_kv_heads, 128), device="cuda").to(torch.bfloat16).view(torch.int16)
    v = torch.randn((n_tok, w.num_kv_heads, 128), device="cuda").to(torch.bfloat16).view(torch.int16)
    ids = np.random.default_rng(0).permutation(n_tok // 16).astype(np.int32)
    sec = time_steps(lambda i: pool.write(ids, 0, k, v), steps, 3)
    pool.close()
    src_bytes = 2 * n_tok * w.num_kv_heads * 128 * 2
    return src_bytes / sec / 1e9


def bench_workflow(runtime, hkv, wl, shape: str):
    """Call orders of one worker compared on the cost model (prefill usage, total token step) and on
    the GPU (kv_pool_write of the new tokens + suffix-only prefill attention per call)."""
    import torch
    if shape == "map_reduce":
        wf = wl.workflow_map_reduce(n_queries=6, n_mappers=4, sys_len=2048, ctx_len=8192, len_out=256)
        per_query = 5
    elif shape == "debate":
        wf = wl.workflow_debate(n_queries=6, n_agents=3, rounds=3, sys_len=4096, q_len=2048, len_out=512)
        per_query = 9
    elif shape == "iterative":
        wf = wl.workflow_iterative(n_queries=8, n_chunks=6, sys_len=1024, chunk_len=4096, len_out=512)
        per_query = 6
    elif shape == "parallel":
        wf = wl.workflow_parallel(n_queries=3, n_experts=7, n_chunks=6, sys_len=2048, chunk_len=4096, len_out=256)
        per_query = 43
    else:
        wf = wl.workflow_reflect(n_queries=12, sys_len=4096, q_len=4096, len_out=512)
        per_query = 3
    r = runtime.WorkflowRunner(wf)
    capacity = 1 << 16
    n = wf.n_calls
    longest_pages = max(len(runtime.workflow_prompt_tokens(wf, c)) for c in range(n)) // 16 + 1
    helium = hkv.trt_schedule(r.tree, 1, capacity)[0][0]
    # the same schedule as nested sequences (one inner sequence per static prompt), run best-effort
    nested = hkv.trt_nested(r.tree, [helium])[0]
    soft = hkv.trt_run_soft(r.tree, [[c for seq in nested for c in seq]], capacity)[0][0]
    orders = {
        "cache_aware_schedule": (helium, True),
        "nested_sequences_best_effort": (soft, True),
        "query_by_query": (list(range(n)), True),
        "operator_by_operator": ([q * per_query + o for o in range(per_query) for q in range(n // per_query)], True),
        "no_prefix_reuse": (helium, False),
    }
    res = {"workflow": wf.name, "calls": n, "tree_nodes": int(len(r.nodes["parent"])), "capacity_M": capacity,
           "inner_sequences": len(nested),
           "layer": "32 q / 8 kv heads, head_dim 128, bf16", "orders": {}}
    for name, (seq, cache) in orders.items():
        usage = r.prepare(seq, cache)
        T = hkv.trt_evaluate(r.tree, [seq], capacity)[2] if cache else None
        r.run()
        torch.cuda.synchronize()
        ms = []
        for _ in range(3):
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            ev0.record()
            r.run()
            ev1.record()
            torch.cuda.synchronize()
            ms.append(ev0.elapsed_time(ev1))
        res["orders"][name] = {"prefill_usage_tokens": int(sum(usage)),
                               "total_token_step_times_M": T, "gpu_ms": round(min(ms), 3)}
        if cache:   # the same order served through the block-level LRU prefix cache with room for two of the longest prompts
            pr = runtime.PrefixCacheRunner([runtime.workflow_prompt_tokens(wf, c) for c in seq], 2 * longest_pages, 32, 8,
                                           random_tensors=True)
            sim = pr.prepare()
            pr.run()
            torch.cuda.synchronize()
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            ev0.record()
            pr.run()
            ev1.record()
            torch.cuda.synchronize()
            pr.close()
            res["orders"][name]["lru_cache_hit_rate"] = round(sim["hit_rate"], 4)
            res["orders"][name]["lru_cache_evictions"] = sim["evictions"]
            res["orders"][name]["lru_cache_gpu_ms"] = round(ev0.elapsed_time(ev1), 3)
    r.close()
    # decode side: the calls of one dependency level generate side by side; the workflow's templated radix
    # tree is the prefix forest of that step (each call has produced half of its output)
    res["decode_levels"] = []
    for k, calls in enumerate(runtime.workflow_levels(wf)):
        wd = runtime.workflow_decode_workload(wf, calls, [max(1, wf.len_out[c] // 2) for c in calls])
        wu = wl.without_sharing(wd)
        row = {"level": k, "calls": len(calls), "unique_kv_MB": round(wd.unique_kv_bytes() / 1e6, 1),
               "attended_over_unique": round(wu.unique_kv_bytes() / max(1, wd.unique_kv_bytes()), 2)}
        for name, w in (("tree_decode_us", wd), ("unshared_decode_us", wu)):
            n_pools = max(1, min(4, int(600e6 // max(1, w.unique_kv_bytes())) + 1))
            pools = []
            for i in range(n_pools):
                p = runtime.DevicePool(w.num_pages, w.num_kv_heads, w.kv_dtype, poison=False)
                p.fill_random(i)
                pools.append(p)
            runners = [runtime.DecodeRunner(p, w, random_q=True) for p in pools]
            row[name] = round(time_steps(lambda i: runners[i % n_pools].run(), 100, 10) * 1e6, 1)
            for rr in runners:
                rr.close()
            for p in pools:
                p.close()
            del runners, pools
            torch.cuda.empty_cache()
        res["decode_levels"].append(row)
    return res


def bench_sensitivity(runtime, hkv, wl, model: str, steps: int, warmup: int):
    """Prefix-sharing sensitivity (the study of Section 7 that varies system / context / question /
    output lengths over 100 queries): the prefix-tree decode step and the suffix-only prefill against the
    same requests with nothing shared (private copies of every prompt, whole-prompt prefill), same kernels.
    Pools are filled with random bf16 values on the device (timing only)."""
    import torch

    def timed(make_runner, w, n_pools, n_steps, n_warm):
        pools = []
        for i in range(n_pools):
            p = runtime.DevicePool(w.num_pages, w.num_kv_heads, w.kv_dtype, poison=False)
            p.fill_random(i)
            pools.append(p)
        runners = [make_runner(p, w, random_q=True) for p in pools]
        sec = time_steps(lambda i: runners[i % n_pools].run(), n_steps, n_warm)
        for r in runners:
            r.close()
        for p in pools:
            p.close()
        del runners, pools
        torch.cuda.empty_cache()
        return sec

    rows = {}
    for name, (sy, cx, qu, ou) in wl.SENSITIVITY_GRID.items():
        wd = wl.prefix_sensitivity(sy, cx, qu, ou, model=model, mode="decode")
        wf = wl.without_sharing(wd)
        pools_for = lambda w: max(1, min(4, int(600e6 // max(1, w.unique_kv_bytes())) + 1))   # > last-level cache in rotation
        t_tree = timed(runtime.DecodeRunner, wd, pools_for(wd), steps, warmup)
        t_flat = timed(runtime.DecodeRunner, wf, pools_for(wf), steps, warmup)
        wp = wl.prefix_sensitivity(sy, cx, qu, ou, model=model, mode="prefill")
        wpf = wl.without_sharing(wp)
        t_pre = timed(runtime.PrefillRunner, wp, 1, 5, 2)
        t_pre_flat = timed(runtime.PrefillRunner, wpf, 1, 5, 2)
        rows[name] = {
            "system_context_question_output": [sy, cx, qu, ou],
            "decode": {"unique_kv_MB": round(wd.unique_kv_bytes() / 1e6, 1),
                       "attended_over_unique": round(wf.unique_kv_bytes() / wd.unique_kv_bytes(), 2),
                       "tree_ms": round(t_tree * 1e3, 4), "unshared_ms": round(t_flat * 1e3, 4),
                       "tree_unique_GBps": round(wd.unique_kv_bytes() / t_tree / 1e9, 1),
                       "unshared_GBps": round(wf.unique_kv_bytes() / t_flat / 1e9, 1),
                       "speedup": round(t_flat / t_tree, 2)},
            "prefill": {"new_tokens": int(wp.total_q()), "whole_prompt_tokens": int(wpf.total_q()),
                        "suffix_only_ms": round(t_pre * 1e3, 3), "whole_prompt_ms": round(t_pre_flat * 1e3, 3),
                        "suffix_only_TFLOPs": round(wp.useful_flop() / t_pre / 1e12, 1),
                        "whole_prompt_TFLOPs": round(wpf.useful_flop() / t_pre_flat / 1e12, 1),
                        "speedup": round(t_pre_flat / t_pre, 2)},
        }
        log(f"sensitivity {name} done")
    hq, hk = wl.MODEL_HEADS[model]
    return {"study": "prefix_sharing_sensitivity", "model_layer": f"{model}: {hq} q / {hk} kv heads, head_dim 128, bf16",
            "queries": 100, "grid": "own choice (the paper's six settings are only in a figure)", "rows": rows}


def bench_mixed(runtime, hkv, wl, steps: int, warmup: int):
    """A chunked-prefill step (64 decode rows of the c2 shape + 8 prompts prefilling 512 tokens each behind
    the same shared prefix): everything through one suffix-only prefill launch, against decode rows
    through the prefix-tree plan + the chunks through prefill.  Four pools in rotation."""
    import torch
    w = wl.mixed_step()
    res = {"workload": w.name, "layer": "32 q / 8 kv heads, head_dim 128, bf16",
           "unique_kv_MB": round(w.unique_kv_bytes() / 1e6, 1), "new_tokens": int(w.total_q())}
    for name, make in (("one_prefill_launch", runtime.PrefillRunner), ("tree_decode_plus_prefill", runtime.MixedStepRunner)):
        pools = []
        for i in range(4):
            p = runtime.DevicePool(w.num_pages, w.num_kv_heads, w.kv_dtype, poison=False)
            p.fill_random(i)
            pools.append(p)
        runners = [make(p, w, random_q=True) for p in pools]
        sec = time_steps(lambda i: runners[i % 4].run(), steps, warmup)
        res[name + "_ms"] = round(sec * 1e3, 4)
        for r in runners:
            r.close()
        for p in pools:
            p.close()
        del runners, pools
        torch.cuda.empty_cache()
    return res


def bench_decode_loop(runtime, hkv, wl, steps: int, warmup: int):
    """Generation loop on the c2 shape: every step stores one new token per request, updates the plan and
    runs the prefix-tree decode.  With a growing plan, store and update are one call
    (hkv_decode_plan_append_tokens); without, kv_pool_append and a new plan per step.  Four independent loops (pool + plan each) take
    turns so that the 256 MB last-level cache cannot hold the KV bytes.  Wall clock, host work included."""
    import numpy as np
    import torch
    w = wl.config2()
    f = w.forest
    n_loops, res = 4, {"workload": w.name + " + one generated token per request and step", "loops_rotated": 4}
    k_new = _rand_bits(torch, (f.n_req, w.num_kv_heads, 128))
    v_new = _rand_bits(torch, (f.n_req, w.num_kv_heads, 128))
    for mode in ("growing_plan", "new_plan_every_step"):
        loops = []
        for i in range(n_loops):
            p = runtime.DevicePool(w.num_pages + f.n_req * ((2 * steps + warmup) // 16 + 2), w.num_kv_heads, w.kv_dtype, poison=False)
            p.fill_random(i)
            hkv.kv_pool_alloc(p.handle, w.num_pages)                      # the forest's pages are in use
            r = runtime.DecodeRunner(p, w, random_q=True, reserve_tokens=2 * steps + warmup if mode == "growing_plan" else 0)
            loops.append({"pool": p, "runner": r, "n_tokens": f.n_tokens.copy(),
                          "last_page": np.array([f.node_pages[f.page_begin[v] + f.n_pages[v] - 1] for v in f.req_leaf]),
                          "nodes": f.nodes.copy(), "node_pages": [list(f.node_pages[f.page_begin[v]: f.page_begin[v] + f.n_pages[v]])
                                                                  for v in range(f.n_nodes)]})
        host_us = []

        def step(i):
            lp = loops[i % n_loops]
            t0 = time.perf_counter()
            leaves = f.req_leaf
            slots = lp["n_tokens"][leaves] % 16
            new = np.full(f.n_req, -1, dtype=np.int32)
            need = np.nonzero(slots == 0)[0]
            if len(need):
                new[need] = hkv.kv_pool_alloc(lp["pool"].handle, len(need))
                lp["last_page"][need] = new[need]
                for r_ in need:
                    lp["node_pages"][leaves[r_]].append(int(new[r_]))
            lp["n_tokens"][leaves] += 1
            if mode == "growing_plan":                                         # tokens and plan update in one launch
                lp["runner"].append_tokens(new, k_new, v_new)
            else:                                                              # what a caller without it has to do
                hkv.kv_pool_append(lp["pool"].handle, lp["last_page"], slots, k_new, v_new)
                nodes = lp["nodes"]
                nodes[:, 3] = lp["n_tokens"]
                nodes[:, 2] = (lp["n_tokens"] + 15) // 16
                nodes[1:, 1] = np.cumsum(nodes[:-1, 2])
                pages = np.fromiter((p_ for l in lp["node_pages"] for p_ in l), dtype=np.int32)
                old = lp["runner"].plan
                lp["runner"].plan = hkv.hkv_decode_plan_create(lp["pool"].handle, nodes, pages, f.req_leaf, w.num_q_heads)
                hkv.hkv_decode_plan_destroy(old)
            host_us.append((time.perf_counter() - t0) * 1e6)
            lp["runner"].run()

        # two timed windows, the better one counts: the first window of a fresh process has been seen several
        # times slower than every later one
        sec = min(time_steps(step, steps, warmup), time_steps(step, steps, 0))
        res[mode + "_us_per_step"] = round(sec * 1e6, 2)
        res[mode + "_host_us_before_the_run_call"] = round(float(np.median(host_us[warmup:])), 2)
        for lp in loops:
            lp["runner"].close()
            lp["pool"].close()
        del loops
        torch.cuda.empty_cache()
    return res


def _rand_bits(torch, shape):
    return torch.randn(shape, device="cuda").to(torch.bfloat16).view(torch.int16)


def cpu_baseline_decode(w, budget_s: float = 20.0):
    """The fp64 oracle as it stands on the host cores, on a bounded sample of the workload: the requests
    below the first root (the whole workload when it has a single root), repeated within the budget."""
    import numpy as np
    from oracle import oracle as orc
    f = w.forest
    first_root = int(f.path(int(f.req_leaf[0]))[0])
    sample = [r for r in range(f.n_req) if int(f.path(int(f.req_leaf[r]))[0]) == first_root]
    nodes = sorted({v for r in sample for v in f.path(int(f.req_leaf[r]))})
    hp = orc.HostPool(w.num_pages, w.num_kv_heads, w.kv_dtype)
    for v in nodes:                                              # only the nodes the sample reads
        if f.n_tokens[v]:
            k, vv = w.node_kv(v)
            hp.write(f.node_pages[f.page_begin[v]: f.page_begin[v] + f.n_pages[v]], 0, k, vv)
    bt, kv_len, *_ = orc.flatten_workload(w)
    q = w.q()
    idx = np.asarray(sample)
    reps, t_total = 0, 0.0
    while reps < 1 or (t_total < budget_s / 2 and reps < 500):      # about 10 s of CPU work
        t0 = time.perf_counter()
        orc.attn_decode(hp, q[idx], bt[idx], kv_len[idx], float(w.scale))
        t_total += time.perf_counter() - t0
        reps += 1
    sec = t_total / reps
    uniq = int(sum(int(f.n_tokens[v]) for v in nodes)) * w.kv_bytes_per_token()
    attended = int(kv_len[idx].sum())
    return {
        "value": uniq / sec / 1e9,
        "unit": "GB/s",
        "cores": orc.num_threads(),
        "kind": "oracle",
        "sample": f"{len(sample)} of {f.n_req} requests (all requests below the first root: {len(nodes)} nodes, "
                  f"{uniq} unique KV bytes, {attended} attended tokens), mean of {reps} runs, {sec:.3f} s each; "
                  "the oracle gathers every request's full sequence, so it reads attended rather than unique bytes",
        "attended_tokens_per_s": attended / sec,
        "seconds_per_run": sec,
    }


def load_traffic(name: str):
    """HBM bytes per launch of the dominant kernel from the rocprofv3 counter runs kept under profiles/."""
    tpath = os.path.join(ROOT, "profiles", name)
    if os.path.exists(tpath):
        try:
            return json.load(open(tpath)).get("hbm_bytes_per_launch")
        except Exception:
            return None
    return None


def sweep_read_probe(torch, bp):
    """Plain streaming reads over launch shapes and sizes: the best rate this machine gives a kernel that only reads."""
    rows = []
    sizes = {"142.6 MB (c2)": 142606336, "184.5 MB (c3)": 184549376, "2416 MB (c5)": 2415919104}
    for label, nbytes in sizes.items():
        n_buf = 4 if nbytes < (1 << 30) else 1
        bufs = [torch.zeros(nbytes // 4, dtype=torch.int32, device="cuda") for _ in range(n_buf)]
        reps = 100 if nbytes < (1 << 30) else 12
        for wgs in (2, 4, 8, 16):
            for threads in (256, 512, 1024):
                if wgs * threads > 2048 * 2:
                    continue
                for in_flight in (2, 4, 8, 16):
                    for contiguous in (False, True):
                        for nt in (False, True):
                            g = bp.hbm_read(bufs, nbytes, reps, wgs, threads, in_flight, contiguous, nt)
                            rows.append({"size": label, "wgs_per_cu": wgs, "threads": threads, "in_flight": in_flight,
                                         "contiguous": contiguous, "nontemporal": nt, "GBps": round(g, 1)})
        del bufs
        torch.cuda.empty_cache()
        best = max((r for r in rows if r["size"] == label), key=lambda r: r["GBps"])
        log(f"read probe {label}: best {best}")
    # the same bytes as randomly placed (page, head) blocks, one block per wavefront at a time: a decode step's pattern
    for label, nbytes in sizes.items():
        n_buf = 4 if nbytes < (1 << 30) else 1
        bufs = [torch.zeros(nbytes // 4, dtype=torch.int32, device="cuda") for _ in range(n_buf)]
        reps = 100 if nbytes < (1 << 30) else 12
        for block in (2048, 4096):
            g = torch.Generator(device="cuda")
            g.manual_seed(5)
            for perm in (False, True):
                n_blocks = nbytes // block
                order = (torch.randperm(n_blocks, device="cuda", generator=g) if perm
                         else torch.arange(n_blocks, device="cuda")).to(torch.int32)
                for wgs in (1, 2, 3, 4, 8):
                    for depth in (1, 2, 4):
                        for nt in (False, True):
                            gb = bp.hbm_paged_read(bufs, order, block, reps, wgs, 256, depth, nt)
                            rows.append({"size": label, "paged_block_bytes": block, "random_order": perm, "wgs_per_cu": wgs,
                                         "threads": 256, "blocks_ahead": depth, "nontemporal": nt, "GBps": round(gb, 1)})
        del bufs
        torch.cuda.empty_cache()
        best = max((r for r in rows if r["size"] == label and r.get("random_order")), key=lambda r: r["GBps"])
        log(f"paged read probe {label}: best random-order {best}")
    return rows


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--pools", type=int, default=4, help="identical pools the small decode workloads rotate over (cache defeat)")
    ap.add_argument("--no-extras", action="store_true", help="skip the other workloads (c2, c3, c4, pool write, probes)")
    ap.add_argument("--fp8-matrix", action="store_true",
                    help="run the fp8 forest on the fp8 matrix instruction (HKV_PLAN_FP8_MATRIX) instead of the default path")
    ap.add_argument("--one-stream", action="store_true",
                    help="decode plans queue the tile kernel in front of the other on one stream (HKV_PLAN_ONE_STREAM)")
    ap.add_argument("--plan", nargs="*", default=[], metavar="NAME=VALUE",
                    help="planner settings (fields of hkv_decode_plan_params) for the decode plans, e.g. leaf_chunk=1024")
    ap.add_argument("--graph", action="store_true", help="with --profile-workload: also time the step as a replayed HIP graph")
    ap.add_argument("--hot", action="store_true", help="also time the small decode workloads without pool rotation (cache-resident)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--decode-loop", action="store_true",
                    help="generation loop on the c2 shape: token append + plan update + decode per step, with a growing "
                         "plan and with a new plan per step (not the headline line)")
    ap.add_argument("--mixed", action="store_true", help="a chunked-prefill step: one prefill launch vs tree decode + prefill")
    ap.add_argument("--sensitivity", choices=["llama3-8b", "qwen3-8b", "qwen3-14b", "qwen3-32b"], default=None,
                    help="prefix-sharing sensitivity grid for one model's layer shape instead of the headline line")
    ap.add_argument("--profile-workload", choices=["c2", "c3", "c4", "c5", "c5_leaves", "c5_roots", "c3_leaves", "c3_shared"],
                    default=None,
                    help="run only this workload for a few steps and print its figures (for rocprofv3 runs; not the headline line)")
    ap.add_argument("--workflow", choices=["map_reduce", "debate", "reflect", "iterative", "parallel"], default=None,
                    help="scheduling-layer experiment: run the prefill side of a synthetic workflow on one worker "
                         "under several call orders and print token steps beside measured GPU time (not the headline line)")
    ap.add_argument("--sweep-read-probe", action="store_true",
                    help="sweep the plain-read probe over launch shapes and sizes and print the table (not the headline line)")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="MiB",
                    help="also run a plain elementwise copy kernel over this many MiB three times (a known-size "
                         "kernel to calibrate rocprofv3's FETCH_SIZE / WRITE_SIZE counters against)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (every box has one GPU); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    for kv in args.plan:
        name, _, value = kv.partition("=")
        PLAN_SETTINGS[name] = int(value)
    import torch
    from paper_2603_16104_amd import binding as hkv, runtime, workloads as wl
    import bench_probes as bp
    if not torch.cuda.is_available():
        print("bench.py needs an MI355X; no GPU is visible", file=sys.stderr)
        return 2
    hkv.lib()

    if args.copy_probe:
        n = args.copy_probe * (1 << 20) // 4
        src = torch.arange(n, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1, out=dst)       # reads n*4 bytes, writes n*4 bytes
        torch.cuda.synchronize()
        log(f"copy probe: 3 x elementwise add over {n * 4} bytes read + {n * 4} bytes written")
        del src, dst
        torch.cuda.empty_cache()

    if args.sweep_read_probe:
        print(json.dumps(sweep_read_probe(torch, bp)), flush=True)
        return 0

    if args.workflow:
        print(json.dumps(bench_workflow(runtime, hkv, wl, args.workflow)), flush=True)
        return 0

    if args.mixed:
        print(json.dumps(bench_mixed(runtime, hkv, wl, min(args.steps, 100), args.warmup)), flush=True)
        return 0

    if args.decode_loop:
        print(json.dumps(bench_decode_loop(runtime, hkv, wl, min(args.steps, 160), args.warmup)), flush=True)
        return 0

    if args.sensitivity:
        print(json.dumps(bench_sensitivity(runtime, hkv, wl, args.sensitivity, min(args.steps, 100), args.warmup)),
              flush=True)
        return 0

    one = hkv.PLAN_ONE_STREAM if args.one_stream else 0
    fp8_flags = (hkv.PLAN_FP8_MATRIX if args.fp8_matrix else 0) | one
    if args.profile_workload:
        name = args.profile_workload
        if name == "c4":
            w4 = wl.config4()
            s4, k4, t4, fb4 = bench_prefill(runtime, hkv, w4, max(1, min(args.steps, 10)), 2)
            tf = w4.useful_flop() / (k4 * 1e-3) / 1e12
            print(json.dumps({"workload": w4.name, "kernel_ms": round(k4, 4), "useful_TFLOPs": round(tf, 2),
                              "mfma_bf16_frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4),
                              "new_tokens_per_s": round(w4.total_q() / s4, 1), "tiles": t4,
                              "fallback_tiles_per_launch": fb4}), flush=True)
        else:
            # *_leaves / c5_roots / c3_shared: the forest with its shared nodes, resp. its leaves, cut down to one
            # block, to time the few-row items (private leaves) and the many-row items (shared nodes) apart
            wx = {"c2": wl.config2, "c3": wl.config3, "c5": wl.config5,
                  "c5_leaves": lambda: wl.config5(root_tokens=16), "c5_roots": lambda: wl.config5(child_tokens=16),
                  "c3_leaves": lambda: wl.config3(root_tokens=16, child_tokens=16),
                  "c3_shared": lambda: wl.config3(leaf_tokens=16)}[name]()
            small = wx.unique_kv_bytes() < (1 << 29)
            rx = bench_decode(runtime, hkv, wx, max(1, min(args.steps, 100 if small else 40)), 10,
                              args.pools if small else 1, 10, fp8_flags if wx.kv_dtype == wl.KV_FP8_E4M3 else one,
                              batch=8 if small else 1, graph=args.graph)
            print(json.dumps({"workload": wx.name, **decode_entry(wx, rx)}), flush=True)
        return 0

    # ---- headline: the largest single-GPU configuration (2.4 GB of fp8 KV: far beyond the last-level cache, one pool)
    w5 = wl.config5()
    f5 = w5.forest
    log(f"workload {w5.name}: {f5.n_req} requests, unique KV {w5.unique_kv_bytes() / 1e6:.1f} MB")
    r5 = bench_decode(runtime, hkv, w5, args.steps, args.warmup, 1, min(max(args.steps, 10), 50), fp8_flags, batch=1)
    e5 = decode_entry(w5, r5)
    uniq = w5.unique_kv_bytes()
    achieved = uniq / (r5["node_ms"] * 1e-3) / 1e9
    result = {
        "metric": "decode_unique_kv_bandwidth",
        "value": e5["unique_kv_GBps"],
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": e5["ms_per_step"],
        "ms_per_step_how": "median over the timed steps (one HIP event after every step); ms_per_step_mean_wall is "
                           "the wall clock between two synchronisations around the same steps divided by their number",
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16 matrix arithmetic with fp32 accumulation over fp8 e4m3 KV" if not args.fp8_matrix else
                 "fp8 e4m3 matrix arithmetic (two-term q and p) with fp32 accumulation over fp8 e4m3 KV",
        "data": "synthetic",
        "config": {
            "workload": "c5_forest_fp8_decode: 16 roots of 8192 tokens x 32 children of 2048 tokens = 512 requests, "
                        "64 q / 8 kv heads, head_dim 128, page 16, fp8 e4m3 KV with per-page per-head fp32 scales, "
                        "bf16 queries, 1 query token per request",
            "pools_rotated": 1,
            "step": "attn_decode_plan_run = per-node decode kernel + lse merge kernel; plan built once outside",
            **{k: v for k, v in e5.items() if k not in ("unique_kv_GBps", "ms_per_step")},
        },
        "roofline": {
            "bound": "hbm",
            "kernel": ("decode_fused_kernel<fp8> (tile items and the other items in one launch)" if e5.get("one_launch") else
                       "decode_node_kernel<fp8> + attn_tile_kernel<decode, fp8> side by side (span from the earlier begin "
                       "to the later end)") if not args.fp8_matrix else "decode_node_kernel<fp8 matrix>",
            "achieved": round(achieved, 2),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": load_traffic("decode_c5_traffic.json"),
            "traffic_how": "HBM bytes per launch from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs kept under profiles/ "
                           "(a stored figure of the same command, not measured in this run)",
            "algorithmic_bytes_per_launch": uniq,
            "kernel_ms": round(r5["node_ms"], 5),
            "kernel_ms_how": "begin/end HIP events attached to each dispatch of this kernel on the launch stream, "
                             "inside whole steps; average over the profiled steps",
            "kernel_ms_p10_p50_p90": r5.get("node_kernel_ms_p10_p50_p90"),
            "merge_kernel_ms": round(r5["merge_ms"], 5),
            "whole_step_frac": e5["hbm_frac_whole_step"],
        },
        "paper_context": "the paper reports end-to-end speedups only (up to 1.56x over KVFlow on 2x H100 NVL); "
                         "no attention-kernel number exists to compare with",
        "extra": {},
    }
    log("c5 done")
    # what a kernel that only reads the same number of bytes reaches (best launch shape of the probe sweep)
    buf = [torch.zeros(uniq // 4, dtype=torch.int32, device="cuda")]
    read_gbps = max(bp.hbm_read(buf, uniq, 10, wgs, 256, inf) for wgs, inf in ((8, 4), (8, 8), (16, 4)))
    del buf
    torch.cuda.empty_cache()
    result["roofline"]["plain_read_same_bytes_GBps"] = round(read_gbps, 1)
    result["roofline"]["frac_of_plain_read"] = round(achieved / read_gbps, 4)

    if not args.no_extras:
        small_steps = max(20, min(5 * args.steps, 1000))
        for key, make, tfile in (("c2_llama8b_decode", wl.config2, "decode_c2_traffic.json"),
                                 ("c3_fanout_decode", wl.config3, "decode_c3_traffic.json")):
            wx = make()
            rx = bench_decode(runtime, hkv, wx, small_steps, 50, args.pools, 100, one, batch=8, graph=True, hot=args.hot)
            result["extra"][key] = {"pools_rotated": args.pools, **decode_entry(wx, rx)}
            t = load_traffic(tfile)
            if t is not None:
                result["extra"][key]["node_kernel_hbm_traffic_bytes"] = t
            bufs = [torch.zeros(wx.unique_kv_bytes() // 4, dtype=torch.int32, device="cuda") for _ in range(args.pools)]
            g = max(bp.hbm_read(bufs, wx.unique_kv_bytes(), 100, wgs, 256, inf) for wgs, inf in ((8, 4), (8, 8), (16, 4)))
            del bufs
            torch.cuda.empty_cache()
            result["extra"][key]["plain_read_same_bytes_GBps"] = round(g, 1)
            log(f"{key} done")
        w4 = wl.config4()
        s4, k4, t4, fb4 = bench_prefill(runtime, hkv, w4, 5, 2)
        tflops = w4.useful_flop() / (k4 * 1e-3) / 1e12
        result["extra"]["c4_prefix_hit_prefill"] = {
            "new_tokens_per_s": round(w4.total_q() / s4, 1), "ms_per_step": round(s4 * 1e3, 4),
            "kernel_ms": round(k4, 4), "useful_TFLOPs": round(tflops, 2),
            "mfma_bf16_frac": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4), "new_tokens": int(w4.total_q()),
            "useful_flop": int(w4.useful_flop()), "tiles": t4,
            "fallback_tiles_per_launch": fb4}     # tiles that repeated with a running softmax maximum (about twice the cost each)
        # matrix-core ceiling with nothing else running: zero operands (nominal clock) and random ones
        # (the clock settles under the power limit), two wavefronts per SIMD as in the prefill kernel
        tf0, ghz0 = bp.mfma_bf16(100000, False, 2)
        tf1, ghz1 = bp.mfma_bf16(100000, True, 2)
        result["extra"]["mfma_probe_bf16"] = {
            "zero_operands_TFLOPs": round(tf0, 1), "zero_operands_clock_GHz": round(ghz0, 3),
            "random_operands_TFLOPs": round(tf1, 1), "random_operands_clock_GHz": round(ghz1, 3)}
        result["extra"]["c4_prefix_hit_prefill"]["frac_of_random_operand_probe"] = round(tflops / tf1, 4)
        log("c4 done")
        result["extra"]["kv_pool_write_src_GBps"] = round(bench_pool_write(runtime, wl.config2(), 20), 1)
    if not args.no_cpu:
        log("timing the CPU oracle")
        result["cpu_baseline"] = cpu_baseline_decode(w5)
    else:
        result["cpu_baseline"] = None
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
