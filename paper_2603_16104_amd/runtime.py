"""Device-memory plumbing around the C ABI: torch owns the HBM buffers and streams, the
library does all the work.  Used by the tests, the smoke check and the bench."""
from __future__ import annotations

from typing import Optional

import numpy as np
import torch

from . import binding as hkv
from . import workloads as wl

# bf16 bit patterns travel as int16 tensors (full torch support); 0x7FC0 is a bf16 NaN, 0x7F the e4m3 NaN
_ELEM = {hkv.BF16: (torch.int16, 0x7FC0), hkv.FP8_E4M3: (torch.uint8, 0x7F), hkv.FP32: (torch.float32, float("nan"))}


class DevicePool:
    """A KV page pool in HBM (library storage format), NaN-poisoned until written."""

    def __init__(self, num_pages: int, num_kv_heads: int, dtype: int, device: str = "cuda:0",
                 free_order: Optional[np.ndarray] = None, poison: bool = True, page_size: int = hkv.PAGE_SIZE):
        self.num_pages, self.num_kv_heads, self.dtype, self.page_size = num_pages, num_kv_heads, dtype, page_size
        tdt, nan_bits = _ELEM[dtype]
        n = num_pages * num_kv_heads * page_size * hkv.HEAD_DIM
        fill = nan_bits if poison else 0
        self.k = torch.full((n,), fill, dtype=tdt, device=device)
        self.v = torch.full((n,), fill, dtype=tdt, device=device)
        self.k_scale = self.v_scale = None
        if dtype == hkv.FP8_E4M3:
            sv = float("nan") if poison else 1.0
            n_sc = num_pages * (page_size // hkv.PAGE_SIZE) * num_kv_heads   # one scale per 16-token block and head
            self.k_scale = torch.full((n_sc,), sv, dtype=torch.float32, device=device)
            self.v_scale = torch.full((n_sc,), sv, dtype=torch.float32, device=device)
        self.handle = hkv.kv_pool_create(num_pages, num_kv_heads, dtype, self.k, self.v, self.k_scale, self.v_scale,
                                         free_order, page_size=page_size)

    def close(self) -> None:
        if self.handle is not None:
            hkv.kv_pool_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def write(self, page_ids, first_slot: int, k_src: torch.Tensor, v_src: torch.Tensor, stream=None) -> None:
        hkv.kv_pool_write(self.handle, page_ids, first_slot, int(k_src.shape[0]), k_src, v_src, stream)

    def fill_random(self, seed: int = 0) -> None:
        """Timing aid for bf16 pools too large to fill through kv_pool_write from host data: every slot
        of every page gets a standard-normal bf16 value drawn on the device (results are not checked)."""
        if self.dtype != hkv.BF16:
            raise ValueError("fill_random: bf16 pools only")
        g = torch.Generator(device=self.k.device)
        g.manual_seed(seed)
        step = 1 << 26
        for t in (self.k, self.v):
            for a in range(0, t.numel(), step):
                b = min(t.numel(), a + step)
                t[a:b] = torch.randn(b - a, device=t.device, generator=g).to(torch.bfloat16).view(torch.int16)
        torch.cuda.synchronize()

    def fill_from(self, workload: wl.Workload, max_chunk_tokens: int = 1 << 16) -> None:
        """kv_pool_write of every node's own tokens into the node's pages."""
        f = workload.forest
        dev = self.k.device
        assert f.page_size == self.page_size and max_chunk_tokens % self.page_size == 0
        for node in range(f.n_nodes):
            nt = int(f.n_tokens[node])
            if nt == 0:
                continue
            k, v = workload.node_kv(node)
            pages = f.node_pages[f.page_begin[node]: f.page_begin[node] + f.n_pages[node]]
            for t0 in range(0, nt, max_chunk_tokens):
                t1 = min(nt, t0 + max_chunk_tokens)
                kd = to_device_bits(k[t0:t1], dev)
                vd = to_device_bits(v[t0:t1], dev)
                self.write(pages[t0 // self.page_size:], 0, kd, vd)
        torch.cuda.synchronize()


def to_device_bits(a: np.ndarray, device="cuda:0") -> torch.Tensor:
    """Host array -> device tensor; uint16 bf16 bit patterns are carried as int16."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(a).to(device)


def _device_random_q(n_tokens: int, num_q_heads: int, device) -> torch.Tensor:
    """Timing aid: standard-normal bf16 queries drawn on the device (bf16 / fp8 pools)."""
    return torch.randn((n_tokens, num_q_heads, hkv.HEAD_DIM), device=device).to(torch.bfloat16).view(torch.int16)


def bf16_tensor_to_f64(t: torch.Tensor) -> np.ndarray:
    """bf16 bit patterns (int16 device tensor) -> float64 numpy; fp32 tensors pass through."""
    if t.dtype == torch.float32:
        return t.cpu().numpy().astype(np.float64)
    b = t.cpu().numpy().view(np.uint16)
    return wl.bf16_bits_to_f32(b).astype(np.float64)


class DecodeRunner:
    """Plan + buffers for repeated decode steps over one forest."""

    def __init__(self, pool: DevicePool, workload: wl.Workload, random_q: bool = False, flags: int = 0,
                 reserve_tokens: int = 0, **settings):
        """reserve_tokens > 0: a decode loop, every request's leaf may grow (append) without a new plan.
        settings: planner settings of hkv_decode_plan_params by name."""
        f = workload.forest
        self.pool, self.workload = pool, workload
        self.plan = hkv.hkv_decode_plan_create_ex(pool.handle, f.nodes, f.node_pages, f.req_leaf,
                                                  workload.num_q_heads, flags, reserve_tokens=reserve_tokens,
                                                  **settings)
        self.ws_bytes = hkv.hkv_decode_plan_workspace_bytes(self.plan)
        dev = pool.k.device
        self.ws = torch.empty(max(self.ws_bytes, 256), dtype=torch.uint8, device=dev)
        self.q = _device_random_q(f.n_req, workload.num_q_heads, dev) if random_q else to_device_bits(workload.q(), dev)
        odt = torch.float32 if pool.dtype == hkv.FP32 else torch.int16      # fp32 pools: fp32 q and out
        self.out = torch.zeros((f.n_req, workload.num_q_heads, hkv.HEAD_DIM), dtype=odt, device=dev)
        self.lse = torch.zeros((f.n_req, workload.num_q_heads), dtype=torch.float32, device=dev)
        self.scale = float(workload.scale)

    def run(self, stream=None) -> None:
        hkv.attn_decode_plan_run(self.plan, self.q, self.scale, self.out, self.lse, self.ws, self.ws_bytes, stream)

    def append(self, new_page_ids=None, stream=None) -> None:
        """Every request's leaf has grown by one token (plans created with reserve_tokens only)."""
        hkv.hkv_decode_plan_append(self.plan, new_page_ids, stream)

    def append_tokens(self, new_page_ids, k_new: torch.Tensor, v_new: torch.Tensor, stream=None) -> None:
        """The same, and the new tokens' K/V ([n_req][Hkv][128]) are stored at the end of the leaves."""
        hkv.hkv_decode_plan_append_tokens(self.plan, new_page_ids, k_new, v_new, stream)

    def close(self) -> None:
        if self.plan is not None:
            hkv.hkv_decode_plan_destroy(self.plan)
            self.plan = None


class PrefillRunner:
    def __init__(self, pool: DevicePool, workload: wl.Workload, random_q: bool = False):
        f = workload.forest
        self.pool, self.workload = pool, workload
        mp = max(1, f.max_pages_per_req())
        self.block_table, self.kv_len, *_ = hkv.prefix_tree_flatten(f.nodes, f.node_pages, f.req_leaf, mp,
                                                                    f.page_size)
        self.cu_q = workload.cu_q()
        self.plan = hkv.hkv_prefill_plan_create(pool.handle, self.cu_q, self.block_table, self.kv_len,
                                                workload.num_q_heads)
        dev = pool.k.device
        tq = workload.total_q()
        self.q = _device_random_q(tq, workload.num_q_heads, dev) if random_q else to_device_bits(workload.q(), dev)
        odt = torch.float32 if pool.dtype == hkv.FP32 else torch.int16      # fp32 pools: fp32 q and out
        self.out = torch.zeros((tq, workload.num_q_heads, hkv.HEAD_DIM), dtype=odt, device=dev)
        self.lse = torch.zeros((tq, workload.num_q_heads), dtype=torch.float32, device=dev)
        self.scale = float(workload.scale)
        self.ws_bytes = hkv.hkv_prefill_plan_workspace_bytes(self.plan)      # fp8 pools: scratch for dequantised pages
        self.ws = torch.empty(max(self.ws_bytes, 256), dtype=torch.uint8, device=dev) if self.ws_bytes else None

    def run(self, stream=None) -> None:
        hkv.attn_prefill_plan_run(self.plan, self.q, self.scale, self.out, self.lse, stream, self.ws, self.ws_bytes)

    def close(self) -> None:
        if self.plan is not None:
            hkv.hkv_prefill_plan_destroy(self.plan)
            self.plan = None


class MixedStepRunner:
    """One engine step that mixes decode rows with chunks of prompts being prefilled (chunked
    prefill): requests bringing one new token go through the prefix-tree decode plan, so the
    shared part of their paths is read once for all of them; requests bringing several go
    through suffix-only prefill.  Both plans are queued back to back on one stream and address
    disjoint rows of one q / out / lse, in the workload's own row order (request by request):
    each plan is told which rows are its own, so the two groups need not be contiguous."""

    def __init__(self, pool: DevicePool, workload: wl.Workload, random_q: bool = False):
        assert workload.mode == "prefill"
        f, dev = workload.forest, pool.k.device
        self.pool, self.workload = pool, workload
        ql = np.asarray(workload.q_len)
        cu = workload.cu_q()
        self.dec_req = np.nonzero(ql == 1)[0]
        self.pre_req = np.nonzero(ql > 1)[0]
        Hq = workload.num_q_heads
        tq = workload.total_q()
        self.q = _device_random_q(tq, Hq, dev) if random_q else to_device_bits(workload.q(), dev)
        self.out = torch.zeros((tq, Hq, hkv.HEAD_DIM), dtype=torch.int16, device=dev)
        self.lse = torch.zeros((tq, Hq), dtype=torch.float32, device=dev)
        self.scale = float(workload.scale)
        self.dec_plan = self.pre_plan = None
        if len(self.dec_req):
            self.dec_plan = hkv.hkv_decode_plan_create_ex(pool.handle, f.nodes, f.node_pages, f.req_leaf[self.dec_req], Hq,
                                                          q_rows=cu[self.dec_req])
            self.ws_bytes = hkv.hkv_decode_plan_workspace_bytes(self.dec_plan)
            self.ws = torch.empty(max(self.ws_bytes, 256), dtype=torch.uint8, device=dev)
        if len(self.pre_req):
            mp = max(1, f.max_pages_per_req())
            bt, kv_len, *_ = hkv.prefix_tree_flatten(f.nodes, f.node_pages, f.req_leaf[self.pre_req], mp,
                                                     f.page_size)
            self.pre_plan = hkv.hkv_prefill_plan_create_rows(pool.handle, cu[self.pre_req], ql[self.pre_req], bt, kv_len, Hq)
            self.pws_bytes = hkv.hkv_prefill_plan_workspace_bytes(self.pre_plan)     # fp8 pools only
            self.pws = torch.empty(max(self.pws_bytes, 256), dtype=torch.uint8, device=dev) if self.pws_bytes else None

    def run(self, stream=None) -> None:
        if self.dec_plan is not None:
            hkv.attn_decode_plan_run(self.dec_plan, self.q, self.scale, self.out, self.lse, self.ws, self.ws_bytes, stream)
        if self.pre_plan is not None:
            hkv.attn_prefill_plan_run(self.pre_plan, self.q, self.scale, self.out, self.lse, stream, self.pws,
                                      self.pws_bytes)

    def close(self) -> None:
        if self.dec_plan is not None:
            hkv.hkv_decode_plan_destroy(self.dec_plan)
            self.dec_plan = None
        if self.pre_plan is not None:
            hkv.hkv_prefill_plan_destroy(self.pre_plan)
            self.pre_plan = None


class WorkflowRunner:
    """Runs the prefill side of a scheduled workflow on one worker through the library: the tree of
    the workflow's prompt templates is the prefix forest, the KV pages of the previous call's path
    stay in the pool, every call allocates and writes pages only for the nodes that are new on its
    path (their token count is the call's prefill usage) and runs suffix-only prefill attention of
    those tokens against the whole path.  Everything a call needs (page ids, plan, source tensors)
    is prepared by `prepare`; `run` only queues GPU work, so that it can be timed."""

    def __init__(self, wf: wl.Workflow, num_q_heads: int = 32, num_kv_heads: int = 8, seed: int = wl.BASE_SEED + 9,
                 device: str = "cuda:0"):
        self.wf, self.Hq, self.Hkv, self.seed, self.device = wf, num_q_heads, num_kv_heads, seed, device
        self.tree = hkv.trt_build(wf.templates, wf.len_out, wf.worker)
        self.nodes = hkv.trt_nodes(self.tree)
        nd = self.nodes
        for v in range(len(nd["parent"])):
            if nd["weight"][v] % hkv.PAGE_SIZE:
                raise ValueError(f"node {v} holds {nd['weight'][v]} tokens: sharing is page-granular, every "
                                 "template segment (and output length) must be a multiple of 16 tokens")
        self.paths = []          # per call: nodes with tokens from the root down to the leaf's parent
        for c in range(wf.n_calls):
            p, v = [], int(nd["parent"][nd["leaf_of_call"][c]])
            while v > 0:
                if nd["weight"][v] > 0:
                    p.append(v)
                v = int(nd["parent"][v])
            self.paths.append(p[::-1])
        longest = max((sum(int(nd["weight"][v]) for v in p) for p in self.paths), default=16)
        self.pool = DevicePool(2 * longest // hkv.PAGE_SIZE + 8, num_kv_heads, hkv.BF16, device)
        self.scale = float(1.0 / np.sqrt(np.float32(hkv.HEAD_DIM)))
        self.steps = []
        self._kv_cache = {}

    def _node_tensors(self, v: int):
        if v not in self._kv_cache:
            n = int(self.nodes["weight"][v])
            k, vv = wl.workflow_node_kv(self.seed, v, n, self.Hkv)
            q = wl.workflow_node_q(self.seed, v, n, self.Hq)
            self._kv_cache[v] = (to_device_bits(k, self.device), to_device_bits(vv, self.device),
                                 to_device_bits(q, self.device))
        return self._kv_cache[v]

    def prepare(self, sequence, cache: bool = True) -> list:
        """Fixes page ids and builds one prefill plan per call of `sequence`.  cache = False models an
        engine without prefix reuse: every call starts from an empty pool.  Returns the calls'
        prefill usage (new tokens)."""
        self.release_steps()
        resident = {}            # node -> page ids
        usage = []
        for c in sequence:
            path = self.paths[c]
            for v in [v for v in resident if (not cache) or v not in path]:
                hkv.kv_pool_release(self.pool.handle, resident.pop(v))
            new = [v for v in path if v not in resident]
            for v in new:
                resident[v] = hkv.kv_pool_alloc(self.pool.handle, int(self.nodes["weight"][v]) // hkv.PAGE_SIZE)
            n_new = sum(int(self.nodes["weight"][v]) for v in new)
            usage.append(n_new)
            step = {"call": c, "new": new, "pages": {v: resident[v].copy() for v in new}, "n_new": n_new, "plan": None}
            if n_new:
                bt = np.concatenate([resident[v] for v in path]).astype(np.int32)
                kv_len = sum(int(self.nodes["weight"][v]) for v in path)
                # the new nodes are the tail of the path (everything below the lowest common ancestor)
                assert path[len(path) - len(new):] == new
                step["plan"] = hkv.hkv_prefill_plan_create(self.pool.handle, np.array([0, n_new], dtype=np.int32),
                                                           bt[None, :], np.array([kv_len], dtype=np.int32), self.Hq)
                step["q"] = torch.cat([self._node_tensors(v)[2] for v in new], dim=0)
                step["out"] = torch.zeros((n_new, self.Hq, hkv.HEAD_DIM), dtype=torch.int16, device=self.device)
                step["block_table"], step["kv_len"] = bt, kv_len
            self.steps.append(step)
        for v in list(resident):
            hkv.kv_pool_release(self.pool.handle, resident.pop(v))
        return usage

    def run(self, stream=None) -> None:
        for st in self.steps:
            for v in st["new"]:
                k, vv, _ = self._node_tensors(v)
                self.pool.write(st["pages"][v], 0, k, vv, stream)
            if st["plan"] is not None:
                hkv.attn_prefill_plan_run(st["plan"], st["q"], self.scale, st["out"], None, stream)

    def release_steps(self) -> None:
        for st in self.steps:
            if st["plan"] is not None:
                hkv.hkv_prefill_plan_destroy(st["plan"])
        self.steps = []

    def close(self) -> None:
        self.release_steps()
        if self.tree is not None:
            hkv.trt_destroy(self.tree)
            self.tree = None
        self.pool.close()


class PrefixCacheRunner:
    """A sequence of prompts (token ids) served one after another through the block-level prefix
    cache under a fixed page budget, as an engine with automatic prefix caching does: acquire the
    prompt's pages (hits come back filled, misses get fresh or evicted pages), write the K/V of the
    uncached tokens, run suffix-only prefill attention for them, release.  `prepare` plays the
    whole sequence through the cache on the host (page assignment is deterministic) and builds one
    plan per prompt; `run` only queues GPU work in the same order, so a page that is evicted and
    handed to a later prompt is overwritten after its last reader in stream order."""

    def __init__(self, prompts, n_pages: int, num_q_heads: int = 8, num_kv_heads: int = 2, seed: int = wl.BASE_SEED + 11,
                 device: str = "cuda:0", random_tensors: bool = False):
        self.prompts, self.Hq, self.Hkv, self.seed, self.device = prompts, num_q_heads, num_kv_heads, seed, device
        self.random_tensors = random_tensors      # timing only: K/V/q drawn on the device instead of per token
        self.pool = DevicePool(n_pages, num_kv_heads, hkv.BF16, device)
        self.cache = hkv.kv_cache_create(self.pool.handle)
        self.scale = float(1.0 / np.sqrt(np.float32(hkv.HEAD_DIM)))
        self.steps = []

    def prepare(self) -> dict:
        hit = total = 0
        for toks in self.prompts:
            n = len(toks)
            pages, cached = hkv.kv_cache_acquire(self.cache, toks)
            hkv.kv_cache_release(self.cache, pages)      # the call is over before the next one is planned
            hit += cached
            total += n
            step = {"pages": np.asarray(pages, dtype=np.int32), "cached": int(cached), "n": n, "plan": None}
            new = n - cached
            if new > 0:
                if self.random_tensors:
                    step["k"] = _device_random_q(new, self.Hkv, self.device)
                    step["v"] = _device_random_q(new, self.Hkv, self.device)
                    step["q"] = _device_random_q(new, self.Hq, self.device)
                else:
                    pos = np.arange(cached, n)
                    k, v = wl.token_kv(self.seed, toks[cached:], pos, self.Hkv)
                    step["k"], step["v"] = to_device_bits(k, self.device), to_device_bits(v, self.device)
                    step["q"] = to_device_bits(wl.token_q(self.seed, toks[cached:], pos, self.Hq), self.device)
                step["out"] = torch.zeros((new, self.Hq, hkv.HEAD_DIM), dtype=torch.int16, device=self.device)
                step["lse"] = torch.zeros((new, self.Hq), dtype=torch.float32, device=self.device)
                step["plan"] = hkv.hkv_prefill_plan_create(self.pool.handle, np.array([0, new], dtype=np.int32),
                                                           step["pages"][None, :], np.array([n], dtype=np.int32), self.Hq)
            self.steps.append(step)
        st = hkv.kv_cache_stats(self.cache)
        return {"hit_rate": hit / max(total, 1), "prompt_tokens": total, "evictions": st["evictions"]}

    def run(self, stream=None) -> None:
        for st in self.steps:
            if st["plan"] is None:
                continue
            self.pool.write(st["pages"][st["cached"] // hkv.PAGE_SIZE:], 0, st["k"], st["v"], stream)
            hkv.attn_prefill_plan_run(st["plan"], st["q"], self.scale, st["out"], st["lse"], stream)

    def close(self) -> None:
        for st in self.steps:
            if st["plan"] is not None:
                hkv.hkv_prefill_plan_destroy(st["plan"])
        self.steps = []
        if self.cache is not None:
            hkv.kv_cache_destroy(self.cache)
            self.cache = None
        self.pool.close()


def workflow_levels(wf: wl.Workflow) -> list:
    """Calls grouped by dependency depth: level 0 quotes no other call's output, level k + 1 quotes
    outputs of level <= k.  The calls of one level can decode side by side."""
    depth = []
    for tmpl in wf.templates:
        deps = [-(s + 1) for s in tmpl if s < 0]
        depth.append(1 + max((depth[d] for d in deps), default=-1))
    return [[c for c, d in enumerate(depth) if d == k] for k in range(max(depth, default=-1) + 1)]


def workflow_decode_workload(wf: wl.Workflow, calls, generated, num_q_heads: int = 32, num_kv_heads: int = 8,
                             seed: int = wl.BASE_SEED + 12) -> wl.Workload:
    """The decode step of a batch of workflow calls running side by side, as a prefix forest: the
    templated radix tree of the workflow (built by the library) restricted to the paths of `calls`,
    omega(v) tokens per node, and under each call's prompt a private node with the `generated[i]`
    tokens it has produced so far (the newest one is the query token's own)."""
    tree = hkv.trt_build(wf.templates, wf.len_out, wf.worker)
    try:
        nd = hkv.trt_nodes(tree)
    finally:
        hkv.trt_destroy(tree)
    keep = set()
    for c in calls:
        v = int(nd["leaf_of_call"][c])
        while v >= 0 and v not in keep:
            keep.add(v)
            v = int(nd["parent"][v])
    order = sorted(keep)                       # preorder numbering: parents stay first
    new_id = {v: i for i, v in enumerate(order)}
    gen = {int(nd["leaf_of_call"][c]): int(g) for c, g in zip(calls, generated)}
    parent = [new_id[int(nd["parent"][v])] if nd["parent"][v] >= 0 else -1 for v in order]
    ntok = [gen.get(v, int(nd["weight"][v])) for v in order]
    leaves = [new_id[int(nd["leaf_of_call"][c])] for c in calls]
    n_used = sum((t + 15) // 16 for t in ntok)
    num_pages = n_used + n_used // 4 + 1
    pages = np.random.default_rng([seed, 0]).permutation(num_pages).astype(np.int32)
    f = wl.make_forest(parent, ntok, leaves, pages)
    return wl.Workload(name=f"{wf.name}_decode_{len(calls)}calls", num_q_heads=num_q_heads, num_kv_heads=num_kv_heads,
                       kv_dtype=wl.KV_BF16, num_pages=num_pages, seed=seed, forest=f, mode="decode")


def workflow_prompt_tokens(wf: wl.Workflow, call: int) -> list:
    """The call's full prompt as token ids: static symbols as they are, a placeholder for call x as
    len_out[x] ids that nothing else uses (what the LLM wrote is not known; only that it is the same
    text wherever it is quoted)."""
    out = []
    for s in wf.templates[call]:
        if s >= 0:
            out.append(int(s))
        else:
            x = -(s + 1)
            out.extend(range((1 << 24) + x * 65536, (1 << 24) + x * 65536 + wf.len_out[x]))
    return out


def simulate_prefix_cache(wf: wl.Workflow, sequence, n_pages: int) -> dict:
    """Host-only: runs the calls of `sequence` one after another through the block-level prefix cache
    (acquire, then release when the call is done) over a pool of n_pages pages and reports the
    prefix-cache hit rate = cached prompt tokens / prompt tokens.  No device memory is touched."""
    pool = hkv.kv_pool_create(n_pages, 1, hkv.BF16, 0x1000, 0x2000)   # addresses are never dereferenced here
    cache = hkv.kv_cache_create(pool)
    hit = total = 0
    try:
        for c in sequence:
            toks = workflow_prompt_tokens(wf, c)
            pages, cached = hkv.kv_cache_acquire(cache, toks)
            hit += cached
            total += len(toks)
            hkv.kv_cache_release(cache, pages)
        st = hkv.kv_cache_stats(cache)
    finally:
        hkv.kv_cache_destroy(cache)
        hkv.kv_pool_destroy(pool)
    return {"hit_rate": hit / max(total, 1), "prompt_tokens": total, "evictions": st["evictions"]}
