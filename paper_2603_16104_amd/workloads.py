"""Seeded synthetic prefix-forest workloads.

This module only *draws inputs*: tree shapes, page-id permutations and N(0,1)
tensors rounded to bf16 bit patterns.  It holds none of the attention
arithmetic, none of the pool-layout indexing and no quantisation: both the
HIP path and the CPU oracle consume what it returns through their own code.

The shapes mirror the prompt structure the paper schedules (a static system
prompt at the root, a per-query context below it, a per-operator suffix at
the leaf: the templated radix tree of Section 5 and the nested sequences of
Algorithm 1) with Llama-3 / Qwen3 class grouped-query head shapes
(Section 7.1, "Models and Testbed").  No dataset item is reproduced; every
tensor is drawn from a fixed-seed generator.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

PAGE_SIZE = 16
HEAD_DIM = 128
BASE_SEED = 20260316

KV_BF16 = 0
KV_FP8_E4M3 = 1
KV_FP32 = 2

BF16_NAN_BITS = 0x7FC0
FP8_NAN_BITS = 0x7F


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even), returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to float32 exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class PrefixForest:
    """Call-level prefix forest: node v holds the tokens of its own prompt segment
    (omega(v) = n_tokens[v]); a request's sequence is the concatenation along root->leaf."""

    parent: np.ndarray       # int32 [n_nodes], -1 for a root; parents precede children
    n_tokens: np.ndarray     # int32 [n_nodes]
    page_begin: np.ndarray   # int32 [n_nodes], offset of the node's first page in node_pages
    n_pages: np.ndarray      # int32 [n_nodes] = ceil(n_tokens / page_size)
    node_pages: np.ndarray   # int32 [sum n_pages], pool page ids
    req_leaf: np.ndarray     # int32 [n_req]
    page_size: int = PAGE_SIZE   # tokens per page (16, 32, 64 or 128)

    @property
    def n_nodes(self) -> int:
        return int(self.parent.shape[0])

    @property
    def n_req(self) -> int:
        return int(self.req_leaf.shape[0])

    @property
    def nodes(self) -> np.ndarray:
        """[n_nodes][4] int32 rows (parent, page_begin, n_pages, n_tokens)."""
        return np.ascontiguousarray(
            np.stack([self.parent, self.page_begin, self.n_pages, self.n_tokens], axis=1), dtype=np.int32
        )

    def path(self, leaf: int) -> List[int]:
        out = []
        v = int(leaf)
        while v >= 0:
            out.append(v)
            v = int(self.parent[v])
        return out[::-1]

    def kv_len(self, r: int) -> int:
        return int(sum(int(self.n_tokens[v]) for v in self.path(int(self.req_leaf[r]))))

    def max_pages_per_req(self) -> int:
        m = 0
        for r in range(self.n_req):
            m = max(m, sum(int(self.n_pages[v]) for v in self.path(int(self.req_leaf[r]))))
        return m

    def unique_tokens(self) -> int:
        """Tokens stored once in the pool and reachable from some request."""
        used = np.zeros(self.n_nodes, dtype=bool)
        for r in range(self.n_req):
            for v in self.path(int(self.req_leaf[r])):
                used[v] = True
        return int(self.n_tokens[used].sum())

    def attended_tokens(self) -> int:
        return int(sum(self.kv_len(r) for r in range(self.n_req)))


def make_forest(parent: Sequence[int], n_tokens: Sequence[int], req_leaf: Sequence[int],
                page_ids: np.ndarray, page_size: int = PAGE_SIZE) -> PrefixForest:
    """Lay the nodes' pages out consecutively over the given (already permuted) pool page ids."""
    parent = np.asarray(parent, dtype=np.int32)
    n_tokens = np.asarray(n_tokens, dtype=np.int32)
    n_pages = ((n_tokens + (page_size - 1)) // page_size).astype(np.int32)
    page_begin = np.zeros_like(n_pages)
    if len(n_pages):
        page_begin[1:] = np.cumsum(n_pages)[:-1]
    total = int(n_pages.sum())
    if total > len(page_ids):
        raise ValueError(f"forest needs {total} pages, only {len(page_ids)} given")
    return PrefixForest(parent, n_tokens, page_begin.astype(np.int32), n_pages,
                        np.ascontiguousarray(page_ids[:total], dtype=np.int32),
                        np.asarray(req_leaf, dtype=np.int32), page_size)


@dataclass
class Workload:
    name: str
    num_q_heads: int
    num_kv_heads: int
    kv_dtype: int
    num_pages: int
    seed: int
    forest: PrefixForest
    mode: str                      # "decode" or "prefill"
    q_len: Optional[np.ndarray] = None   # prefill: int32 [n_req] new tokens (= leaf n_tokens)
    src_dtype: str = "bf16"        # dtype of Q and of the K/V handed to the pool writer
    notes: str = ""

    @property
    def group(self) -> int:
        return self.num_q_heads // self.num_kv_heads

    @property
    def page_size(self) -> int:
        return self.forest.page_size

    @property
    def scale(self) -> np.float32:
        return np.float32(1.0 / np.sqrt(np.float32(HEAD_DIM)))

    def _draw(self, tag: Tuple[int, ...], shape) -> np.ndarray:
        rng = np.random.default_rng([self.seed, *tag])
        x = rng.standard_normal(size=shape, dtype=np.float32)
        if self.src_dtype == "fp32":
            return x
        return f32_to_bf16_bits(x)

    def node_kv(self, node: int) -> Tuple[np.ndarray, np.ndarray]:
        """K and V of the node's own tokens, each [n_tokens][Hkv][128] (uint16 bf16 bits or float32)."""
        n = int(self.forest.n_tokens[node])
        shape = (n, self.num_kv_heads, HEAD_DIM)
        return self._draw((1, node), shape), self._draw((2, node), shape)

    def total_q(self) -> int:
        if self.mode == "decode":
            return self.forest.n_req
        return int(self.q_len.sum())

    def cu_q(self) -> np.ndarray:
        cu = np.zeros(self.forest.n_req + 1, dtype=np.int32)
        if self.mode == "decode":
            cu[1:] = np.arange(1, self.forest.n_req + 1)
        else:
            cu[1:] = np.cumsum(self.q_len)
        return cu

    def q(self) -> np.ndarray:
        """[total_q][Hq][128] query tokens."""
        return self._draw((3,), (self.total_q(), self.num_q_heads, HEAD_DIM))

    def kv_bytes_per_token(self) -> int:
        es = {KV_BF16: 2, KV_FP8_E4M3: 1, KV_FP32: 4}[self.kv_dtype]
        return 2 * self.num_kv_heads * HEAD_DIM * es

    def unique_kv_bytes(self) -> int:
        return self.forest.unique_tokens() * self.kv_bytes_per_token()

    def pair_count(self) -> int:
        """Causally visible (query token, key token) pairs, per q-head."""
        f = self.forest
        if self.mode == "decode":
            return f.attended_tokens()
        tot = 0
        for r in range(f.n_req):
            s = int(self.q_len[r])
            p = f.kv_len(r) - s
            tot += s * p + s * (s + 1) // 2
        return tot

    def useful_flop(self) -> int:
        return 4 * HEAD_DIM * self.num_q_heads * self.pair_count()


def _perm(seed: int, num_pages: int) -> np.ndarray:
    return np.random.default_rng([seed, 0]).permutation(num_pages).astype(np.int32)


def config1(seed: int = BASE_SEED + 1) -> Tuple[Workload, Workload]:
    """Tiny prefix tree: returns (prefill workload, decode workload) over the same pool pages.

    root 256 tokens -> 4 private branches of 32 -> 4 new-token segments of 16 (prefilled)
    -> 4 single decode tokens, each alone in a fresh page.
    """
    parent = [-1] + [0] * 4 + [1, 2, 3, 4] + [5, 6, 7, 8]
    ntok = [256] + [32] * 4 + [16] * 4 + [1] * 4
    pages = _perm(seed, 128)
    f_dec = make_forest(parent, ntok, [9, 10, 11, 12], pages)
    f_pre = make_forest(parent[:9], ntok[:9], [5, 6, 7, 8], pages)
    common = dict(num_q_heads=8, num_kv_heads=2, kv_dtype=KV_BF16, num_pages=128, seed=seed)
    pre = Workload(name="c1_tiny_prefill", forest=f_pre, mode="prefill",
                   q_len=np.full(4, 16, dtype=np.int32), **common)
    dec = Workload(name="c1_tiny_decode", forest=f_dec, mode="decode", **common)
    return pre, dec


def _pool_pages(n_used: int) -> int:
    return int(n_used + n_used // 4)


def config2(seed: int = BASE_SEED + 2, n_req: int = 64, root_tokens: int = 2048,
            private_tokens: int = 512) -> Workload:
    """Llama-3-8B-shaped decode: one shared system-prompt root, one private context per request."""
    parent = [-1] + [0] * n_req
    ntok = [root_tokens] + [private_tokens] * n_req
    n_used = sum((t + 15) // 16 for t in ntok)
    num_pages = _pool_pages(n_used)
    f = make_forest(parent, ntok, list(range(1, n_req + 1)), _perm(seed, num_pages))
    return Workload(name="c2_llama8b_decode", num_q_heads=32, num_kv_heads=8, kv_dtype=KV_BF16,
                    num_pages=num_pages, seed=seed, forest=f, mode="decode")


def config3(seed: int = BASE_SEED + 3, root_tokens: int = 4096, child_tokens: int = 1024,
            leaf_tokens: int = 256) -> Workload:
    """Speculative fan-out tree: 4096 -> 8 x 1024 -> 128 x 256."""
    parent = [-1] + [0] * 8
    ntok = [root_tokens] + [child_tokens] * 8
    leaves = []
    for c in range(8):
        for _ in range(16):
            parent.append(1 + c)
            ntok.append(leaf_tokens)
            leaves.append(len(parent) - 1)
    n_used = sum((t + 15) // 16 for t in ntok)
    num_pages = _pool_pages(n_used)
    f = make_forest(parent, ntok, leaves, _perm(seed, num_pages))
    return Workload(name="c3_fanout_decode", num_q_heads=32, num_kv_heads=8, kv_dtype=KV_BF16,
                    num_pages=num_pages, seed=seed, forest=f, mode="decode")


def config4(seed: int = BASE_SEED + 4, n_req: int = 32, prefix_tokens: int = 8192,
            lo: int = 768, hi: int = 1024) -> Workload:
    """Prefix-hit prefill: every request prefills s_r ~ U{lo..hi} new tokens over a shared cached prefix."""
    s = np.random.default_rng([seed, 7]).integers(lo, hi + 1, size=n_req).astype(np.int32)
    parent = [-1] + [0] * n_req
    ntok = [prefix_tokens] + [int(x) for x in s]
    n_used = sum((t + 15) // 16 for t in ntok)
    num_pages = _pool_pages(n_used)
    f = make_forest(parent, ntok, list(range(1, n_req + 1)), _perm(seed, num_pages))
    return Workload(name="c4_prefix_hit_prefill", num_q_heads=32, num_kv_heads=8, kv_dtype=KV_BF16,
                    num_pages=num_pages, seed=seed, forest=f, mode="prefill", q_len=s)


def config5(seed: int = BASE_SEED + 5, n_roots: int = 16, children: int = 32,
            root_tokens: int = 8192, child_tokens: int = 2048) -> Workload:
    """Large forest, 70B-shaped layer, KV stored as fp8 e4m3 with per-page per-head scales."""
    parent, ntok, leaves = [], [], []
    for _ in range(n_roots):
        parent.append(-1)
        ntok.append(root_tokens)
    for r in range(n_roots):
        for _ in range(children):
            parent.append(r)
            ntok.append(child_tokens)
            leaves.append(len(parent) - 1)
    n_used = sum((t + 15) // 16 for t in ntok)
    num_pages = _pool_pages(n_used)
    f = make_forest(parent, ntok, leaves, _perm(seed, num_pages))
    return Workload(name="c5_forest_fp8_decode", num_q_heads=64, num_kv_heads=8, kv_dtype=KV_FP8_E4M3,
                    num_pages=num_pages, seed=seed, forest=f, mode="decode")


# (query heads, KV heads) of one layer of the model families the evaluation names (Section 7,
# "Sensitivity Analysis": Llama-3.1-8B, Qwen3-8B/14B/32B); head_dim is 128 for all of them.
MODEL_HEADS = {"llama3-8b": (32, 8), "qwen3-8b": (32, 8), "qwen3-14b": (40, 8), "qwen3-32b": (64, 8)}

# (system, context, question, output) token lengths.  The prefix-sharing sensitivity study (Section 7)
# varies exactly these four; its six settings are only in a figure, so this grid is our own choice:
# from almost nothing shared to almost everything shared.
SENSITIVITY_GRID = {
    "P1": (256, 0, 256, 128),
    "P2": (2048, 0, 256, 128),
    "P3": (256, 2048, 128, 128),
    "P4": (2048, 2048, 128, 128),
    "P5": (1024, 8192, 64, 256),
    "P6": (4096, 4096, 512, 512),
}


def prefix_sensitivity(system: int, context: int, question: int, output: int, *, model: str = "qwen3-14b",
                       n_contexts: int = 10, questions_per_context: int = 10, mode: str = "decode",
                       kv_dtype: int = KV_BF16, seed: int = BASE_SEED + 6) -> Workload:
    """Fixed system prompt -> one shared context per group of queries -> one question per query
    (100 queries by default, as in the study).  Shared segments are rounded up to whole pages.
    decode: every query has produced half of its `output` tokens; its leaf holds question + those.
    prefill: the system prompt and the contexts are cached, every query prefills its question."""
    up = lambda t: (t + PAGE_SIZE - 1) // PAGE_SIZE * PAGE_SIZE
    hq, hk = MODEL_HEADS[model]
    leaf_tokens = question + (output // 2 if mode == "decode" else 0)
    parent, ntok, leaves = [-1], [up(system)], []
    for _ in range(n_contexts):
        ctx = 0
        if context > 0:
            parent.append(0)
            ntok.append(up(context))
            ctx = len(parent) - 1
        for _ in range(questions_per_context):
            parent.append(ctx)
            ntok.append(leaf_tokens)
            leaves.append(len(parent) - 1)
    n_used = sum((t + 15) // 16 for t in ntok)
    num_pages = _pool_pages(n_used)
    f = make_forest(parent, ntok, leaves, _perm(seed, num_pages))
    q_len = np.full(len(leaves), question, dtype=np.int32) if mode == "prefill" else None
    return Workload(name=f"sens_{model}_{system}_{context}_{question}_{output}_{mode}", num_q_heads=hq,
                    num_kv_heads=hk, kv_dtype=kv_dtype, num_pages=num_pages, seed=seed, forest=f, mode=mode,
                    q_len=q_len)


def mixed_step(n_decode: int = 64, n_prefill: int = 8, root_tokens: int = 2048, private_tokens: int = 512,
               chunk_tokens: int = 512, model: str = "llama3-8b", seed: int = BASE_SEED + 7) -> Workload:
    """One step of an engine with chunked prefill: n_decode requests that bring one new token (context
    = shared root + private_tokens, the new token is the last of them) next to n_prefill requests that
    prefill a chunk of chunk_tokens new tokens right behind the shared root."""
    hq, hk = MODEL_HEADS[model]
    parent = [-1] + [0] * (n_decode + n_prefill)
    ntok = [root_tokens] + [private_tokens] * n_decode + [chunk_tokens] * n_prefill
    q_len = np.asarray([1] * n_decode + [chunk_tokens] * n_prefill, dtype=np.int32)
    n_used = sum((t + 15) // 16 for t in ntok)
    num_pages = _pool_pages(n_used)
    f = make_forest(parent, ntok, list(range(1, n_decode + n_prefill + 1)), _perm(seed, num_pages))
    return Workload(name=f"mixed_{n_decode}dec_{n_prefill}x{chunk_tokens}pre", num_q_heads=hq, num_kv_heads=hk,
                    kv_dtype=KV_BF16, num_pages=num_pages, seed=seed, forest=f, mode="prefill", q_len=q_len)


def without_sharing(w: Workload) -> Workload:
    """The same requests with nothing shared: every request owns a private copy of its whole path
    (one root node per request).  decode: each request still has one query token; prefill: each
    request prefills its whole prompt (no cached prefix).  What a paged engine without prefix reuse
    would hold and read."""
    f = w.forest
    total = [int(sum(f.n_tokens[v] for v in f.path(int(leaf)))) for leaf in f.req_leaf]
    n_used = sum((t + 15) // 16 for t in total)
    num_pages = _pool_pages(n_used)
    flat = make_forest([-1] * len(total), total, list(range(len(total))), _perm(w.seed, num_pages))
    q_len = np.asarray(total, dtype=np.int32) if w.mode == "prefill" else None
    return Workload(name=w.name + "_unshared", num_q_heads=w.num_q_heads, num_kv_heads=w.num_kv_heads,
                    kv_dtype=w.kv_dtype, num_pages=num_pages, seed=w.seed, forest=flat, mode=w.mode, q_len=q_len,
                    src_dtype=w.src_dtype)


def random_forest_workload(seed: int, *, n_roots: int = 2, depth: int = 3, fanout: int = 3,
                           max_node_pages: int = 5, num_q_heads: int = 8, num_kv_heads: int = 2,
                           kv_dtype: int = KV_BF16, mode: str = "decode", ragged: bool = True,
                           zero_weight_nodes: bool = True, src_dtype: str = "bf16",
                           extra_pages: int = 7, ragged_internal: bool = False,
                           page_size: int = PAGE_SIZE) -> Workload:
    """Small random forest for tests: internal nodes are page aligned (unless ragged_internal: then they
    may end inside a page, which only the tree decode accepts), leaves may be ragged, and (as in the
    paper's tree, where the root and the leaves carry no tokens) some nodes are empty."""
    rng = np.random.default_rng([seed, 11])
    parent: List[int] = []
    ntok: List[int] = []
    leaves: List[int] = []

    def grow(par: int, level: int) -> None:
        idx = len(parent)
        parent.append(par)
        is_leaf = level == depth - 1 or (level > 0 and rng.random() < 0.25)
        if is_leaf:
            if zero_weight_nodes and rng.random() < 0.15:
                t = 0
            elif ragged:
                t = int(rng.integers(1, max_node_pages * page_size + 1))
            else:
                t = int(rng.integers(1, max_node_pages + 1)) * page_size
            ntok.append(t)
            leaves.append(idx)
            return
        if zero_weight_nodes and rng.random() < 0.2:
            ntok.append(0)
        elif ragged_internal:
            ntok.append(int(rng.integers(1, max_node_pages * page_size + 1)))
        else:
            ntok.append(int(rng.integers(1, max_node_pages + 1)) * page_size)
        for _ in range(int(rng.integers(1, fanout + 1))):
            grow(idx, level + 1)

    # Nodes must be parent-first: grow() appends a node before its children.
    for _ in range(n_roots):
        grow(-1, 0)
    # Some requests may stop at an internal (page-aligned) node as well.
    req_leaf = list(leaves)
    internal = [v for v in range(len(parent)) if v not in set(leaves)]
    for v in internal:
        if rng.random() < 0.3:
            req_leaf.append(v)
    order = rng.permutation(len(req_leaf))
    req_leaf = [req_leaf[i] for i in order]
    n_used = sum((t + page_size - 1) // page_size for t in ntok)
    num_pages = n_used + extra_pages
    f = make_forest(parent, ntok, req_leaf, _perm(seed, num_pages), page_size)
    q_len = None
    if mode == "prefill":
        # new tokens = the request's last node; everything above it is the cached prefix
        q_len = np.asarray([ntok[v] for v in req_leaf], dtype=np.int32)
    return Workload(name=f"random_{seed}", num_q_heads=num_q_heads, num_kv_heads=num_kv_heads,
                    kv_dtype=kv_dtype, num_pages=num_pages, seed=seed, forest=f, mode=mode,
                    q_len=q_len, src_dtype=src_dtype)


def all_configs():
    c1p, c1d = config1()
    return {"c1_prefill": c1p, "c1_decode": c1d, "c2": config2(), "c3": config3(),
            "c4": config4(), "c5": config5()}


# ---------------------------------------------------------------------------------------------
# Workflow shapes for the scheduling layer: lists of LLM calls with prefix templates.
# A template is a list of int symbols: s >= 0 static token id, s < 0 the output of call -(s+1).
# Only the structure of the paper's primitive workflows is used (Section 7, "Workloads": map-reduce,
# multi-agent debate, reflection, iterative refinement, parallel chains); token ids and lengths are synthetic.


class Workflow:
    def __init__(self, name: str):
        self.name = name
        self.templates: List[List[int]] = []
        self.len_out: List[int] = []
        self.worker: List[int] = []
        self._next_token = 0

    def fresh_tokens(self, n: int) -> List[int]:
        """n static token ids that occur nowhere else (so that only intended prefixes are shared)."""
        t = list(range(self._next_token, self._next_token + n))
        self._next_token += n
        return t

    def add(self, template: List[int], len_out: int, worker: int = 0) -> int:
        self.templates.append(list(template))
        self.len_out.append(int(len_out))
        self.worker.append(int(worker))
        return len(self.templates) - 1

    @staticmethod
    def out(call: int) -> int:
        return -(call + 1)

    @property
    def n_calls(self) -> int:
        return len(self.templates)


def workflow_map_reduce(n_queries: int = 4, n_mappers: int = 3, sys_len: int = 64, ctx_len: int = 128,
                        len_out: int = 32, n_workers: int = 1) -> Workflow:
    """Per query: n_mappers calls [mapper system prompt | query context], one reducer
    [reducer system prompt | query context | all mapper outputs]."""
    w = Workflow("map_reduce")
    map_sys = [w.fresh_tokens(sys_len) for _ in range(n_mappers)]
    red_sys = w.fresh_tokens(sys_len)
    for q in range(n_queries):
        ctx = w.fresh_tokens(ctx_len)
        wk = q % n_workers
        ms = [w.add(map_sys[m] + ctx, len_out, wk) for m in range(n_mappers)]
        w.add(red_sys + ctx + [Workflow.out(m) for m in ms], len_out, wk)
    return w


def workflow_debate(n_queries: int = 3, n_agents: int = 3, rounds: int = 2, sys_len: int = 64, q_len: int = 48,
                    len_out: int = 32, n_workers: int = 1) -> Workflow:
    """Round 1: every agent answers [agent system prompt | question]; every later round appends the
    answers of all agents in all earlier rounds."""
    w = Workflow("debate")
    sys_p = [w.fresh_tokens(sys_len) for _ in range(n_agents)]
    for q in range(n_queries):
        question = w.fresh_tokens(q_len)
        wk = q % n_workers
        history: List[int] = []               # answers of all earlier rounds, in order
        for _ in range(rounds):
            cur = [w.add(sys_p[a] + question + [Workflow.out(c) for c in history], len_out, wk)
                   for a in range(n_agents)]
            history = history + cur
    return w


def workflow_reflect(n_queries: int = 4, sys_len: int = 64, q_len: int = 48, len_out: int = 32,
                     n_workers: int = 1) -> Workflow:
    """answer -> critique of the answer -> revised answer, per query; the three roles have their own
    system prompts."""
    w = Workflow("reflect")
    s_ans, s_crit, s_rev = (w.fresh_tokens(sys_len) for _ in range(3))
    for q in range(n_queries):
        question = w.fresh_tokens(q_len)
        wk = q % n_workers
        a = w.add(s_ans + question, len_out, wk)
        c = w.add(s_crit + question + [Workflow.out(a)], len_out, wk)
        w.add(s_rev + question + [Workflow.out(a), Workflow.out(c)], len_out, wk)
    return w


def workflow_iterative(n_queries: int = 4, n_chunks: int = 6, sys_len: int = 64, chunk_len: int = 96, len_out: int = 32,
                       n_workers: int = 1) -> Workflow:
    """Iterative refinement: per input item its chunks are summarised one after the other by one summariser,
    [system prompt | chunk j | summary so far] (the first call has no summary yet)."""
    w = Workflow("iterative")
    sys_first, sys_refine = w.fresh_tokens(sys_len), w.fresh_tokens(sys_len)
    for q in range(n_queries):
        wk = q % n_workers
        prev = -1
        for j in range(n_chunks):
            chunk = w.fresh_tokens(chunk_len)
            prev = w.add((sys_first if j == 0 else sys_refine) + chunk + ([Workflow.out(prev)] if j else []), len_out, wk)
    return w


def workflow_parallel(n_queries: int = 3, n_experts: int = 7, n_chunks: int = 6, sys_len: int = 64, chunk_len: int = 96,
                      len_out: int = 32, n_workers: int = 1) -> Workflow:
    """Parallel chains: per input item every expert reads every chunk, [expert system prompt | chunk]; a
    writer aggregates all insights, [writer system prompt | all expert outputs]."""
    w = Workflow("parallel")
    exp_sys = [w.fresh_tokens(sys_len) for _ in range(n_experts)]
    writer_sys = w.fresh_tokens(sys_len)
    for q in range(n_queries):
        wk = q % n_workers
        chunks = [w.fresh_tokens(chunk_len) for _ in range(n_chunks)]
        insights = [w.add(exp_sys[e] + chunks[k], len_out, wk) for e in range(n_experts) for k in range(n_chunks)]
        w.add(writer_sys + [Workflow.out(c) for c in insights], len_out, wk)
    return w


def random_workflow(seed: int, n_calls: int = 12, vocab: int = 6, max_len: int = 10, max_out: int = 9,
                    n_workers: int = 1, p_placeholder: float = 0.2) -> Workflow:
    """Small random templates over a tiny vocabulary (many accidental shared prefixes, splits at every
    depth), placeholders only to earlier calls (acyclic by construction, then shuffled)."""
    rng = np.random.default_rng([seed, 13])
    w = Workflow(f"random_{seed}")
    perm = rng.permutation(n_calls)           # call i of the build order gets index perm[i]
    tmpl = [None] * n_calls
    for i in range(n_calls):
        t = []
        for _ in range(int(rng.integers(0, max_len + 1))):
            if i > 0 and rng.random() < p_placeholder:
                t.append(-(int(perm[int(rng.integers(0, i))]) + 1))
            else:
                t.append(int(rng.integers(0, vocab)))
        tmpl[int(perm[i])] = t
    for i in range(n_calls):
        w.add(tmpl[i], int(rng.integers(0, max_out + 1)), int(rng.integers(0, n_workers)))
    return w


def workflow_node_kv(seed: int, node: int, n_tokens: int, num_kv_heads: int) -> Tuple[np.ndarray, np.ndarray]:
    """K and V (bf16 bits, [n_tokens][Hkv][128]) of the tokens of one tree node of a workflow: the same
    node always yields the same bits, whichever call brings it into the cache."""
    shape = (n_tokens, num_kv_heads, HEAD_DIM)
    k = np.random.default_rng([seed, 21, node]).standard_normal(size=shape, dtype=np.float32)
    v = np.random.default_rng([seed, 22, node]).standard_normal(size=shape, dtype=np.float32)
    return f32_to_bf16_bits(k), f32_to_bf16_bits(v)


def workflow_node_q(seed: int, node: int, n_tokens: int, num_q_heads: int) -> np.ndarray:
    """Query rows (bf16 bits, [n_tokens][Hq][128]) of the tokens of one tree node."""
    x = np.random.default_rng([seed, 23, node]).standard_normal(size=(n_tokens, num_q_heads, HEAD_DIM), dtype=np.float32)
    return f32_to_bf16_bits(x)


# ---- token-level synthetic tensors (for engines that cache by token prefix)

def _hash_normal(seed: int, tag: int, token_ids, positions, heads: int) -> np.ndarray:
    """[n][heads][128] float32, approximately standard normal, a pure function of (seed, tag, token id,
    position, head, dim): a counter-based generator (64-bit mix of the coordinates, sum of four
    24-bit uniforms), so that equal (token, position) pairs give equal values in whatever call or
    order they are asked for."""
    ids = np.asarray(token_ids, dtype=np.uint64)[:, None, None]
    pos = np.asarray(positions, dtype=np.uint64)[:, None, None]
    h = np.arange(heads, dtype=np.uint64)[None, :, None]
    d = np.arange(HEAD_DIM, dtype=np.uint64)[None, None, :]
    with np.errstate(over="ignore"):
        x = (ids * np.uint64(0x9E3779B97F4A7C15) + pos * np.uint64(0xC2B2AE3D27D4EB4F) + h * np.uint64(0x165667B19E3779F9) +
             d * np.uint64(0xD6E8FEB86659FD93) + np.uint64(seed) * np.uint64(0xA0761D6478BD642F) + np.uint64(tag))
        acc = np.zeros(x.shape, dtype=np.float64)
        for r in range(4):
            x = x + np.uint64(0x9E3779B97F4A7C15)
            z = x
            z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
            z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
            z = z ^ (z >> np.uint64(31))
            acc += (z >> np.uint64(40)).astype(np.float64) * (1.0 / (1 << 24))
    return ((acc - 2.0) * np.sqrt(3.0)).astype(np.float32)


def token_kv(seed: int, token_ids, positions, num_kv_heads: int) -> Tuple[np.ndarray, np.ndarray]:
    """K and V (bf16 bits, [n][Hkv][128]) of tokens given by (id, position in their prompt)."""
    return (f32_to_bf16_bits(_hash_normal(seed, 1, token_ids, positions, num_kv_heads)),
            f32_to_bf16_bits(_hash_normal(seed, 2, token_ids, positions, num_kv_heads)))


def token_q(seed: int, token_ids, positions, num_q_heads: int) -> np.ndarray:
    """Query rows (bf16 bits, [n][Hq][128]) of the same tokens."""
    return f32_to_bf16_bits(_hash_normal(seed, 3, token_ids, positions, num_q_heads))


def shared_prefix_prompts(seed: int, n_prompts: int = 12, n_systems: int = 2, n_contexts: int = 3,
                          system_len: int = 48, context_len: int = 40, question_lo: int = 5,
                          question_hi: int = 60) -> List[List[int]]:
    """Token-id prompts with the structure of the evaluated workflows (system prompt, shared context,
    private question), lengths deliberately not page-aligned, in an order that revisits prefixes."""
    rng = np.random.default_rng([seed, 31])
    systems = [list(rng.integers(0, 30000, size=system_len + int(rng.integers(0, 9)))) for _ in range(n_systems)]
    contexts = [list(rng.integers(0, 30000, size=context_len + int(rng.integers(0, 17)))) for _ in range(n_contexts)]
    prompts = []
    for _ in range(n_prompts):
        sy = systems[int(rng.integers(0, n_systems))]
        cx = contexts[int(rng.integers(0, n_contexts))]
        qu = list(rng.integers(0, 30000, size=int(rng.integers(question_lo, question_hi + 1))))
        prompts.append([int(t) for t in sy + cx + qu])
    return prompts
