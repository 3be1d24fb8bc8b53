"""CPU-only tests of the C-ABI library: it loads, exports what the header declares, and its host
logic (pool bookkeeping, forest flattening, token usage, work planning, argument validation) is
right.  Integer outputs are compared bit-exactly with the oracle.  No kernel is launched."""
import os
import re

import numpy as np
import pytest

from paper_2603_16104_amd import binding as hkv
from paper_2603_16104_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE_K, FAKE_V = 0x10000, 0x20000     # never dereferenced on the host


@pytest.fixture(scope="module", autouse=True)
def built():
    if not os.path.exists(hkv.LIB_PATH):
        from paper_2603_16104_amd import build
        build.build(force=True)
    hkv.lib()


def fake_pool(num_pages=64, num_kv_heads=2, dtype=hkv.BF16, **kw):
    scales = dict(k_scale=0x30000, v_scale=0x40000) if dtype == hkv.FP8_E4M3 else {}
    return hkv.kv_pool_create(num_pages, num_kv_heads, dtype, FAKE_K, FAKE_V, **scales, **kw)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "heliumkv.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b([a-z_0-9]+)\s*\(", header)) - {"defined", "sizeof"}
    declared = {d for d in declared if d.startswith(("kv_pool", "hkv_", "prefix_tree", "attn_", "lse_merge", "trt_", "kv_cache"))}
    assert len(declared) >= 30
    L = hkv.lib()
    for name in sorted(declared):
        assert hasattr(L, name), f"{name} is declared in heliumkv.h but not exported"
    assert declared == set(hkv.EXPORTS), declared ^ set(hkv.EXPORTS)


# ------------------------------------------------------------------------------ pool bookkeeping

def test_pool_create_validation():
    with pytest.raises(hkv.HkvError) as e:
        hkv.kv_pool_create(8, 2, hkv.BF16, FAKE_K, FAKE_V, page_size=48)
    assert e.value.code == hkv.ESHAPE
    for ps in (16, 32, 64, 128):
        pool = hkv.kv_pool_create(8, 2, hkv.BF16, FAKE_K, FAKE_V, page_size=ps)
        assert hkv.kv_pool_page_size(pool) == ps
        hkv.kv_pool_destroy(pool)
    with pytest.raises(hkv.HkvError) as e:
        hkv.kv_pool_create(8, 2, hkv.BF16, FAKE_K, FAKE_V, head_dim=64)
    assert e.value.code == hkv.ESHAPE
    with pytest.raises(hkv.HkvError) as e:
        hkv.kv_pool_create(8, 2, hkv.FP8_E4M3, FAKE_K, FAKE_V)          # scales missing
    assert e.value.code == hkv.ESHAPE
    with pytest.raises(hkv.HkvError) as e:
        hkv.kv_pool_create(8, 2, 7, FAKE_K, FAKE_V)                    # unknown dtype
    assert e.value.code == hkv.ESHAPE
    hkv.kv_pool_destroy(hkv.kv_pool_create(8, 2, hkv.FP32, FAKE_K, FAKE_V))
    with pytest.raises(hkv.HkvError) as e:
        hkv.kv_pool_create(8, 2, hkv.BF16, None, FAKE_V)
    assert e.value.code == hkv.EINVAL
    with pytest.raises(hkv.HkvError) as e:
        hkv.kv_pool_create(4, 2, hkv.BF16, FAKE_K, FAKE_V, free_order=[0, 1, 1, 3])
    assert e.value.code == hkv.EINVAL
    assert "permutation" in str(e.value)
    hkv.kv_pool_destroy(fake_pool())


def test_pool_alloc_retain_release_matches_model():
    rng = np.random.default_rng(0)
    n = 40
    order = rng.permutation(n).astype(np.int32)
    pool = fake_pool(n, free_order=order)
    free = list(order)
    ref = [0] * n
    held = []
    for step in range(300):
        op = rng.integers(0, 3)
        if op == 0:
            k = int(rng.integers(0, 6))
            if k > len(free):
                with pytest.raises(hkv.HkvError) as e:
                    hkv.kv_pool_alloc(pool, k)
                assert e.value.code == hkv.ENOMEM
                continue
            got = hkv.kv_pool_alloc(pool, k)
            exp = [free.pop(0) for _ in range(k)]
            assert list(got) == exp                     # deterministic, bit-exact page ids
            for p in exp:
                ref[p] = 1
            held += exp
        elif op == 1 and held:
            ids = list(rng.choice(held, size=min(3, len(held)), replace=False))
            hkv.kv_pool_retain(pool, ids)
            for p in ids:
                ref[p] += 1
            held += ids
        elif op == 2 and held:
            k = int(rng.integers(1, min(4, len(held)) + 1))
            idx = sorted(rng.choice(len(held), size=k, replace=False), reverse=True)
            ids = [held.pop(i) for i in idx]
            hkv.kv_pool_release(pool, ids)
            for p in ids:
                ref[p] -= 1
                if ref[p] == 0:
                    free.append(p)
        assert hkv.kv_pool_num_free(pool) == len(free)
    for p in range(n):
        assert hkv.kv_pool_refcount(pool, p) == ref[p]
    with pytest.raises(hkv.HkvError) as e:
        hkv.kv_pool_retain(pool, [n])
    assert e.value.code == hkv.ERANGE
    if free:
        with pytest.raises(hkv.HkvError) as e:
            hkv.kv_pool_release(pool, [int(free[0])])
        assert e.value.code == hkv.EINVAL
    hkv.kv_pool_destroy(pool)


def test_pool_copy_on_write_host_side():
    """Without a device only the cases that queue no copy can run: sole holders keep their pages; every
    error leaves the pool as it was."""
    pool = fake_pool(4)
    a = hkv.kv_pool_alloc(pool, 3)
    assert list(hkv.kv_pool_copy_on_write(pool, a, stream=0)) == list(a)       # single references: in place
    assert [hkv.kv_pool_refcount(pool, int(p)) for p in a] == [1, 1, 1] and hkv.kv_pool_num_free(pool) == 1
    hkv.kv_pool_retain(pool, a[:2])                                           # two shared pages, one free page
    for ids, code in (([int(a[0]), int(a[0])], hkv.EINVAL), ([3], hkv.EINVAL), ([4], hkv.ERANGE),
                      ([int(a[0]), int(a[1])], hkv.ENOMEM)):
        with pytest.raises(hkv.HkvError) as e:
            hkv.kv_pool_copy_on_write(pool, ids, stream=0)
        assert e.value.code == code, ids
        assert [hkv.kv_pool_refcount(pool, p) for p in range(4)] == [2, 2, 1, 0] and hkv.kv_pool_num_free(pool) == 1
    hkv.kv_pool_destroy(pool)


def test_pool_write_validates_before_touching_the_device():
    pool = fake_pool(8)
    for args, code in (((np.array([9], dtype=np.int32), 0, 4), hkv.ERANGE),
                       ((np.array([-1], dtype=np.int32), 0, 4), hkv.ERANGE),
                       ((np.array([1], dtype=np.int32), 16, 4), hkv.EINVAL),
                       ((np.array([1], dtype=np.int32), 0, -1), hkv.EINVAL)):
        with pytest.raises(hkv.HkvError) as e:
            hkv.kv_pool_write(pool, args[0], args[1], args[2], 0x50000, 0x60000, stream=0)
        assert e.value.code == code
    with pytest.raises(hkv.HkvError) as e:                                              # more than 65536 pages in one call
        hkv.kv_pool_write(pool, np.zeros(65537, dtype=np.int32), 1, 65536 * 16, 0x50000, 0x60000, stream=0)
    assert e.value.code == hkv.EINVAL and "65537 pages" in str(e.value)
    hkv.kv_pool_write(pool, np.zeros(0, dtype=np.int32), 0, 0, None, None, stream=0)    # empty write is a no-op
    p8 = fake_pool(8, dtype=hkv.FP8_E4M3)          # fp8 pages may be continued at any slot: same checks apply
    with pytest.raises(hkv.HkvError) as e:
        hkv.kv_pool_write(p8, np.array([8], dtype=np.int32), 3, 4, 0x50000, 0x60000, stream=0)
    assert e.value.code == hkv.ERANGE
    hkv.kv_pool_destroy(pool)
    hkv.kv_pool_destroy(p8)


# ------------------------------------------------------------------------------ forest indexing (bit-exact vs oracle)

def _all_forests():
    out = [wl.random_forest_workload(s, depth=4, fanout=3, n_roots=3).forest for s in range(100, 112)]
    c1p, c1d = wl.config1()
    out += [c1p.forest, c1d.forest, wl.config2().forest, wl.config3().forest, wl.config4().forest,
            wl.config5().forest]
    return out


def test_flatten_bit_exact_against_oracle(oracle):
    for f in _all_forests():
        mp = max(1, f.max_pages_per_req()) + 1
        got = hkv.prefix_tree_flatten(f.nodes, f.node_pages, f.req_leaf, mp)
        exp = oracle.flatten_tree(f.nodes, f.node_pages, f.req_leaf, mp)
        for g, e, name in zip(got, exp, ("block_table", "kv_len", "node_req_indptr", "node_req_idx", "node_tok_start")):
            assert np.array_equal(g, e), name


def test_flatten_error_codes():
    pages = np.arange(8, dtype=np.int32)
    ok = np.array([[-1, 0, 1, 16], [0, 1, 1, 5]], dtype=np.int32)
    hkv.prefix_tree_flatten(ok, pages, [1], 4)
    cases = [(np.array([[0, 0, 1, 16]], dtype=np.int32), [0], 4, hkv.ETREE),
             (np.array([[-1, 0, 1, 12], [0, 1, 1, 5]], dtype=np.int32), [1], 4, hkv.ETREE),
             (np.array([[-1, 0, 2, 16]], dtype=np.int32), [0], 4, hkv.ETREE),
             (np.array([[-1, 7, 2, 32]], dtype=np.int32), [0], 4, hkv.ERANGE),
             (ok, [2], 4, hkv.ERANGE),
             (ok, [1], 1, hkv.ENOMEM)]
    for nodes, leaves, mp, code in cases:
        with pytest.raises(hkv.HkvError) as e:
            hkv.prefix_tree_flatten(nodes, pages, leaves, mp)
        assert e.value.code == code, (nodes, code, str(e.value))


def test_prefill_usage_bit_exact_against_oracle(oracle):
    rng = np.random.default_rng(1)
    for f in _all_forests()[:14]:
        calls = rng.integers(0, f.n_nodes, size=25).astype(np.int32)
        assert np.array_equal(hkv.prefix_tree_prefill_usage(f.nodes, calls), oracle.prefill_usage(f.nodes, calls))
    pre, _ = wl.config1()
    assert list(hkv.prefix_tree_prefill_usage(pre.forest.nodes, [5, 6, 7, 8])) == [304, 48, 48, 48]


# ------------------------------------------------------------------------------ decode planning

def _check_decode_plan(w, oracle):
    f = w.forest
    pool = fake_pool(w.num_pages, w.num_kv_heads, w.kv_dtype)
    plan = hkv.hkv_decode_plan_create(pool, f.nodes, f.node_pages, f.req_leaf, w.num_q_heads, hkv.PLAN_HOST_ONLY)
    items = hkv.hkv_decode_plan_items(plan)
    G = w.group
    _, kv_len, indptr, idx, tok_start = oracle.flatten_tree(f.nodes, f.node_pages, f.req_leaf,
                                                            max(1, f.max_pages_per_req()))
    max_parts = hkv.hkv_decode_plan_max_parts(plan)
    counts = hkv.hkv_decode_plan_part_counts(plan, f.n_req)
    assert hkv.hkv_decode_plan_num_parts(plan) == f.n_req * w.num_q_heads * max_parts
    assert hkv.hkv_decode_plan_workspace_bytes(plan) >= hkv.hkv_decode_plan_num_parts(plan) * 264
    covered = [np.zeros((w.num_kv_heads, int(kv_len[r])), dtype=np.int32) for r in range(f.n_req)]
    slots = [np.zeros((w.num_kv_heads, max_parts), dtype=np.int32) for _ in range(f.n_req)]
    n_tile = hkv.hkv_decode_plan_num_tile_items(plan)          # the last n_tile items belong to the 256-row tile kernel
    n_rows_items = len(items) - n_tile
    for i, (page_off, n_tok, kv_head, req_off, n_req, slot, tok_begin, node) in enumerate(items):
        assert 1 <= n_tok and tok_begin % 16 == 0 and tok_begin + n_tok <= f.n_tokens[node]
        assert page_off == f.page_begin[node] + tok_begin // 16
        if i >= n_rows_items:
            assert 128 <= (indptr[node + 1] - indptr[node]) * G and 1 <= n_req <= max(1, 256 // G) and n_tok <= 8192
        else:
            assert 1 <= n_req and n_req * G <= 64
            if n_req * G > 16:
                assert n_tok <= 2048                       # what the LDS-staged path can index
        assert indptr[node] <= req_off and req_off + n_req <= indptr[node + 1]
        if tok_begin + n_tok < f.n_tokens[node]:
            assert n_tok % 16 == 0                     # only a node's last chunk may end inside a page
        for r in idx[req_off: req_off + n_req]:
            a = tok_start[node] + tok_begin
            covered[r][kv_head, a: a + n_tok] += 1
            slots[r][kv_head, slot] += 1
    assert (items[:, 2] == np.arange(len(items)) % w.num_kv_heads).all(), "item index mod Hkv is the KV head"
    assert (n_tile == 0) == (hkv.hkv_decode_plan_tile_workgroups(plan) == 0)
    assert hkv.hkv_decode_plan_tile_workgroups(plan) <= min(n_tile, 256)
    # forests with more items than the 768 resident workgroups: the short items of at most 16 rows come last
    # and share a workgroup four at a time
    rows_items = items[:n_rows_items]
    limit = 768 if w.kv_dtype == wl.KV_FP8_E4M3 else 384
    short = ((rows_items[:, 4] * G <= 16) & (rows_items[:, 1] <= limit) if n_rows_items > 768
             else np.zeros(n_rows_items, dtype=bool))
    n_single = int((~short).sum())
    assert not short[:n_single].any() and short[n_single:].all()
    assert hkv.hkv_decode_plan_num_workgroups(plan) == n_single + (n_rows_items - n_single + 3) // 4
    for r in range(f.n_req):
        assert (covered[r] == 1).all(), "every (request, kv head, token) is read by exactly one item"
        assert (slots[r][:, :counts[r]] == 1).all() and (slots[r][:, counts[r]:] == 0).all()
    hkv.hkv_decode_plan_destroy(plan)
    hkv.kv_pool_destroy(pool)
    return items


def test_decode_plan_covers_every_token_once(oracle):
    for seed in range(120, 128):
        hq, hk = [(8, 2), (8, 1), (4, 4), (16, 1)][seed % 4]
        _check_decode_plan(wl.random_forest_workload(seed, depth=4, fanout=3, n_roots=2, max_node_pages=40,
                                                     num_q_heads=hq, num_kv_heads=hk), oracle)
    _, c1d = wl.config1()
    for w in (c1d, wl.config2(), wl.config3(), wl.config5()):
        _check_decode_plan(w, oracle)


def test_decode_plan_accepts_nodes_that_end_inside_a_page(oracle):
    """bf16 / fp8 decode plans read every node through its own pages: parents may hold any token count.
    Every (request, KV head, token) is still covered exactly once; flat tables, prefill and fp32 pools
    keep the whole-page rule."""
    for seed in range(140, 146):
        w = wl.random_forest_workload(seed, depth=4, fanout=3, n_roots=2, max_node_pages=30, ragged_internal=True,
                                      kv_dtype=wl.KV_FP8_E4M3 if seed % 2 else wl.KV_BF16)
        f = w.forest
        has_child = np.zeros(f.n_nodes, dtype=bool)
        has_child[f.parent[f.parent >= 0]] = True
        if not (has_child & (f.n_tokens % 16 != 0)).any():
            continue
        pool = fake_pool(w.num_pages, w.num_kv_heads, w.kv_dtype)
        plan = hkv.hkv_decode_plan_create(pool, f.nodes, f.node_pages, f.req_leaf, w.num_q_heads, hkv.PLAN_HOST_ONLY)
        items = hkv.hkv_decode_plan_items(plan)
        tok_start = np.zeros(f.n_nodes, dtype=np.int64)
        for v in range(f.n_nodes):
            if f.parent[v] >= 0:
                tok_start[v] = tok_start[f.parent[v]] + f.n_tokens[f.parent[v]]
        under = [[r for r in range(f.n_req) if v in f.path(int(f.req_leaf[r]))] for v in range(f.n_nodes)]
        covered = [np.zeros((w.num_kv_heads, f.kv_len(r)), dtype=np.int32) for r in range(f.n_req)]
        pos = {v: 0 for v in range(f.n_nodes)}
        indptr = np.cumsum([0] + [len(u) for u in under])
        for page_off, n_tok, kv_head, req_off, n_req, slot, tok_begin, node in items:
            assert page_off == f.page_begin[node] + tok_begin // 16 and tok_begin + n_tok <= f.n_tokens[node]
            for r in under[node][req_off - indptr[node]: req_off - indptr[node] + n_req]:
                covered[r][kv_head, tok_start[node] + tok_begin: tok_start[node] + tok_begin + n_tok] += 1
        assert all((c == 1).all() for c in covered)
        hkv.hkv_decode_plan_destroy(plan)
        with pytest.raises(hkv.HkvError) as e:
            hkv.prefix_tree_flatten(f.nodes, f.node_pages, f.req_leaf, 4096)
        assert e.value.code == hkv.ETREE
        p32 = fake_pool(w.num_pages, w.num_kv_heads, hkv.FP32)
        with pytest.raises(hkv.HkvError) as e:
            hkv.hkv_decode_plan_create(p32, f.nodes, f.node_pages, f.req_leaf, w.num_q_heads, hkv.PLAN_HOST_ONLY)
        assert e.value.code == hkv.ETREE
        hkv.kv_pool_destroy(p32)
        hkv.kv_pool_destroy(pool)


def test_tree_verification_plan_error_codes():
    pool = fake_pool(16, 2)
    nodes = np.array([[-1, 0, 1, 16], [0, 1, 2, 20]], dtype=np.int32)
    pages = np.array([3, 4, 5], dtype=np.int32)
    ok = [0b001, 0b011, 0b101]
    hkv.hkv_decode_plan_destroy(hkv.hkv_decode_plan_create_tree(pool, nodes, pages, [1], 3, ok, 4, hkv.PLAN_HOST_ONLY))
    for T, masks, code in ((3, [0b001, 0b001, 0b101], hkv.EINVAL),       # token 1 does not see itself
                           (3, [0b001, 0b011, 0b1101], hkv.EINVAL),      # a bit beyond the drafted tokens
                           (65, [1] * 65, hkv.EINVAL),                   # more than 64 drafted tokens
                           (21, [(1 << (t + 1)) - 1 for t in range(21)], hkv.EINVAL)):   # the leaf holds only 20 tokens
        with pytest.raises(hkv.HkvError) as e:
            hkv.hkv_decode_plan_create_tree(pool, nodes, pages, [1], T, masks, 4, hkv.PLAN_HOST_ONLY)
        assert e.value.code == code, (T, masks)
    p32 = fake_pool(16, 2, dtype=hkv.FP32)
    with pytest.raises(hkv.HkvError) as e:
        hkv.hkv_decode_plan_create_tree(p32, nodes, pages, [1], 3, ok, 4, hkv.PLAN_HOST_ONLY)
    assert e.value.code == hkv.ESHAPE
    hkv.kv_pool_destroy(p32)
    hkv.kv_pool_destroy(pool)


def test_decode_plan_sizes_of_benchmark_configs(oracle):
    items = _check_decode_plan(wl.config2(), oracle)
    # 4 chunks x 4 row groups x 8 heads of the root, one item per workgroup, heavy first; then the 64 leaves of
    # 512 tokens x 8 heads as two pieces of 256 each, four to a workgroup (one wavefront streams a piece)
    assert len(items) == 128 + 1024
    assert (items[:128, 4] == 16).all() and (items[:128, 1] == 512).all()
    assert (items[128:, 4] == 1).all() and (items[128:, 1] == 256).all()
    pool = fake_pool(wl.config2().num_pages, 8)
    f = wl.config2().forest
    plan = hkv.hkv_decode_plan_create(pool, f.nodes, f.node_pages, f.req_leaf, 32, hkv.PLAN_HOST_ONLY)
    assert hkv.hkv_decode_plan_num_workgroups(plan) == 128 + 256 and hkv.hkv_decode_plan_max_parts(plan) == 6
    hkv.hkv_decode_plan_destroy(plan)
    hkv.kv_pool_destroy(pool)
    # a forest too small to fill the chip in that mode keeps its leaves whole (8 requests: 16 root + 64 leaf items)
    small = _check_decode_plan(wl.config2(n_req=8), oracle)
    assert (small[small[:, 4] == 1][:, 1] >= 256).all() and len(small) < 768


def test_many_row_and_few_row_items_are_dispatched_side_by_side():
    """c5: 2048 items of the shared roots (64 query rows each) and 4096 items of the private leaves (8 rows, too
    long for the four-to-a-workgroup mode).  Both classes are spread evenly over the work list, heavy before
    light within a class; the planner setting `interleave` restores one class after the other; the items are the same."""
    w = wl.config5()
    f = w.forest
    pool = fake_pool(w.num_pages, w.num_kv_heads, dtype=hkv.FP8_E4M3)

    def items_of(**settings):      # tile_min_gflop: keeps the roots out of the 256-row tile kernel here
        plan = hkv.hkv_decode_plan_create_ex(pool, f.nodes, f.node_pages, f.req_leaf, w.num_q_heads, hkv.PLAN_HOST_ONLY,
                                             tile_min_gflop=1000000, **settings)
        it = hkv.hkv_decode_plan_items(plan).copy()
        assert hkv.hkv_decode_plan_num_workgroups(plan) == len(it)
        hkv.hkv_decode_plan_destroy(plan)
        return it

    mixed = items_of()
    many = mixed[:, 4] * (w.num_q_heads // w.num_kv_heads) > 16
    assert many.sum() == 2048 and (~many).sum() == 4096
    # every window of 48 consecutive items holds its share of both classes (8 and 16 per 24)
    for b in range(0, len(mixed), 48):
        assert many[b:b + 48].sum() == 16
    for cls in (many, ~many):
        cost = mixed[cls, 1].astype(np.int64)
        assert (np.diff(cost) <= 0).all()
    apart = items_of(interleave=-1)
    many_apart = apart[:, 4] * (w.num_q_heads // w.num_kv_heads) > 16
    assert many_apart[:2048].all() and not many_apart[2048:].any()
    assert sorted(map(tuple, mixed.tolist())) == sorted(map(tuple, apart.tolist()))
    assert (mixed[many] == apart[many_apart]).all() and (mixed[~many] == apart[~many_apart]).all()
    hkv.kv_pool_destroy(pool)


def test_large_many_row_share_goes_to_the_tile_kernel(oracle):
    """c5: the 16 roots (256 query rows per KV head, 137 GFLOP) become items of the 256-row tile: one request
    group of 32 per root and KV head, the root's 8192 tokens in one item, 64 persistent workgroups of two items
    each (two items take about as long as streaming the step's bytes); the private
    leaves (8 rows each) are the other items, so both kinds go out as one launch unless the caller says
    otherwise.  c2 and c3 (2 and 9 GFLOP of such work) and plans with several query tokens per request have
    no tile items."""
    w = wl.config5()
    f = w.forest
    items = _check_decode_plan(w, oracle)
    pool = fake_pool(w.num_pages, w.num_kv_heads, dtype=hkv.FP8_E4M3)
    plan = hkv.hkv_decode_plan_create(pool, f.nodes, f.node_pages, f.req_leaf, w.num_q_heads, hkv.PLAN_HOST_ONLY)
    n_tile = hkv.hkv_decode_plan_num_tile_items(plan)
    assert n_tile == 16 * 8 and len(items) == n_tile + 4096
    tiles = items[-n_tile:]
    assert (tiles[:, 4] == 32).all() and (tiles[:, 1] == 8192).all() and (tiles[:, 7] < 16).all()
    assert hkv.hkv_decode_plan_tile_workgroups(plan) == 64 and hkv.hkv_decode_plan_is_fused(plan)
    assert (items[:-n_tile, 4] == 1).all()
    hkv.hkv_decode_plan_destroy(plan)
    two = hkv.hkv_decode_plan_create_ex(pool, f.nodes, f.node_pages, f.req_leaf, w.num_q_heads, hkv.PLAN_HOST_ONLY, fused=-1,
                                        tile_chunk=2048, tile_workgroups=96)
    assert not hkv.hkv_decode_plan_is_fused(two) and hkv.hkv_decode_plan_num_tile_items(two) == 16 * 8 * 4
    assert hkv.hkv_decode_plan_tile_workgroups(two) == 96
    hkv.hkv_decode_plan_destroy(two)
    # a forest with a node shared by 64 rows besides the big one keeps two kernels: such items synchronise per step
    mixed = wl.make_forest([-1, 0] + [1] * 8 + [0] * 56, [4096, 512] + [64] * 64, list(range(2, 66)), np.arange(4096 // 16 + 512 // 16 + 64 * 4, dtype=np.int32))
    mp = fake_pool(len(mixed.node_pages), 8)
    plan = hkv.hkv_decode_plan_create_ex(mp, mixed.nodes, mixed.node_pages, mixed.req_leaf, 64, hkv.PLAN_HOST_ONLY, tile_min_gflop=-1)
    assert hkv.hkv_decode_plan_num_tile_items(plan) > 0 and not hkv.hkv_decode_plan_is_fused(plan)
    hkv.hkv_decode_plan_destroy(plan)
    hkv.kv_pool_destroy(mp)
    multi = hkv.hkv_decode_plan_create_multi(pool, f.nodes, f.node_pages, f.req_leaf, 2, w.num_q_heads, hkv.PLAN_HOST_ONLY)
    assert hkv.hkv_decode_plan_num_tile_items(multi) == 0
    hkv.hkv_decode_plan_destroy(multi)
    hkv.kv_pool_destroy(pool)
    for small in (wl.config2(), wl.config3()):
        sp = fake_pool(small.num_pages, small.num_kv_heads)
        plan = hkv.hkv_decode_plan_create(sp, small.forest.nodes, small.forest.node_pages, small.forest.req_leaf,
                                          small.num_q_heads, hkv.PLAN_HOST_ONLY)
        assert hkv.hkv_decode_plan_num_tile_items(plan) == 0 and hkv.hkv_decode_plan_tile_workgroups(plan) == 0
        hkv.hkv_decode_plan_destroy(plan)
        hkv.kv_pool_destroy(sp)


def test_decode_plan_create_ex_equals_the_four_creators_and_checks_its_settings():
    """With NULL settings the call plans as hkv_decode_plan_create; tokens_per_req, visible and reserve_tokens
    select the other three creators' plans (same items); a setting outside its range is EINVAL and names the field;
    settings change the cut into items, never the coverage."""
    w = wl.config2(n_req=12)
    f = w.forest
    pool = fake_pool(w.num_pages, w.num_kv_heads)
    args = (pool, f.nodes, f.node_pages, f.req_leaf)

    def items(plan):
        it = hkv.hkv_decode_plan_items(plan).copy()
        hkv.hkv_decode_plan_destroy(plan)
        return it

    H = hkv.PLAN_HOST_ONLY
    assert (items(hkv.hkv_decode_plan_create(*args, w.num_q_heads, H)) == items(hkv.hkv_decode_plan_create_ex(*args, w.num_q_heads, H))).all()
    assert (items(hkv.hkv_decode_plan_create_multi(*args, 3, w.num_q_heads, H)) ==
            items(hkv.hkv_decode_plan_create_ex(*args, w.num_q_heads, H, tokens_per_req=3))).all()
    vis = np.tile(np.array([1, 3, 5], dtype=np.uint64), f.n_req)
    assert (items(hkv.hkv_decode_plan_create_tree(*args, 3, vis, w.num_q_heads, H)) ==
            items(hkv.hkv_decode_plan_create_ex(*args, w.num_q_heads, H, tokens_per_req=3, visible=vis))).all()
    assert (items(hkv.hkv_decode_plan_create_growing(*args, w.num_q_heads, 40, H)) ==
            items(hkv.hkv_decode_plan_create_ex(*args, w.num_q_heads, H, reserve_tokens=40))).all()
    base = items(hkv.hkv_decode_plan_create_ex(*args, w.num_q_heads, H))
    cut = items(hkv.hkv_decode_plan_create_ex(*args, w.num_q_heads, H, leaf_chunk=64, shared_chunk=128, max_rows=32))
    assert len(cut) > len(base) and cut[:, 1].sum() * 1 >= base[:, 1].sum()
    bad = [dict(leaf_chunk=24), dict(shared_chunk=4096), dict(max_rows=8), dict(max_rows=128), dict(pack=4), dict(stages=2),
           dict(stages=6), dict(interleave=-2), dict(tile_min_rows=64), dict(tile_chunk=40), dict(tile_chunk=16384), dict(fused=1), dict(fused=-2),
           dict(tile_workgroups=-1), dict(large_batch_updates=2), dict(tokens_per_req=17), dict(tokens_per_req=65, visible=np.zeros(65 * f.n_req, dtype=np.uint64)),
           dict(reserve_tokens=-1), dict(reserve_tokens=8, tokens_per_req=2)]
    for kw in bad:
        with pytest.raises(hkv.HkvError) as e:
            hkv.hkv_decode_plan_create_ex(*args, w.num_q_heads, H, **kw)
        assert e.value.code == hkv.EINVAL, (kw, str(e.value))
        name = next(k for k in kw if k != "visible")
        assert name in str(e.value) or "query tokens" in str(e.value) or "growing" in str(e.value), str(e.value)
    with pytest.raises(TypeError):
        hkv.hkv_decode_plan_create_ex(*args, w.num_q_heads, H, no_such_setting=1)
    hkv.kv_pool_destroy(pool)


def test_row_lists_of_a_mixed_step():
    """q_rows of a decode plan and q_row_begin / q_len of a prefill plan: what is accepted, and that the
    prefill tiles address the rows asked for."""
    w = wl.config2(n_req=6)
    f = w.forest
    pool = fake_pool(w.num_pages, w.num_kv_heads)
    args = (pool, f.nodes, f.node_pages, f.req_leaf, w.num_q_heads, hkv.PLAN_HOST_ONLY)
    hkv.hkv_decode_plan_destroy(hkv.hkv_decode_plan_create_ex(*args, q_rows=[9, 0, 4, 2, 30, 7]))
    for rows in ([9, 0, 4, 2, 30, 9], [0, 1, 2, 3, 4, -1]):
        with pytest.raises(hkv.HkvError) as e:
            hkv.hkv_decode_plan_create_ex(*args, q_rows=rows)
        assert e.value.code == hkv.EINVAL and "q_rows" in str(e.value)
    with pytest.raises(ValueError):
        hkv.hkv_decode_plan_create_ex(*args, q_rows=[0, 1, 2])
    hkv.hkv_decode_plan_destroy(hkv.hkv_decode_plan_create_ex(*args, tokens_per_req=2, q_rows=np.arange(12)[::-1]))
    p32 = fake_pool(w.num_pages, w.num_kv_heads, dtype=hkv.FP32)
    with pytest.raises(hkv.HkvError) as e:
        hkv.hkv_decode_plan_create_ex(p32, *args[1:], q_rows=[0, 1, 2, 3, 4, 5])
    assert e.value.code == hkv.ESHAPE
    # prefill: three requests of 70, 0 and 5 new tokens at rows 100.., (none), 3..
    bt = np.tile(np.arange(8, dtype=np.int32), (3, 1))
    kv_len, q_len, begin = [100, 40, 128], [70, 0, 5], [100, 0, 3]
    plan = hkv.hkv_prefill_plan_create_rows(pool, begin, q_len, bt, kv_len, w.num_q_heads, hkv.PLAN_HOST_ONLY)
    tiles = hkv.hkv_prefill_plan_tiles(plan)            # (req, q_begin, n_q, kv_head, q_row0, prefix_len, kv_len, bt_off)
    same = hkv.hkv_prefill_plan_create(pool, [0, 70, 70, 75], bt, kv_len, w.num_q_heads, hkv.PLAN_HOST_ONLY)
    ref = hkv.hkv_prefill_plan_tiles(same)
    assert np.array_equal(np.delete(tiles, 4, axis=1), np.delete(ref, 4, axis=1))
    assert np.array_equal(tiles[:, 4], np.asarray(begin)[tiles[:, 0]] + tiles[:, 1])
    for pl in (plan, same):
        hkv.hkv_prefill_plan_destroy(pl)
    for b, n in (([0, 50, 69], [70, 0, 5]), ([0, 0, -1], [70, 0, 5]), ([0, 0, 80], [70, -1, 5])):
        with pytest.raises(hkv.HkvError) as e:
            hkv.hkv_prefill_plan_create_rows(pool, b, n, bt, kv_len, w.num_q_heads, hkv.PLAN_HOST_ONLY)
        assert e.value.code == hkv.EINVAL, str(e.value)
    with pytest.raises(hkv.HkvError) as e:
        hkv.hkv_prefill_plan_create_rows(p32, begin, q_len, bt, kv_len, w.num_q_heads, hkv.PLAN_HOST_ONLY)
    assert e.value.code == hkv.ESHAPE
    hkv.kv_pool_destroy(pool)
    hkv.kv_pool_destroy(p32)


def test_decode_plan_error_codes():
    pool = fake_pool(16, 2)
    nodes = np.array([[-1, 0, 1, 16], [0, 1, 1, 5]], dtype=np.int32)
    pages = np.array([3, 4], dtype=np.int32)
    cases = [(nodes, pages, [1], 3, hkv.ESHAPE),                                    # 3 q heads over 2 kv heads
             (nodes, np.array([3, 16], dtype=np.int32), [1], 4, hkv.ERANGE),        # page id outside the pool
             (nodes, pages, [5], 4, hkv.ERANGE),
             (np.array([[-1, 0, 2, 10], [0, 1, 1, 5]], dtype=np.int32), pages, [1], 4, hkv.ETREE),  # 10 tokens are 1 page
             (np.array([[0, 0, 1, 16], [-1, 1, 1, 5]], dtype=np.int32), pages, [1], 4, hkv.ETREE)]   # parent after child
    for n, p, leaves, hq, code in cases:
        with pytest.raises(hkv.HkvError) as e:
            hkv.hkv_decode_plan_create(pool, n, p, leaves, hq, hkv.PLAN_HOST_ONLY)
        assert e.value.code == code, str(e.value)
    plan = hkv.hkv_decode_plan_create(pool, nodes, pages, [1], 4, hkv.PLAN_HOST_ONLY)
    with pytest.raises(hkv.HkvError) as e:          # a host-only plan cannot run
        hkv.attn_decode_plan_run(plan, 0x1000, 1.0, 0x2000, None, 0x3000, 1 << 20, stream=0)
    assert e.value.code == hkv.EINVAL and "host-only" in str(e.value)
    with pytest.raises(hkv.HkvError) as e:
        hkv.attn_decode_plan_run(plan, 0x1001, 1.0, 0x2000, None, 0x3000, 1 << 20, stream=0)   # unaligned q
    assert e.value.code == hkv.EINVAL
    assert hkv.attn_decode_workspace_bytes(pool, nodes, pages, [1], 4) == hkv.hkv_decode_plan_workspace_bytes(plan)
    hkv.hkv_decode_plan_destroy(plan)
    hkv.kv_pool_destroy(pool)


# ------------------------------------------------------------------------------ prefill planning

def _check_prefill_plan(w, oracle):
    f = w.forest
    bt, kv_len, *_ = oracle.flatten_tree(f.nodes, f.node_pages, f.req_leaf, max(1, f.max_pages_per_req()))
    cu = w.cu_q()
    pool = fake_pool(w.num_pages, w.num_kv_heads, w.kv_dtype)
    plan = hkv.hkv_prefill_plan_create(pool, cu, bt, kv_len, w.num_q_heads, hkv.PLAN_HOST_ONLY)
    tiles = hkv.hkv_prefill_plan_tiles(plan)
    tq = 256 // w.group
    covered = np.zeros((w.num_kv_heads, int(cu[-1])), dtype=np.int32)
    for req, q_begin, n_q, kv_head, q_row0, prefix_len, kvl, bt_off in tiles:
        assert 1 <= n_q <= tq and q_begin % tq == 0
        assert q_row0 == cu[req] + q_begin and q_begin + n_q <= cu[req + 1] - cu[req]
        assert kvl == kv_len[req] and prefix_len == kv_len[req] - (cu[req + 1] - cu[req])
        assert bt_off == req * bt.shape[1]
        covered[kv_head, q_row0: q_row0 + n_q] += 1
    assert (covered == 1).all()
    # longest key range first
    ext = tiles[:, 5] + tiles[:, 1] + tiles[:, 2]
    assert (np.diff(ext[::w.num_kv_heads]) <= 0).all()
    hkv.hkv_prefill_plan_destroy(plan)
    hkv.kv_pool_destroy(pool)
    return tiles


def test_prefill_plan_covers_every_new_token_once(oracle):
    for seed in range(130, 136):
        hq, hk = [(8, 2), (8, 1), (4, 4), (4, 2)][seed % 4]
        _check_prefill_plan(wl.random_forest_workload(seed, mode="prefill", num_q_heads=hq, num_kv_heads=hk,
                                                      max_node_pages=30), oracle)
    c1p, _ = wl.config1()
    _check_prefill_plan(c1p, oracle)
    tiles = _check_prefill_plan(wl.config4(), oracle)
    assert len(tiles) == 3712


def test_prefill_plan_error_codes():
    pool = fake_pool(16, 2)
    bt = np.array([[1, 2, 3, -1]], dtype=np.int32)
    cases = [([0, 8], bt, [40], 4, hkv.OK),
             ([0, 8], bt, [4], 4, hkv.EINVAL),              # fewer keys than new tokens
             ([1, 8], bt, [40], 4, hkv.EINVAL),             # cu_q must start at 0
             ([0, 8], bt, [80], 4, hkv.ENOMEM),             # needs 5 pages, table has 4
             ([0, 8], bt, [60], 4, hkv.ERANGE),             # reaches the -1 entry
             ([0, 8], bt, [40], 6, hkv.OK),                 # group of 3 heads: 85 tokens x 3 heads per tile
             ([0, 8], bt, [40], 18, hkv.OK),                # group of 9 heads
             ([0, 8], bt, [40], 34, hkv.ESHAPE),            # group of 17 heads: beyond the supported 16
             ([0, 8], bt, [40], 5, hkv.ESHAPE)]             # 5 query heads over 2 KV heads
    for cu, b, kvl, hq, code in cases:
        if code == hkv.OK:
            hkv.hkv_prefill_plan_destroy(hkv.hkv_prefill_plan_create(pool, cu, b, kvl, hq, hkv.PLAN_HOST_ONLY))
            continue
        with pytest.raises(hkv.HkvError) as e:
            hkv.hkv_prefill_plan_create(pool, cu, b, kvl, hq, hkv.PLAN_HOST_ONLY)
        assert e.value.code == code, str(e.value)
    # fp8 pools: the batch's distinct pages are dequantised into a workspace of 8 KiB per page and KV head
    p8 = fake_pool(16, 2, dtype=hkv.FP8_E4M3)
    bt2 = np.array([[1, 2, 3, -1], [1, 2, 7, 9]], dtype=np.int32)          # pages 1 and 2 are shared
    plan = hkv.hkv_prefill_plan_create(p8, [0, 8, 8 + 20], bt2, [40, 60], 4, hkv.PLAN_HOST_ONLY)
    assert hkv.hkv_prefill_plan_workspace_bytes(plan) == 5 * 2 * 8192
    hkv.hkv_prefill_plan_destroy(plan)
    plan = hkv.hkv_prefill_plan_create(pool, [0, 8], bt, [40], 4, hkv.PLAN_HOST_ONLY)
    assert hkv.hkv_prefill_plan_workspace_bytes(plan) == 0
    hkv.hkv_prefill_plan_destroy(plan)
    hkv.kv_pool_destroy(pool)
    hkv.kv_pool_destroy(p8)


def test_merge_argument_validation():
    with pytest.raises(hkv.HkvError) as e:
        hkv.lse_merge(0x1000, 0x2000, 0x3000, 0x4000, 4, 0x5000, 7, stream=0)
    assert e.value.code == hkv.ESHAPE
    with pytest.raises(hkv.HkvError) as e:
        hkv.lse_merge(None, 0x2000, 0x3000, 0x4000, 4, 0x5000, hkv.BF16, stream=0)
    assert e.value.code == hkv.EINVAL
    hkv.lse_merge(None, None, None, None, 0, None, hkv.BF16, stream=0)              # nothing to do
    with pytest.raises(hkv.HkvError) as e:
        hkv.lse_merge_dense(0x1000, 0x2000, 0x3000, 0, 4, 8, 0x5000, hkv.BF16, stream=0)
    assert e.value.code == hkv.EINVAL
    with pytest.raises(hkv.HkvError) as e:
        hkv.lse_merge_dense(0x1004, 0x2000, 0x3000, 4, 4, 8, 0x5000, hkv.BF16, stream=0)
    assert e.value.code == hkv.EINVAL
    assert hkv.attn_prefill_workspace_bytes(1000, 32) == 0


def test_decode_several_query_tokens_errors():
    f = wl.make_forest([-1, 0], [32, 3], [1], np.arange(4, dtype=np.int32))
    pool = fake_pool(8, 2)
    with pytest.raises(hkv.HkvError) as e:
        hkv.hkv_decode_plan_create_multi(pool, f.nodes, f.node_pages, f.req_leaf, 4, 4, hkv.PLAN_HOST_ONLY)   # leaf holds 3 tokens
    assert e.value.code == hkv.EINVAL
    with pytest.raises(hkv.HkvError) as e:
        hkv.hkv_decode_plan_create_multi(pool, f.nodes, f.node_pages, f.req_leaf, 17, 4, hkv.PLAN_HOST_ONLY)
    assert e.value.code == hkv.EINVAL
    plan = hkv.hkv_decode_plan_create_multi(pool, f.nodes, f.node_pages, f.req_leaf, 3, 4, hkv.PLAN_HOST_ONLY)
    assert hkv.hkv_decode_plan_part_counts(plan, 3).tolist() == [2, 2, 2]       # three query rows, root + leaf each
    hkv.hkv_decode_plan_destroy(plan)


# ------------------------------------------------------------------------------ seeded input generators

def test_token_level_inputs_are_a_function_of_token_and_position():
    """What a prefix cache relies on: the K/V of a (token id, position) pair do not depend on the call that
    asks for them; different pairs, heads, tensors and seeds differ; values look standard normal."""
    ids, pos = np.array([5, 9, 5, 5]), np.array([0, 1, 2, 0])
    k, v = wl.token_kv(3, ids, pos, 2)
    assert k.shape == (4, 2, 128) and k.dtype == np.uint16
    assert np.array_equal(k[0], k[3]) and np.array_equal(v[0], v[3])
    assert not np.array_equal(k[0], k[2]) and not np.array_equal(k[0], v[0]) and not np.array_equal(k[0, 0], k[0, 1])
    k2, _ = wl.token_kv(3, ids[1:3], pos[1:3], 2)
    assert np.array_equal(k2, k[1:3])
    assert not np.array_equal(wl.token_kv(4, ids, pos, 2)[0], k)
    x = wl._hash_normal(1, 3, np.arange(500), np.arange(500) % 7, 4)
    assert abs(float(x.mean())) < 0.01 and abs(float(x.std()) - 1.0) < 0.01 and float(np.abs(x).max()) <= 2 * np.sqrt(3.0)
    prompts = wl.shared_prefix_prompts(3)
    assert len({tuple(p[:40]) for p in prompts}) <= 2          # at most two distinct system prompts


# ------------------------------------------------------------------------------ pages of 32, 64, 128 tokens

def _as_16_token_forest(f, P):
    """The same forest over 16-token pages: page p of P = 16 S tokens is the blocks p S .. p S + S - 1."""
    S = P // 16
    pages, begin, count = [], [], []
    for v in range(f.n_nodes):
        nb = (int(f.n_tokens[v]) + 15) // 16
        begin.append(len(pages))
        count.append(nb)
        pages += [int(f.node_pages[f.page_begin[v] + b // S]) * S + b % S for b in range(nb)]
    return wl.PrefixForest(f.parent, f.n_tokens, np.asarray(begin, dtype=np.int32), np.asarray(count, dtype=np.int32),
                           np.asarray(pages, dtype=np.int32), f.req_leaf)


@pytest.mark.parametrize("P", [32, 64, 128])
def test_flatten_with_larger_pages_bit_exact_against_oracle(oracle, P):
    for seed in range(130, 134):
        f = wl.random_forest_workload(seed, depth=4, fanout=3, n_roots=2, page_size=P).forest
        mp = max(1, f.max_pages_per_req()) + 1
        got = hkv.prefix_tree_flatten(f.nodes, f.node_pages, f.req_leaf, mp, P)
        exp = oracle.flatten_tree(f.nodes, f.node_pages, f.req_leaf, mp, P)
        for g, e in zip(got, exp):
            assert np.array_equal(g, e)
        with pytest.raises(hkv.HkvError) as e:          # page counts fit only the page size they were made for
            hkv.prefix_tree_flatten(f.nodes, f.node_pages, f.req_leaf, mp, 16)
        assert e.value.code == hkv.ETREE
    with pytest.raises(hkv.HkvError) as e:
        hkv.prefix_tree_flatten(f.nodes, f.node_pages, f.req_leaf, mp, 48)
    assert e.value.code == hkv.ESHAPE


@pytest.mark.parametrize("kv_dtype", [wl.KV_BF16, wl.KV_FP8_E4M3])
@pytest.mark.parametrize("P", [32, 64, 128])
def test_plans_over_larger_pages_equal_plans_over_their_16_token_blocks(oracle, P, kv_dtype):
    """The planners work on 16-token blocks: a forest over P-token pages gives the work items and tiles
    of the same forest written over the blocks those pages consist of."""
    S = P // 16
    for seed, ragged_internal in ((140, False), (141, False), (142, True)):
        w = wl.random_forest_workload(seed, depth=4, fanout=3, n_roots=2, max_node_pages=6, page_size=P,
                                      kv_dtype=kv_dtype, ragged_internal=ragged_internal)
        f, f16 = w.forest, _as_16_token_forest(w.forest, P)
        big, small = fake_pool(w.num_pages, w.num_kv_heads, kv_dtype, page_size=P), fake_pool(w.num_pages * S, w.num_kv_heads, kv_dtype)
        a = hkv.hkv_decode_plan_create(big, f.nodes, f.node_pages, f.req_leaf, w.num_q_heads, hkv.PLAN_HOST_ONLY)
        b = hkv.hkv_decode_plan_create(small, f16.nodes, f16.node_pages, f16.req_leaf, w.num_q_heads, hkv.PLAN_HOST_ONLY)
        assert np.array_equal(hkv.hkv_decode_plan_items(a), hkv.hkv_decode_plan_items(b))
        assert np.array_equal(hkv.hkv_decode_plan_part_counts(a, f.n_req), hkv.hkv_decode_plan_part_counts(b, f.n_req))
        assert hkv.hkv_decode_plan_workspace_bytes(a) == hkv.hkv_decode_plan_workspace_bytes(b)
        hkv.hkv_decode_plan_destroy(a)
        hkv.hkv_decode_plan_destroy(b)
        if not ragged_internal:
            wp = wl.random_forest_workload(seed, depth=4, fanout=3, n_roots=2, max_node_pages=6, page_size=P,
                                           kv_dtype=kv_dtype, mode="prefill")
            fp = wp.forest
            mp = max(1, fp.max_pages_per_req())
            bt, kv_len, *_ = oracle.flatten_tree(fp.nodes, fp.node_pages, fp.req_leaf, mp, P)
            bt16 = np.where(bt[:, :, None] >= 0, bt[:, :, None] * S + np.arange(S)[None, None, :], 0).reshape(fp.n_req, mp * S)
            a = hkv.hkv_prefill_plan_create(big, wp.cu_q(), np.maximum(bt, 0), kv_len, wp.num_q_heads, hkv.PLAN_HOST_ONLY)
            b = hkv.hkv_prefill_plan_create(small, wp.cu_q(), bt16.astype(np.int32), kv_len, wp.num_q_heads, hkv.PLAN_HOST_ONLY)
            assert np.array_equal(hkv.hkv_prefill_plan_tiles(a), hkv.hkv_prefill_plan_tiles(b))
            assert hkv.hkv_prefill_plan_workspace_bytes(a) == hkv.hkv_prefill_plan_workspace_bytes(b)
            hkv.hkv_prefill_plan_destroy(a)
            hkv.hkv_prefill_plan_destroy(b)
        hkv.kv_pool_destroy(big)
        hkv.kv_pool_destroy(small)


def test_larger_pages_argument_checks():
    pool = fake_pool(8, page_size=64)
    # a parent of 32 tokens ends inside a 64-token page: fine for the bf16 decode plan, ETREE for flat tables
    nodes = np.array([[-1, 0, 1, 32], [0, 1, 1, 70]], dtype=np.int32)
    with pytest.raises(hkv.HkvError) as e:              # 70 tokens need two 64-token pages
        hkv.hkv_decode_plan_create(pool, nodes, [0, 1], [1], 8, hkv.PLAN_HOST_ONLY)
    assert e.value.code == hkv.ETREE
    nodes[1, 2] = 2
    plan = hkv.hkv_decode_plan_create(pool, nodes, [0, 1, 2], [1], 8, hkv.PLAN_HOST_ONLY)
    hkv.hkv_decode_plan_destroy(plan)
    with pytest.raises(hkv.HkvError) as e:
        hkv.prefix_tree_flatten(nodes, [0, 1, 2], [1], 4, 64)
    assert e.value.code == hkv.ETREE
    with pytest.raises(hkv.HkvError) as e:              # page id beyond the pool's 8 pages
        hkv.hkv_decode_plan_create(pool, nodes, [0, 1, 8], [1], 8, hkv.PLAN_HOST_ONLY)
    assert e.value.code == hkv.ERANGE
    with pytest.raises(hkv.HkvError) as e:              # first_slot must lie inside the first page
        hkv.kv_pool_write(pool, [0, 1], 64, 4, 0x50000, 0x60000, stream=0)
    assert e.value.code == hkv.EINVAL
    with pytest.raises(hkv.HkvError) as e:              # slot 60 + 10 tokens reach into a second page: its id is checked
        hkv.kv_pool_write(pool, [0, 9], 60, 10, 0x50000, 0x60000, stream=0)
    assert e.value.code == hkv.ERANGE
    # prefill: a request of 130 tokens needs three 64-token pages
    with pytest.raises(hkv.HkvError) as e:
        hkv.hkv_prefill_plan_create(pool, [0, 10], np.zeros((1, 2), dtype=np.int32), [130], 8, hkv.PLAN_HOST_ONLY)
    assert e.value.code == hkv.ENOMEM
    plan = hkv.hkv_prefill_plan_create(pool, [0, 10], np.array([[0, 1, 2]], dtype=np.int32), [130], 8, hkv.PLAN_HOST_ONLY)
    hkv.hkv_prefill_plan_destroy(plan)
    hkv.kv_pool_destroy(pool)


def test_fp8_matrix_flag_is_for_fp8_pools():
    nodes, pages = np.array([[-1, 0, 2, 32]], dtype=np.int32), [0, 1]
    pool = fake_pool(4)
    with pytest.raises(hkv.HkvError) as e:
        hkv.hkv_decode_plan_create(pool, nodes, pages, [0], 8, hkv.PLAN_HOST_ONLY | hkv.PLAN_FP8_MATRIX)
    assert e.value.code == hkv.ESHAPE
    hkv.kv_pool_destroy(pool)
    p8 = fake_pool(4, dtype=hkv.FP8_E4M3)
    a = hkv.hkv_decode_plan_create(p8, nodes, pages, [0], 8, hkv.PLAN_HOST_ONLY | hkv.PLAN_FP8_MATRIX)
    b = hkv.hkv_decode_plan_create(p8, nodes, pages, [0], 8, hkv.PLAN_HOST_ONLY)
    assert np.array_equal(hkv.hkv_decode_plan_items(a), hkv.hkv_decode_plan_items(b))      # same work list, other arithmetic
    hkv.hkv_decode_plan_destroy(a)
    hkv.hkv_decode_plan_destroy(b)
    hkv.kv_pool_destroy(p8)


# ------------------------------------------------------------------------------ plans that grow with the decode loop

def _grown(f, page_size, steps, next_page):
    """The forest after `steps` appends to every request's leaf; new pages are taken from next_page()."""
    n_tokens, n_pages = f.n_tokens.copy(), f.n_pages.copy()
    lists = [list(f.node_pages[f.page_begin[v]: f.page_begin[v] + f.n_pages[v]]) for v in range(f.n_nodes)]
    log = []
    for _ in range(steps):
        new = np.full(f.n_req, -1, dtype=np.int32)
        for r, v in enumerate(f.req_leaf):
            if n_tokens[v] % page_size == 0:
                new[r] = next_page()
                lists[v].append(int(new[r]))
                n_pages[v] += 1
            n_tokens[v] += 1
        log.append(new)
    begin = np.concatenate([[0], np.cumsum(n_pages)[:-1]]).astype(np.int32)
    g = wl.PrefixForest(f.parent, n_tokens, begin, n_pages, np.asarray([p for l in lists for p in l], dtype=np.int32),
                        f.req_leaf, page_size)
    return g, log


@pytest.mark.parametrize("page_size", [16, 64])
@pytest.mark.parametrize("kv_dtype", [wl.KV_BF16, wl.KV_FP8_E4M3])
def test_growing_plan_covers_the_grown_forest(oracle, page_size, kv_dtype):
    """After k appends the work list covers every (request, KV head, token) of the grown forest exactly once and has
    kept its chunking: only the leaves' last chunks got longer (which blocks they read is checked on the GPU)."""
    H, Hq, S = 2, 8, page_size // 16
    parent = [-1, 0, 0, 1, 1, 2]
    ntok = [4 * page_size, 2 * page_size, page_size, 5, page_size - 1, 3 * page_size]     # leaves 3, 4, 5 of requests 0, 1, 2
    pages = np.random.default_rng(3).permutation(200).astype(np.int32)
    f = wl.make_forest(parent, ntok, [3, 4, 5], pages, page_size)
    used = int(f.n_pages.sum())
    pool = fake_pool(200, H, kv_dtype, page_size=page_size)
    steps = 2 * page_size + 3
    plan = hkv.hkv_decode_plan_create_growing(pool, f.nodes, f.node_pages, f.req_leaf, Hq, steps, hkv.PLAN_HOST_ONLY)
    before = hkv.hkv_decode_plan_items(plan)
    fresh = iter(pages[used:].tolist())
    g, log = _grown(f, page_size, steps, lambda: next(fresh))
    for new in log:
        hkv.hkv_decode_plan_append(plan, new, stream=0)
    with pytest.raises(hkv.HkvError) as e:                     # the reserve is used up
        hkv.hkv_decode_plan_append(plan, np.zeros(3, dtype=np.int32), stream=0)
    assert e.value.code == hkv.ENOMEM
    items = hkv.hkv_decode_plan_items(plan)
    assert len(items) == len(before) and np.array_equal(items[:, [0, 2, 3, 4, 5, 6, 7]], before[:, [0, 2, 3, 4, 5, 6, 7]])
    assert ((items[:, 1] - before[:, 1]) == np.where(np.isin(items[:, 7], [3, 4, 5]) & (items[:, 1] != before[:, 1]), steps, 0)).all()
    covered = {r: np.zeros((H, int(g.kv_len(r))), dtype=np.int32) for r in range(3)}
    starts = {v: sum(int(g.n_tokens[u]) for u in g.path(v)[:-1]) for v in range(g.n_nodes)}
    members = {v: [r for r in range(3) if v in g.path(int(g.req_leaf[r]))] for v in range(g.n_nodes)}
    for page_off, n_tok, kv_head, req_off, n_req, slot, tok_begin, node in items:
        for r in members[node]:
            a = starts[node] + tok_begin
            covered[r][kv_head, a: a + n_tok] += 1
    for r in range(3):
        assert (covered[r] == 1).all()
    hkv.hkv_decode_plan_destroy(plan)
    hkv.kv_pool_destroy(pool)


def test_growing_plan_argument_checks():
    pool = fake_pool(16, 2)
    nodes = np.array([[-1, 0, 1, 16], [0, 1, 1, 5], [0, 2, 1, 16]], dtype=np.int32)
    pages = np.array([3, 4, 5], dtype=np.int32)
    mk = lambda n, leaves, reserve=8, p=pool: hkv.hkv_decode_plan_create_growing(p, n, pages, leaves, 4, reserve, hkv.PLAN_HOST_ONLY)
    for leaves, code in (([0], hkv.ETREE),            # the leaf has children
                         ([1, 1], hkv.ETREE),         # two requests on one leaf
                         ([3], hkv.ERANGE)):
        with pytest.raises(hkv.HkvError) as e:
            mk(nodes, leaves)
        assert e.value.code == code, str(e.value)
    empty = nodes.copy()
    empty[1] = [0, 1, 0, 0]
    with pytest.raises(hkv.HkvError) as e:                # a leaf without a token
        mk(empty, [1])
    assert e.value.code == hkv.ETREE
    with pytest.raises(hkv.HkvError) as e:
        mk(nodes, [1], reserve=0)
    assert e.value.code == hkv.EINVAL
    p32 = fake_pool(16, 2, hkv.FP32)
    with pytest.raises(hkv.HkvError) as e:
        mk(nodes, [1], p=p32)
    assert e.value.code == hkv.ESHAPE
    plan = mk(nodes, [1, 2])
    with pytest.raises(hkv.HkvError) as e:                # request 1 (16 tokens in its leaf) opens a page: none given
        hkv.hkv_decode_plan_append(plan, None, stream=0)
    assert e.value.code == hkv.EINVAL
    with pytest.raises(hkv.HkvError) as e:
        hkv.hkv_decode_plan_append(plan, [0, 16], stream=0)
    assert e.value.code == hkv.ERANGE
    before = hkv.hkv_decode_plan_items(plan)
    assert np.array_equal(before, hkv.hkv_decode_plan_items(plan))      # the failed calls changed nothing
    hkv.hkv_decode_plan_append(plan, [-1, 7], stream=0)                  # request 0 still has room in its page
    plain = hkv.hkv_decode_plan_create(pool, nodes, pages, [1], 4, hkv.PLAN_HOST_ONLY)
    with pytest.raises(hkv.HkvError) as e:
        hkv.hkv_decode_plan_append(plain, None, stream=0)
    assert e.value.code == hkv.EINVAL
    for p in (plan, plain):
        hkv.hkv_decode_plan_destroy(p)
    with pytest.raises(hkv.HkvError) as e:                # append writes: checked before anything is queued
        hkv.kv_pool_append(pool, [1, 16], [0, 3], 0x50000, 0x60000, stream=0)
    assert e.value.code == hkv.ERANGE
    with pytest.raises(hkv.HkvError) as e:
        hkv.kv_pool_append(pool, [1, 2], [0, 16], 0x50000, 0x60000, stream=0)
    assert e.value.code == hkv.EINVAL
    with pytest.raises(hkv.HkvError) as e:
        hkv.kv_pool_append(p32, [1], [0], 0x50000, 0x60000, stream=0)
    assert e.value.code == hkv.ESHAPE
    hkv.kv_pool_append(pool, [], [], None, None, stream=0)
    for ids, slots in (([1, 2, 1], [3, 0, 4]), ([5, 5], [0, 15])):     # two tokens into one 16-token block
        with pytest.raises(hkv.HkvError) as e:
            hkv.kv_pool_append(pool, ids, slots, 0x50000, 0x60000, stream=0)
        assert e.value.code == hkv.EINVAL and "two tokens" in str(e.value)
    got = hkv.kv_pool_alloc(pool, 2)
    hkv.kv_pool_retain(pool, got[:1])                                   # first page now has two owners
    with pytest.raises(hkv.HkvError) as e:
        hkv.kv_pool_append(pool, got, [0, 0], 0x50000, 0x60000, stream=0)
    assert e.value.code == hkv.EINVAL and "owners" in str(e.value) and f"page {got[0]}" in str(e.value)
    p64 = fake_pool(8, 2, page_size=64)                                 # 64-token pages: blocks 0 and 1 of page 3 differ
    with pytest.raises(hkv.HkvError) as e:
        hkv.kv_pool_append(p64, [3, 3, 3], [1, 17, 30], 0x50000, 0x60000, stream=0)
    assert e.value.code == hkv.EINVAL and "block 1 of page 3" in str(e.value)
    hkv.kv_pool_destroy(pool)
    hkv.kv_pool_destroy(p32)
    hkv.kv_pool_destroy(p64)


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; with --gpus above 1 it says so and exits before touching a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in (r.stdout + r.stderr)
