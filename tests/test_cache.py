"""Block-level prefix cache: the plain-Python oracle (oracle/cache.py) against the invariants the
policy must satisfy, then the library's host implementation against the oracle, bit for bit.
All CPU (the pool's device pointers are never touched)."""
import numpy as np
import pytest

from oracle import cache as OC
from paper_2603_16104_amd import binding as hkv
from tests.test_host_library import fake_pool


def random_trace(seed, n_ops=300, n_prompts=12, vocab=5, max_blocks=7):
    """acquire / release / unpin operations over a small family of prompts with many shared prefixes."""
    rng = np.random.default_rng(seed)
    stems = [rng.integers(0, vocab, size=16 * int(rng.integers(1, 4))).tolist() for _ in range(4)]
    prompts = []
    for _ in range(n_prompts):
        stem = stems[int(rng.integers(0, len(stems)))]
        tail = rng.integers(0, vocab, size=int(rng.integers(0, 16 * (max_blocks - 3)))).tolist()
        prompts.append(stem + tail)
    ops, live = [], 0
    for _ in range(n_ops):
        r = rng.random()
        if live and r < 0.45:
            ops.append(("release", int(rng.integers(0, 1 << 30))))
            live -= 1
        elif r < 0.5:
            ops.append(("unpin", int(rng.integers(0, 1 << 30))))
        else:
            ops.append(("acquire", int(rng.integers(0, n_prompts)), bool(rng.random() < 0.15)))
            live += 1
    return prompts, ops


def replay(cache_acquire, cache_release, cache_unpin, prompts, ops):
    """Runs a trace through either implementation; returns the observable history."""
    live, pinned, history = [], [], []
    for op in ops:
        if op[0] == "acquire":
            try:
                pages, cached = cache_acquire(prompts[op[1]], op[2])
                pages = [int(p) for p in pages]
                history.append(("A", pages, cached))
                live.append(pages)
                if op[2]:
                    pinned.append(pages)
            except (MemoryError, hkv.HkvError):
                history.append(("A", "full"))
        elif op[0] == "release" and live:
            pages = live.pop(op[1] % len(live))
            cache_release(pages)
            history.append(("R", pages))
        elif op[0] == "unpin" and pinned:
            pages = pinned.pop(op[1] % len(pinned))
            cache_unpin(pages)
            history.append(("U", pages))
    return history


# ------------------------------------------------------------------ oracle pins

def test_oracle_cache_hits_are_exactly_the_shared_full_blocks():
    c = OC.PrefixCache(32)
    a = list(range(40))                       # 2 full blocks + 8 tokens
    pa, ca = c.acquire(a)
    assert ca == 0 and len(pa) == 3 and len(set(pa)) == 3
    b = a[:32] + [99] * 20                    # shares both full blocks, then diverges
    pb, cb = c.acquire(b)
    assert cb == 32 and pb[:2] == pa[:2] and pb[2] not in pa
    d = a[:20] + [7] * 30                     # shares one full block only (the second differs inside)
    pd, cd = c.acquire(d)
    assert cd == 16 and pd[0] == pa[0] and pd[1] != pa[1]
    e = [1] + a[1:]                           # differs in the first token: nothing shared
    pe, ce = c.acquire(e)
    assert ce == 0 and not set(pe) & set(pa)
    # a block in the middle that is equal but follows a different prefix is NOT shared
    f = [5] * 16 + a[16:32]
    pf, cf = c.acquire(f)
    assert cf == 0 and pf[1] != pa[1]


def test_oracle_cache_eviction_order_and_protection():
    c = OC.PrefixCache(6)
    s1, s2, s3 = [1] * 32, [2] * 32, [3] * 32
    p1, _ = c.acquire(s1)
    p2, _ = c.acquire(s2)
    p3, _ = c.acquire(s3)                      # pool full: 6 blocks
    with pytest.raises(MemoryError):
        c.acquire([4] * 16)                    # everything is in use
    c.release(p2)                              # s2 released first -> older last use
    c.release(p1)
    p4, _ = c.acquire([4] * 16)                # must evict: candidates are the LEAF blocks of s2 and s1
    assert c.evicted_pages == [p2[1]]          # least recently used leaf; never the prefix block p2[0] first
    assert p4 == [p2[1]]
    p5, _ = c.acquire([5] * 16)
    assert c.evicted_pages == [p2[1], p2[0]]   # now s2's first block is a leaf and still the oldest
    # a hit refreshes the last use: s1 (released long ago) is touched again and released AFTER p4, so p4's
    # block, although created later, is now the least recently used leaf
    c.release(p4)
    q1, cached = c.acquire(s1)
    assert cached == 32 and q1 == p1
    c.release(q1)
    p6, _ = c.acquire([6] * 16)
    assert c.evicted_pages[-1] == p4[0]
    # pinned blocks survive pressure
    c2 = OC.PrefixCache(4)
    pp, _ = c2.acquire([9] * 32, pin=True)
    c2.release(pp)
    x, _ = c2.acquire([8] * 32)
    c2.release(x)
    y, _ = c2.acquire([7] * 32)                # evicts x's blocks, not the pinned ones
    assert set(c2.evicted_pages) == set(x) and not set(y) & set(pp)
    with pytest.raises(MemoryError):
        c2.acquire([6] * 48)                   # 3 pages wanted, 2 evictable... y is live: nothing to evict
    c2.release(y)
    c2.unpin(pp)
    z, _ = c2.acquire([6] * 64)                # now the formerly pinned blocks may go as well
    assert len(z) == 4 and set(pp) <= set(c2.evicted_pages)


@pytest.mark.parametrize("seed", range(8))
def test_oracle_cache_invariants_on_random_traces(seed):
    """After every operation: no page is owned twice; a cached block's parent is cached; hits + misses
    account for every full block asked for; pages handed out for new blocks are never pages that a
    live sequence still holds."""
    prompts, ops = random_trace(seed)
    n_pages = 24
    c = OC.PrefixCache(n_pages)
    live = []

    def check():
        owned = list(c.by_page) + list(c.private) + list(c.free)
        assert sorted(owned) == list(range(n_pages))
        for b in c.by_page.values():
            assert b.parent is c.root or c.by_page.get(b.parent.page) is b.parent
            assert b.ref >= 0 and b.pin >= 0
        held = [p for pages in live for p in pages]
        for p in held:
            assert p in c.private or c.by_page[p].ref > 0

    def acq(tokens, pin):
        before = set(p for pages in live for p in pages)
        pages, cached = c.acquire(tokens, pin)
        assert cached % 16 == 0 and cached <= len(tokens)
        fresh = pages[cached // 16:]
        assert not set(fresh) & before
        live.append(list(pages))
        check()
        return pages, cached

    def rel(pages):
        live.remove(list(pages))
        c.release(pages)
        check()

    replay(acq, rel, lambda p: (c.unpin(p), check()), prompts, ops)
    full_blocks_asked = c.hits + c.misses
    assert full_blocks_asked > 0 and c.evictions > 0


# ------------------------------------------------------------------ library against the oracle

@pytest.mark.parametrize("seed,page", [(s, 16) for s in range(10)] + [(10, 32), (11, 32), (12, 64)])
def test_library_cache_matches_oracle(seed, page):
    prompts, ops = random_trace(100 + seed, n_ops=400)
    n_pages = [16, 24, 40][seed % 3]
    order = np.random.default_rng(seed).permutation(n_pages).astype(np.int32) if seed % 2 else None
    oc = OC.PrefixCache(n_pages, None if order is None else order.tolist(), block=page)
    exp = replay(oc.acquire, oc.release, oc.unpin, prompts, ops)
    pool = fake_pool(n_pages, 2, free_order=order, page_size=page)
    cache = hkv.kv_cache_create(pool)
    try:
        got = replay(lambda t, p: hkv.kv_cache_acquire(cache, t, p, page), lambda p: hkv.kv_cache_release(cache, p),
                     lambda p: hkv.kv_cache_unpin(cache, p), prompts, ops)
        assert got == exp
        st = hkv.kv_cache_stats(cache)
        assert (st["hits"], st["misses"], st["evictions"], st["cached_blocks"]) == (oc.hits, oc.misses, oc.evictions,
                                                                                   oc.num_cached_blocks())
        assert hkv.kv_pool_num_free(pool) == len(oc.free)
    finally:
        hkv.kv_cache_destroy(cache)
    assert hkv.kv_pool_num_free(pool) == n_pages          # everything went back to the pool
    hkv.kv_pool_destroy(pool)


@pytest.mark.parametrize("impl", ["oracle", "library"])
def test_failed_acquire_leaves_no_block_that_a_later_call_could_hit(impl):
    """A call that runs out of pages had already entered its first new blocks; they never held KV.  After it
    fails and room is made, the same prompt must come back with nothing cached (and stats as if the failed
    call had not happened), while the hits the failed call took are released again."""
    if impl == "oracle":
        c = OC.PrefixCache(4)
        acquire, release = c.acquire, c.release
        stats = lambda: (c.hits, c.misses, c.num_cached_blocks(), len(c.free))
        err = MemoryError
    else:
        pool = fake_pool(4, 2)
        cache = hkv.kv_cache_create(pool)
        acquire = lambda t: hkv.kv_cache_acquire(cache, t)
        release = lambda p: hkv.kv_cache_release(cache, p)

        def stats():
            st = hkv.kv_cache_stats(cache)
            return st["hits"], st["misses"], st["cached_blocks"], hkv.kv_pool_num_free(pool)
        err = hkv.HkvError
    a = [1] * 16 + [2] * 24                   # 2 full blocks + a private one: 3 of 4 pages
    pa, _ = acquire(a)
    before = stats()
    b = [1] * 16 + [3] * 48                   # hits a's first block, then needs 3 pages: 1 free, nothing evictable
    with pytest.raises(err):
        acquire(b)
    assert stats() == before
    release(pa)                               # a's blocks become evictable; its private page is free again
    pb, cached = acquire(b)
    assert cached == 16 and pb[0] == pa[0] and len(pb) == 4, "only the block a had filled may count as cached"
    release(pb)
    pc, cached = acquire([1] * 16 + [3] * 48)
    assert cached == 64 and list(pc) == list(pb)
    if impl == "library":
        hkv.kv_cache_destroy(cache)
        hkv.kv_pool_destroy(pool)


def test_library_cache_errors():
    pool = fake_pool(4, 2)
    cache = hkv.kv_cache_create(pool)
    pages, cached = hkv.kv_cache_acquire(cache, [1] * 40)
    assert cached == 0 and len(pages) == 3
    with pytest.raises(hkv.HkvError) as e:
        hkv.kv_cache_acquire(cache, [2] * 40)            # 3 more pages, 1 free, nothing evictable
    assert e.value.code == hkv.ENOMEM
    # the failed call holds nothing and leaves nothing: the block it had created is gone again, its page free
    st = hkv.kv_cache_stats(cache)
    assert (st["cached_blocks"], st["misses"], st["evictions"]) == (2, 2, 0) and hkv.kv_pool_num_free(pool) == 1
    extra, _ = hkv.kv_cache_acquire(cache, [3] * 16)
    assert hkv.kv_cache_stats(cache)["evictions"] == 0
    hkv.kv_cache_release(cache, extra)
    with pytest.raises(hkv.HkvError) as e:
        hkv.kv_cache_release(cache, extra)               # released twice
    assert e.value.code == hkv.ERANGE
    hkv.kv_cache_release(cache, pages)
    hkv.kv_cache_destroy(cache)
    hkv.kv_pool_destroy(pool)


def test_schedule_and_cache_hit_rate_under_pressure():
    """Host-only end-to-end: scheduled call orders run through the block-level cache with room for two
    prompts.  For map-reduce the cache-aware order keeps each role's system prompt hot and beats the
    query-by-query order by a wide margin; for reflect both orders reuse the same tokens.  (For debate the
    query-by-query order can reuse more under tight capacity, because a query's later rounds extend its own
    earlier prompts: the cost model only counts reuse between consecutive calls, and the order it picks is
    not the best one for an LRU cache.  Nothing is asserted there beyond consistency.)"""
    from paper_2603_16104_amd import runtime, workloads as wl
    res = {}
    for wf in (wl.workflow_map_reduce(n_queries=5, n_mappers=3), wl.workflow_debate(n_queries=4, n_agents=3, rounds=2),
               wl.workflow_reflect(n_queries=6)):
        tree = hkv.trt_build(wf.templates, wf.len_out, wf.worker)
        order = hkv.trt_schedule(tree, 1, 4096)[0][0]
        hkv.trt_destroy(tree)
        longest = max(len(runtime.workflow_prompt_tokens(wf, c)) for c in range(wf.n_calls)) // 16 + 1
        smart = runtime.simulate_prefix_cache(wf, order, 2 * longest)
        naive = runtime.simulate_prefix_cache(wf, list(range(wf.n_calls)), 2 * longest)
        roomy = runtime.simulate_prefix_cache(wf, order, 64 * longest)
        assert smart["prompt_tokens"] == naive["prompt_tokens"] == roomy["prompt_tokens"]
        assert roomy["evictions"] == 0 and roomy["hit_rate"] >= max(smart["hit_rate"], naive["hit_rate"])
        res[wf.name] = (smart["hit_rate"], naive["hit_rate"])
    assert res["map_reduce"][0] > 5 * res["map_reduce"][1]
    assert res["reflect"][0] >= res["reflect"][1] > 0.3
