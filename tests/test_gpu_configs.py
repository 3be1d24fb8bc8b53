"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration the
bench times (plan objects, default work splitting).  Configurations 2 and 3 are compared with the
oracle element by element, and so is every request of configurations 4 and 5 through the oracle's matrix
form of the definition (which tests/test_oracle_pins.py pins to the row-by-row routine and to brute force;
some rows go through the row-by-row routine too)."""
import numpy as np
import pytest

from paper_2603_16104_amd import workloads as wl
from test_gpu_parity import check_close, check_lse, both_pools, gpu  # noqa: F401  (gpu is a fixture)

pytestmark = pytest.mark.gpu


def _decode_full(gpu, oracle, w):
    import torch
    hp, dp = both_pools(gpu, oracle, w)
    exp_o, exp_l = oracle.run_workload(w, hp)
    r = gpu.DecodeRunner(dp, w)
    r.run()
    torch.cuda.synchronize()
    got_o, got_l = gpu.bf16_tensor_to_f64(r.out), r.lse.cpu().numpy()
    # second run on the same plan must give the same bits (no state carried in the workspace)
    first = r.out.clone()
    r.run()
    torch.cuda.synchronize()
    assert torch.equal(first, r.out)
    r.close()
    dp.close()
    res = check_close(got_o, exp_o, w.name)
    check_lse(got_l, exp_l, w.name)
    print(f"{w.name}: max_abs {res[0]:.3e} rel_l2 {res[1]:.3e}")


@pytest.mark.timeout(300)
def test_config2_full(gpu, oracle):
    _decode_full(gpu, oracle, wl.config2())


@pytest.mark.timeout(300)
def test_config2_generation_loop(gpu, oracle):
    """Configuration 2 as a generation loop: 35 steps of one new token per request through the growing plan
    (store and plan update in one call), the configuration the decode-loop bench times; every request opens a
    new page twice on the way.  Outputs of the last step against the oracle over the grown forest, pool bytes
    against the oracle's pool."""
    import torch
    w = wl.config2()
    f = w.forest
    hp, dp = both_pools(gpu, oracle, w)
    steps = 35
    free = [p for p in range(w.num_pages) if p not in set(f.node_pages.tolist())]
    assert len(free) >= 3 * f.n_req
    r = gpu.DecodeRunner(dp, w, reserve_tokens=steps)
    n_tokens = f.n_tokens.copy()
    pages_of = {int(v): list(f.node_pages[f.page_begin[v]: f.page_begin[v] + f.n_pages[v]]) for v in f.req_leaf}
    rng = np.random.default_rng(9)
    for step in range(steps):
        k = wl.f32_to_bf16_bits(rng.standard_normal((f.n_req, w.num_kv_heads, 128)).astype(np.float32))
        v = wl.f32_to_bf16_bits(rng.standard_normal((f.n_req, w.num_kv_heads, 128)).astype(np.float32))
        new = np.full(f.n_req, -1, dtype=np.int32)
        for i, leaf in enumerate(f.req_leaf):
            if n_tokens[leaf] % 16 == 0:
                new[i] = free.pop(0)
                pages_of[int(leaf)].append(int(new[i]))
            hp.write([pages_of[int(leaf)][-1]], int(n_tokens[leaf] % 16), k[i:i + 1], v[i:i + 1])
            n_tokens[leaf] += 1
        r.append_tokens(new, gpu.to_device_bits(k), gpu.to_device_bits(v))
        r.run()
    torch.cuda.synchronize()
    assert np.array_equal(dp.k.cpu().numpy().view(np.uint16), hp.k) and np.array_equal(dp.v.cpu().numpy().view(np.uint16), hp.v)
    n_pg = (n_tokens + 15) // 16
    lists = [pages_of[v] if v in pages_of else list(f.node_pages[f.page_begin[v]: f.page_begin[v] + f.n_pages[v]])
             for v in range(f.n_nodes)]
    g = wl.PrefixForest(f.parent, n_tokens, np.concatenate([[0], np.cumsum(n_pg)[:-1]]).astype(np.int32), n_pg.astype(np.int32),
                        np.asarray([p for l in lists for p in l], dtype=np.int32), f.req_leaf)
    wg = wl.Workload(name="c2_grown", num_q_heads=w.num_q_heads, num_kv_heads=w.num_kv_heads, kv_dtype=w.kv_dtype,
                     num_pages=w.num_pages, seed=w.seed, forest=g, mode="decode")
    exp_o, exp_l = oracle.run_workload(wg, hp)
    res = check_close(gpu.bf16_tensor_to_f64(r.out), exp_o, "c2 generation loop")
    check_lse(r.lse.cpu().numpy(), exp_l, "c2 generation loop")
    print(f"c2 generation loop: max_abs {res[0]:.3e} rel_l2 {res[1]:.3e}")
    r.close()
    dp.close()


@pytest.mark.timeout(300)
def test_config3_full(gpu, oracle):
    _decode_full(gpu, oracle, wl.config3())


# ---- configurations 4 and 5 at full size: the GPU runs once per module, the oracle checks it in slices (each a
# test of its own, so that none runs for minutes without a sign of life)

@pytest.fixture(scope="module")
def c4_run(gpu, oracle):
    import torch
    w = wl.config4()
    hp, dp = both_pools(gpu, oracle, w)
    r = gpu.PrefillRunner(dp, w)
    r.run()
    torch.cuda.synchronize()
    got_o, got_l = gpu.bf16_tensor_to_f64(r.out), r.lse.cpu().numpy()
    obt, okv, *_ = oracle.flatten_workload(w)
    # indexing outputs bit-exact against the oracle's own tree walk
    assert np.array_equal(r.block_table, obt) and np.array_equal(r.kv_len, okv)
    r.close()
    dp.close()
    return w, hp, w.q(), obt, okv, got_o, got_l


@pytest.mark.timeout(300)
@pytest.mark.parametrize("part", [0, 1, 2, 3])
def test_config4_every_request(gpu, oracle, c4_run, part):
    """Every new token of all 32 requests (eight per test) against the oracle's matrix form of the same
    definition (pinned to the row-by-row routine and to brute force in tests/test_oracle_pins.py)."""
    w, hp, q, obt, okv, got_o, got_l = c4_run
    assert np.isfinite(got_o).all() and np.isfinite(got_l).all()
    reqs = list(range(part, w.forest.n_req, 4))
    exp_o, exp_l, rows = oracle.attn_matrix_form(hp, q, w.cu_q(), obt, okv, float(w.scale), requests=reqs)
    res = check_close(got_o[rows], exp_o, w.name)
    check_lse(got_l[rows], exp_l, w.name)
    print(f"{w.name}: requests {reqs}, {len(rows)} query tokens x {w.num_q_heads} heads: max_abs {res[0]:.3e} rel_l2 {res[1]:.3e}")


@pytest.mark.timeout(300)
def test_config4_tile_boundaries_of_every_request(gpu, oracle, c4_run):
    """The kernel works on tiles of 256 query rows of one KV head = 256 / G consecutive new tokens of a request.
    First and last token of every such tile of every request (the last tile is ragged), plus tokens drawn at
    random: a quick check that names the tile when one is dropped, doubled or given the wrong causal limit;
    a handful of tokens go through the row-by-row C routine as well."""
    w, hp, q, obt, okv, got_o, got_l = c4_run
    cu = w.cu_q()
    tile = 256 // (w.num_q_heads // w.num_kv_heads)
    rng = np.random.default_rng(4)
    tokens = {}
    for r in range(w.forest.n_req):
        s = int(cu[r + 1] - cu[r])
        edge = {t for b in range(0, s, tile) for t in (b, min(s, b + tile) - 1)}
        tokens[r] = sorted(edge | {int(x) for x in rng.integers(0, s, 6)})
    exp_o, exp_l, rows = oracle.attn_matrix_form(hp, q, cu, obt, okv, float(w.scale), tokens=tokens)
    res = check_close(got_o[rows], exp_o, w.name)
    check_lse(got_l[rows], exp_l, w.name)
    print(f"{w.name}: {len(rows)} tile-boundary and random query tokens of all {w.forest.n_req} requests: max_abs {res[0]:.3e} rel_l2 {res[1]:.3e}")
    some = rows[rng.integers(0, len(rows), 12)]
    req = np.searchsorted(cu, some, side="right") - 1
    lens = okv[req] - (cu[req + 1] - cu[req]) + (some - cu[req]) + 1
    row_o, row_l = oracle.attn_decode(hp, q[some], obt[req], lens.astype(np.int32), float(w.scale))
    check_close(got_o[some], row_o, w.name + " (row by row)")
    check_lse(got_l[some], row_l, w.name + " (row by row)")


@pytest.fixture(scope="module")
def c5_run(gpu, oracle):
    """The fp8 forest in both pools: every node's seeded K/V is drawn once, quantised by the oracle into its pool
    and by kv_pool_write into the device pool; bytes and scales of both pools are compared as a whole."""
    import torch
    from concurrent.futures import ThreadPoolExecutor
    w = wl.config5()
    f = w.forest
    hp = oracle.HostPool(w.num_pages, w.num_kv_heads, w.kv_dtype)
    dp = gpu.DevicePool(w.num_pages, w.num_kv_heads, w.kv_dtype)

    def host_side(v):       # nodes own disjoint pages: their writes into the oracle's pool do not meet
        k, vv = w.node_kv(v)
        hp.write(f.node_pages[f.page_begin[v]: f.page_begin[v] + f.n_pages[v]], 0, k, vv)
        return v, k, vv

    with ThreadPoolExecutor(max_workers=8) as ex:
        for v, k, vv in ex.map(host_side, [v for v in range(f.n_nodes) if f.n_tokens[v] > 0]):
            dp.write(f.node_pages[f.page_begin[v]: f.page_begin[v] + f.n_pages[v]], 0, gpu.to_device_bits(k), gpu.to_device_bits(vv))
    torch.cuda.synchronize()
    print("c5: both pools filled", flush=True)
    used = np.sort(f.node_pages)
    for name, per_page in (("k", 16 * 128 * w.num_kv_heads), ("v", 16 * 128 * w.num_kv_heads),
                           ("k_scale", w.num_kv_heads), ("v_scale", w.num_kv_heads)):
        g = getattr(dp, name).cpu().numpy().reshape(w.num_pages, per_page)[used]
        o = getattr(hp, name).reshape(w.num_pages, per_page)[used]
        assert np.array_equal(g.view(np.uint8), o.view(np.uint8)), f"{name}: the pools differ"
    r = gpu.DecodeRunner(dp, w)
    r.run()
    torch.cuda.synchronize()
    got_o, got_l = gpu.bf16_tensor_to_f64(r.out), r.lse.cpu().numpy()
    first = r.out.clone()
    r.run()
    torch.cuda.synchronize()
    assert torch.equal(first, r.out)
    r.close()
    dp.close()
    bt, kv_len, *_ = oracle.flatten_workload(w)
    return w, hp, w.q(), bt, kv_len, got_o, got_l


@pytest.mark.timeout(600)
@pytest.mark.parametrize("part", [0, 1, 2, 3])
def test_config5_every_request(gpu, oracle, c5_run, part):
    """All 512 requests of the fp8 forest (every root, every row of every 256-row tile of the shared nodes, every
    private leaf), 128 per test, element by element against the oracle's matrix form over the oracle's own pool;
    eight of them through the row-by-row C routine as well."""
    w, hp, q, bt, kv_len, got_o, got_l = c5_run
    assert np.isfinite(got_o).all() and np.isfinite(got_l).all()
    reqs = list(range(part, w.forest.n_req, 4))        # every root has requests in every part
    cu = np.arange(w.forest.n_req + 1, dtype=np.int32)
    exp_o, exp_l, rows = oracle.attn_matrix_form(hp, q, cu, bt, kv_len, float(w.scale), requests=reqs)
    assert np.array_equal(rows, reqs)
    res = check_close(got_o[rows], exp_o, w.name)
    check_lse(got_l[rows], exp_l, w.name)
    print(f"{w.name}: {len(reqs)} requests x {w.num_q_heads} heads: max_abs {res[0]:.3e} rel_l2 {res[1]:.3e}")
    some = reqs[::16]
    row_o, row_l = oracle.run_workload(w, hp, req_subset=some)
    check_close(got_o[some], row_o, w.name + " (row by row)")
    check_lse(got_l[some], row_l, w.name + " (row by row)")


@pytest.mark.timeout(600)
def test_pool_beyond_4_gib_per_buffer(gpu, oracle):
    """Byte offsets inside the K and V buffers beyond 2^32: a 140 000-page bf16 pool (4.6 GB per buffer)
    whose forest sits in the highest pages.  Pool writer, copy-on-write copy, both decode paths and
    prefill are compared with the oracle run on a compact twin (same nodes and seeded K/V, page ids
    renumbered 0..n-1; the oracle's invariance under page renumbering is pinned on the CPU)."""
    import torch
    from paper_2603_16104_amd import binding as hkv
    num_pages, Hq, Hkv = 140_000, 32, 8
    rng = np.random.default_rng(77)
    parent = [-1] + [0] * 22
    ntok = [256] + [int(t) for t in rng.integers(20, 130, size=22)]
    n_used = sum((t + 15) // 16 for t in ntok)
    high = (num_pages - 1 - rng.permutation(4000)[:n_used]).astype(np.int32)      # scattered over the top 4000 pages
    if num_pages - 1 in high:                                      # the very last page belongs to the root
        j = int(np.nonzero(high == num_pages - 1)[0][0])
        high[0], high[j] = high[j], high[0]
    else:
        high[0] = num_pages - 1
    leaves = list(range(1, 23))
    for mode in ("decode", "prefill"):
        q_len = np.asarray(ntok[1:], dtype=np.int32) if mode == "prefill" else None
        big = wl.Workload(name="beyond_4gib_" + mode, num_q_heads=Hq, num_kv_heads=Hkv, kv_dtype=wl.KV_BF16, num_pages=num_pages,
                          seed=41, forest=wl.make_forest(parent, ntok, leaves, high), mode=mode, q_len=q_len)
        twin = wl.Workload(name="twin_" + mode, num_q_heads=Hq, num_kv_heads=Hkv, kv_dtype=wl.KV_BF16, num_pages=n_used,
                           seed=41, forest=wl.make_forest(parent, ntok, leaves, np.arange(n_used, dtype=np.int32)), mode=mode,
                           q_len=q_len)
        hp = oracle.HostPool(n_used, Hkv, wl.KV_BF16)
        hp.fill_from(twin)
        exp_o, exp_l = oracle.run_workload(twin, hp)
        dp = gpu.DevicePool(num_pages, Hkv, wl.KV_BF16, poison=False)
        dp.fill_from(big)
        # the bytes written to the highest page equal the oracle's for its twin page
        per_page = Hkv * 16 * 128
        top = dp.k.view(num_pages, per_page)[num_pages - 1].cpu().numpy().view(np.uint16)
        assert np.array_equal(top, hp.k.reshape(n_used, per_page)[0])
        r = (gpu.DecodeRunner if mode == "decode" else gpu.PrefillRunner)(dp, big)
        r.run()
        torch.cuda.synchronize()
        res = check_close(gpu.bf16_tensor_to_f64(r.out), exp_o, big.name)
        check_lse(r.lse.cpu().numpy(), exp_l, big.name)
        print(f"{big.name}: max_abs {res[0]:.3e} rel_l2 {res[1]:.3e}")
        r.close()
        if mode == "decode":   # copy-on-write of the highest page into a fresh one, bytes compared on the device
            held = hkv.kv_pool_alloc(dp.handle, num_pages)          # every page: so that page num_pages-1 is allocated
            hkv.kv_pool_release(dp.handle, held[:10])              # ten free pages at the tail of the free list
            hkv.kv_pool_retain(dp.handle, [num_pages - 1])
            new = hkv.kv_pool_copy_on_write(dp.handle, [num_pages - 1])
            torch.cuda.synchronize()
            assert int(new[0]) != num_pages - 1
            for t in (dp.k, dp.v):
                tv = t.view(num_pages, per_page)
                assert torch.equal(tv[int(new[0])], tv[num_pages - 1])
        dp.close()
        del dp
        torch.cuda.empty_cache()


@pytest.mark.timeout(600)
@pytest.mark.parametrize("kv_dtype", [wl.KV_BF16, wl.KV_FP8_E4M3])
def test_pool_write_largest_single_call(gpu, oracle, kv_dtype):
    """kv_pool_write at its documented limit of 65536 pages (1 048 576 tokens) in one call, ragged at both
    ends (first_slot 5, last page partly filled): bytes and scales bit-exact."""
    import torch
    from paper_2603_16104_amd import binding as hkv
    n_pages, H, first = 65536, 1, 5
    n_tok = n_pages * 16 - first - 9
    rng = np.random.default_rng(23)
    k = wl.f32_to_bf16_bits(rng.standard_normal((n_tok, H, 128), dtype=np.float32))
    v = wl.f32_to_bf16_bits(rng.standard_normal((n_tok, H, 128), dtype=np.float32))
    ids = rng.permutation(n_pages + 7).astype(np.int32)[:n_pages]
    hp = oracle.HostPool(n_pages + 7, H, kv_dtype)
    dp = gpu.DevicePool(n_pages + 7, H, kv_dtype)
    if kv_dtype == wl.KV_FP8_E4M3:      # a continued fp8 page needs its first slots written before
        head_k = wl.f32_to_bf16_bits(rng.standard_normal((first, H, 128), dtype=np.float32))
        hp.write(ids[:1], 0, head_k, head_k)
        dp.write(ids[:1], 0, gpu.to_device_bits(head_k), gpu.to_device_bits(head_k))
    hp.write(ids, first, k, v)
    dp.write(ids, first, gpu.to_device_bits(k), gpu.to_device_bits(v))
    torch.cuda.synchronize()
    assert np.array_equal(dp.k.cpu().numpy().view(hp.k.dtype), hp.k) and np.array_equal(dp.v.cpu().numpy().view(hp.v.dtype), hp.v)
    if kv_dtype == wl.KV_FP8_E4M3:
        used = np.zeros(n_pages + 7, dtype=bool)
        used[ids] = True
        for name in ("k_scale", "v_scale"):
            g, o = getattr(dp, name).cpu().numpy()[used], getattr(hp, name)[used]
            assert np.array_equal(g.view(np.uint32), o.view(np.uint32)), name
    dp.close()


@pytest.mark.timeout(600)
def test_very_long_shared_prefix(gpu, oracle):
    """A 65 536-token prefix shared by 24 requests: decode (the prefix is cut into many LDS-staged chunks and
    every row collects 30+ partials) element by element, prefill of 150-250 new tokens per request on
    sampled query tokens (the page-id window of the prefill kernel is refilled hundreds of times)."""
    import torch
    rng = np.random.default_rng(5)
    n_req, Hq, Hkv, root = 24, 4, 1, 65536
    s = [int(x) for x in rng.integers(150, 251, size=n_req)]
    parent, ntok = [-1] + [0] * n_req, [root] + s
    n_used = sum((t + 15) // 16 for t in ntok)
    pages = rng.permutation(n_used + 11).astype(np.int32)
    f = wl.make_forest(parent, ntok, list(range(1, n_req + 1)), pages)
    common = dict(num_q_heads=Hq, num_kv_heads=Hkv, kv_dtype=wl.KV_BF16, num_pages=n_used + 11, seed=61, forest=f)
    wd = wl.Workload(name="long_prefix_decode", mode="decode", **common)
    hp, dp = both_pools(gpu, oracle, wd)
    exp_o, exp_l = oracle.run_workload(wd, hp)
    r = gpu.DecodeRunner(dp, wd)
    r.run()
    torch.cuda.synchronize()
    res = check_close(gpu.bf16_tensor_to_f64(r.out), exp_o, wd.name)
    check_lse(r.lse.cpu().numpy(), exp_l, wd.name)
    from paper_2603_16104_amd import binding as hkv
    print(f"{wd.name}: max_abs {res[0]:.3e} rel_l2 {res[1]:.3e}, {hkv.hkv_decode_plan_max_parts(r.plan)} partials per row")
    r.close()
    wp = wl.Workload(name="long_prefix_prefill", mode="prefill", q_len=np.asarray(s, dtype=np.int32), **common)
    pr = gpu.PrefillRunner(dp, wp)
    pr.run()
    torch.cuda.synchronize()
    got_o, got_l = gpu.bf16_tensor_to_f64(pr.out), pr.lse.cpu().numpy()
    assert np.isfinite(got_o).all()
    obt, okv, *_ = oracle.flatten_workload(wp)
    cu, q = wp.cu_q(), wp.q()
    rows, qs, bts, lens = [], [], [], []
    for _ in range(12):
        req = int(rng.integers(0, n_req))
        i = int(rng.choice([0, 1, 63, 64, s[req] - 1, int(rng.integers(0, s[req]))]))
        rows.append(cu[req] + i)
        qs.append(q[cu[req] + i])
        bts.append(obt[req])
        lens.append(okv[req] - s[req] + i + 1)
    e_o, e_l = oracle.attn_decode(hp, np.stack(qs), np.stack(bts), np.array(lens, dtype=np.int32), float(wp.scale))
    res = check_close(got_o[rows], e_o, wp.name)
    check_lse(got_l[rows], e_l, wp.name)
    print(f"{wp.name}: sampled {len(rows)} query tokens: max_abs {res[0]:.3e} rel_l2 {res[1]:.3e}")
    pr.close()
    dp.close()
