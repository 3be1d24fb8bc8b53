"""GPU parity of the second decode kernel: nodes shared by 128 query rows or more run as items of the
256-row tile kernel (the prefill kernel's loop with partial results as output), next to the kernel
that streams the other nodes.  By default only forests with a large share of such work take that
route, so these tests switch the threshold off and compare, element by element, with the fp64 oracle."""
import numpy as np
import pytest

from paper_2603_16104_amd import workloads as wl
from test_gpu_parity import check_close, check_lse, both_pools, gpu, plan_settings, _FixedWorkload  # noqa: F401  (gpu is a fixture)

pytestmark = pytest.mark.gpu


@pytest.fixture
def tiles_on(monkeypatch):
    plan_settings(monkeypatch, tile_min_gflop=-1)


def shared_root_workload(seed, hq, hkv_, n_req, root_tokens, kv_dtype, mid_tokens=0):
    """A root shared by every request (optionally a second shared node below it) and ragged private leaves."""
    rng = np.random.default_rng([seed, 3])
    parent, ntok = [-1], [root_tokens]
    top = 0
    if mid_tokens:
        parent.append(0)
        ntok.append(mid_tokens)
        top = 1
    leaves = []
    for _ in range(n_req):
        parent.append(top)
        ntok.append(int(rng.integers(1, 90)))
        leaves.append(len(parent) - 1)
    n_used = sum((t + 15) // 16 for t in ntok)
    pages = np.random.default_rng([seed, 0]).permutation(n_used + 9).astype(np.int32)
    f = wl.make_forest(parent, ntok, leaves, pages)
    return wl.Workload(name=f"shared_root_{seed}", num_q_heads=hq, num_kv_heads=hkv_, kv_dtype=kv_dtype,
                       num_pages=n_used + 9, seed=seed, forest=f, mode="decode")


def run_tiled(gpu, oracle, w, flags=0, expect_tiles=True):
    import torch
    from paper_2603_16104_amd import binding as hkv
    hp, dp = both_pools(gpu, oracle, w)
    exp_o, exp_l = oracle.run_workload(w, hp)
    r = gpu.DecodeRunner(dp, w, flags=flags)
    assert (hkv.hkv_decode_plan_num_tile_items(r.plan) > 0) == expect_tiles
    r.run()
    torch.cuda.synchronize()
    got_o, got_l = gpu.bf16_tensor_to_f64(r.out), r.lse.cpu().numpy()
    first = r.out.clone()
    r.run()                                           # the same bits again: nothing is carried between runs
    torch.cuda.synchronize()
    assert torch.equal(first, r.out)
    r.close()
    dp.close()
    res = check_close(got_o, exp_o, w.name)
    check_lse(got_l, exp_l, w.name)
    return first, res


@pytest.mark.parametrize("kv_dtype", [wl.KV_BF16, wl.KV_FP8_E4M3])
@pytest.mark.parametrize("hq,hkv_,n_req,root_tokens", [
    (32, 8, 64, 1040),      # 256 rows: one full tile per chunk and KV head
    (8, 2, 70, 1509),       # 280 rows: two request groups of 35; the root ends inside a page
    (8, 1, 40, 777),        # G = 8: 320 rows, two groups of 20
    (5, 1, 60, 300),        # G = 5: 51 requests per tile at most, two groups of 30
    (4, 4, 130, 200),       # G = 1: 130 requests in one tile
    (16, 1, 8, 64),         # exactly 128 rows, one 64-token block
    (8, 2, 33, 31),         # fewer tokens than one 32-token step
])
def test_tile_decode_shared_root(gpu, oracle, tiles_on, kv_dtype, hq, hkv_, n_req, root_tokens):
    w = shared_root_workload(11, hq, hkv_, n_req, root_tokens, kv_dtype)
    _, res = run_tiled(gpu, oracle, w)
    print(f"{w.name} {hq}/{hkv_} x {n_req} requests, root {root_tokens}: max_abs {res[0]:.3e} rel_l2 {res[1]:.3e}")


@pytest.mark.parametrize("kv_dtype", [wl.KV_BF16, wl.KV_FP8_E4M3])
@pytest.mark.parametrize("chunk", [256, 400, 2048])
def test_tile_decode_chunks_and_two_shared_levels(gpu, oracle, tiles_on, monkeypatch, kv_dtype, chunk):
    """A 2100-token root and a 330-token node below it, both shared by 48 requests x 4 heads: several chunks per
    node (the last one ragged), partial slots of two tiled nodes and of the private leaves in one merge."""
    plan_settings(monkeypatch, tile_chunk=chunk)
    w = shared_root_workload(12, 8, 2, 48, 2100, kv_dtype, mid_tokens=330)
    run_tiled(gpu, oracle, w)


@pytest.mark.parametrize("kv_dtype", [wl.KV_BF16, wl.KV_FP8_E4M3])
def test_tile_decode_on_one_stream_gives_the_same_bits(gpu, oracle, tiles_on, kv_dtype):
    from paper_2603_16104_amd import binding as hkv
    w = shared_root_workload(13, 8, 2, 50, 1200, kv_dtype)
    both, _ = run_tiled(gpu, oracle, w)
    one, _ = run_tiled(gpu, oracle, w, flags=hkv.PLAN_ONE_STREAM)
    import torch
    assert torch.equal(both, one)


@pytest.mark.parametrize("kv_dtype", [wl.KV_BF16, wl.KV_FP8_E4M3])
@pytest.mark.parametrize("beta", [4.9, 8.0, 30.0])
def test_tile_decode_late_dominant_key(gpu, oracle, tiles_on, kv_dtype, beta):
    """A key deep inside the shared root whose score exceeds everything before it by 55 / 90 / 340 nats: the tile
    kernel keeps one softmax reference per row (the maximum of its first 32 scores); the first case stays inside
    that reference's range, the others must take its running-maximum fallback."""
    rng = np.random.default_rng(78)
    n_req, root, hot = 40, 700, 611
    base = shared_root_workload(14, 8, 2, n_req, root, kv_dtype)
    f = base.forest
    u = rng.standard_normal(128).astype(np.float32)
    u *= np.sqrt(128.0) / np.linalg.norm(u)
    kv = {}
    for v in range(f.n_nodes):
        n = int(f.n_tokens[v])
        k = (0.05 * rng.standard_normal((n, 2, 128))).astype(np.float32)
        vv = rng.standard_normal((n, 2, 128)).astype(np.float32)
        kv[v] = [k, vv]
    kv[0][0][hot] = beta * u
    q = np.broadcast_to(u, (n_req, 8, 128)).astype(np.float32) + 0.05 * rng.standard_normal((n_req, 8, 128)).astype(np.float32)
    w = _FixedWorkload(base, {n: (wl.f32_to_bf16_bits(k), wl.f32_to_bf16_bits(v)) for n, (k, v) in kv.items()},
                       wl.f32_to_bf16_bits(q))
    import torch
    hp, dp = both_pools(gpu, oracle, w)
    exp_o, exp_l = oracle.run_workload(w, hp)
    r = gpu.DecodeRunner(dp, w)
    r.run()
    torch.cuda.synchronize()
    got_o, got_l = gpu.bf16_tensor_to_f64(r.out), r.lse.cpu().numpy()
    r.close()
    dp.close()
    check_close(got_o, exp_o, w.name)
    assert np.abs(got_l - exp_l).max() <= 2e-3 + 1e-6 * np.abs(exp_l).max()


def test_tile_decode_is_graph_capturable(gpu, oracle, tiles_on):
    """The fork to the plan's own stream and the join before the merge are event edges, so a caller may capture
    the step in a HIP graph: several replays, with eager work in between, must each reproduce the eager result."""
    import torch
    from paper_2603_16104_amd import binding as hkv
    w = shared_root_workload(15, 32, 8, 40, 900, wl.KV_BF16)
    hp, dp = both_pools(gpu, oracle, w)
    r = gpu.DecodeRunner(dp, w)
    assert hkv.hkv_decode_plan_num_tile_items(r.plan) > 0
    r.run()
    torch.cuda.synchronize()
    ref_o, ref_l = r.out.clone(), r.lse.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        r.run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        r.run()
    for rep in range(4):
        r.out.fill_(7)
        r.lse.fill_(3.0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(r.out, ref_o) and torch.equal(r.lse, ref_l), f"replay {rep}"
        r.out.float().sum().item()                   # eager work between replays
    del g
    r.close()
    dp.close()


@pytest.mark.parametrize("kv_dtype", [wl.KV_BF16, wl.KV_FP8_E4M3])
@pytest.mark.parametrize("T", [1, 2])
def test_decode_rows_anywhere_in_q_and_out(gpu, oracle, tiles_on, kv_dtype, T):
    """hkv_decode_plan_params.q_rows: the plan's rows are scattered over a q / out / lse three times as long
    (every third row, in a shuffled order); both kernels read their query rows from there, the merge writes
    there, the rows in between keep what they held.  70 requests x 4 heads under one root (tile kernel) with
    ragged leaves (the other kernel); with two query tokens per request as well."""
    import torch
    from paper_2603_16104_amd import binding as hkv
    w = shared_root_workload(21, 8, 2, 70, 1104, kv_dtype)      # whole pages: the oracle walks a flat block table
    f = w.forest
    hp, dp = both_pools(gpu, oracle, w)
    n_rows = f.n_req * T
    q = wl.f32_to_bf16_bits(np.random.default_rng(3).standard_normal((n_rows, w.num_q_heads, 128)).astype(np.float32))
    bt, kv_len, *_ = oracle.flatten_workload(w)
    exp_o, exp_l = oracle.attn_prefill(hp, q, np.arange(f.n_req + 1, dtype=np.int32) * T, bt, kv_len, float(w.scale))
    rows = (3 * np.random.default_rng(4).permutation(n_rows) + 1).astype(np.int32)
    q_big = np.zeros((3 * n_rows, w.num_q_heads, 128), dtype=np.uint16)
    q_big[:] = 0x7FC0                                   # a row read by mistake poisons its output
    q_big[rows] = q
    plan = hkv.hkv_decode_plan_create_ex(dp.handle, f.nodes, f.node_pages, f.req_leaf, w.num_q_heads, tokens_per_req=T,
                                         q_rows=rows)
    assert (hkv.hkv_decode_plan_num_tile_items(plan) > 0) == (T == 1)      # plans of several query tokens keep to one kernel
    nb = hkv.hkv_decode_plan_workspace_bytes(plan)
    ws = torch.empty(max(nb, 256), dtype=torch.uint8, device="cuda")
    out = torch.full((3 * n_rows, w.num_q_heads, 128), 0x1234, dtype=torch.int16, device="cuda")
    lse = torch.full((3 * n_rows, w.num_q_heads), 7.5, dtype=torch.float32, device="cuda")
    hkv.attn_decode_plan_run(plan, gpu.to_device_bits(q_big), float(w.scale), out, lse, ws, nb)
    torch.cuda.synchronize()
    idx = torch.from_numpy(rows.astype(np.int64)).cuda()
    check_close(gpu.bf16_tensor_to_f64(out[idx]), exp_o, w.name)
    check_lse(lse[idx].cpu().numpy(), exp_l, w.name)
    other = np.setdiff1d(np.arange(3 * n_rows), rows)
    oi = torch.from_numpy(other).cuda()
    assert bool((out[oi] == 0x1234).all()) and bool((lse[oi] == 7.5).all()), "rows of other work were written"
    hkv.hkv_decode_plan_destroy(plan)
    dp.close()
