"""GPU parity over random forests x random planner settings: every case draws a forest (shared roots over private
leaves, optionally a second shared level; any node may end inside a page), a head shape, a pool type and a set of
hkv_decode_plan_params / flags, builds the plan through hkv_decode_plan_create_ex and compares the step, element by
element, with the fp64 oracle.  The draws reach the one-launch path, the two-kernel path (tile kernel beside the
kernel that streams the other nodes, on one or two streams), plans without tile items, ragged chunks of every
kind and the fp8 matrix instruction."""
import numpy as np
import pytest

from paper_2603_16104_amd import workloads as wl
from test_gpu_parity import check_close, check_lse, both_pools, gpu  # noqa: F401  (gpu is a fixture)

pytestmark = pytest.mark.gpu

HEADS = [(32, 8), (64, 8), (16, 1), (8, 2), (16, 2), (12, 3), (8, 1)]


def draw_case(seed):
    rng = np.random.default_rng([seed, 77])
    hq, hk = HEADS[rng.integers(len(HEADS))]
    G = hq // hk
    kv_dtype = [wl.KV_BF16, wl.KV_FP8_E4M3][rng.integers(2)]
    parent, ntok, leaves = [], [], []
    for _ in range(int(rng.integers(1, 4))):
        parent.append(-1)
        ntok.append(int(rng.integers(1, 200)) * 16 if rng.random() < 0.7 else int(rng.integers(1, 3000)))
        top = len(parent) - 1
        if rng.random() < 0.4:
            parent.append(top)
            ntok.append(int(rng.integers(1, 900)))
            top = len(parent) - 1
        for _ in range(int(rng.integers(max(1, 100 // G), 400 // G + 2))):
            parent.append(top)
            ntok.append(int(rng.integers(0, 120)))
            leaves.append(len(parent) - 1)
    n_used = sum((t + 15) // 16 for t in ntok)
    pages = np.random.default_rng([seed, 0]).permutation(n_used + 9).astype(np.int32)
    w = wl.Workload(name=f"random_plan_{seed}", num_q_heads=hq, num_kv_heads=hk, kv_dtype=kv_dtype, num_pages=n_used + 9,
                    seed=seed, forest=wl.make_forest(parent, ntok, leaves, pages), mode="decode")
    st, flags = {}, 0
    pick = lambda p: rng.random() < p  # noqa: E731
    if pick(0.6): st["tile_min_gflop"] = -1
    if pick(0.3): st["tile_min_rows"] = int(rng.choice([128, 160, 200, 256]))
    if pick(0.15): st["fused"] = -1
    if pick(0.4): st["max_rows"] = int(rng.choice([16, 32, 48, 64]))
    if pick(0.4): st["leaf_chunk"] = int(rng.choice([16, 64, 256, 1024]))
    if pick(0.4): st["shared_chunk"] = int(rng.choice([16, 128, 512, 2048]))
    if pick(0.4): st["tile_chunk"] = int(rng.choice([16, 64, 400, 2048, 8192]))
    if pick(0.3): st["pack"] = int(rng.integers(1, 4))
    if pick(0.3): st["stages"] = int(rng.integers(3, 6))
    if pick(0.3): st["tile_workgroups"] = int(rng.choice([1, 3, 64]))
    if pick(0.2): st["interleave"] = int(rng.choice([-1, 1, 4]))
    from paper_2603_16104_amd import binding as hkv
    if pick(0.2): flags |= hkv.PLAN_ONE_STREAM
    if kv_dtype == wl.KV_FP8_E4M3 and pick(0.1): flags |= hkv.PLAN_FP8_MATRIX
    return w, st, flags


def test_random_forests_and_planner_settings(gpu, oracle):
    import torch
    from paper_2603_16104_amd import binding as hkv
    seen = {"one_launch": 0, "two_kernels": 0, "no_tiles": 0}
    for seed in range(9000, 9040):
        w, st, flags = draw_case(seed)
        f, hq = w.forest, w.num_q_heads
        hp, dp = both_pools(gpu, oracle, w)
        exp_o, exp_l = oracle.run_workload(w, hp)
        plan = hkv.hkv_decode_plan_create_ex(dp.handle, f.nodes, f.node_pages, f.req_leaf, hq, flags, **st)
        nb = hkv.hkv_decode_plan_workspace_bytes(plan)
        ws = torch.empty(max(nb, 256), dtype=torch.uint8, device="cuda")
        out = torch.zeros((f.n_req, hq, 128), dtype=torch.int16, device="cuda")
        lse = torch.zeros((f.n_req, hq), dtype=torch.float32, device="cuda")
        hkv.attn_decode_plan_run(plan, gpu.to_device_bits(w.q()), float(w.scale), out, lse, ws, nb)
        torch.cuda.synchronize()
        tiles, fused = hkv.hkv_decode_plan_num_tile_items(plan), hkv.hkv_decode_plan_is_fused(plan)
        seen["one_launch" if fused else "two_kernels" if tiles else "no_tiles"] += 1
        hkv.hkv_decode_plan_destroy(plan)
        dp.close()
        what = f"{w.name} {hq}/{w.num_kv_heads} dtype {w.kv_dtype} flags {flags} {st}"
        check_close(gpu.bf16_tensor_to_f64(out), exp_o, what)
        check_lse(lse.cpu().numpy(), exp_l, what)
    print(seen)
    assert min(seen.values()) >= 3, seen      # the draws do reach all three launch shapes
