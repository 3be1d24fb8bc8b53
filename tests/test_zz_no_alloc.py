"""attn_decode_plan_run_static, the decode step for callers that cannot allocate device memory,
against attn_decode_plan_run with a caller-owned workspace: same kernels, so the outputs must be
identical bit for bit (and with that inside the max-abs 2e-2 / relative-L2 5e-3 bound against the
oracle that the other parity tests hold attn_decode_plan_run to).  Two calls in a row share the
library's static workspace; the second has the smaller input, so it runs over what the first left."""
import numpy as np
import pytest

from paper_2603_16104_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need an MI355X"
    from paper_2603_16104_amd import binding, runtime
    binding.lib()
    return runtime


def _run_both(gpu, oracle, w, kv_dtype):
    import torch
    from paper_2603_16104_amd import binding as hkv
    hp = oracle.HostPool(w.num_pages, w.num_kv_heads, w.kv_dtype, page_size=w.page_size)
    hp.fill_from(w)
    dp = gpu.DevicePool(w.num_pages, w.num_kv_heads, w.kv_dtype, page_size=w.page_size)
    dp.fill_from(w)
    r = gpu.DecodeRunner(dp, w)
    assert 0 < r.ws_bytes <= hkv.hkv_static_workspace_bytes()
    r.run()                                               # caller-owned workspace
    torch.cuda.synchronize()
    ref_out, ref_lse = r.out.clone(), r.lse.clone()
    r.out.fill_(0x7FC0)                                   # bf16 NaN bits: every row must be written again
    r.lse.fill_(float("nan"))
    hkv.attn_decode_plan_run_static(r.plan, r.q, r.scale, r.out, r.lse)
    torch.cuda.synchronize()
    got_out, got_lse = r.out.cpu().numpy(), r.lse.cpu().numpy()
    assert np.array_equal(got_out, ref_out.cpu().numpy()), "static-workspace run differs from the workspace run"
    assert np.array_equal(got_lse.view(np.uint32), ref_lse.cpu().numpy().view(np.uint32))
    exp_o, exp_lse = oracle.run_workload(w, hp)
    got = gpu.bf16_tensor_to_f64(r.out)
    err = np.abs(got - exp_o).max()
    rel = np.linalg.norm((got - exp_o).ravel()) / np.linalg.norm(exp_o.ravel())
    assert np.isfinite(got).all()
    assert err <= 2e-2 and rel <= 5e-3, (err, rel)
    fin = np.isfinite(exp_lse)                            # a request whose path holds no token: lse = -inf on both sides
    assert np.array_equal(np.isneginf(got_lse), np.isneginf(exp_lse))
    assert np.abs(got_lse[fin] - exp_lse[fin]).max() <= 2e-3
    r.close()
    dp.close()


@pytest.mark.parametrize("kv_dtype", [wl.KV_BF16, wl.KV_FP8_E4M3])
def test_static_workspace_run_equals_workspace_run_twice(gpu, oracle, kv_dtype):
    big = wl.random_forest_workload(71, kv_dtype=kv_dtype, n_roots=2, depth=3, fanout=3, max_node_pages=9)
    small = wl.random_forest_workload(72, kv_dtype=kv_dtype, n_roots=1, depth=2, fanout=2, max_node_pages=3)
    assert small.forest.n_req < big.forest.n_req
    _run_both(gpu, oracle, big, kv_dtype)
    _run_both(gpu, oracle, small, kv_dtype)               # smaller input over the first call's leftovers


def test_static_workspace_limit_is_an_error(gpu):
    """A plan whose partials exceed the static array is refused with ENOMEM before anything is queued."""
    import torch
    from paper_2603_16104_amd import binding as hkv
    n_req, Hq = 2048, 64                                   # 2048 * 64 rows x 2 partials of 264 B = 69 MB > 32 MiB
    parent = [-1] + [0] * n_req
    w_tokens = [16] * (n_req + 1)
    pages = np.arange(n_req + 1, dtype=np.int32)
    f = wl.make_forest(parent, w_tokens, list(range(1, n_req + 1)), pages)
    dp = gpu.DevicePool(n_req + 1, 8, hkv.BF16, poison=False)
    plan = hkv.hkv_decode_plan_create(dp.handle, f.nodes, f.node_pages, f.req_leaf, Hq)
    assert hkv.hkv_decode_plan_workspace_bytes(plan) > hkv.hkv_static_workspace_bytes()
    q = torch.zeros((n_req, Hq, 128), dtype=torch.int16, device="cuda")
    out = torch.zeros_like(q)
    with pytest.raises(hkv.HkvError) as e:
        hkv.attn_decode_plan_run_static(plan, q, 0.1, out, None)
    assert e.value.code == hkv.ENOMEM
    hkv.hkv_decode_plan_destroy(plan)
    dp.close()
