"""Device-memory plumbing around the C ABI: torch owns the HBM buffers and streams, the
library does all the work.  Used by the tests, the smoke check and the bench."""
from __future__ import annotations

from typing import Optional

import numpy as np
import torch

from . import binding as hkv
from . import workloads as wl

# bf16 bit patterns travel as int16 tensors (full torch support); 0x7FC0 is a bf16 NaN, 0x7F the e4m3 NaN
_ELEM = {hkv.BF16: (torch.int16, 0x7FC0), hkv.FP8_E4M3: (torch.uint8, 0x7F)}


class DevicePool:
    """A KV page pool in HBM (library storage format), NaN-poisoned until written."""

    def __init__(self, num_pages: int, num_kv_heads: int, dtype: int, device: str = "cuda:0",
                 free_order: Optional[np.ndarray] = None, poison: bool = True):
        self.num_pages, self.num_kv_heads, self.dtype = num_pages, num_kv_heads, dtype
        tdt, nan_bits = _ELEM[dtype]
        n = num_pages * num_kv_heads * hkv.PAGE_SIZE * hkv.HEAD_DIM
        fill = nan_bits if poison else 0
        self.k = torch.full((n,), fill, dtype=tdt, device=device)
        self.v = torch.full((n,), fill, dtype=tdt, device=device)
        self.k_scale = self.v_scale = None
        if dtype == hkv.FP8_E4M3:
            sv = float("nan") if poison else 1.0
            self.k_scale = torch.full((num_pages * num_kv_heads,), sv, dtype=torch.float32, device=device)
            self.v_scale = torch.full((num_pages * num_kv_heads,), sv, dtype=torch.float32, device=device)
        self.handle = hkv.kv_pool_create(num_pages, num_kv_heads, dtype, self.k, self.v, self.k_scale, self.v_scale,
                                         free_order)

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

    def fill_from(self, workload: wl.Workload, max_chunk_tokens: int = 1 << 16) -> None:
        """kv_pool_write of every node's own tokens into the node's pages."""
        f = workload.forest
        dev = self.k.device
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
                self.write(pages[t0 // 16:], 0, kd, vd)
        torch.cuda.synchronize()


def to_device_bits(a: np.ndarray, device="cuda:0") -> torch.Tensor:
    """Host array -> device tensor; uint16 bf16 bit patterns are carried as int16."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(a).to(device)


def bf16_tensor_to_f64(t: torch.Tensor) -> np.ndarray:
    """bf16 bit patterns (int16 device tensor) -> float64 numpy."""
    b = t.cpu().numpy().view(np.uint16)
    return wl.bf16_bits_to_f32(b).astype(np.float64)


class DecodeRunner:
    """Plan + buffers for repeated decode steps over one forest."""

    def __init__(self, pool: DevicePool, workload: wl.Workload):
        f = workload.forest
        self.pool, self.workload = pool, workload
        self.plan = hkv.hkv_decode_plan_create(pool.handle, f.nodes, f.node_pages, f.req_leaf, workload.num_q_heads)
        self.ws_bytes = hkv.hkv_decode_plan_workspace_bytes(self.plan)
        dev = pool.k.device
        self.ws = torch.empty(max(self.ws_bytes, 256), dtype=torch.uint8, device=dev)
        self.q = to_device_bits(workload.q(), dev)
        self.out = torch.zeros((f.n_req, workload.num_q_heads, hkv.HEAD_DIM), dtype=torch.int16, device=dev)
        self.lse = torch.zeros((f.n_req, workload.num_q_heads), dtype=torch.float32, device=dev)
        self.scale = float(workload.scale)

    def run(self, stream=None) -> None:
        hkv.attn_decode_plan_run(self.plan, self.q, self.scale, self.out, self.lse, self.ws, self.ws_bytes, stream)

    def close(self) -> None:
        if self.plan is not None:
            hkv.hkv_decode_plan_destroy(self.plan)
            self.plan = None


class PrefillRunner:
    def __init__(self, pool: DevicePool, workload: wl.Workload):
        f = workload.forest
        self.pool, self.workload = pool, workload
        mp = max(1, f.max_pages_per_req())
        self.block_table, self.kv_len, *_ = hkv.prefix_tree_flatten(f.nodes, f.node_pages, f.req_leaf, mp)
        self.cu_q = workload.cu_q()
        self.plan = hkv.hkv_prefill_plan_create(pool.handle, self.cu_q, self.block_table, self.kv_len,
                                                workload.num_q_heads)
        dev = pool.k.device
        tq = workload.total_q()
        self.q = to_device_bits(workload.q(), dev)
        self.out = torch.zeros((tq, workload.num_q_heads, hkv.HEAD_DIM), dtype=torch.int16, device=dev)
        self.lse = torch.zeros((tq, workload.num_q_heads), dtype=torch.float32, device=dev)
        self.scale = float(workload.scale)

    def run(self, stream=None) -> None:
        hkv.attn_prefill_plan_run(self.plan, self.q, self.scale, self.out, self.lse, stream)

    def close(self) -> None:
        if self.plan is not None:
            hkv.hkv_prefill_plan_destroy(self.plan)
            self.plan = None
