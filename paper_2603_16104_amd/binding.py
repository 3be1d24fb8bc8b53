"""Thin ctypes binding of libheliumkv.so: argument marshalling only.

Function names match the C ABI in include/heliumkv.h.  Device buffers are passed as
torch tensors (their data_ptr() is used) or as raw integer addresses; host arrays as
numpy int32 arrays.  Every step of the path runs inside the library's HIP kernels;
there is no Python or CPU fallback, and loading fails loudly when the library has
not been built.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libheliumkv.so")

OK, EINVAL, ERANGE, ESHAPE, ETREE, ENOMEM, EHIP = 0, -1, -2, -3, -4, -5, -6
BF16, FP8_E4M3, FP32 = 0, 1, 2
PLAN_HOST_ONLY, PLAN_FP8_MATRIX, PLAN_ONE_STREAM = 1, 2, 4
PAGE_SIZE, HEAD_DIM = 16, 128

EXPORTS = [
    "hkv_last_error", "kv_pool_create", "kv_pool_destroy", "kv_pool_alloc", "kv_pool_retain", "kv_pool_release", "kv_pool_copy_on_write",
    "kv_pool_num_free", "kv_pool_page_size", "kv_pool_refcount", "kv_pool_write", "kv_pool_append", "prefix_tree_flatten",
    "hkv_decode_plan_create_growing", "hkv_decode_plan_append", "hkv_decode_plan_append_tokens",
    "prefix_tree_flatten_paged", "prefix_tree_prefill_usage",
    "lse_merge", "hkv_decode_plan_create", "hkv_decode_plan_create_multi", "hkv_decode_plan_create_tree", "hkv_decode_plan_create_ex", "hkv_prefill_plan_create_rows", "hkv_prefill_plan_fallback_tiles", "hkv_decode_plan_destroy", "hkv_decode_plan_workspace_bytes",
    "hkv_decode_plan_num_items", "hkv_decode_plan_num_workgroups", "hkv_decode_plan_num_parts", "hkv_decode_plan_items",
    "hkv_decode_plan_max_parts", "hkv_decode_plan_part_counts", "lse_merge_dense", "attn_decode_plan_run",
    "attn_decode_plan_run_static", "hkv_static_workspace_bytes",
    "hkv_decode_plan_set_profiling", "hkv_decode_plan_elapsed_ms", "hkv_decode_plan_elapsed_kernels_ms",
    "hkv_decode_plan_num_tile_items", "hkv_decode_plan_tile_workgroups", "hkv_decode_plan_is_fused",
    "attn_decode_prefix_tree", "attn_decode_workspace_bytes", "hkv_prefill_plan_create", "hkv_prefill_plan_destroy",
    "hkv_prefill_plan_num_tiles", "hkv_prefill_plan_tiles", "attn_prefill_plan_run", "attn_prefill_plan_run_ws", "hkv_prefill_plan_workspace_bytes", "attn_prefill_with_prefix",
    "attn_prefill_workspace_bytes",
    "kv_cache_create", "kv_cache_destroy", "kv_cache_acquire", "kv_cache_release", "kv_cache_unpin", "kv_cache_stats",
    "trt_build", "trt_destroy", "trt_num_nodes", "trt_num_syms", "trt_num_calls", "trt_nodes", "trt_prefill_usage",
    "trt_evaluate", "trt_schedule", "trt_partition", "trt_nested", "trt_run_soft",
]


class HkvError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"heliumkv error {code}: {msg}")
        self.code = code


class PoolDesc(C.Structure):
    _fields_ = [("num_pages", C.c_int32), ("page_size", C.c_int32), ("num_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("dtype", C.c_int32), ("k_pages", C.c_void_p), ("v_pages", C.c_void_p),
                ("k_scale", C.c_void_p), ("v_scale", C.c_void_p), ("free_order", C.c_void_p)]


_lib = None


def lib():
    """Loads the built library; raises if it is missing (build it with __graft_entry__.build())."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build the HIP library first "
                               "(python -c 'import __graft_entry__ as g; g.build()'); there is no fallback path")
        L = C.CDLL(LIB_PATH)
        L.hkv_last_error.restype = C.c_char_p
        for name in ("hkv_decode_plan_workspace_bytes", "attn_decode_workspace_bytes", "attn_prefill_workspace_bytes",
                     "hkv_prefill_plan_workspace_bytes", "hkv_static_workspace_bytes"):
            getattr(L, name).restype = C.c_size_t
        _lib = L
    return _lib


def last_error() -> str:
    return lib().hkv_last_error().decode()


def _check(rc: int) -> int:
    if rc < 0:
        raise HkvError(rc, last_error())
    return rc


def _dev(t) -> C.c_void_p:
    """Device address of a torch tensor, a raw int address, or None."""
    if t is None:
        return C.c_void_p(None)
    if isinstance(t, int):
        return C.c_void_p(t)
    return C.c_void_p(t.data_ptr())


def _host_i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _hp(a: Optional[np.ndarray]) -> C.c_void_p:
    return C.c_void_p(None) if a is None else a.ctypes.data_as(C.c_void_p)


def _stream(stream) -> C.c_void_p:
    if stream is None:
        import torch
        return C.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return C.c_void_p(stream)
    return C.c_void_p(stream.cuda_stream)


def _nodes(nodes) -> np.ndarray:
    n = np.ascontiguousarray(nodes, dtype=np.int32).reshape(-1, 4)
    return n


# ----------------------------------------------------------------------------------------- pool
def kv_pool_create(num_pages: int, num_kv_heads: int, dtype: int, k_pages, v_pages, k_scale=None, v_scale=None,
                   free_order=None, page_size: int = PAGE_SIZE, head_dim: int = HEAD_DIM) -> C.c_void_p:
    fo = None if free_order is None else _host_i32(free_order)
    d = PoolDesc(num_pages, page_size, num_kv_heads, head_dim, dtype, _dev(k_pages), _dev(v_pages), _dev(k_scale),
                 _dev(v_scale), _hp(fo))
    out = C.c_void_p()
    _check(lib().kv_pool_create(C.byref(d), C.byref(out)))
    return out


def kv_pool_destroy(pool) -> None:
    _check(lib().kv_pool_destroy(pool))


def kv_pool_alloc(pool, n: int) -> np.ndarray:
    ids = np.empty(max(n, 0), dtype=np.int32)
    _check(lib().kv_pool_alloc(pool, C.c_int32(n), _hp(ids)))
    return ids


def kv_pool_retain(pool, ids) -> None:
    ids = _host_i32(ids)
    _check(lib().kv_pool_retain(pool, C.c_int32(len(ids)), _hp(ids)))


def kv_pool_release(pool, ids) -> None:
    ids = _host_i32(ids)
    _check(lib().kv_pool_release(pool, C.c_int32(len(ids)), _hp(ids)))


def kv_pool_copy_on_write(pool, ids, stream=None) -> np.ndarray:
    """Returns the ids to write through: shared pages are replaced by private copies."""
    ids = _host_i32(ids).copy()
    _check(lib().kv_pool_copy_on_write(pool, C.c_int32(len(ids)), _hp(ids), _stream(stream)))
    return ids


def kv_pool_num_free(pool) -> int:
    return _check(lib().kv_pool_num_free(pool))


def kv_pool_page_size(pool) -> int:
    return _check(lib().kv_pool_page_size(pool))


def kv_pool_refcount(pool, page_id: int) -> int:
    return _check(lib().kv_pool_refcount(pool, C.c_int32(page_id)))


def kv_pool_write(pool, page_ids, first_slot: int, n_tokens: int, k_src, v_src, stream=None) -> None:
    ids = _host_i32(page_ids)
    page = kv_pool_page_size(pool)
    need = (first_slot + n_tokens + page - 1) // page if n_tokens > 0 else 0
    if len(ids) < need:
        raise HkvError(EINVAL, f"kv_pool_write: {need} page ids needed, {len(ids)} given")
    _check(lib().kv_pool_write(pool, _hp(ids), C.c_int32(first_slot), C.c_int32(n_tokens), _dev(k_src), _dev(v_src),
                               _stream(stream) if n_tokens > 0 else C.c_void_p(None)))


def kv_pool_append(pool, page_ids, slots, k_src, v_src, stream=None) -> None:
    """One new token for each of len(page_ids) sequences: row i goes to slot slots[i] of page page_ids[i]."""
    ids, sl = _host_i32(page_ids), _host_i32(slots)
    if len(ids) != len(sl):
        raise HkvError(EINVAL, "kv_pool_append: page_ids and slots differ in length")
    _check(lib().kv_pool_append(pool, _hp(ids), _hp(sl), C.c_int32(len(ids)), _dev(k_src), _dev(v_src),
                                _stream(stream) if len(ids) > 0 else C.c_void_p(None)))


# ----------------------------------------------------------------------------------------- forest
def prefix_tree_flatten(nodes, node_pages, req_leaf, max_pages: int, page_size: int = PAGE_SIZE):
    nodes, node_pages, req_leaf = _nodes(nodes), _host_i32(node_pages), _host_i32(req_leaf)
    n_nodes, n_req = nodes.shape[0], req_leaf.shape[0]
    bt = np.empty((n_req, max_pages), dtype=np.int32)
    kv_len = np.empty(n_req, dtype=np.int32)
    indptr = np.empty(n_nodes + 1, dtype=np.int32)
    idx = np.empty(max(1, n_nodes * max(1, n_req)), dtype=np.int32)
    tok_start = np.empty(n_nodes, dtype=np.int32)
    if page_size == PAGE_SIZE:
        _check(lib().prefix_tree_flatten(_hp(nodes), C.c_int32(n_nodes), _hp(node_pages), C.c_int32(len(node_pages)),
                                         _hp(req_leaf), C.c_int32(n_req), C.c_int32(max_pages), _hp(bt), _hp(kv_len),
                                         _hp(indptr), _hp(idx), _hp(tok_start)))
    else:
        _check(lib().prefix_tree_flatten_paged(_hp(nodes), C.c_int32(n_nodes), _hp(node_pages),
                                               C.c_int32(len(node_pages)), _hp(req_leaf), C.c_int32(n_req),
                                               C.c_int32(page_size), C.c_int32(max_pages), _hp(bt), _hp(kv_len),
                                               _hp(indptr), _hp(idx), _hp(tok_start)))
    return bt, kv_len, indptr, idx[: indptr[-1]].copy(), tok_start


def prefix_tree_prefill_usage(nodes, calls) -> np.ndarray:
    nodes, calls = _nodes(nodes), _host_i32(calls)
    out = np.empty(len(calls), dtype=np.int64)
    _check(lib().prefix_tree_prefill_usage(_hp(nodes), C.c_int32(nodes.shape[0]), _hp(calls), C.c_int32(len(calls)),
                                           _hp(out)))
    return out


# ----------------------------------------------------------------------------------------- merge
def lse_merge(o_parts, lse_parts, row_indptr, part_idx, n_rows: int, out, out_dtype: int, lse_out=None,
              stream=None) -> None:
    _check(lib().lse_merge(_dev(o_parts), _dev(lse_parts), _dev(row_indptr), _dev(part_idx), C.c_int32(n_rows),
                           _dev(out), C.c_int32(out_dtype), _dev(lse_out),
                           _stream(stream) if n_rows > 0 else C.c_void_p(None)))


def lse_merge_dense(o_parts, lse_parts, part_count, rows_per_count: int, max_parts: int, n_rows: int, out,
                    out_dtype: int, lse_out=None, stream=None) -> None:
    _check(lib().lse_merge_dense(_dev(o_parts), _dev(lse_parts), _dev(part_count), C.c_int32(rows_per_count),
                                 C.c_int32(max_parts), C.c_int32(n_rows), _dev(out), C.c_int32(out_dtype),
                                 _dev(lse_out), _stream(stream) if n_rows > 0 else C.c_void_p(None)))


# ----------------------------------------------------------------------------------------- decode
def hkv_decode_plan_create_growing(pool, nodes, node_pages, req_leaf, num_q_heads: int, reserve_tokens: int,
                                   flags: int = 0) -> C.c_void_p:
    nodes, node_pages, req_leaf = _nodes(nodes), _host_i32(node_pages), _host_i32(req_leaf)
    out = C.c_void_p()
    _check(lib().hkv_decode_plan_create_growing(pool, _hp(nodes), C.c_int32(nodes.shape[0]), _hp(node_pages),
                                                C.c_int32(len(node_pages)), _hp(req_leaf), C.c_int32(len(req_leaf)),
                                                C.c_int32(num_q_heads), C.c_int32(reserve_tokens), C.c_uint32(flags),
                                                C.byref(out)))
    return out


def hkv_decode_plan_append(plan, new_page_ids=None, stream=None) -> None:
    ids = None if new_page_ids is None else _host_i32(new_page_ids)
    _check(lib().hkv_decode_plan_append(plan, _hp(ids), _stream(stream)))


def hkv_decode_plan_append_tokens(plan, new_page_ids, k_src, v_src, stream=None) -> None:
    ids = None if new_page_ids is None else _host_i32(new_page_ids)
    _check(lib().hkv_decode_plan_append_tokens(plan, _hp(ids), _dev(k_src), _dev(v_src), _stream(stream)))


def hkv_decode_plan_create(pool, nodes, node_pages, req_leaf, num_q_heads: int, flags: int = 0) -> C.c_void_p:
    nodes, node_pages, req_leaf = _nodes(nodes), _host_i32(node_pages), _host_i32(req_leaf)
    out = C.c_void_p()
    _check(lib().hkv_decode_plan_create(pool, _hp(nodes), C.c_int32(nodes.shape[0]), _hp(node_pages),
                                        C.c_int32(len(node_pages)), _hp(req_leaf), C.c_int32(len(req_leaf)),
                                        C.c_int32(num_q_heads), C.c_uint32(flags), C.byref(out)))
    return out


def hkv_decode_plan_create_multi(pool, nodes, node_pages, req_leaf, tokens_per_req: int, num_q_heads: int,
                                 flags: int = 0) -> C.c_void_p:
    nodes, node_pages, req_leaf = _nodes(nodes), _host_i32(node_pages), _host_i32(req_leaf)
    out = C.c_void_p()
    _check(lib().hkv_decode_plan_create_multi(pool, _hp(nodes), C.c_int32(nodes.shape[0]), _hp(node_pages),
                                              C.c_int32(len(node_pages)), _hp(req_leaf), C.c_int32(len(req_leaf)),
                                              C.c_int32(tokens_per_req), C.c_int32(num_q_heads), C.c_uint32(flags),
                                              C.byref(out)))
    return out


def hkv_decode_plan_create_tree(pool, nodes, node_pages, req_leaf, tokens_per_req: int, visible, num_q_heads: int,
                                flags: int = 0) -> C.c_void_p:
    """visible: [n_req * tokens_per_req] uint64 masks over each request's drafted tokens."""
    nodes, node_pages, req_leaf = _nodes(nodes), _host_i32(node_pages), _host_i32(req_leaf)
    visible = np.ascontiguousarray(visible, dtype=np.uint64)
    if len(visible) != len(req_leaf) * tokens_per_req:
        raise ValueError("visible must hold one mask per request and drafted token")
    out = C.c_void_p()
    _check(lib().hkv_decode_plan_create_tree(pool, _hp(nodes), C.c_int32(nodes.shape[0]), _hp(node_pages),
                                             C.c_int32(len(node_pages)), _hp(req_leaf), C.c_int32(len(req_leaf)),
                                             C.c_int32(tokens_per_req), _hp(visible), C.c_int32(num_q_heads),
                                             C.c_uint32(flags), C.byref(out)))
    return out


class DecodePlanParams(C.Structure):
    """hkv_decode_plan_params: what to plan (query tokens per request, visibility masks, room to grow) and the
    planner's settings; every field left 0 keeps the library's choice."""
    _fields_ = [("tokens_per_req", C.c_int32), ("visible", C.c_void_p), ("reserve_tokens", C.c_int32),
                ("q_rows", C.c_void_p)] + [
        (name, C.c_int32) for name in ("leaf_chunk", "shared_chunk", "max_rows", "pack", "pack_tokens", "stages",
                                       "interleave", "tile_min_rows", "tile_min_gflop", "tile_workgroups",
                                       "tile_chunk", "large_batch_updates", "fused")]


def hkv_decode_plan_create_ex(pool, nodes, node_pages, req_leaf, num_q_heads: int, flags: int = 0, visible=None,
                              q_rows=None, **params) -> C.c_void_p:
    """params: fields of hkv_decode_plan_params by name (tokens_per_req, reserve_tokens, leaf_chunk, pack, ...);
    q_rows: the row of q / out / lse of every row of the plan."""
    nodes, node_pages, req_leaf = _nodes(nodes), _host_i32(node_pages), _host_i32(req_leaf)
    st = DecodePlanParams()
    known = {name for name, _ in DecodePlanParams._fields_} - {"visible", "q_rows"}
    for name, value in params.items():
        if name not in known:
            raise TypeError(f"hkv_decode_plan_create_ex: no setting named {name!r}")
        setattr(st, name, int(value))
    if visible is not None:
        visible = np.ascontiguousarray(visible, dtype=np.uint64)
        if len(visible) != len(req_leaf) * max(1, st.tokens_per_req):
            raise ValueError("visible must hold one mask per request and drafted token")
        st.visible = visible.ctypes.data
    if q_rows is not None:
        q_rows = _host_i32(q_rows)
        if len(q_rows) != len(req_leaf) * max(1, st.tokens_per_req):
            raise ValueError("q_rows must hold one row per request and query token")
        st.q_rows = q_rows.ctypes.data
    out = C.c_void_p()
    _check(lib().hkv_decode_plan_create_ex(pool, _hp(nodes), C.c_int32(nodes.shape[0]), _hp(node_pages),
                                           C.c_int32(len(node_pages)), _hp(req_leaf), C.c_int32(len(req_leaf)),
                                           C.c_int32(num_q_heads), C.c_uint32(flags), C.byref(st), C.byref(out)))
    return out


def hkv_decode_plan_destroy(plan) -> None:
    _check(lib().hkv_decode_plan_destroy(plan))


def hkv_decode_plan_workspace_bytes(plan) -> int:
    return int(lib().hkv_decode_plan_workspace_bytes(plan))


def hkv_decode_plan_items(plan) -> np.ndarray:
    n = _check(lib().hkv_decode_plan_num_items(plan))
    items = np.empty((n, 8), dtype=np.int32)
    _check(lib().hkv_decode_plan_items(plan, _hp(items)))
    return items


def hkv_decode_plan_num_workgroups(plan) -> int:
    return _check(lib().hkv_decode_plan_num_workgroups(plan))


def hkv_decode_plan_num_parts(plan) -> int:
    return _check(lib().hkv_decode_plan_num_parts(plan))


def hkv_decode_plan_max_parts(plan) -> int:
    return _check(lib().hkv_decode_plan_max_parts(plan))


def hkv_decode_plan_part_counts(plan, n_req: int) -> np.ndarray:
    cnt = np.empty(n_req, dtype=np.int32)
    _check(lib().hkv_decode_plan_part_counts(plan, _hp(cnt)))
    return cnt


def attn_decode_plan_run(plan, q, scale: float, out, lse_out, workspace, workspace_bytes: int, stream=None) -> None:
    _check(lib().attn_decode_plan_run(plan, _dev(q), C.c_float(scale), _dev(out), _dev(lse_out), _dev(workspace),
                                      C.c_size_t(workspace_bytes), _stream(stream)))


def hkv_static_workspace_bytes() -> int:
    return int(lib().hkv_static_workspace_bytes())


def attn_decode_plan_run_static(plan, q, scale: float, out, lse_out, stream=None) -> None:
    _check(lib().attn_decode_plan_run_static(plan, _dev(q), C.c_float(scale), _dev(out), _dev(lse_out), _stream(stream)))


def hkv_decode_plan_set_profiling(plan, mode) -> None:
    """mode: 0/False off, 1/True begin and end events on both kernel dispatches."""
    _check(lib().hkv_decode_plan_set_profiling(plan, C.c_int32(int(mode))))


def hkv_decode_plan_elapsed_ms(plan):
    a, b = C.c_float(), C.c_float()
    _check(lib().hkv_decode_plan_elapsed_ms(plan, C.byref(a), C.byref(b)))
    return float(a.value), float(b.value)


def hkv_decode_plan_elapsed_kernels_ms(plan):
    """(kernel over the few-row items, tile kernel) of the most recent profiled run, milliseconds."""
    a, b = C.c_float(), C.c_float()
    _check(lib().hkv_decode_plan_elapsed_kernels_ms(plan, C.byref(a), C.byref(b)))
    return float(a.value), float(b.value)


def hkv_decode_plan_num_tile_items(plan) -> int:
    return _check(lib().hkv_decode_plan_num_tile_items(plan))


def hkv_decode_plan_is_fused(plan) -> bool:
    return bool(lib().hkv_decode_plan_is_fused(plan))


def hkv_decode_plan_tile_workgroups(plan) -> int:
    return _check(lib().hkv_decode_plan_tile_workgroups(plan))


def attn_decode_prefix_tree(pool, q, nodes, node_pages, req_leaf, num_q_heads: int, scale: float, out, lse_out,
                            workspace, workspace_bytes: int, stream=None) -> None:
    nodes, node_pages, req_leaf = _nodes(nodes), _host_i32(node_pages), _host_i32(req_leaf)
    _check(lib().attn_decode_prefix_tree(pool, _dev(q), _hp(nodes), C.c_int32(nodes.shape[0]), _hp(node_pages),
                                         C.c_int32(len(node_pages)), _hp(req_leaf), C.c_int32(len(req_leaf)),
                                         C.c_int32(num_q_heads), C.c_float(scale), _dev(out), _dev(lse_out),
                                         _dev(workspace), C.c_size_t(workspace_bytes), _stream(stream)))


def attn_decode_workspace_bytes(pool, nodes, node_pages, req_leaf, num_q_heads: int) -> int:
    nodes, node_pages, req_leaf = _nodes(nodes), _host_i32(node_pages), _host_i32(req_leaf)
    n = int(lib().attn_decode_workspace_bytes(pool, _hp(nodes), C.c_int32(nodes.shape[0]), _hp(node_pages),
                                              C.c_int32(len(node_pages)), _hp(req_leaf), C.c_int32(len(req_leaf)),
                                              C.c_int32(num_q_heads)))
    return n


# ----------------------------------------------------------------------------------------- prefill
def hkv_prefill_plan_create(pool, cu_q, block_table, kv_len, num_q_heads: int, flags: int = 0) -> C.c_void_p:
    cu_q, kv_len = _host_i32(cu_q), _host_i32(kv_len)
    bt = _host_i32(block_table).reshape(len(kv_len), -1) if len(kv_len) else _host_i32(block_table).reshape(0, 0)
    out = C.c_void_p()
    _check(lib().hkv_prefill_plan_create(pool, _hp(cu_q), _hp(bt), C.c_int32(bt.shape[1] if bt.ndim == 2 else 0),
                                         _hp(kv_len), C.c_int32(len(kv_len)), C.c_int32(num_q_heads),
                                         C.c_uint32(flags), C.byref(out)))
    return out


def hkv_prefill_plan_create_rows(pool, q_row_begin, q_len, block_table, kv_len, num_q_heads: int,
                                 flags: int = 0) -> C.c_void_p:
    q_row_begin, q_len, kv_len = _host_i32(q_row_begin), _host_i32(q_len), _host_i32(kv_len)
    if not len(q_row_begin) == len(q_len) == len(kv_len):
        raise ValueError("q_row_begin, q_len and kv_len hold one entry per request")
    bt = _host_i32(block_table).reshape(len(kv_len), -1) if len(kv_len) else _host_i32(block_table).reshape(0, 0)
    out = C.c_void_p()
    _check(lib().hkv_prefill_plan_create_rows(pool, _hp(q_row_begin), _hp(q_len), _hp(bt),
                                              C.c_int32(bt.shape[1] if bt.ndim == 2 else 0), _hp(kv_len),
                                              C.c_int32(len(kv_len)), C.c_int32(num_q_heads), C.c_uint32(flags),
                                              C.byref(out)))
    return out


def hkv_prefill_plan_fallback_tiles(plan) -> int:
    n = C.c_int64()
    _check(lib().hkv_prefill_plan_fallback_tiles(plan, C.byref(n)))
    return int(n.value)


def hkv_prefill_plan_destroy(plan) -> None:
    _check(lib().hkv_prefill_plan_destroy(plan))


def hkv_prefill_plan_tiles(plan) -> np.ndarray:
    n = _check(lib().hkv_prefill_plan_num_tiles(plan))
    tiles = np.empty((n, 8), dtype=np.int32)
    _check(lib().hkv_prefill_plan_tiles(plan, _hp(tiles)))
    return tiles


def attn_prefill_plan_run(plan, q, scale: float, out, lse_out=None, stream=None, workspace=None,
                          workspace_bytes: int = 0) -> None:
    """workspace: device scratch of hkv_prefill_plan_workspace_bytes(plan) bytes (fp8 pools only)."""
    _check(lib().attn_prefill_plan_run_ws(plan, _dev(q), C.c_float(scale), _dev(out), _dev(lse_out), _dev(workspace),
                                          C.c_size_t(workspace_bytes), _stream(stream)))


def hkv_prefill_plan_workspace_bytes(plan) -> int:
    return int(lib().hkv_prefill_plan_workspace_bytes(plan))


def attn_prefill_with_prefix(pool, q, cu_q, block_table, kv_len, num_q_heads: int, scale: float, out, lse_out=None,
                             workspace=None, workspace_bytes: int = 0, stream=None) -> None:
    cu_q, kv_len = _host_i32(cu_q), _host_i32(kv_len)
    bt = _host_i32(block_table).reshape(len(kv_len), -1) if len(kv_len) else _host_i32(block_table).reshape(0, 0)
    _check(lib().attn_prefill_with_prefix(pool, _dev(q), _hp(cu_q), _hp(bt), C.c_int32(bt.shape[1]), _hp(kv_len),
                                          C.c_int32(len(kv_len)), C.c_int32(num_q_heads), C.c_float(scale), _dev(out),
                                          _dev(lse_out), _dev(workspace), C.c_size_t(workspace_bytes),
                                          _stream(stream)))


def attn_prefill_workspace_bytes(total_q: int, num_q_heads: int) -> int:
    return int(lib().attn_prefill_workspace_bytes(C.c_int32(total_q), C.c_int32(num_q_heads)))


# ---------------------------------------------------------------------------------------------
# scheduling layer (host only)


def _host_i64(n: int) -> np.ndarray:
    return np.zeros(max(n, 0), dtype=np.int64)


def trt_build(templates, len_out, worker=None) -> C.c_void_p:
    """templates: list of int sequences (symbols); returns the tree handle."""
    indptr = np.zeros(len(templates) + 1, dtype=np.int32)
    for i, t in enumerate(templates):
        indptr[i + 1] = indptr[i] + len(t)
    syms = _host_i32([s for t in templates for s in t])
    lo = _host_i32(len_out)
    wk = _host_i32(worker) if worker is not None else None
    out = C.c_void_p()
    _check(lib().trt_build(_hp(indptr), _hp(syms), _hp(lo), _hp(wk) if wk is not None else None,
                           C.c_int32(len(templates)), C.byref(out)))
    return out


def trt_destroy(tree) -> None:
    _check(lib().trt_destroy(tree))


def trt_nodes(tree) -> dict:
    n, ns, nc = (_check(lib().trt_num_nodes(tree)), _check(lib().trt_num_syms(tree)), _check(lib().trt_num_calls(tree)))
    parent, call, sb, sl = (np.zeros(n, dtype=np.int32) for _ in range(4))
    weight = _host_i64(n)
    syms, leaf = np.zeros(ns, dtype=np.int32), np.zeros(nc, dtype=np.int32)
    _check(lib().trt_nodes(tree, _hp(parent), _hp(weight), _hp(call), _hp(sb), _hp(sl), _hp(syms), _hp(leaf)))
    return {"parent": parent, "weight": weight, "call": call, "seg_begin": sb, "seg_len": sl, "syms": syms,
            "leaf_of_call": leaf}


def trt_prefill_usage(tree, calls) -> np.ndarray:
    calls = _host_i32(calls)
    u = _host_i64(len(calls))
    _check(lib().trt_prefill_usage(tree, _hp(calls), C.c_int32(len(calls)), _hp(u)))
    return u


def _sigma_arrays(sigma):
    indptr = np.zeros(len(sigma) + 1, dtype=np.int32)
    for i, s in enumerate(sigma):
        indptr[i + 1] = indptr[i] + len(s)
    return indptr, _host_i32([c for s in sigma for c in s])


def trt_evaluate(tree, sigma, capacity: int):
    """sigma: one list of calls per worker.  Returns (B, C, T)."""
    nc = _check(lib().trt_num_calls(tree))
    indptr, flat = _sigma_arrays(sigma)
    B, Cc, T = _host_i64(nc), _host_i64(nc), C.c_int64(0)
    _check(lib().trt_evaluate(tree, _hp(indptr), _hp(flat), C.c_int32(len(sigma)), C.c_int64(capacity), _hp(B),
                              _hp(Cc), C.byref(T)))
    return B, Cc, int(T.value)


def trt_schedule(tree, n_workers: int, capacity: int):
    """Returns (sigma as a list of lists, B, C, T)."""
    nc = _check(lib().trt_num_calls(tree))
    indptr, flat = np.zeros(n_workers + 1, dtype=np.int32), np.zeros(nc, dtype=np.int32)
    B, Cc, T = _host_i64(nc), _host_i64(nc), C.c_int64(0)
    _check(lib().trt_schedule(tree, C.c_int32(n_workers), C.c_int64(capacity), _hp(indptr), _hp(flat), _hp(B), _hp(Cc),
                              C.byref(T)))
    return [flat[indptr[i]:indptr[i + 1]].tolist() for i in range(n_workers)], B, Cc, int(T.value)


def trt_partition(templates, len_out, n_workers: int) -> np.ndarray:
    """Worker of every call (PartitionWorkflow)."""
    indptr = np.zeros(len(templates) + 1, dtype=np.int32)
    for i, t in enumerate(templates):
        indptr[i + 1] = indptr[i] + len(t)
    syms = _host_i32([s for t in templates for s in t])
    lo = _host_i32(len_out)
    worker = np.zeros(len(templates), dtype=np.int32)
    _check(lib().trt_partition(_hp(indptr), _hp(syms), _hp(lo), C.c_int32(len(templates)), C.c_int32(n_workers),
                               _hp(worker)))
    return worker


def trt_nested(tree, sigma):
    """sigma: one list of calls per worker.  Returns per worker the list of inner sequences (lists of calls)."""
    nc = _check(lib().trt_num_calls(tree))
    indptr, flat = _sigma_arrays(sigma)
    seq_indptr = np.zeros(len(sigma) + 1, dtype=np.int32)
    seq_begin, nested = np.zeros(nc + 1, dtype=np.int32), np.zeros(nc, dtype=np.int32)
    _check(lib().trt_nested(tree, _hp(indptr), _hp(flat), C.c_int32(len(sigma)), _hp(seq_indptr), _hp(seq_begin),
                            _hp(nested)))
    return [[nested[seq_begin[s]:seq_begin[s + 1]].tolist() for s in range(seq_indptr[i], seq_indptr[i + 1])]
            for i in range(len(sigma))]


def trt_run_soft(tree, order, capacity: int):
    """order: one priority list of calls per worker.  Returns (realised sigma, B, C, T)."""
    nc = _check(lib().trt_num_calls(tree))
    indptr, flat = _sigma_arrays(order)
    sigma = np.zeros(nc, dtype=np.int32)
    B, Cc, T = _host_i64(nc), _host_i64(nc), C.c_int64(0)
    _check(lib().trt_run_soft(tree, _hp(indptr), _hp(flat), C.c_int32(len(order)), C.c_int64(capacity), _hp(sigma),
                              _hp(B), _hp(Cc), C.byref(T)))
    return [sigma[indptr[i]:indptr[i + 1]].tolist() for i in range(len(order))], B, Cc, int(T.value)


# ---------------------------------------------------------------------------------------------
# block-level prefix cache (host only)


def kv_cache_create(pool) -> C.c_void_p:
    out = C.c_void_p()
    _check(lib().kv_cache_create(pool, C.byref(out)))
    return out


def kv_cache_destroy(cache) -> None:
    _check(lib().kv_cache_destroy(cache))


def kv_cache_acquire(cache, tokens, pin: bool = False, page_size: int = PAGE_SIZE):
    """Returns (page ids of the sequence's blocks, number of leading tokens already cached);
    page_size is the page size of the pool the cache was created over."""
    tokens = _host_i32(tokens)
    pages = np.zeros((len(tokens) + page_size - 1) // page_size, dtype=np.int32)
    cached = C.c_int32(0)
    _check(lib().kv_cache_acquire(cache, _hp(tokens), C.c_int32(len(tokens)), C.c_int32(1 if pin else 0), _hp(pages),
                                  C.byref(cached)))
    return pages, int(cached.value)


def kv_cache_release(cache, pages) -> None:
    pages = _host_i32(pages)
    _check(lib().kv_cache_release(cache, _hp(pages), C.c_int32(len(pages))))


def kv_cache_unpin(cache, pages) -> None:
    pages = _host_i32(pages)
    _check(lib().kv_cache_unpin(cache, _hp(pages), C.c_int32(len(pages))))


def kv_cache_stats(cache) -> dict:
    v = [C.c_int64(0) for _ in range(4)]
    _check(lib().kv_cache_stats(cache, *[C.byref(x) for x in v]))
    return dict(zip(("cached_blocks", "hits", "misses", "evictions"), (int(x.value) for x in v)))
