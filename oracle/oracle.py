"""ctypes front end of the CPU oracle (oracle/oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
bench's cpu_baseline leg.  The product package never imports this module.
It marshals numpy arrays into the C functions and holds a host copy of a KV
pool; it contains no attention arithmetic of its own.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle.so")
_SRC = os.path.join(_HERE, "oracle.c")

BF16, FP8_E4M3, FP32 = 0, 1, 2
PAGE, D = 16, 128


def build(force: bool = False) -> str:
    """Compile oracle.c with gcc (double precision, OpenMP over independent rows)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", _SO, _SRC, "-lm"])
    return _SO


class _Pool(C.Structure):
    _fields_ = [("num_pages", C.c_int32), ("num_kv_heads", C.c_int32), ("dtype", C.c_int32),
                ("page_size", C.c_int32), ("k_pages", C.c_void_p), ("v_pages", C.c_void_p),
                ("k_scale", C.c_void_p), ("v_scale", C.c_void_p)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_SO)
        L.orc_e4m3_value.restype = C.c_double
        L.orc_e4m3_value.argtypes = [C.c_uint8]
        L.orc_e4m3_encode.restype = C.c_uint8
        L.orc_e4m3_encode.argtypes = [C.c_float]
        L.oracle_num_threads.restype = C.c_int
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    if a is None:
        return None
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.c_void_p)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _elem_np(dtype: int):
    return {BF16: np.uint16, FP8_E4M3: np.uint8, FP32: np.float32}[dtype]


def _src_dtype(a: np.ndarray) -> int:
    if a.dtype == np.uint16:
        return BF16
    if a.dtype == np.float32:
        return FP32
    raise TypeError(f"expected uint16 (bf16 bits) or float32, got {a.dtype}")


class HostPool:
    """Host copy of a KV page pool in the library's documented storage format.

    Unused pages and slots are filled with NaN so that anything read by mistake shows."""

    def __init__(self, num_pages: int, num_kv_heads: int, dtype: int, poison: bool = True, page_size: int = PAGE):
        assert page_size in (16, 32, 64, 128)
        self.num_pages, self.num_kv_heads, self.dtype, self.page_size = num_pages, num_kv_heads, dtype, page_size
        n = num_pages * num_kv_heads * page_size * D
        et = _elem_np(dtype)
        if dtype == BF16:
            fill = 0x7FC0 if poison else 0
        elif dtype == FP8_E4M3:
            fill = 0x7F if poison else 0
        else:
            fill = np.nan if poison else 0.0
        self.k = np.full(n, fill, dtype=et)
        self.v = np.full(n, fill, dtype=et)
        self.k_scale = self.v_scale = None
        if dtype == FP8_E4M3:
            n_sc = num_pages * (page_size // PAGE) * num_kv_heads      # one scale per 16-slot block and head
            self.k_scale = np.full(n_sc, np.nan if poison else 1.0, dtype=np.float32)
            self.v_scale = np.full(n_sc, np.nan if poison else 1.0, dtype=np.float32)

    def _c(self) -> _Pool:
        return _Pool(self.num_pages, self.num_kv_heads, self.dtype, self.page_size, _p(self.k), _p(self.v),
                     _p(self.k_scale), _p(self.v_scale))

    def write(self, page_ids, first_slot: int, k_src: np.ndarray, v_src: np.ndarray) -> None:
        page_ids = _i32(page_ids)
        k_src, v_src = np.ascontiguousarray(k_src), np.ascontiguousarray(v_src)
        n_tokens = k_src.shape[0]
        assert k_src.shape == v_src.shape == (n_tokens, self.num_kv_heads, D)
        assert len(page_ids) >= (first_slot + n_tokens + self.page_size - 1) // self.page_size
        pc = self._c()
        rc = lib().oracle_kv_write(C.byref(pc), _p(self.k), _p(self.v), _p(self.k_scale), _p(self.v_scale),
                                   _p(page_ids), C.c_int32(first_slot), C.c_int32(n_tokens), _p(k_src),
                                   _p(v_src), C.c_int32(_src_dtype(k_src)))
        if rc:
            raise ValueError(f"oracle_kv_write failed: {rc}")

    def copy_page(self, src: int, dst: int) -> None:
        """Private copy of a whole page (every head's K and V block and, for fp8, its scales): what a
        forked sequence needs before it continues inside a partially filled page others still hold."""
        n = self.num_kv_heads * self.page_size * D
        self.k[dst * n:(dst + 1) * n] = self.k[src * n:(src + 1) * n]
        self.v[dst * n:(dst + 1) * n] = self.v[src * n:(src + 1) * n]
        if self.k_scale is not None:
            h = self.num_kv_heads * (self.page_size // PAGE)
            self.k_scale[dst * h:(dst + 1) * h] = self.k_scale[src * h:(src + 1) * h]
            self.v_scale[dst * h:(dst + 1) * h] = self.v_scale[src * h:(src + 1) * h]

    def fill_from(self, workload) -> None:
        """Write every node's own tokens into the node's pages."""
        f = workload.forest
        for v in range(f.n_nodes):
            if f.n_tokens[v] == 0:
                continue
            k, vv = workload.node_kv(v)
            self.write(f.node_pages[f.page_begin[v]: f.page_begin[v] + f.n_pages[v]], 0, k, vv)


def flatten_tree(nodes, node_pages, req_leaf, max_pages: int, page_size: int = PAGE):
    nodes, node_pages, req_leaf = _i32(nodes).reshape(-1, 4), _i32(node_pages), _i32(req_leaf)
    n_nodes, n_req = nodes.shape[0], req_leaf.shape[0]
    bt = np.empty((n_req, max_pages), dtype=np.int32)
    kv_len = np.empty(n_req, dtype=np.int32)
    indptr = np.empty(n_nodes + 1, dtype=np.int32)
    idx = np.empty(max(1, n_nodes * max(1, n_req)), dtype=np.int32)
    tok_start = np.empty(n_nodes, dtype=np.int32)
    rc = lib().oracle_flatten_tree(_p(nodes), C.c_int32(n_nodes), _p(node_pages), C.c_int32(len(node_pages)),
                                   _p(req_leaf), C.c_int32(n_req), C.c_int32(page_size), C.c_int32(max_pages),
                                   _p(bt), _p(kv_len),
                                   _p(indptr), _p(idx), _p(tok_start))
    if rc:
        raise ValueError(f"oracle_flatten_tree failed: {rc}")
    return bt, kv_len, indptr, idx[: indptr[-1]].copy(), tok_start


def prefill_usage(nodes, calls) -> np.ndarray:
    nodes, calls = _i32(nodes).reshape(-1, 4), _i32(calls)
    out = np.empty(len(calls), dtype=np.int64)
    rc = lib().oracle_prefill_usage(_p(nodes), C.c_int32(nodes.shape[0]), _p(calls), C.c_int32(len(calls)), _p(out))
    if rc:
        raise ValueError(f"oracle_prefill_usage failed: {rc}")
    return out


def attn_decode(pool: HostPool, q: np.ndarray, block_table, kv_len, scale: float,
                seg: Optional[Tuple[np.ndarray, np.ndarray]] = None):
    q = np.ascontiguousarray(q)
    block_table, kv_len = _i32(block_table), _i32(kv_len)
    n_req, Hq = q.shape[0], q.shape[1]
    assert q.shape[2] == D and block_table.shape[0] == n_req
    out = np.empty((n_req, Hq, D), dtype=np.float64)
    lse = np.empty((n_req, Hq), dtype=np.float64)
    sb = se = None
    if seg is not None:
        sb, se = _i32(seg[0]), _i32(seg[1])
    pc = pool._c()
    rc = lib().oracle_attn_decode(C.byref(pc), _p(q), C.c_int32(_src_dtype(q)), _p(block_table),
                                  C.c_int32(block_table.shape[1]), _p(kv_len), _p(sb), _p(se), C.c_int32(n_req),
                                  C.c_int32(Hq), C.c_float(scale), _p(out), _p(lse))
    if rc:
        raise ValueError(f"oracle_attn_decode failed: {rc}")
    return out, lse


def attn_decode_tree(pool: HostPool, q: np.ndarray, nodes, node_pages, req_leaf, scale: float, leaf_visible=None,
                     tail_len: int = 0, tail_mask=None):
    """One query token per request over the token segments on its root-to-leaf path, read straight from
    the forest (nodes may end inside a page anywhere).  leaf_visible[r]: how many tokens of its last node
    request r sees (default: all).  tail_len / tail_mask[r]: the last tail_len tokens of the last node
    are drafted tokens of which request r sees number j iff bit j of tail_mask[r] is set."""
    q = np.ascontiguousarray(q)
    nodes, node_pages, req_leaf = _i32(nodes).reshape(-1, 4), _i32(node_pages), _i32(req_leaf)
    n_req, Hq = q.shape[0], q.shape[1]
    assert q.shape[2] == D and len(req_leaf) == n_req
    out = np.empty((n_req, Hq, D), dtype=np.float64)
    lse = np.empty((n_req, Hq), dtype=np.float64)
    lv = None if leaf_visible is None else _i32(leaf_visible)
    tm = None if tail_mask is None else np.ascontiguousarray(tail_mask, dtype=np.uint64)
    assert tm is None or len(tm) == n_req
    pc = pool._c()
    rc = lib().oracle_attn_decode_tree(C.byref(pc), _p(q), C.c_int32(_src_dtype(q)), _p(nodes), C.c_int32(nodes.shape[0]),
                                       _p(node_pages), C.c_int32(len(node_pages)), _p(req_leaf), _p(lv),
                                       C.c_int32(tail_len), _p(tm), C.c_int32(n_req), C.c_int32(Hq), C.c_float(scale),
                                       _p(out), _p(lse))
    if rc:
        raise ValueError(f"oracle_attn_decode_tree failed: {rc}")
    return out, lse


def attn_prefill(pool: HostPool, q: np.ndarray, cu_q, block_table, kv_len, scale: float):
    q = np.ascontiguousarray(q)
    cu_q, block_table, kv_len = _i32(cu_q), _i32(block_table), _i32(kv_len)
    total, Hq = q.shape[0], q.shape[1]
    n_req = len(kv_len)
    assert int(cu_q[-1]) == total
    out = np.empty((total, Hq, D), dtype=np.float64)
    lse = np.empty((total, Hq), dtype=np.float64)
    pc = pool._c()
    rc = lib().oracle_attn_prefill(C.byref(pc), _p(q), C.c_int32(_src_dtype(q)), _p(cu_q), _p(block_table),
                                   C.c_int32(block_table.shape[1]), _p(kv_len), C.c_int32(n_req), C.c_int32(Hq),
                                   C.c_float(scale), _p(out), _p(lse))
    if rc:
        raise ValueError(f"oracle_attn_prefill failed: {rc}")
    return out, lse


def gather_kv(pool: HostPool, pages, kv_len: int):
    """K and V of one sequence as double arrays [kv_len][Hkv][128] (read through the page list)."""
    pages = _i32(pages)
    k = np.empty((kv_len, pool.num_kv_heads, D), dtype=np.float64)
    v = np.empty_like(k)
    pc = pool._c()
    rc = lib().oracle_gather_kv(C.byref(pc), _p(pages), C.c_int32(kv_len), _p(k), _p(v))
    if rc:
        raise ValueError(f"oracle_gather_kv failed: {rc}")
    return k, v


def _q_as_double(q: np.ndarray) -> np.ndarray:
    if q.dtype == np.uint16:       # bf16 bit patterns
        return (q.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return q.astype(np.float64)


def attn_matrix_form(pool: HostPool, q: np.ndarray, cu_q, block_table, kv_len, scale: float, requests=None,
                     tokens=None):
    """Suffix attention of whole requests with matrix products as steps (Section 5: a call computes its
    uncached suffix against the whole prompt): request r brings s_r = cu_q[r+1] - cu_q[r] query tokens at
    positions kv_len_r - s_r ..; token i of them sees keys 0 .. kv_len_r - s_r + i.  Per request and KV head
    S = scale * Q K^T, masked, m = row max, P = exp(S - m), l = row sum, O = P V / l, lse = m + ln l:
    the same definition as oracle_attn_prefill / oracle_attn_decode (s_r = 1), evaluated for all rows of a
    request at once, so that complete requests of the large configurations finish in seconds.
    requests: which requests to compute (default all); tokens: {request: indices of its new tokens to compute}
    for requests of which only some rows are wanted (default: all of a request's tokens).
    Returns (out [rows][Hq][128], lse [rows][Hq], rows) with rows = the global q row of every computed row,
    in order."""
    cu_q, block_table, kv_len = _i32(cu_q), _i32(block_table), _i32(kv_len)
    Hq, Hk = q.shape[1], pool.num_kv_heads
    G = Hq // Hk
    requests = range(len(kv_len)) if requests is None else requests
    outs, lses, rows = [], [], []
    sc = float(np.float32(scale))
    for r in requests:
        a, b = int(cu_q[r]), int(cu_q[r + 1])
        s, T = b - a, int(kv_len[r])
        which = np.arange(s) if tokens is None or r not in tokens else np.asarray(tokens[r], dtype=np.int64)
        assert ((which >= 0) & (which < s)).all()
        k, v = gather_kv(pool, block_table[r], T)
        qd = _q_as_double(q[a + which])                             # [n][Hq][128]
        o = np.zeros((len(which), Hq, D))
        l_ = np.full((len(which), Hq), -np.inf)
        if T > 0 and len(which):
            visible = np.arange(T)[None, :] <= (T - s + which)[:, None]             # [n][T]
            for j in range(Hk):                                     # KV head j serves q heads j*G .. j*G + G - 1
                kh, vh = np.ascontiguousarray(k[:, j, :]), np.ascontiguousarray(v[:, j, :])     # [T][128]
                for h in range(j * G, (j + 1) * G):
                    S = sc * (np.ascontiguousarray(qd[:, h, :]) @ kh.T)     # [n][T]
                    S[~visible] = -np.inf
                    m = S.max(axis=1, keepdims=True)
                    P = np.exp(S - m)
                    l = P.sum(axis=1, keepdims=True)
                    o[:, h, :] = (P @ vh) / l
                    l_[:, h] = (m + np.log(l))[:, 0]
        outs.append(o)
        lses.append(l_)
        rows.append(a + which)
    if not outs:
        return np.zeros((0, Hq, D)), np.zeros((0, Hq)), np.zeros(0, dtype=np.int64)
    return np.concatenate(outs), np.concatenate(lses), np.concatenate(rows)


def attn_probs(pool: HostPool, q_row: np.ndarray, pages, kv_len: int, q_head: int, num_q_heads: int, scale: float):
    """q_row: [Hq][128] of one token; returns the softmax weights over the kv_len tokens."""
    q_row, pages = np.ascontiguousarray(q_row), _i32(pages)
    probs = np.empty(kv_len, dtype=np.float64)
    pc = pool._c()
    lib().oracle_attn_probs(C.byref(pc), _p(q_row), C.c_int32(_src_dtype(q_row)), _p(pages), C.c_int32(kv_len),
                            C.c_int32(q_head), C.c_int32(num_q_heads), C.c_float(scale), _p(probs))
    return probs


def lse_merge(o_parts, lse_parts, row_indptr, part_idx):
    o_parts = np.ascontiguousarray(o_parts, dtype=np.float64)
    lse_parts = np.ascontiguousarray(lse_parts, dtype=np.float64)
    row_indptr, part_idx = _i32(row_indptr), _i32(part_idx)
    n_rows = len(row_indptr) - 1
    out = np.empty((n_rows, D), dtype=np.float64)
    lse = np.empty(n_rows, dtype=np.float64)
    lib().oracle_lse_merge(_p(o_parts), _p(lse_parts), _p(row_indptr), _p(part_idx), C.c_int32(n_rows), _p(out), _p(lse))
    return out, lse


def e4m3_value(code: int) -> float:
    return float(lib().orc_e4m3_value(C.c_uint8(code)))


def e4m3_encode(x: float) -> int:
    return int(lib().orc_e4m3_encode(C.c_float(x)))


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def max_pages_per_request(nodes, req_leaf) -> int:
    """Pages on the longest root-to-leaf path among the requests (parents come before children)."""
    nodes, req_leaf = _i32(nodes).reshape(-1, 4), _i32(req_leaf)
    along = np.zeros(nodes.shape[0], dtype=np.int64)
    for v in range(nodes.shape[0]):
        par = int(nodes[v, 0])
        along[v] = int(nodes[v, 2]) + (along[par] if par >= 0 else 0)
    return int(along[req_leaf].max()) if len(req_leaf) else 0


def flatten_workload(workload):
    f = workload.forest
    mp = max(1, max_pages_per_request(f.nodes, f.req_leaf))
    return flatten_tree(f.nodes, f.node_pages, f.req_leaf, mp, f.page_size)


def run_workload(workload, pool: Optional[HostPool] = None, req_subset=None):
    """Whole-workload oracle result (out, lse).  req_subset (decode only) restricts to some requests."""
    if pool is None:
        pool = HostPool(workload.num_pages, workload.num_kv_heads, workload.kv_dtype, page_size=workload.page_size)
        pool.fill_from(workload)
    f = workload.forest
    q = workload.q()
    has_child = np.zeros(f.n_nodes, dtype=bool)
    has_child[f.parent[f.parent >= 0]] = True
    if workload.mode == "decode" and bool(np.any(has_child & (f.n_tokens % f.page_size != 0))):
        # a node with children ends inside a page: no flat block table exists, walk the forest
        idx = np.arange(f.n_req) if req_subset is None else np.asarray(req_subset)
        return attn_decode_tree(pool, q[idx], f.nodes, f.node_pages, f.req_leaf[idx], float(workload.scale))
    bt, kv_len, _, _, _ = flatten_workload(workload)
    if workload.mode == "decode":
        if req_subset is not None:
            idx = np.asarray(req_subset)
            return attn_decode(pool, q[idx], bt[idx], kv_len[idx], float(workload.scale))
        return attn_decode(pool, q, bt, kv_len, float(workload.scale))
    return attn_prefill(pool, q, workload.cu_q(), bt, kv_len, float(workload.scale))
