"""Pins of the CPU oracle against things other than itself (CPU only).

The paper prints no number for attention, so the oracle is pinned by what the
mathematics fixes: brute force on contiguous unpaged tensors, a library routine
(PyTorch CPU float64 scaled_dot_product_attention), closed forms, invariants
(page permutation, sharing vs private copies, causality), the log-sum-exp split
identity, the token-usage equation of Section 5 evaluated on explicit token
strings, and a library float8 conversion.
"""
import math
import os

import numpy as np
import pytest
import torch

from paper_2603_16104_amd import workloads as wl

D, PAGE = 128, 16


# ------------------------------------------------------------------ independent helpers

def _as_f64(x):
    if x.dtype == np.uint16:
        return wl.bf16_bits_to_f32(x).astype(np.float64)
    return x.astype(np.float64)


def logical_kv(w, r):
    """Contiguous K, V [kv_len][Hkv][D] of request r built from node tensors, never touching a pool."""
    ks, vs = [], []
    for node in w.forest.path(int(w.forest.req_leaf[r])):
        if w.forest.n_tokens[node] == 0:
            continue
        k, v = w.node_kv(node)
        ks.append(_as_f64(k))
        vs.append(_as_f64(v))
    if not ks:
        z = np.zeros((0, w.num_kv_heads, D))
        return z, z
    return np.concatenate(ks), np.concatenate(vs)


def brute_attention(qv, K, V, scale):
    """Dense softmax attention of one query vector, pure numpy on contiguous [T][D] arrays."""
    if K.shape[0] == 0:
        return np.zeros(D), -np.inf
    s = (K @ qv) * scale
    m = s.max()
    e = np.exp(s - m)
    return (e[:, None] * V).sum(0) / e.sum(), m + math.log(e.sum())


def brute_workload(w):
    q = _as_f64(w.q())
    scale = float(w.scale)
    G = w.group
    out = np.zeros((w.total_q(), w.num_q_heads, D))
    lse = np.zeros((w.total_q(), w.num_q_heads))
    cu = w.cu_q()
    for r in range(w.forest.n_req):
        K, V = logical_kv(w, r)
        T = K.shape[0]
        nq = cu[r + 1] - cu[r]
        for i in range(nq):
            vis = T if w.mode == "decode" else T - nq + i + 1
            for h in range(w.num_q_heads):
                o, l = brute_attention(q[cu[r] + i, h], K[:vis, h // G], V[:vis, h // G], scale)
                out[cu[r] + i, h], lse[cu[r] + i, h] = o, l
    return out, lse


def oracle_pool(orc, w):
    pool = orc.HostPool(w.num_pages, w.num_kv_heads, w.kv_dtype)
    pool.fill_from(w)
    return pool


# ------------------------------------------------------------------ brute force and library routine

@pytest.mark.parametrize("seed,mode", [(1, "decode"), (2, "decode"), (3, "prefill"), (4, "prefill")])
def test_brute_force_small_forests(oracle, seed, mode):
    w = wl.random_forest_workload(seed, mode=mode, max_node_pages=2, depth=3, fanout=2)
    out, lse = oracle.run_workload(w)
    bout, blse = brute_workload(w)
    assert np.abs(out - bout).max() <= 1e-12
    fin = np.isfinite(blse)
    assert np.array_equal(np.isfinite(lse), fin)
    assert np.abs(lse[fin] - blse[fin]).max() <= 1e-12


def test_brute_force_fp32_source(oracle):
    w = wl.random_forest_workload(9, mode="decode", kv_dtype=wl.KV_FP32, src_dtype="fp32", max_node_pages=2)
    out, lse = oracle.run_workload(w)
    bout, blse = brute_workload(w)
    assert np.abs(out - bout).max() <= 1e-12


def test_config1_against_brute_force(oracle):
    pre, dec = wl.config1()
    for w in (pre, dec):
        out, lse = oracle.run_workload(w)
        bout, blse = brute_workload(w)
        assert np.abs(out - bout).max() <= 1e-12
        assert np.abs(lse - blse).max() <= 1e-12
    assert dec.forest.kv_len(0) == 305 and pre.forest.kv_len(0) == 304
    assert pre.pair_count() == 4 * 4744


def test_library_sdpa_float64(oracle):
    """Prefill on gathered contiguous K/V equals torch's float64 SDPA with an explicit boolean mask."""
    w = wl.random_forest_workload(5, mode="prefill", max_node_pages=3, zero_weight_nodes=False)
    out, _ = oracle.run_workload(w)
    q = _as_f64(w.q())
    cu = w.cu_q()
    G = w.group
    for r in range(w.forest.n_req):
        K, V = logical_kv(w, r)
        T, nq = K.shape[0], cu[r + 1] - cu[r]
        if nq == 0:
            continue
        qt = torch.from_numpy(q[cu[r]:cu[r + 1]]).permute(1, 0, 2)               # [Hq][nq][D]
        kt = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(G, dim=0)     # [Hq][T][D]
        vt = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(G, dim=0)
        pos = torch.arange(nq)[:, None] + (T - nq)
        mask = torch.arange(T)[None, :] <= pos
        ref = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, attn_mask=mask, scale=float(w.scale))
        assert np.abs(ref.permute(1, 0, 2).numpy() - out[cu[r]:cu[r + 1]]).max() <= 1e-12


@pytest.mark.parametrize("seed,mode,kv", [(1, "decode", "bf16"), (3, "prefill", "bf16"), (4, "prefill", "fp8"),
                                          (2, "decode", "fp8"), (7, "prefill", "fp32")])
def test_matrix_form_against_brute_force_and_row_form(oracle, seed, mode, kv):
    """attn_matrix_form (whole requests through matrix products) against the brute force on K/V built from the
    node tensors, never touching a pool (bf16 / fp32 pools store them exactly), and against the row-by-row C
    routine over the same pool (all pool types): ragged forests, empty nodes, requests with 0, 1 and several
    new tokens.  A transposed operand, a mask shifted by one or a wrong head group fails either."""
    kv_dtype = {"bf16": wl.KV_BF16, "fp8": wl.KV_FP8_E4M3, "fp32": wl.KV_FP32}[kv]
    w = wl.random_forest_workload(seed, mode=mode, max_node_pages=3, depth=3, fanout=2, kv_dtype=kv_dtype,
                                  src_dtype="fp32" if kv == "fp32" else "bf16")
    pool = oracle_pool(oracle, w)
    bt, kv_len, *_ = oracle.flatten_workload(w)
    out, lse, rows = oracle.attn_matrix_form(pool, w.q(), w.cu_q(), bt, kv_len, float(w.scale))
    assert np.array_equal(rows, np.arange(w.total_q()))
    rout, rlse = oracle.run_workload(w, pool)
    fin = np.isfinite(rlse)
    assert np.array_equal(np.isfinite(lse), fin)
    assert np.abs(out - rout).max() <= 1e-12 and np.abs(lse[fin] - rlse[fin]).max() <= 1e-12
    if kv != "fp8":
        bout, blse = brute_workload(w)
        assert np.abs(out - bout).max() <= 1e-12 and np.abs(lse[fin] - blse[fin]).max() <= 1e-12
    # a subset of requests: the same rows, in the order asked for
    if w.forest.n_req >= 2:
        sub = [w.forest.n_req - 1, 0]
        so, sl, srows = oracle.attn_matrix_form(pool, w.q(), w.cu_q(), bt, kv_len, float(w.scale), requests=sub)
        assert np.abs(so - out[srows]).max() <= 1e-12 and np.array_equal(np.isfinite(sl), np.isfinite(lse[srows]))
        cu = w.cu_q()
        assert np.array_equal(srows, np.concatenate([np.arange(cu[r], cu[r + 1]) for r in sub]))
    # some tokens of a request only
    cu = w.cu_q()
    big = int(np.argmax(np.diff(cu)))
    n_new = int(cu[big + 1] - cu[big])
    pick = sorted({0, n_new - 1, n_new // 2})
    to, tl, trows = oracle.attn_matrix_form(pool, w.q(), w.cu_q(), bt, kv_len, float(w.scale), requests=[big],
                                            tokens={big: pick})
    assert np.array_equal(trows, cu[big] + np.array(pick))
    assert np.abs(to - out[trows]).max() <= 1e-12 and np.abs(tl - lse[trows]).max() <= 1e-12


def test_matrix_form_closed_form_running_mean(oracle):
    """Equal keys give equal scores, so new token i returns the mean of the values it may see: with
    V_t = t in every dimension and a prefix of p tokens, out_i = (p + i) / 2 and lse_i = s0 + ln(p + i + 1)."""
    T, s, H = 45, 7, 2
    K = np.ones((T, H, D), dtype=np.float32)
    V = np.broadcast_to(np.arange(T, dtype=np.float32)[:, None, None], (T, H, D)).copy()
    pool = oracle.HostPool(3, H, oracle.FP32)
    pages = np.array([2, 0, 1], dtype=np.int32)
    pool.write(pages, 0, K, V)
    q = np.full((s, 4, D), 0.25, dtype=np.float32)
    scale = 0.5
    out, lse, _ = oracle.attn_matrix_form(pool, q, [0, s], pages[None, :], [T], scale)
    p = T - s
    for i in range(s):
        assert np.abs(out[i] - (p + i) / 2).max() <= 1e-12
        assert np.abs(lse[i] - (scale * 0.25 * D + math.log(p + i + 1))).max() <= 1e-12


# ------------------------------------------------------------------ invariants

def test_page_permutation_invariance(oracle):
    w = wl.random_forest_workload(6, mode="decode")
    out_a, lse_a = oracle.run_workload(w)
    # same logical tokens, different physical pages
    perm = np.random.default_rng(123).permutation(w.num_pages).astype(np.int32)
    f = w.forest
    w2 = wl.Workload(**{**w.__dict__, "forest": wl.PrefixForest(f.parent, f.n_tokens, f.page_begin, f.n_pages,
                                                                perm[f.node_pages], f.req_leaf)})
    out_b, lse_b = oracle.run_workload(w2)
    assert np.array_equal(out_a, out_b) and np.array_equal(lse_a, lse_b)


def test_shared_equals_private_copies(oracle):
    """Section 2 ("Scope"): optimised execution returns what naive execution returns.  A forest whose
    requests share pages gives bit-identical oracle output to one where every request owns copies."""
    w = wl.random_forest_workload(7, mode="decode")
    out_s, lse_s = oracle.run_workload(w)
    f = w.forest
    # private chains: request r gets its own copy of every node on its path
    parent, ntok, leaves, src = [], [], [], []
    for r in range(f.n_req):
        prev = -1
        for node in f.path(int(f.req_leaf[r])):
            parent.append(prev)
            ntok.append(int(f.n_tokens[node]))
            src.append(node)
            prev = len(parent) - 1
        leaves.append(prev)
    n_used = sum((t + 15) // 16 for t in ntok)
    f2 = wl.make_forest(parent, ntok, leaves, np.random.default_rng(5).permutation(n_used + 3).astype(np.int32))
    pool = oracle.HostPool(n_used + 3, w.num_kv_heads, w.kv_dtype)
    for i, node in enumerate(src):
        if ntok[i]:
            k, v = w.node_kv(node)
            pool.write(f2.node_pages[f2.page_begin[i]: f2.page_begin[i] + f2.n_pages[i]], 0, k, v)
    bt, kv_len, *_ = oracle.flatten_tree(f2.nodes, f2.node_pages, f2.req_leaf, max(1, f2.max_pages_per_req()))
    out_p, lse_p = oracle.attn_decode(pool, w.q(), bt, kv_len, float(w.scale))
    assert np.array_equal(out_s, out_p) and np.array_equal(lse_s, lse_p)


def test_softmax_rows_sum_to_one(oracle):
    w = wl.random_forest_workload(8, mode="decode", zero_weight_nodes=False)
    pool = oracle_pool(oracle, w)
    bt, kv_len, *_ = oracle.flatten_workload(w)
    q = w.q()
    for r in range(w.forest.n_req):
        for h in (0, w.num_q_heads - 1):
            p = oracle.attn_probs(pool, q[r], bt[r], int(kv_len[r]), h, w.num_q_heads, float(w.scale))
            assert abs(p.sum() - 1.0) <= 1e-14 * max(1, len(p))
            assert (p >= 0).all() and (p <= 1).all()


def test_causality_and_unreferenced_pages(oracle):
    w = wl.random_forest_workload(10, mode="prefill", zero_weight_nodes=False, max_node_pages=3)
    pool = oracle_pool(oracle, w)
    bt, kv_len, *_ = oracle.flatten_workload(w)
    cu = w.cu_q()
    out, lse = oracle.attn_prefill(pool, w.q(), cu, bt, kv_len, float(w.scale))
    r = int(np.argmax(cu[1:] - cu[:-1]))
    nq = int(cu[r + 1] - cu[r])
    assert nq >= 2
    # perturb the last token's K/V of request r: every earlier query row must be bit-identical
    last = int(kv_len[r]) - 1
    page, slot = int(bt[r, last // PAGE]), last % PAGE
    pool2 = oracle_pool(oracle, w)
    H = w.num_kv_heads
    kblk = pool2.k.reshape(w.num_pages, H, 4, PAGE, 32)
    vblk = pool2.v.reshape(w.num_pages, H, D, PAGE)
    kblk[page, :, :, slot, :] = wl.f32_to_bf16_bits(np.float32(3.0))
    vblk[page, :, :, slot] = wl.f32_to_bf16_bits(np.float32(-5.0))
    out2, _ = oracle.attn_prefill(pool2, w.q(), cu, bt, kv_len, float(w.scale))
    assert np.array_equal(out[cu[r]:cu[r + 1] - 1], out2[cu[r]:cu[r + 1] - 1])
    assert not np.array_equal(out[cu[r + 1] - 1], out2[cu[r + 1] - 1])
    # a page no request references may hold anything
    unused = sorted(set(range(w.num_pages)) - set(int(x) for x in w.forest.node_pages))
    pool3 = oracle_pool(oracle, w)
    pool3.k.reshape(w.num_pages, -1)[unused] = 0x1234
    out3, _ = oracle.attn_prefill(pool3, w.q(), cu, bt, kv_len, float(w.scale))
    assert np.array_equal(out, out3)


def test_prefill_equals_successive_decodes(oracle):
    w = wl.random_forest_workload(12, mode="prefill", zero_weight_nodes=False, max_node_pages=2)
    pool = oracle_pool(oracle, w)
    bt, kv_len, *_ = oracle.flatten_workload(w)
    cu = w.cu_q()
    q = w.q()
    out, lse = oracle.attn_prefill(pool, q, cu, bt, kv_len, float(w.scale))
    for r in range(w.forest.n_req):
        nq = int(cu[r + 1] - cu[r])
        for i in range(nq):
            klen = np.array([kv_len[r] - nq + i + 1], dtype=np.int32)
            o1, l1 = oracle.attn_decode(pool, q[cu[r] + i: cu[r] + i + 1], bt[r:r + 1], klen, float(w.scale))
            assert np.array_equal(o1[0], out[cu[r] + i]) and np.array_equal(l1[0], lse[cu[r] + i])


# ------------------------------------------------------------------ closed forms

def _single_request_pool(oracle, K, V, seed=0, Hkv=1):
    T = K.shape[0]
    n_pages = max(1, (T + 15) // 16)
    pages = np.random.default_rng(seed).permutation(n_pages + 2).astype(np.int32)
    pool = oracle.HostPool(n_pages + 2, Hkv, oracle.BF16)
    if T:
        pool.write(pages[:n_pages], 0, wl.f32_to_bf16_bits(K), wl.f32_to_bf16_bits(V))
    bt = pages[:n_pages][None, :].copy()
    return pool, bt


def test_closed_forms(oracle):
    rng = np.random.default_rng(0)
    scale = float(np.float32(1 / math.sqrt(128)))
    T = 37
    K = rng.standard_normal((T, 1, D)).astype(np.float32)
    V = rng.standard_normal((T, 1, D)).astype(np.float32)
    Kb, Vb = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(K)), wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(V))
    q = wl.f32_to_bf16_bits(rng.standard_normal((1, 2, D)).astype(np.float32))
    pool, bt = _single_request_pool(oracle, K, V)
    # kv_len = 1 -> output is V_0 exactly, lse = s_0
    o, l = oracle.attn_decode(pool, q, bt, [1], scale)
    assert np.array_equal(o[0, 0], Vb[0, 0].astype(np.float64))
    s0 = scale * float(wl.bf16_bits_to_f32(q)[0, 0].astype(np.float64) @ Kb[0, 0].astype(np.float64))
    assert abs(l[0, 0] - s0) <= 1e-13
    # q = 0 -> uniform weights: mean of V, lse = ln T
    q0 = np.zeros((1, 2, D), dtype=np.uint16)
    o, l = oracle.attn_decode(pool, q0, bt, [T], scale)
    assert np.abs(o[0, 1] - Vb[:, 0].astype(np.float64).mean(0)).max() <= 1e-14
    assert abs(l[0, 1] - math.log(T)) <= 1e-14
    # all keys identical -> mean of V again, lse = s + ln T
    Ksame = np.repeat(K[:1], T, axis=0)
    pool2, bt2 = _single_request_pool(oracle, Ksame, V, seed=1)
    o, l = oracle.attn_decode(pool2, q, bt2, [T], scale)
    assert np.abs(o[0, 0] - Vb[:, 0].astype(np.float64).mean(0)).max() <= 1e-13
    assert abs(l[0, 0] - (s0 + math.log(T))) <= 1e-12
    # constant V -> that constant
    Vc = np.full((T, 1, D), 0.75, dtype=np.float32)
    pool3, bt3 = _single_request_pool(oracle, K, Vc, seed=2)
    o, _ = oracle.attn_decode(pool3, q, bt3, [T], scale)
    assert np.abs(o - 0.75).max() <= 1e-14
    # one key aligned with q and huge -> output tends to that token's V
    qf = wl.bf16_bits_to_f32(q)[0, 0]
    Kbig = K.copy()
    Kbig[11, 0] = 64.0 * qf
    pool4, bt4 = _single_request_pool(oracle, Kbig, V, seed=3)
    o, _ = oracle.attn_decode(pool4, q, bt4, [T], scale)
    assert np.abs(o[0, 0] - Vb[11, 0]).max() <= 1e-9
    # prefill, no cached prefix: token 0 sees only itself
    qp = wl.f32_to_bf16_bits(rng.standard_normal((T, 2, D)).astype(np.float32))
    o, _ = oracle.attn_prefill(pool, qp, [0, T], bt, [T], scale)
    assert np.array_equal(o[0, 0], Vb[0, 0].astype(np.float64))
    # empty sequence -> zeros and -inf
    o, l = oracle.attn_decode(pool, q, bt, [0], scale)
    assert (o == 0).all() and np.isneginf(l).all()


# ------------------------------------------------------------------ log-sum-exp combine

def test_lse_split_identity(oracle):
    w = wl.random_forest_workload(13, mode="decode", zero_weight_nodes=True, max_node_pages=4)
    pool = oracle_pool(oracle, w)
    bt, kv_len, indptr, idx, tok_start = oracle.flatten_workload(w)
    q = w.q()
    scale = float(w.scale)
    full_o, full_l = oracle.attn_decode(pool, q, bt, kv_len, scale)
    rng = np.random.default_rng(3)
    n_req, Hq = q.shape[0], q.shape[1]
    # split every request at random points, one empty segment included
    n_seg = 4
    cuts = np.zeros((n_req, n_seg + 1), dtype=np.int32)
    for r in range(n_req):
        c = np.sort(rng.integers(0, kv_len[r] + 1, size=n_seg - 2))
        cuts[r] = np.concatenate([[0], c, [kv_len[r], kv_len[r]]])      # last segment is empty
    o_parts, l_parts = [], []
    for s in range(n_seg):
        o, l = oracle.attn_decode(pool, q, bt, kv_len, scale, seg=(cuts[:, s], cuts[:, s + 1]))
        o_parts.append(o.reshape(-1, D))
        l_parts.append(l.reshape(-1))
    o_parts, l_parts = np.concatenate(o_parts), np.concatenate(l_parts)
    rows = n_req * Hq
    indp = np.arange(rows + 1, dtype=np.int32) * n_seg
    pidx = (np.arange(rows)[:, None] + rows * np.arange(n_seg)[None, :]).reshape(-1).astype(np.int32)
    mo, ml = oracle.lse_merge(o_parts, l_parts, indp, pidx)
    fin = np.isfinite(full_l.reshape(-1))
    assert np.abs(mo - full_o.reshape(-1, D)).max() <= 1e-12
    assert np.abs(ml[fin] - full_l.reshape(-1)[fin]).max() <= 1e-12
    assert np.array_equal(np.isneginf(ml), ~fin)
    # order of the partials does not matter
    pidx2 = pidx.reshape(rows, n_seg)[:, ::-1].reshape(-1).copy()
    mo2, ml2 = oracle.lse_merge(o_parts, l_parts, indp, pidx2)
    assert np.abs(mo2 - mo).max() <= 1e-12
    # split at node boundaries (what the shared-node decode does) also reproduces the whole
    f = w.forest
    for r in range(n_req):
        path = f.path(int(f.req_leaf[r]))
        ob, lb = [], []
        for node in path:
            b = np.array([tok_start[node]], dtype=np.int32)
            e = b + f.n_tokens[node]
            o, l = oracle.attn_decode(pool, q[r:r + 1], bt[r:r + 1], kv_len[r:r + 1], scale, seg=(b, e))
            ob.append(o[0])
            lb.append(l[0])
        ob, lb = np.stack(ob, 1).reshape(-1, D), np.stack(lb, 1).reshape(-1)   # [Hq*len(path)]
        indp_r = np.arange(Hq + 1, dtype=np.int32) * len(path)
        mo, ml = oracle.lse_merge(ob, lb, indp_r, np.arange(Hq * len(path), dtype=np.int32))
        assert np.abs(mo - full_o[r]).max() <= 1e-12


def test_lse_merge_closed_forms(oracle):
    # two partials with equal lse average; -inf partial is ignored; all -inf gives (0, -inf); empty row too
    o = np.zeros((4, D))
    o[0], o[1], o[2], o[3] = 1.0, 3.0, 100.0, np.nan
    lse = np.array([0.5, 0.5, -np.inf, -np.inf])
    indptr = np.array([0, 3, 5, 5], dtype=np.int32)
    pidx = np.array([0, 1, 2, 2, 3], dtype=np.int32)
    mo, ml = oracle.lse_merge(o, lse, indptr, pidx)
    assert np.abs(mo[0] - 2.0).max() <= 1e-15 and abs(ml[0] - (0.5 + math.log(2))) <= 1e-15
    assert (mo[1] == 0).all() and np.isneginf(ml[1])
    assert (mo[2] == 0).all() and np.isneginf(ml[2])
    # weights follow exp(lse): lse = ln 1, ln 3 -> weights 1/4, 3/4
    lse2 = np.array([0.0, math.log(3.0)])
    mo, ml = oracle.lse_merge(o[:2], lse2, np.array([0, 2], dtype=np.int32), np.array([0, 1], dtype=np.int32))
    assert np.abs(mo[0] - (0.25 * 1 + 0.75 * 3)).max() <= 1e-15 and abs(ml[0] - math.log(4.0)) <= 1e-15


# ------------------------------------------------------------------ tree indexing and token usage

def py_flatten(f, max_pages):
    """Independent pure-Python walk of the forest."""
    n_req = f.n_req
    bt = -np.ones((n_req, max_pages), dtype=np.int32)
    kv_len = np.zeros(n_req, dtype=np.int32)
    members = [[] for _ in range(f.n_nodes)]
    for r in range(n_req):
        pages = []
        for node in f.path(int(f.req_leaf[r])):
            members[node].append(r)
            pages += [int(x) for x in f.node_pages[f.page_begin[node]: f.page_begin[node] + f.n_pages[node]]]
            kv_len[r] += f.n_tokens[node]
        bt[r, :len(pages)] = pages
    indptr = np.cumsum([0] + [len(m) for m in members]).astype(np.int32)
    idx = np.array([r for m in members for r in sorted(m)], dtype=np.int32)
    tok_start = np.array([sum(int(f.n_tokens[u]) for u in f.path(v)[:-1]) for v in range(f.n_nodes)], dtype=np.int32)
    return bt, kv_len, indptr, idx, tok_start


@pytest.mark.parametrize("seed", range(20, 26))
def test_flatten_tree_against_python_walk(oracle, seed):
    w = wl.random_forest_workload(seed, depth=4, fanout=3, n_roots=3)
    f = w.forest
    mp = max(1, f.max_pages_per_req()) + 2
    got = oracle.flatten_tree(f.nodes, f.node_pages, f.req_leaf, mp)
    exp = py_flatten(f, mp)
    for g, e in zip(got, exp):
        assert np.array_equal(g, e)


def test_flatten_tree_rejects_malformed(oracle):
    pages = np.arange(8, dtype=np.int32)
    ok = np.array([[-1, 0, 1, 16], [0, 1, 1, 5]], dtype=np.int32)
    oracle.flatten_tree(ok, pages, [1], 4)
    for bad in (np.array([[0, 0, 1, 16]], dtype=np.int32),                      # parent not before child
                np.array([[-1, 0, 1, 12], [0, 1, 1, 5]], dtype=np.int32),       # shared node not page aligned
                np.array([[-1, 0, 2, 16]], dtype=np.int32)):                    # page count does not match tokens
        with pytest.raises(ValueError):
            oracle.flatten_tree(bad, pages, [0], 4)
    with pytest.raises(ValueError):
        oracle.flatten_tree(ok, pages, [1], 1)                                   # max_pages too small
    with pytest.raises(ValueError):
        oracle.flatten_tree(ok, pages, [2], 4)                                   # leaf out of range


def _token_strings(f, rng):
    """Explicit token-id strings per node such that sibling segments start with different tokens
    (the radix-tree property); roots differ too."""
    seg = {}
    for v in range(f.n_nodes):
        seg[v] = [int(x) for x in rng.integers(0, 50, size=int(f.n_tokens[v]))]
        if seg[v]:
            seg[v][0] = 1000 + v
    return seg


@pytest.mark.parametrize("seed", range(30, 36))
def test_prefill_usage_equals_uncached_suffix_of_token_strings(oracle, seed):
    """u_p of Section 5: tokens of call j that are not shared with call j-1 (consecutive calls on one
    worker).  Checked against the longest common prefix of explicit token strings."""
    w = wl.random_forest_workload(seed, depth=4, fanout=3, n_roots=2, zero_weight_nodes=False)
    f = w.forest
    rng = np.random.default_rng(seed)
    seg = _token_strings(f, rng)
    calls = rng.integers(0, f.n_nodes, size=12).astype(np.int32)
    strings = [sum((seg[v] for v in f.path(int(l))), []) for l in calls]
    exp = []
    for j, s in enumerate(strings):
        if j == 0:
            exp.append(len(s))
            continue
        p = strings[j - 1]
        lcp = 0
        while lcp < min(len(p), len(s)) and p[lcp] == s[lcp]:
            lcp += 1
        exp.append(len(s) - lcp)
    got = oracle.prefill_usage(f.nodes, calls)
    assert [int(x) for x in got] == exp


def test_prefill_usage_golden_config1(oracle):
    pre, _ = wl.config1()
    path = os.path.join(os.path.dirname(__file__), "golden", "c1_token_usage.txt")
    n = 0
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        calls, exp = line.split("|")
        got = oracle.prefill_usage(pre.forest.nodes, [int(x) for x in calls.split()])
        assert [int(x) for x in got] == [int(x) for x in exp.split()]
        n += 1
    assert n == 3
    # with root and branch cached, the prefilled suffix is the 16-token leaf segment
    assert int(pre.q_len.sum()) == 64 and all(pre.forest.kv_len(r) - 16 == 288 for r in range(4))


# ------------------------------------------------------------------ pool format and fp8

def test_pool_layout_matches_documented_format(oracle):
    """K block: 64-byte dimension chunks, chunk-major then slot; V block: dimension-major, slot-minor."""
    rng = np.random.default_rng(4)
    H, T = 2, 48
    k = rng.integers(0, 65535, size=(T, H, D)).astype(np.uint16)
    v = rng.integers(0, 65535, size=(T, H, D)).astype(np.uint16)
    pages = np.array([5, 1, 3], dtype=np.int32)
    pool = oracle.HostPool(7, H, oracle.BF16)
    pool.write(pages, 0, k, v)
    kk = pool.k.reshape(7, H, 4, PAGE, 32)
    vv = pool.v.reshape(7, H, D, PAGE)
    exp_k = k.reshape(3, PAGE, H, 4, 32).transpose(0, 2, 3, 1, 4)
    exp_v = v.reshape(3, PAGE, H, D).transpose(0, 2, 3, 1)
    assert np.array_equal(kk[pages], exp_k) and np.array_equal(vv[pages], exp_v)
    # appending at a slot offset touches only those slots
    pool2 = oracle.HostPool(7, H, oracle.BF16)
    pool2.write(pages, 0, k[:20], v[:20])
    pool2.write(pages[1:], 4, k[20:], v[20:])
    assert np.array_equal(pool2.k, pool.k) and np.array_equal(pool2.v, pool.v)
    # fp8 block: one byte per element, 64 dimensions per chunk
    pool8 = oracle.HostPool(7, H, oracle.FP8_E4M3)
    pool8.write(pages, 0, wl.f32_to_bf16_bits(rng.standard_normal((T, H, D)).astype(np.float32)),
                wl.f32_to_bf16_bits(rng.standard_normal((T, H, D)).astype(np.float32)))
    assert pool8.k.size == 7 * H * PAGE * D and np.isfinite(pool8.k_scale[pages[0] * H]).all()


def test_e4m3_against_library_conversion(oracle):
    codes = torch.arange(256, dtype=torch.uint8)
    ref = codes.view(torch.float8_e4m3fn).to(torch.float64).numpy()
    ours = np.array([oracle.e4m3_value(c) for c in range(256)])
    assert np.array_equal(np.isnan(ref), np.isnan(ours))
    ok = ~np.isnan(ref)
    assert np.array_equal(ref[ok], ours[ok])
    assert ours[0x7E] == 448.0
    # encode(decode(c)) == c for every finite code except negative zero's sign-preserving twin
    for c in range(256):
        if np.isnan(ours[c]):
            continue
        assert oracle.e4m3_encode(float(ours[c])) == c
    # round-to-nearest-even inside the range agrees with the library conversion
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.uniform(-448, 448, 4000), rng.standard_normal(4000) * 0.01,
                        0.5 * (ours[:0x7E] + ours[1:0x7F])]).astype(np.float32)   # exact midpoints too
    ref_codes = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = np.array([oracle.e4m3_encode(float(t)) for t in x], dtype=np.uint8)
    assert np.array_equal(got, ref_codes)
    # saturation
    assert oracle.e4m3_encode(1e9) == 0x7E and oracle.e4m3_encode(-500.0) == 0xFE


def test_fp8_pool_write_quantisation(oracle):
    """Per (page, head) scale = amax/448 in float; codes = RNE(x / scale); dequantised pool drives attention."""
    rng = np.random.default_rng(2)
    H, T = 2, 40                          # last page holds 8 tokens
    k = rng.standard_normal((T, H, D)).astype(np.float32)
    v = rng.standard_normal((T, H, D)).astype(np.float32)
    k[16:32, 1] = 0.0                     # an all-zero block -> scale 1
    kb, vb = wl.f32_to_bf16_bits(k), wl.f32_to_bf16_bits(v)
    kf, vf = wl.bf16_bits_to_f32(kb), wl.bf16_bits_to_f32(vb)
    pages = np.array([2, 0, 3], dtype=np.int32)
    pool = oracle.HostPool(4, H, oracle.FP8_E4M3)
    pool.write(pages, 0, kb, vb)
    kk = pool.k.reshape(4, H, 2, PAGE, 64)
    vv = pool.v.reshape(4, H, D, PAGE)
    for i, pg in enumerate(pages):
        n = min(16, T - 16 * i)
        for h in range(H):
            for src, codes, scales in ((kf, kk[pg, h].transpose(1, 0, 2).reshape(PAGE, D), pool.k_scale),
                                       (vf, vv[pg, h].T, pool.v_scale)):
                blk = src[16 * i: 16 * i + n, h]
                amax = np.abs(blk).max()
                sc = np.float32(amax) / np.float32(448.0) if amax > 0 else np.float32(1.0)
                assert scales[pg * H + h] == sc
                ref = torch.from_numpy((blk / sc).astype(np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
                assert np.array_equal(codes[:n], ref)
                if n < 16:
                    assert (codes[n:] == 0x7F).all()       # untouched poison
    # attention through the fp8 pool equals brute force on the dequantised values
    deq_k = np.zeros((T, H, D))
    deq_v = np.zeros((T, H, D))
    lut = np.array([oracle.e4m3_value(c) for c in range(256)])
    for i, pg in enumerate(pages):
        n = min(16, T - 16 * i)
        for h in range(H):
            deq_k[16 * i:16 * i + n, h] = lut[kk[pg, h].transpose(1, 0, 2).reshape(PAGE, D)[:n]] * float(pool.k_scale[pg * H + h])
            deq_v[16 * i:16 * i + n, h] = lut[vv[pg, h].T[:n]] * float(pool.v_scale[pg * H + h])
    q = wl.f32_to_bf16_bits(rng.standard_normal((1, 4, D)).astype(np.float32))
    scale = float(np.float32(1 / math.sqrt(128)))
    o, l = oracle.attn_decode(pool, q, pages[None, :], [T], scale)
    qf = wl.bf16_bits_to_f32(q).astype(np.float64)
    for h in range(4):
        bo, bl = brute_attention(qf[0, h], deq_k[:, h // 2], deq_v[:, h // 2], scale)
        assert np.abs(o[0, h] - bo).max() <= 1e-12 and abs(l[0, h] - bl) <= 1e-12
    # quantisation error of the round trip stays within half an e4m3 step (relative 2^-4) of amax scale
    assert np.abs(deq_k - kf).max() <= np.abs(kf).max() * 2.0 ** -4


def test_fp8_append_running_scale(oracle):
    """Continuing an fp8 page (first_slot > 0).  Pinned by what the rule must reduce to:
    (a) tokens whose magnitude does not exceed the page's amax leave scale and earlier codes untouched,
        and the page ends up byte-identical to writing all its tokens in one call (that path is pinned
        against the library float8 conversion above);
    (b) a louder token raises the scale to amax_new/448 exactly, maps itself to +-448, and moves every
        earlier dequantised value by at most half a step of the new grid at that value;
    (c) the scale never shrinks."""
    import torch
    rng = np.random.default_rng(9)
    H = 2
    x = rng.standard_normal((16, H, D)).astype(np.float32)
    x[0, :, 0] = 5.0                                   # the page's amax sits in its first token
    kb = wl.f32_to_bf16_bits(x)
    whole = oracle.HostPool(3, H, oracle.FP8_E4M3)
    whole.write([1], 0, kb, kb)
    grown = oracle.HostPool(3, H, oracle.FP8_E4M3)
    for a, b in ((0, 1), (1, 2), (2, 9), (9, 16)):
        grown.write([1], a, kb[a:b], kb[a:b])
    assert np.array_equal(grown.k, whole.k) and np.array_equal(grown.v, whole.v)          # (a)
    assert np.array_equal(grown.k_scale[H:2 * H], whole.k_scale[H:2 * H])
    assert np.all(grown.k_scale[H:2 * H] == np.float32(5.0) / np.float32(448.0))

    lut = np.array([oracle.e4m3_value(c) for c in range(256)])
    p = oracle.HostPool(3, H, oracle.FP8_E4M3)
    quiet = wl.f32_to_bf16_bits((0.1 * rng.standard_normal((5, H, D))).astype(np.float32))
    p.write([2], 0, quiet, quiet)
    s_old = p.k_scale[2 * H: 3 * H].copy()
    blk = lambda pool: pool.k.reshape(3, H, 2, PAGE, 64)[2]           # [head][chunk][slot][64]
    before = lut[blk(p)[:, :, :5]] * s_old[:, None, None, None].astype(np.float64)
    loud = np.zeros((1, H, D), dtype=np.float32)
    loud[0, :, 3] = [-7.0, 3.5]
    loud_b = wl.f32_to_bf16_bits(loud)
    p.write([2], 5, loud_b, loud_b)
    s_new = p.k_scale[2 * H: 3 * H]
    assert np.array_equal(s_new, (np.float32([7.0, 3.5]) / np.float32(448.0)).astype(np.float32))      # (b)
    assert blk(p)[0, 0, 5, 3] == 0xFE and blk(p)[1, 0, 5, 3] == 0x7E                  # -448 and +448
    after = lut[blk(p)[:, :, :5]] * s_new[:, None, None, None].astype(np.float64)
    # half a step of the e4m3 grid at magnitude m is at most m * 2^-4 (normal range) or 2^-10 (subnormal), times the scale
    step = np.maximum(np.abs(before) * 2.0 ** -4, 2.0 ** -10 * s_new[:, None, None, None])
    assert np.all(np.abs(after - before) <= step * (1 + 1e-6))
    assert np.abs(after - before).max() > 0                                         # it really was re-encoded
    # reference for the re-encoding itself: the library float8 conversion of value * s_old / s_new
    for h in range(H):
        v = (lut[grown_codes := blk(oracle_pool_copy(oracle, quiet, H))[h, :, :5]].astype(np.float32) * s_old[h]) / s_new[h]
        ref = torch.from_numpy(v.astype(np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        assert np.array_equal(blk(p)[h, :, :5], ref)
    p.write([2], 6, quiet[:3], quiet[:3])
    assert np.array_equal(p.k_scale[2 * H: 3 * H], s_new)                              # (c)


def oracle_pool_copy(oracle, quiet, H):
    """The page of the test above as it was before the loud token (a fresh pool written the same way)."""
    q = oracle.HostPool(3, H, oracle.FP8_E4M3)
    q.write([2], 0, quiet, quiet)
    return q


def _fork_scenario(seed: int, H: int):
    """One parent sequence of 40 tokens (its third page holds 8), continued three ways."""
    rng = np.random.default_rng(seed)
    mk = lambda n: wl.f32_to_bf16_bits(rng.standard_normal((n, H, D)).astype(np.float32))
    return {"parent": (mk(40), mk(40)), "a": (mk(3), mk(3)), "b": (mk(5), mk(5)), "c": (mk(12), mk(12))}


@pytest.mark.parametrize("dtype_name", ["BF16", "FP8_E4M3"])
def test_forked_sequences_through_page_copies(oracle, dtype_name):
    """A sequence forked inside a partially filled page: after a private copy of that page and divergent
    appends, every branch's pool content and attention equal those of the same branch written alone into
    pages of its own (same write calls, so fp8 scales take the same history), and the siblings' appends
    leave one another's pages untouched."""
    dt = getattr(oracle, dtype_name)
    H, Hq = 2, 4
    tok = _fork_scenario(31, H)
    kp, vp = tok["parent"]
    shared = oracle.HostPool(12, H, dt)
    shared.write([0, 1, 2], 0, kp, vp)                 # parent: pages 0, 1 full, page 2 holds 8 tokens
    shared.copy_page(2, 3)                             # branch b
    shared.copy_page(2, 4)                             # branch c
    shared.write([2], 8, *tok["a"])                    # the parent itself goes on in place
    shared.write([3], 8, *tok["b"])
    shared.write([4, 5], 8, *tok["c"])                 # runs over into a fresh page
    tables = {"a": [0, 1, 2], "b": [0, 1, 3], "c": [0, 1, 4, 5]}
    q = np.random.default_rng(5).standard_normal((1, Hq, D)).astype(np.float32)
    for name, table in tables.items():
        own = oracle.HostPool(12, H, dt)
        kb, vb = tok[name]
        own_table = [7, 8, 9, 10][:len(table)]
        own.write(own_table[:3], 0, kp, vp)
        own.write(own_table[2:], 8, kb, vb)
        n = 40 + kb.shape[0]
        nb = H * PAGE * D
        for ps, po in zip(table, own_table):
            assert np.array_equal(shared.k[ps * nb:(ps + 1) * nb], own.k[po * nb:(po + 1) * nb]), (name, ps)
            assert np.array_equal(shared.v[ps * nb:(ps + 1) * nb], own.v[po * nb:(po + 1) * nb]), (name, ps)
        bt = lambda t: np.asarray([t + [-1] * (4 - len(t))], dtype=np.int32)
        o1, l1 = oracle.attn_decode(shared, q, bt(table), [n], 0.1)
        o2, l2 = oracle.attn_decode(own, q, bt(own_table), [n], 0.1)
        assert np.array_equal(o1, o2) and np.array_equal(l1, l2)


# ------------------------------------------------------------------ attention read straight from the forest

@pytest.mark.parametrize("seed", [11, 12, 13])
def test_tree_walk_decode_equals_block_table_decode_on_aligned_forests(oracle, seed):
    """Where a flat block table exists (nodes with children hold whole pages), walking the forest node by
    node must give the table-based result bit for bit (same token order, same arithmetic)."""
    w = wl.random_forest_workload(seed, max_node_pages=3, depth=4, fanout=3)
    pool = oracle_pool(oracle, w)
    f = w.forest
    bt, kv_len, *_ = oracle.flatten_workload(w)
    o1, l1 = oracle.attn_decode(pool, w.q(), bt, kv_len, float(w.scale))
    o2, l2 = oracle.attn_decode_tree(pool, w.q(), f.nodes, f.node_pages, f.req_leaf, float(w.scale))
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)


@pytest.mark.parametrize("seed,kv", [(21, "bf16"), (22, "bf16"), (23, "fp32")])
def test_tree_walk_decode_brute_force_with_ragged_internal_nodes(oracle, seed, kv):
    """Nodes with children that end inside a page: against dense numpy attention over each request's
    sequence assembled from the node tensors without any pool."""
    w = wl.random_forest_workload(seed, max_node_pages=2, depth=4, fanout=2, ragged_internal=True,
                                  src_dtype="fp32" if kv == "fp32" else "bf16",
                                  kv_dtype=wl.KV_FP32 if kv == "fp32" else wl.KV_BF16)
    f = w.forest
    has_child = np.zeros(f.n_nodes, dtype=bool)
    has_child[f.parent[f.parent >= 0]] = True
    assert (has_child & (f.n_tokens % 16 != 0)).any(), "the case must hold a ragged node with children"
    out, lse = oracle.run_workload(w)
    bout, blse = brute_workload(w)
    assert np.abs(out - bout).max() <= 1e-12
    fin = np.isfinite(blse)
    assert np.array_equal(np.isfinite(lse), fin) and np.abs(lse[fin] - blse[fin]).max() <= 1e-12


def test_tree_walk_decode_leaf_visibility(oracle):
    """leaf_visible cuts the request's last node: equal to the same forest with that node shortened."""
    w = wl.random_forest_workload(31, max_node_pages=2, depth=3, fanout=2, ragged_internal=True, zero_weight_nodes=False)
    f = w.forest
    pool = oracle_pool(oracle, w)
    vis = np.maximum(f.n_tokens[f.req_leaf] - 3, 0).astype(np.int32)
    o1, l1 = oracle.attn_decode_tree(pool, w.q(), f.nodes, f.node_pages, f.req_leaf, float(w.scale), leaf_visible=vis)
    q = _as_f64(w.q())
    for r in range(f.n_req):
        K, V = logical_kv(w, r)
        T = K.shape[0] - (int(f.n_tokens[f.req_leaf[r]]) - int(vis[r]))
        for h in range(w.num_q_heads):
            o, l = brute_attention(q[r, h], K[:T, h // w.group], V[:T, h // w.group], float(w.scale))
            assert np.abs(o1[r, h] - o).max() <= 1e-12
            assert (np.isneginf(l) and np.isneginf(l1[r, h])) or abs(l1[r, h] - l) <= 1e-12


def _draft_tree(widths):
    """Parents of the drafted tokens of one tree in topological order (-1: child of the context)."""
    parents, level = [], [-1]
    for wd in widths:
        nxt = []
        for p in level:
            for _ in range(wd):
                parents.append(p)
                nxt.append(len(parents) - 1)
        level = nxt
    return parents


def _ancestor_masks(parents):
    masks = []
    for t in range(len(parents)):
        m, v = 0, t
        while v >= 0:
            m |= 1 << v
            v = parents[v]
        masks.append(m)
    return masks


def test_drafted_token_masks_equal_one_node_per_drafted_token(oracle):
    """Two formulations of the verification of a tree of drafted tokens must agree bit for bit in the oracle:
    (A) the drafted tokens are the last T tokens of the request's leaf node and every query row carries a
    bit mask of the drafted tokens it sees (its ancestors and itself); (B) every drafted token is a forest
    node of its own under the context, the forest being the mask (pinned above against dense attention)."""
    H, Hq, ctx_len = 2, 4, 37
    parents = _draft_tree((2, 2, 1))                 # 2 + 4 + 4 = 10 drafted tokens
    T = len(parents)
    rng = np.random.default_rng(19)
    mk = lambda n: wl.f32_to_bf16_bits(rng.standard_normal((n, H, D)).astype(np.float32))
    root_kv, ctx_kv, draft_kv = (mk(32), mk(32)), (mk(ctx_len), mk(ctx_len)), (mk(T), mk(T))
    q = wl.f32_to_bf16_bits(rng.standard_normal((T, Hq, D)).astype(np.float32))
    # (A) root -> one leaf holding context + drafted tokens
    n_leaf = ctx_len + T
    pa = oracle.HostPool(2 + (n_leaf + 15) // 16, H, oracle.BF16)
    pa.write([0, 1], 0, *root_kv)
    leaf_pages = list(range(2, 2 + (n_leaf + 15) // 16))
    pa.write(leaf_pages, 0, np.concatenate([ctx_kv[0], draft_kv[0]]), np.concatenate([ctx_kv[1], draft_kv[1]]))
    nodes_a = np.array([[-1, 0, 2, 32], [0, 2, len(leaf_pages), n_leaf]], dtype=np.int32)
    oa, la = oracle.attn_decode_tree(pa, q, nodes_a, np.array([0, 1] + leaf_pages, dtype=np.int32), [1] * T, 0.1,
                                     tail_len=T, tail_mask=_ancestor_masks(parents))
    # (B) root -> context -> one node per drafted token
    n_ctx_pages = (ctx_len + 15) // 16
    pb = oracle.HostPool(2 + n_ctx_pages + T, H, oracle.BF16)
    pb.write([0, 1], 0, *root_kv)
    pb.write(list(range(2, 2 + n_ctx_pages)), 0, *ctx_kv)
    rows_b = [[-1, 0, 2, 32], [0, 2, n_ctx_pages, ctx_len]]
    for t in range(T):
        pb.write([2 + n_ctx_pages + t], 0, draft_kv[0][t:t + 1], draft_kv[1][t:t + 1])
        rows_b.append([1 if parents[t] < 0 else 2 + parents[t], 2 + n_ctx_pages + t, 1, 1])
    ob, lb = oracle.attn_decode_tree(pb, q, np.array(rows_b, dtype=np.int32), np.arange(2 + n_ctx_pages + T, dtype=np.int32),
                                     [2 + t for t in range(T)], 0.1)
    assert np.array_equal(oa, ob) and np.array_equal(la, lb)
    # and a causal run is the mask with bits 0..t: equal to leaf_visible
    oc, lc = oracle.attn_decode_tree(pa, q, nodes_a, np.array([0, 1] + leaf_pages, dtype=np.int32), [1] * T, 0.1,
                                     tail_len=T, tail_mask=[(1 << (t + 1)) - 1 for t in range(T)])
    od, ld = oracle.attn_decode_tree(pa, q, nodes_a, np.array([0, 1] + leaf_pages, dtype=np.int32), [1] * T, 0.1,
                                     leaf_visible=[ctx_len + t + 1 for t in range(T)])
    assert np.array_equal(oc, od) and np.array_equal(lc, ld)


# ------------------------------------------------------------------ pages of 32, 64 and 128 tokens

@pytest.mark.parametrize("dtype_name", ["BF16", "FP8_E4M3", "FP32"])
@pytest.mark.parametrize("P", [32, 64, 128])
def test_larger_pages_are_runs_of_16_token_blocks(oracle, dtype_name, P):
    """A page of P = 16 S tokens is the S consecutive 16-token blocks p S .. p S + S - 1 of the same
    buffers: writing a sequence through P-token pages [p0, p1, ..] leaves, bit for bit, what writing it
    through the 16-token pages [p0 S, p0 S + 1, .., p1 S, ..] leaves (the 16-token format is pinned above),
    in one piece and in appended pieces that start inside a page and inside a block."""
    dtype = getattr(oracle, dtype_name)
    rng = np.random.default_rng(P)
    S, H, n_big = P // 16, 2, 5
    T = 2 * P + 21
    amp = np.linspace(0.2, 5.0, T)[:, None, None]             # growing magnitudes: fp8 scales rise on appends
    kf = (amp * rng.standard_normal((T, H, D))).astype(np.float32)
    vf = (amp[::-1] * rng.standard_normal((T, H, D))).astype(np.float32)
    k, v = (kf, vf) if dtype == oracle.FP32 else (wl.f32_to_bf16_bits(kf), wl.f32_to_bf16_bits(vf))
    big = np.array([3, 0, 4], dtype=np.int32)
    small = (big[:, None] * S + np.arange(S)[None, :]).reshape(-1).astype(np.int32)
    for cuts in ([0, T], [0, 5, 16, 21, P + 3, P + 4, 2 * P - 1, T]):
        a_pool = oracle.HostPool(n_big, H, dtype, page_size=P)
        b_pool = oracle.HostPool(n_big * S, H, dtype)
        for a, b in zip(cuts[:-1], cuts[1:]):
            a_pool.write(big[a // P:], a % P, k[a:b], v[a:b])
            b_pool.write(small[a // 16:], a % 16, k[a:b], v[a:b])
        for name in ("k", "v") + (("k_scale", "v_scale") if dtype == oracle.FP8_E4M3 else ()):
            x, y = getattr(a_pool, name), getattr(b_pool, name)
            assert x.shape == y.shape and np.array_equal(x.view(np.uint8), y.view(np.uint8)), (name, cuts)
    # and attention reads them back the same way: a P-page table against the equivalent 16-token table
    q = rng.standard_normal((1, 4, D)).astype(np.float32)
    q = q if dtype == oracle.FP32 else wl.f32_to_bf16_bits(q)
    o1, l1 = oracle.attn_decode(a_pool, q, big[None, :], np.array([T], dtype=np.int32), 0.09)
    o2, l2 = oracle.attn_decode(b_pool, q, small[None, :], np.array([T], dtype=np.int32), 0.09)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)
    a_pool.copy_page(3, 1)
    big2 = np.array([1, 0, 4], dtype=np.int32)
    o3, l3 = oracle.attn_decode(a_pool, q, big2[None, :], np.array([T], dtype=np.int32), 0.09)
    assert np.array_equal(o1, o3) and np.array_equal(l1, l3)


@pytest.mark.parametrize("P", [32, 64])
@pytest.mark.parametrize("seed,mode", [(5, "decode"), (6, "prefill")])
def test_brute_force_small_forests_with_larger_pages(oracle, P, seed, mode):
    w = wl.random_forest_workload(seed, mode=mode, page_size=P, max_node_pages=2, depth=3, fanout=2)
    assert w.page_size == P and (w.forest.n_pages == (w.forest.n_tokens + P - 1) // P).all()
    got_o, got_l = oracle.run_workload(w)
    exp_o, exp_l = brute_workload(w)
    assert np.abs(got_o - exp_o).max() <= 1e-12
    fin = np.isfinite(exp_l)
    assert np.array_equal(np.isneginf(got_l), np.isneginf(exp_l)) and np.abs(got_l[fin] - exp_l[fin]).max() <= 1e-12


@pytest.mark.parametrize("P", [32, 128])
def test_tree_walk_with_larger_pages_and_ragged_internal_nodes(oracle, P):
    w = wl.random_forest_workload(77, page_size=P, max_node_pages=2, depth=3, fanout=2, ragged_internal=True)
    f = w.forest
    has_child = np.zeros(f.n_nodes, dtype=bool)
    has_child[f.parent[f.parent >= 0]] = True
    assert (has_child & (f.n_tokens % P != 0)).any()
    got_o, got_l = oracle.run_workload(w)
    exp_o, exp_l = brute_workload(w)
    assert np.abs(got_o - exp_o).max() <= 1e-12


@pytest.mark.parametrize("P", [32, 64])
def test_flatten_tree_with_larger_pages_against_python_walk(oracle, P):
    w = wl.random_forest_workload(27, depth=4, fanout=3, n_roots=3, page_size=P)
    f = w.forest
    mp = max(1, f.max_pages_per_req()) + 2
    got = oracle.flatten_tree(f.nodes, f.node_pages, f.req_leaf, mp, P)
    for g, e in zip(got, py_flatten(f, mp)):
        assert np.array_equal(g, e)
    with pytest.raises(ValueError):                # the same forest is malformed for another page size
        oracle.flatten_tree(f.nodes, f.node_pages, f.req_leaf, mp, 16)
