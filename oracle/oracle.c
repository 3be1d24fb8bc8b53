/*
 * CPU oracle for attention over a paged, prefix-shared KV pool.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP library is checked against.  Only tests, the smoke check and the
 * bench's cpu_baseline leg may build, load or call it.  It shares no code,
 * header, table or constant with the HIP path and must never be reached from
 * the product path.
 *
 * What it computes.  The paper (Section 5, "Proactive Cache Management" and
 * the token-usage cost model) fixes the problem, not a kernel: the KV cache
 * of a prompt prefix shared by many LLM calls is stored once, block by block,
 * and a call processes only the tokens below the part of its root-to-leaf
 * path that is already cached.  Section 2 ("Scope") requires optimised
 * execution to return what naive execution returns.  Sharing pages and
 * combining per-node partial results therefore has to equal, up to rounding,
 * ordinary softmax attention of every query over the full key/value sequence
 * of its own request.  This oracle is that ordinary definition written out
 * in double precision: walk the tree to get each request's page list, gather
 * its keys and values one token at a time through the page table, and apply
 * max-subtracted softmax attention.  No tiling, no sharing, no partial
 * results (the one log-sum-exp combine below is the definition of that
 * operation itself, kept separate).
 *
 * Pool layout (the documented storage format of the library, indexed here by
 * this file's own code).  Storage is an array of blocks of 16 token slots; a
 * page of P = 16*S tokens (S = 1, 2, 4, 8) is the blocks p*S .. p*S + S - 1,
 * slot s of the page being slot s % 16 of block b = p*S + s / 16.  For block b
 * and KV head h, the K block and the V block each hold 16*128 elements and
 * start at element (b*Hkv + h)*2048.  Inside a K block the 128 dimensions are cut into
 * chunks of 64 bytes (C = 64/sizeof(element) dimensions); element (slot t,
 * dim d) sits at (d / C)*16*C + t*C + d % C.  Inside a V block the layout is
 * dimension-major: element (t, d) sits at d*16 + t.  fp8 pools carry two
 * float arrays k_scale[b*Hkv + h], v_scale[b*Hkv + h]; the stored value is
 * code * scale.
 *
 * Every function is pinned by tests/test_oracle_*.py against brute force,
 * closed forms, a library routine and invariants; nothing here is "parity
 * unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_BLOCK 16 /* token slots per storage block */
#define ORC_D 128

enum { ORC_BF16 = 0, ORC_FP8_E4M3 = 1, ORC_FP32 = 2 };

typedef struct {
    int32_t num_pages;
    int32_t num_kv_heads;
    int32_t dtype;
    int32_t page_size; /* tokens per page: 16, 32, 64 or 128 */
    const void *k_pages;
    const void *v_pages;
    const float *k_scale; /* fp8 only */
    const float *v_scale; /* fp8 only */
} orc_pool;

/* ---------------------------------------------------------------- element decoding */

static double bf16_to_double(uint16_t b) {
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* OCP 8-bit float, 4 exponent bits (bias 7), 3 mantissa bits, no infinities,
 * S.1111.111 is NaN, largest finite value 448. */
double orc_e4m3_value(uint8_t c) {
    int s = c >> 7, e = (c >> 3) & 15, m = c & 7;
    double v;
    if (e == 15 && m == 7) return NAN;
    if (e == 0)
        v = ldexp((double)m / 8.0, -6);
    else
        v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return s ? -v : v;
}

/* Round-to-nearest-even onto the e4m3 grid, saturating at +-448.  The grid spacing around a is
 * 2^(e-3) with e = floor(log2 a), but never finer than the subnormal spacing 2^-9; a / spacing is
 * rounded to the nearest integer with ties to even (rint under the default rounding mode), which
 * may carry into the next binade, and the code is read off the rounded value. */
uint8_t orc_e4m3_encode(float y) {
    if (isnan(y)) return 0x7F;
    uint8_t sign = signbit(y) ? 0x80 : 0x00;
    double a = fabs((double)y);
    if (a >= 448.0) return (uint8_t)(sign | 0x7E);
    int e;
    (void)frexp(a, &e); /* a = f * 2^e with f in [0.5, 1)  ->  floor(log2 a) = e - 1 */
    e -= 1;
    if (a == 0.0 || e < -6) e = -6;
    double spacing = ldexp(1.0, e - 3);
    double v = rint(a / spacing) * spacing; /* exact: a / spacing < 16 has few significant bits */
    if (v > 448.0) v = 448.0;
    int code;
    if (v < ldexp(1.0, -6)) {
        code = (int)(v / ldexp(1.0, -9)); /* subnormal: mantissa in units of 2^-9 */
    } else {
        int e2;
        double f = frexp(v, &e2); /* v = f * 2^e2, f in [0.5, 1) -> v = (2f) * 2^(e2-1) */
        code = ((e2 - 1 + 7) << 3) | (int)((2.0 * f - 1.0) * 8.0);
    }
    return (uint8_t)(sign | code);
}

static size_t elem_size(int dtype) { return dtype == ORC_BF16 ? 2 : dtype == ORC_FP8_E4M3 ? 1 : 4; }

/* storage block that holds slot `slot` (0 .. page_size - 1) of page `page` */
static size_t block_of(const orc_pool *p, int page, int slot) {
    return (size_t)page * (size_t)(p->page_size / ORC_BLOCK) + (size_t)(slot / ORC_BLOCK);
}

static size_t k_offset(const orc_pool *p, int page, int head, int slot, int d) {
    size_t C = 64 / elem_size(p->dtype);
    size_t block = (block_of(p, page, slot) * p->num_kv_heads + head) * (ORC_BLOCK * ORC_D);
    return block + (size_t)(d / C) * ORC_BLOCK * C + (size_t)(slot % ORC_BLOCK) * C + (size_t)(d % C);
}

static size_t v_offset(const orc_pool *p, int page, int head, int slot, int d) {
    size_t block = (block_of(p, page, slot) * p->num_kv_heads + head) * (ORC_BLOCK * ORC_D);
    return block + (size_t)d * ORC_BLOCK + (size_t)(slot % ORC_BLOCK);
}

static double load_elem(const orc_pool *p, const void *base, const float *scale, size_t off, int page, int slot,
                        int head) {
    switch (p->dtype) {
    case ORC_BF16: return bf16_to_double(((const uint16_t *)base)[off]);
    case ORC_FP8_E4M3:
        return orc_e4m3_value(((const uint8_t *)base)[off]) *
               (double)scale[block_of(p, page, slot) * p->num_kv_heads + head];
    default: return (double)((const float *)base)[off];
    }
}

static double load_k(const orc_pool *p, int page, int head, int slot, int d) {
    return load_elem(p, p->k_pages, p->k_scale, k_offset(p, page, head, slot, d), page, slot, head);
}
static double load_v(const orc_pool *p, int page, int head, int slot, int d) {
    return load_elem(p, p->v_pages, p->v_scale, v_offset(p, page, head, slot, d), page, slot, head);
}

static double load_q(const void *q, int q_dtype, size_t idx) {
    return q_dtype == ORC_FP32 ? (double)((const float *)q)[idx] : bf16_to_double(((const uint16_t *)q)[idx]);
}

/* ---------------------------------------------------------------- tree indexing */

/* nodes: [n_nodes][4] = (parent, page_begin, n_pages, n_tokens), parents before children.
 * Section 5 defines path(r, l) as the nodes from the root down to the leaf; a call's
 * prompt is the concatenation of their token segments.  Returns 0, or a negative code:
 * -1 bad argument, -2 index out of range, -4 malformed tree, -5 max_pages too small.
 * page_size: tokens per page of the forest (a node of n tokens holds ceil(n / page_size) pages). */
int oracle_flatten_tree(const int32_t *nodes, int32_t n_nodes, const int32_t *node_pages, int32_t n_node_pages,
                        const int32_t *req_leaf, int32_t n_req, int32_t page_size, int32_t max_pages,
                        int32_t *block_table, int32_t *kv_len, int32_t *node_req_indptr, int32_t *node_req_idx,
                        int32_t *node_tok_start) {
    if (n_nodes < 0 || n_req < 0 || max_pages < 0 || page_size <= 0) return -1;
    int *has_child = (int *)calloc((size_t)n_nodes + 1, sizeof(int));
    for (int v = 0; v < n_nodes; ++v) {
        int par = nodes[4 * v], pb = nodes[4 * v + 1], np = nodes[4 * v + 2], nt = nodes[4 * v + 3];
        if (par < -1 || par >= v) { free(has_child); return -4; }
        if (nt < 0 || np != (nt + page_size - 1) / page_size) { free(has_child); return -4; }
        if (pb < 0 || pb + np > n_node_pages) { free(has_child); return -2; }
        if (par >= 0) has_child[par] = 1;
    }
    for (int v = 0; v < n_nodes; ++v)
        if (has_child[v] && nodes[4 * v + 3] % page_size != 0) { free(has_child); return -4; }
    free(has_child);

    /* token offset at which each node's segment starts along its root path */
    for (int v = 0; v < n_nodes; ++v) {
        int par = nodes[4 * v];
        node_tok_start[v] = par < 0 ? 0 : node_tok_start[par] + nodes[4 * par + 3];
    }
    /* per request: page list along root -> leaf */
    int *stack = (int *)malloc(sizeof(int) * ((size_t)n_nodes + 1));
    for (int r = 0; r < n_req; ++r) {
        int leaf = req_leaf[r];
        if (leaf < 0 || leaf >= n_nodes) { free(stack); return -2; }
        int depth = 0;
        for (int v = leaf; v >= 0; v = nodes[4 * v]) stack[depth++] = v;
        int n = 0, len = 0;
        for (int i = depth - 1; i >= 0; --i) {
            int v = stack[i];
            for (int j = 0; j < nodes[4 * v + 2]; ++j) {
                if (n >= max_pages) { free(stack); return -5; }
                block_table[(size_t)r * max_pages + n++] = node_pages[nodes[4 * v + 1] + j];
            }
            len += nodes[4 * v + 3];
        }
        for (; n < max_pages; ++n) block_table[(size_t)r * max_pages + n] = -1;
        kv_len[r] = len;
    }
    /* node -> requests whose path passes through it, ascending request order */
    int pos = 0;
    for (int v = 0; v < n_nodes; ++v) {
        node_req_indptr[v] = pos;
        for (int r = 0; r < n_req; ++r) {
            int on_path = 0;
            for (int u = req_leaf[r]; u >= 0; u = nodes[4 * u])
                if (u == v) on_path = 1;
            if (on_path) node_req_idx[pos++] = r;
        }
    }
    node_req_indptr[n_nodes] = pos;
    free(stack);
    return 0;
}

/* Prefill token usage u_p of Section 5 ("Token usage"): the first call of a worker's
 * schedule processes every token on path(r, l_1); call j > 1 processes only the tokens on
 * the path from the lowest common ancestor of l_{j-1} and l_j (exclusive) down to l_j. */
int oracle_prefill_usage(const int32_t *nodes, int32_t n_nodes, const int32_t *calls, int32_t n_calls,
                         int64_t *u_p) {
    for (int j = 0; j < n_calls; ++j) {
        int l = calls[j];
        if (l < 0 || l >= n_nodes) return -2;
        int lca = -1; /* -1: nothing shared (also when the two leaves sit under different roots) */
        if (j > 0) {
            for (int a = calls[j - 1]; a >= 0 && lca < 0; a = nodes[4 * a])
                for (int b = l; b >= 0; b = nodes[4 * b])
                    if (a == b) { lca = a; break; }
        }
        int64_t s = 0;
        for (int v = l; v >= 0 && v != lca; v = nodes[4 * v]) s += nodes[4 * v + 3];
        u_p[j] = s;
    }
    return 0;
}

/* ---------------------------------------------------------------- pool writer */

static void store_bf16_or_f32(void *base, int dtype, size_t off, const void *src, int src_dtype, size_t sidx) {
    if (dtype == ORC_BF16)
        ((uint16_t *)base)[off] = ((const uint16_t *)src)[sidx];
    else
        ((float *)base)[off] = src_dtype == ORC_FP32 ? ((const float *)src)[sidx]
                                                     : (float)bf16_to_double(((const uint16_t *)src)[sidx]);
}

static float src_as_float(const void *src, int src_dtype, size_t i) {
    return src_dtype == ORC_FP32 ? ((const float *)src)[i] : (float)bf16_to_double(((const uint16_t *)src)[i]);
}

/* Store n_tokens consecutive tokens ([n_tokens][Hkv][128], bf16 bits or float) into the pages
 * page_ids[0..], starting at slot first_slot (< page size) of page_ids[0].  This is the "precompute and keep
 * the KV cache" step of Section 5 seen from the pool.  bf16/fp32 pools: plain copy.  fp8 pools:
 * a (16-slot block, head) block written from its slot 0 gets scale = amax/448 over the tokens written into it
 * (1 if amax is 0), computed in float, and code = RNE(x / scale) with the division in float.
 * A block that is continued (first block of a call, first_slot % 16 > 0) keeps a running scale:
 * scale' = max(scale, amax_new/448); when the scale grows, the codes already in slots below
 * first_slot % 16 are re-encoded as RNE(value(code) * scale / scale'), product and quotient in float;
 * the scale never shrinks.  Returns 0 or a negative code as in oracle_flatten_tree. */
int oracle_kv_write(orc_pool *p, void *k_pages, void *v_pages, float *k_scale, float *v_scale,
                    const int32_t *page_ids, int32_t first_slot, int32_t n_tokens, const void *k_src,
                    const void *v_src, int32_t src_dtype) {
    int H = p->num_kv_heads, P = p->page_size;
    if (n_tokens < 0 || first_slot < 0 || first_slot >= P) return -1;
    if (p->dtype == ORC_BF16 && src_dtype != ORC_BF16) return -1;
    int n_pg = (first_slot + n_tokens + P - 1) / P;
    for (int i = 0; i < n_pg; ++i)
        if (page_ids[i] < 0 || page_ids[i] >= p->num_pages) return -2;
    if (p->dtype != ORC_FP8_E4M3) {
        for (int t = 0; t < n_tokens; ++t) {
            int page = page_ids[(first_slot + t) / P], slot = (first_slot + t) % P;
            for (int h = 0; h < H; ++h)
                for (int d = 0; d < ORC_D; ++d) {
                    size_t s = ((size_t)t * H + h) * ORC_D + d;
                    store_bf16_or_f32(k_pages, p->dtype, k_offset(p, page, h, slot, d), k_src, src_dtype, s);
                    store_bf16_or_f32(v_pages, p->dtype, v_offset(p, page, h, slot, d), v_src, src_dtype, s);
                }
        }
        return 0;
    }
    /* fp8: one scale per storage block of 16 slots; walk the blocks the tokens land in */
    int g0 = first_slot / ORC_BLOCK;      /* first block touched, counted along the listed pages */
    int fs = first_slot % ORC_BLOCK;      /* first slot written in it */
    int n_blk = (fs + n_tokens + ORC_BLOCK - 1) / ORC_BLOCK;
    for (int i = 0; i < n_blk; ++i) {
        int at = (g0 + i) * ORC_BLOCK;                              /* slot along the listed pages */
        int page = page_ids[at / P], base = at % P;                 /* the block's first slot in its page */
        size_t blk = block_of(p, page, base);
        int s_lo = i == 0 ? fs : 0;                                /* first slot written in this block */
        int t0 = i == 0 ? 0 : i * ORC_BLOCK - fs;                  /* token that lands in slot s_lo */
        int t1 = (i + 1) * ORC_BLOCK - fs < n_tokens ? (i + 1) * ORC_BLOCK - fs : n_tokens;
        for (int h = 0; h < H; ++h)
            for (int which = 0; which < 2; ++which) {
                const void *src = which ? v_src : k_src;
                uint8_t *codes = (uint8_t *)(which ? v_pages : k_pages);
                float *scales = which ? v_scale : k_scale;
                float amax = 0.0f;
                for (int t = t0; t < t1; ++t)
                    for (int d = 0; d < ORC_D; ++d) {
                        float a = fabsf(src_as_float(src, src_dtype, ((size_t)t * H + h) * ORC_D + d));
                        if (a > amax) amax = a;
                    }
                float scale;
                if (s_lo == 0) {
                    scale = amax > 0.0f ? amax / 448.0f : 1.0f;
                } else {
                    float old = scales[blk * H + h];
                    float cand = amax > 0.0f ? amax / 448.0f : 0.0f;
                    scale = old >= cand ? old : cand;   /* an unset (NaN) old scale gives cand */
                    if (!(scale > 0.0f)) scale = 1.0f;
                    if (scale > old)
                        for (int sl = 0; sl < s_lo; ++sl)
                            for (int d = 0; d < ORC_D; ++d) {
                                size_t off = which ? v_offset(p, page, h, base + sl, d) : k_offset(p, page, h, base + sl, d);
                                float v = (float)orc_e4m3_value(codes[off]) * old;
                                codes[off] = orc_e4m3_encode(v / scale);
                            }
                }
                scales[blk * H + h] = scale;
                for (int t = t0; t < t1; ++t)
                    for (int d = 0; d < ORC_D; ++d) {
                        float x = src_as_float(src, src_dtype, ((size_t)t * H + h) * ORC_D + d);
                        float y = x / scale;
                        int sl = base + s_lo + (t - t0);
                        size_t off = which ? v_offset(p, page, h, sl, d) : k_offset(p, page, h, sl, d);
                        codes[off] = orc_e4m3_encode(y);
                    }
            }
    }
    return 0;
}

/* ---------------------------------------------------------------- attention */

/* Softmax attention of one query vector over the tokens [t0, t1) of one request, read through
 * its page list: s_t = scale * <q, K_t>, m = max s_t, p_t = exp(s_t - m), l = sum p_t,
 * o = sum p_t V_t / l, lse = m + ln l.  An empty range gives o = 0, lse = -inf.
 * probs (optional, length t1 - t0) receives p_t / l. */
static void attend_range(const orc_pool *p, const int32_t *pages, int kv_head, const double *qv, double scale,
                         int t0, int t1, double *o, double *lse, double *probs) {
    int n = t1 - t0;
    for (int d = 0; d < ORC_D; ++d) o[d] = 0.0;
    if (n <= 0) {
        *lse = -INFINITY;
        return;
    }
    double *s = (double *)malloc(sizeof(double) * (size_t)n);
    double m = -INFINITY;
    for (int t = t0; t < t1; ++t) {
        int page = pages[t / p->page_size], slot = t % p->page_size;
        double acc = 0.0;
        for (int d = 0; d < ORC_D; ++d) acc += qv[d] * load_k(p, page, kv_head, slot, d);
        s[t - t0] = scale * acc;
        if (s[t - t0] > m) m = s[t - t0];
    }
    double l = 0.0;
    for (int i = 0; i < n; ++i) {
        s[i] = exp(s[i] - m);
        l += s[i];
    }
    for (int t = t0; t < t1; ++t) {
        int page = pages[t / p->page_size], slot = t % p->page_size;
        double w = s[t - t0];
        for (int d = 0; d < ORC_D; ++d) o[d] += w * load_v(p, page, kv_head, slot, d);
    }
    for (int d = 0; d < ORC_D; ++d) o[d] /= l;
    if (probs)
        for (int i = 0; i < n; ++i) probs[i] = s[i] / l;
    *lse = m + log(l);
    free(s);
}

static int check_pages(const orc_pool *p, const int32_t *pages, int kv_len) {
    int n = (kv_len + p->page_size - 1) / p->page_size;
    for (int i = 0; i < n; ++i)
        if (pages[i] < 0 || pages[i] >= p->num_pages) return -2;
    return 0;
}

/* Attention of one query token per request over tokens [seg_begin[r], seg_end[r]) of that
 * request's sequence (pass NULL, NULL for the whole sequence [0, kv_len[r])).
 * q: [n_req][Hq][128]; out: [n_req][Hq][128] double; lse: [n_req][Hq] double.
 * q-head h reads KV head h / (Hq / Hkv).  scale is the float the GPU receives, widened. */
int oracle_attn_decode(const orc_pool *p, const void *q, int32_t q_dtype, const int32_t *block_table,
                       int32_t max_pages, const int32_t *kv_len, const int32_t *seg_begin,
                       const int32_t *seg_end, int32_t n_req, int32_t num_q_heads, float scale, double *out,
                       double *lse) {
    if (num_q_heads <= 0 || num_q_heads % p->num_kv_heads) return -3;
    int G = num_q_heads / p->num_kv_heads;
    for (int r = 0; r < n_req; ++r) {
        if (kv_len[r] < 0 || kv_len[r] > max_pages * p->page_size) return -1;
        int rc = check_pages(p, block_table + (size_t)r * max_pages, kv_len[r]);
        if (rc) return rc;
    }
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int r = 0; r < n_req; ++r)
        for (int h = 0; h < num_q_heads; ++h) {
            double qv[ORC_D];
            for (int d = 0; d < ORC_D; ++d) qv[d] = load_q(q, q_dtype, ((size_t)r * num_q_heads + h) * ORC_D + d);
            int t0 = seg_begin ? seg_begin[r] : 0, t1 = seg_end ? seg_end[r] : kv_len[r];
            size_t o = (size_t)r * num_q_heads + h;
            attend_range(p, block_table + (size_t)r * max_pages, h / G, qv, (double)scale, t0, t1, out + o * ORC_D,
                         lse + o, NULL);
        }
    return 0;
}

/* The same attention taken straight from the forest (Section 5, templated radix tree: a call's
 * prompt is the concatenation of the token segments on the path from the root to its leaf), for
 * forests whose nodes may end inside a page anywhere: request r's sequence is, node by node from
 * the root down to req_leaf[r], token t of node v = slot t % P of page node_pages[page_begin_v +
 * t / P] (P the pool's page size).  nodes: [n_nodes][4] = parent, page_begin, n_pages, n_tokens (parents first).
 * leaf_visible (optional): of its last node request r sees only the first leaf_visible[r] tokens
 * (one of several query tokens of a call, which must not see the call's newer tokens).
 * tail_len, tail_mask (optional, instead of leaf_visible): the last tail_len tokens of the last node
 * are drafted tokens of which request r sees number j iff bit j of tail_mask[r] is set (its ancestors
 * in the tree of drafts and itself); everything before them it sees.
 * Plain definition: all scores, their maximum, the exponentials, the weighted sum. */
int oracle_attn_decode_tree(const orc_pool *p, const void *q, int32_t q_dtype, const int32_t *nodes, int32_t n_nodes,
                            const int32_t *node_pages, int32_t n_node_pages, const int32_t *req_leaf,
                            const int32_t *leaf_visible, int32_t tail_len, const uint64_t *tail_mask, int32_t n_req,
                            int32_t num_q_heads, float scale, double *out, double *lse) {
    if (tail_mask && (leaf_visible || tail_len < 1 || tail_len > 64)) return -1;
    if (num_q_heads <= 0 || num_q_heads % p->num_kv_heads) return -3;
    int G = num_q_heads / p->num_kv_heads;
    for (int v = 0; v < n_nodes; ++v) {
        const int32_t *nd = nodes + 4 * (size_t)v;
        if (nd[0] < -1 || nd[0] >= v || nd[3] < 0 || nd[2] != (nd[3] + p->page_size - 1) / p->page_size) return -4;
        if (nd[1] < 0 || (int64_t)nd[1] + nd[2] > n_node_pages) return -2;
        for (int j = 0; j < nd[2]; ++j)
            if (node_pages[nd[1] + j] < 0 || node_pages[nd[1] + j] >= p->num_pages) return -2;
    }
    for (int r = 0; r < n_req; ++r)
        if (req_leaf[r] < 0 || req_leaf[r] >= n_nodes) return -2;
#pragma omp parallel for schedule(dynamic)
    for (int r = 0; r < n_req; ++r) {
        /* the request's tokens in sequence order as (page, slot) pairs */
        int depth = 0, total = 0;
        for (int v = req_leaf[r]; v >= 0; v = nodes[4 * (size_t)v]) ++depth;
        int *chain = (int *)malloc(sizeof(int) * (size_t)(depth > 0 ? depth : 1));
        int i = depth;
        for (int v = req_leaf[r]; v >= 0; v = nodes[4 * (size_t)v]) chain[--i] = v;
        for (i = 0; i < depth; ++i) {
            int nt = nodes[4 * (size_t)chain[i] + 3];
            if (i == depth - 1 && leaf_visible && leaf_visible[r] < nt) nt = leaf_visible[r] < 0 ? 0 : leaf_visible[r];
            total += nt;
        }
        int *pg = (int *)malloc(sizeof(int) * (size_t)(total > 0 ? total : 1));
        int *sl = (int *)malloc(sizeof(int) * (size_t)(total > 0 ? total : 1));
        int n = 0;
        for (i = 0; i < depth; ++i) {
            const int32_t *nd = nodes + 4 * (size_t)chain[i];
            int nt = nd[3];
            if (i == depth - 1 && leaf_visible && leaf_visible[r] < nt) nt = leaf_visible[r] < 0 ? 0 : leaf_visible[r];
            for (int t = 0; t < nt; ++t) {
                if (i == depth - 1 && tail_mask && t >= nt - tail_len && !((tail_mask[r] >> (t - (nt - tail_len))) & 1u))
                    continue; /* a drafted token that is no ancestor of this one */
                pg[n] = node_pages[nd[1] + t / p->page_size];
                sl[n] = t % p->page_size;
                ++n;
            }
        }
        total = n;
        double *s = (double *)malloc(sizeof(double) * (size_t)(total > 0 ? total : 1));
        for (int h = 0; h < num_q_heads; ++h) {
            size_t row = (size_t)r * num_q_heads + h;
            double *o = out + row * ORC_D;
            for (int d = 0; d < ORC_D; ++d) o[d] = 0.0;
            if (total == 0) {
                lse[row] = -INFINITY;
                continue;
            }
            double qv[ORC_D];
            for (int d = 0; d < ORC_D; ++d) qv[d] = load_q(q, q_dtype, row * ORC_D + d);
            double m = -INFINITY;
            for (int t = 0; t < total; ++t) {
                double acc = 0.0;
                for (int d = 0; d < ORC_D; ++d) acc += qv[d] * load_k(p, pg[t], h / G, sl[t], d);
                s[t] = (double)scale * acc;
                if (s[t] > m) m = s[t];
            }
            double l = 0.0;
            for (int t = 0; t < total; ++t) {
                s[t] = exp(s[t] - m);
                l += s[t];
            }
            for (int t = 0; t < total; ++t)
                for (int d = 0; d < ORC_D; ++d) o[d] += s[t] * load_v(p, pg[t], h / G, sl[t], d);
            for (int d = 0; d < ORC_D; ++d) o[d] /= l;
            lse[row] = m + log(l);
        }
        free(s);
        free(sl);
        free(pg);
        free(chain);
    }
    return 0;
}

/* Suffix-only prefill (Section 5: a call processes only the tokens that are not already
 * cached).  Request r has s_r = cu_q[r+1] - cu_q[r] new tokens whose K/V are already in the
 * pool at positions prefix_len_r .. kv_len_r - 1, prefix_len_r = kv_len_r - s_r.  New token i
 * sits at absolute position a = prefix_len_r + i and attends every key t <= a.
 * q/out: [cu_q[n_req]][Hq][128]; lse: [cu_q[n_req]][Hq]. */
int oracle_attn_prefill(const orc_pool *p, const void *q, int32_t q_dtype, const int32_t *cu_q,
                        const int32_t *block_table, int32_t max_pages, const int32_t *kv_len, int32_t n_req,
                        int32_t num_q_heads, float scale, double *out, double *lse) {
    if (num_q_heads <= 0 || num_q_heads % p->num_kv_heads) return -3;
    int G = num_q_heads / p->num_kv_heads;
    if (n_req > 0 && cu_q[0] != 0) return -1;
    for (int r = 0; r < n_req; ++r) {
        int s = cu_q[r + 1] - cu_q[r];
        if (s < 0 || kv_len[r] < s || kv_len[r] > max_pages * p->page_size) return -1;
        int rc = check_pages(p, block_table + (size_t)r * max_pages, kv_len[r]);
        if (rc) return rc;
    }
    for (int r = 0; r < n_req; ++r) {
        int s = cu_q[r + 1] - cu_q[r];
        int prefix_len = kv_len[r] - s;
#pragma omp parallel for collapse(2) schedule(dynamic)
        for (int i = 0; i < s; ++i)
            for (int h = 0; h < num_q_heads; ++h) {
                double qv[ORC_D];
                size_t row = (size_t)(cu_q[r] + i) * num_q_heads + h;
                for (int d = 0; d < ORC_D; ++d) qv[d] = load_q(q, q_dtype, row * ORC_D + d);
                attend_range(p, block_table + (size_t)r * max_pages, h / G, qv, (double)scale, 0,
                             prefix_len + i + 1, out + row * ORC_D, lse + row, NULL);
            }
    }
    return 0;
}

/* The keys and values of one sequence, read through its page list and widened to double (fp8: code value
 * times the block's scale): k_out, v_out [kv_len][Hkv][128].  For the matrix form of the attention in
 * oracle.py, which needs the operands as arrays. */
int oracle_gather_kv(const orc_pool *p, const int32_t *pages, int32_t kv_len, double *k_out, double *v_out) {
    if (kv_len < 0) return -1;
    int rc = check_pages(p, pages, kv_len);
    if (rc) return rc;
#pragma omp parallel for schedule(static)
    for (int t = 0; t < kv_len; ++t) {
        int page = pages[t / p->page_size], slot = t % p->page_size;
        for (int h = 0; h < p->num_kv_heads; ++h)
            for (int d = 0; d < ORC_D; ++d) {
                size_t o = ((size_t)t * p->num_kv_heads + h) * ORC_D + d;
                k_out[o] = load_k(p, page, h, slot, d);
                v_out[o] = load_v(p, page, h, slot, d);
            }
    }
    return 0;
}

/* Normalised attention weights p_t / l of one (request, q-head) over its whole sequence;
 * exposed so that tests can check the softmax itself. */
int oracle_attn_probs(const orc_pool *p, const void *q, int32_t q_dtype, const int32_t *pages, int32_t kv_len,
                      int32_t q_head, int32_t num_q_heads, float scale, double *probs) {
    int G = num_q_heads / p->num_kv_heads;
    double qv[ORC_D], o[ORC_D], lse;
    for (int d = 0; d < ORC_D; ++d) qv[d] = load_q(q, q_dtype, (size_t)q_head * ORC_D + d);
    attend_range(p, pages, q_head / G, qv, (double)scale, 0, kv_len, o, &lse, probs);
    return 0;
}

/* Log-sum-exp combine of partial attention results: output row i owns the partials
 * part_idx[row_indptr[i] .. row_indptr[i+1]); with M = max lse_n,
 *   lse = M + ln sum_n exp(lse_n - M),   o = sum_n exp(lse_n - lse) o_n.
 * A partial with lse = -inf contributes nothing; a row with no finite partial gives
 * o = 0, lse = -inf. */
void oracle_lse_merge(const double *o_parts, const double *lse_parts, const int32_t *row_indptr,
                      const int32_t *part_idx, int32_t n_rows, double *out, double *lse_out) {
    for (int i = 0; i < n_rows; ++i) {
        double M = -INFINITY;
        for (int k = row_indptr[i]; k < row_indptr[i + 1]; ++k)
            if (lse_parts[part_idx[k]] > M) M = lse_parts[part_idx[k]];
        for (int d = 0; d < ORC_D; ++d) out[(size_t)i * ORC_D + d] = 0.0;
        if (M == -INFINITY) {
            lse_out[i] = -INFINITY;
            continue;
        }
        double z = 0.0;
        for (int k = row_indptr[i]; k < row_indptr[i + 1]; ++k) z += exp(lse_parts[part_idx[k]] - M);
        double L = M + log(z);
        for (int k = row_indptr[i]; k < row_indptr[i + 1]; ++k) {
            int n = part_idx[k];
            if (lse_parts[n] == -INFINITY) continue;
            double w = exp(lse_parts[n] - L);
            for (int d = 0; d < ORC_D; ++d) out[(size_t)i * ORC_D + d] += w * o_parts[(size_t)n * ORC_D + d];
        }
        lse_out[i] = L;
    }
}

int oracle_num_threads(void) {
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
