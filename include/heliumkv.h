/*
 * heliumkv: attention over a paged KV pool whose pages are shared through a prefix forest.
 *
 * C ABI of the MI355X (gfx950) library.  Every step behind these calls runs in hand-written
 * HIP kernels; there is no CPU fallback.  The operations are the GPU side of the proactive KV
 * caching and cache-aware scheduling of the Helium paper:
 *   - Section 5, "Proactive Cache Management": the KV cache of a prompt prefix shared by many
 *     LLM calls is computed once, kept in GPU memory block by block, and reused.
 *   - Section 5, "Token usage" (equation for u_p): a call processes only the tokens below the
 *     part of its root-to-leaf path that is already cached.
 *   - Section 5, templated radix tree T = (V, E, E'): prompts form a prefix tree; omega(v) is
 *     the number of tokens of node v's own segment and may be zero.
 *   - Section 2, "Scope": the optimised execution must return what naive execution returns, so
 *     every result here equals plain softmax attention of a query over its request's whole
 *     key/value sequence (up to floating-point rounding).
 *
 * Conventions
 *   - Every function returns HKV_OK (0) or a negative HKV_E* code and never throws.
 *     hkv_last_error() returns a thread-local message for the last failure on this thread.
 *   - "host" pointers are ordinary CPU memory read during the call; the caller may free or
 *     reuse them as soon as the call returns.  "device" pointers are HIP device memory of the
 *     current device, owned by the caller, and must stay valid until the work queued on
 *     `stream` has finished.  The library never frees caller memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Kernel launches are
 *     asynchronous on it.  All argument validation happens on the host before anything is
 *     queued, so a failing call has no effect on device memory.
 *   - Threads: objects (pools, plans, caches, trees) carry no locks.  Calls on different objects
 *     may run on different threads at once; calls on one object, and calls on a plan or cache and
 *     on the pool it was created over, must be serialised by the caller.  A plan's workspace and
 *     device index buffers belong to one run at a time: queue runs of one plan on one stream, or
 *     order them with events.
 *   - Geometry: head dimension 128; page size 16 tokens, or 32, 64 or 128 (a page of 16*S tokens
 *     is S consecutive 16-token blocks, see below).  Anything else is HKV_ESHAPE.  Where the text
 *     below says "16" about pages of a forest, a block table or a write, read the pool's page
 *     size; the storage format and the fp8 scales are always per 16-token block.
 *   - Grouped-query attention: query head h reads KV head h / (num_q_heads / num_kv_heads).
 *
 * Pool storage format (device memory owned by the caller, layout fixed by this library).
 *   Storage is an array of 16-token blocks.  With page size 16 block b is page b; with page size
 *   16*S page p is the blocks p*S .. p*S + S - 1, block p*S + j holding slots 16j .. 16j + 15 of
 *   the page (so a page is one contiguous range of the buffers, S times the 16-token size).
 *   For block b and KV head h, the K block and the V block each hold 16*128 elements and start
 *   at element (b*num_kv_heads + h)*2048 of k_pages / v_pages.
 *     K block: the 128 dimensions are cut into chunks of 64 bytes (C = 64/sizeof(element)
 *              dimensions: 32 for bf16, 64 for fp8, 16 for fp32); element (slot t, dim d) is at
 *              (d / C)*16*C + t*C + d % C.
 *     V block: dimension-major; element (slot t, dim d) is at d*16 + t.
 *   Both orders hand a 64-lane wavefront its matrix-core operands as 16-byte contiguous loads
 *   and make every (page, head) block one contiguous 4 KiB (bf16) / 2 KiB (fp8) burst.
 *   fp8 pools (OCP e4m3, no infinities, max 448) carry k_scale and v_scale, float
 *   [num_pages * S][num_kv_heads] (one scale per 16-token block and head); the stored value is
 *   code * scale.
 *   Slots past the end of a sequence and unreferenced pages may hold anything, NaN included.
 */
#ifndef HELIUMKV_H
#define HELIUMKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HKV_PAGE_SIZE 16
#define HKV_HEAD_DIM 128

enum {
    HKV_OK = 0,
    HKV_EINVAL = -1, /* null pointer, negative size, inconsistent lengths */
    HKV_ERANGE = -2, /* page id, node id or request id outside its range */
    HKV_ESHAPE = -3, /* unsupported geometry or dtype combination */
    HKV_ETREE = -4,  /* malformed forest: parent after child, page count != ceil(tokens/16); where a
                        flat block table is involved also a node with children whose token count
                        is not a multiple of 16 */
    HKV_ENOMEM = -5, /* pool exhausted, workspace or output table too small */
    HKV_EHIP = -6    /* a HIP runtime call failed (message holds the HIP error string) */
};

/* Pool element types.  bf16 and fp8 pools are the throughput paths (matrix cores, bf16 q and out).
 * An fp32 pool selects the full-precision path: k_src / v_src of kv_pool_write, q, and out of the
 * attention calls are then fp32 as well, all arithmetic is fp32 on the vector ALUs, one wavefront
 * per (query token, query head) without sharing between requests, no workspace is needed, and
 * results agree with exact attention to about 1e-6 (the bound asked of fp32 inputs is 1e-4).
 * fp32 block format: K in 64-byte chunks of 16 floats ((d/16)*256 + slot*16 + d%16), V
 * dimension-major (d*16 + slot). */
enum { HKV_BF16 = 0, HKV_FP8_E4M3 = 1, HKV_FP32 = 2 };

typedef struct hkv_pool hkv_pool;
typedef struct hkv_decode_plan hkv_decode_plan;
typedef struct hkv_prefill_plan hkv_prefill_plan;

/* Thread-local text of the last error returned on the calling thread ("" if none). */
const char *hkv_last_error(void);

/* ------------------------------------------------------------------------------------------
 * KV page pool (Section 5, "Proactive Cache Management"; Section 6, pinned prefix blocks).
 * The pool object is host metadata over caller-owned device buffers: a free list, a
 * reference count per page (the number of holders that pin it) and the buffer addresses.
 */
typedef struct {
    int32_t num_pages;
    int32_t page_size;    /* 16, 32, 64 or 128 tokens */
    int32_t num_kv_heads;
    int32_t head_dim;     /* must be 128 */
    int32_t dtype;        /* HKV_BF16, HKV_FP8_E4M3 or HKV_FP32 */
    void *k_pages;        /* device, num_pages*(page_size/16)*num_kv_heads*2048 elements, format above */
    void *v_pages;        /* device, same size */
    float *k_scale;       /* device, [num_pages*(page_size/16)][num_kv_heads]; fp8 pools only, else NULL */
    float *v_scale;       /* device, same */
    const int32_t *free_order; /* host, optional permutation of 0..num_pages-1: the order in
                                  which kv_pool_alloc hands pages out; NULL = ascending */
} hkv_pool_desc;

/* Creates the host-side pool object.  Borrows the device pointers; copies free_order.
 * EINVAL: null desc/out or buffers, num_pages <= 0, free_order not a permutation.
 * ESHAPE: page_size not 16/32/64/128, head_dim != 128, dtype not storable, scales missing for fp8. */
int kv_pool_create(const hkv_pool_desc *desc, hkv_pool **out);

/* Frees host metadata and any cached plan.  Waits for the device to be idle first if a cached
 * plan holds device index buffers.  Never touches the caller's page buffers. */
int kv_pool_destroy(hkv_pool *pool);

/* Pops n pages from the free list in free_order (deterministic), sets their reference count to
 * 1 and writes their ids to ids_out (host, n entries).  ENOMEM (nothing allocated) if fewer
 * than n pages are free. */
int kv_pool_alloc(hkv_pool *pool, int32_t n, int32_t *ids_out);

/* Adds one reference to each listed page (a further request or tree node pins it).
 * ERANGE: id outside the pool; EINVAL: page not allocated.  Nothing changes on error. */
int kv_pool_retain(hkv_pool *pool, int32_t n, const int32_t *ids /* host */);

/* Drops one reference from each listed page; a page whose count reaches 0 returns to the
 * tail of the free list in the order listed.  Errors as kv_pool_retain. */
int kv_pool_release(hkv_pool *pool, int32_t n, const int32_t *ids /* host */);

/* Copy-on-write before one holder writes into pages that others may hold too (a sequence forked
 * from another continues inside the last, partially filled page; sharing itself stays whole
 * pages, Section 6).  For each listed page: with a single reference it stays as it is; otherwise
 * the next free page is taken (reference count 1), the whole page (K and V blocks of every head
 * and, for fp8 pools, its scales) is copied to it on `stream`, one reference of the old page is
 * dropped and ids[i] is replaced by the new id.  Work queued earlier on `stream` that writes the
 * old page is seen by the copy; the old page must not be written on other streams meanwhile.
 *   ids: host, n entries, in/out, no page twice.
 * ERANGE / EINVAL as kv_pool_retain, EINVAL for a page listed twice, ENOMEM if fewer pages are
 * free than copies are needed; nothing changes on these errors. */
int kv_pool_copy_on_write(hkv_pool *pool, int32_t n, int32_t *ids /* host, in/out */, void *stream);

/* Number of free pages, or a negative error code. */
int32_t kv_pool_num_free(const hkv_pool *pool);

/* Tokens per page of the pool (16, 32, 64 or 128), or a negative error code. */
int32_t kv_pool_page_size(const hkv_pool *pool);

/* Reference count of one page (0 = free), or a negative error code. */
int32_t kv_pool_refcount(const hkv_pool *pool, int32_t page_id);

/* Stores the K/V of n_tokens consecutive tokens of one sequence into the pool: token i goes to
 * page page_ids[(first_slot + i) / P], slot (first_slot + i) % P, P the pool's page size
 * (first_slot < P).  This is the "compute the prefix KV once and keep it" step seen from the pool.
 *   page_ids: host, ceil((first_slot + n_tokens)/P) entries; one call touches at most 65536
 *   16-token blocks.
 *   k_src, v_src: device, [n_tokens][num_kv_heads][128] bf16.
 * bf16 pools: plain scatter into the block format.  fp8 pools: a (16-token block, head) block
 * written from its slot 0 gets scale = amax/448 over the tokens written into it by this call (1
 * if amax == 0) and code = round-to-nearest-even(x / scale), saturated to +-448, all in float.
 * A block that is continued (the first block of a call with first_slot % 16 > 0, e.g. decode
 * appending a token) keeps a running scale: scale' = max(scale, amax_new/448); if the scale
 * grows, the codes already in the block's slots below first_slot % 16 are re-encoded as
 * RNE(value(code) * scale / scale') (a second rounding of those tokens); the scale never
 * shrinks.  Those slots of such a block must have been written before.  Slots not written keep
 * their contents.  n_tokens == 0 is a no-op.
 * EINVAL / ERANGE / ESHAPE as above; the ids are checked before anything is queued. */
int kv_pool_write(hkv_pool *pool, const int32_t *page_ids, int32_t first_slot, int32_t n_tokens,
                  const void *k_src, const void *v_src, void *stream);

/* The decode step's write: one new token for each of n sequences in one launch.  Token i (row i
 * of k_src / v_src, device, [n][num_kv_heads][128] bf16) goes to slot slots[i] (0 .. page size - 1)
 * of page page_ids[i]; page_ids and slots are host arrays of n entries (n <= 32768).  Same
 * arithmetic as kv_pool_write with n_tokens = 1 (fp8: the block's running scale, re-encoding of
 * its earlier codes if the scale grows).  No two tokens of one call may go to the same 16-token
 * block, and no token to a page that has more than one owner (kv_pool_refcount > 1: such a page is
 * shared, kv_pool_copy_on_write gives the writer its own): EINVAL, checked before anything is queued.
 * bf16 and fp8 pools (ESHAPE for fp32 pools: use kv_pool_write). */
int kv_pool_append(hkv_pool *pool, const int32_t *page_ids, const int32_t *slots, int32_t n,
                   const void *k_src, const void *v_src, void *stream);

/* ------------------------------------------------------------------------------------------
 * Prefix forest (the call-level templated radix tree of Section 5: every leaf is one LLM
 * call, a call's prompt is the concatenation of the token segments on path(root, leaf)).
 */
typedef struct {
    int32_t parent;     /* index of the parent node, -1 for a root; must be < own index */
    int32_t page_begin; /* offset of this node's first page id in node_pages */
    int32_t n_pages;    /* == ceil(n_tokens / 16) */
    int32_t n_tokens;   /* omega(v) >= 0.  prefix_tree_flatten, prefill and fp32 pools need a multiple
                           of 16 in every node that has children (positions along a path must map
                           to pages without gaps); the bf16 / fp8 decode plans do not */
} hkv_node;

/* Host-only, integer-only.  Expands the forest into what the kernels index with:
 *   block_table     [n_req][max_pages]  page ids along root -> leaf, padded with -1
 *   kv_len          [n_req]             sum of n_tokens along the path
 *   node_req_indptr [n_nodes + 1], node_req_idx [<= n_nodes*n_req]
 *                                       CSR: the requests whose path contains the node,
 *                                       ascending request index
 *   node_tok_start  [n_nodes]           token offset of the node's segment within such a path
 * Any output pointer may be NULL to skip it.  All pointers are host memory.
 * ETREE / ERANGE as documented on the codes; ENOMEM if a path needs more than max_pages.
 * prefix_tree_flatten is the 16-token-page case of prefix_tree_flatten_paged, which takes the page
 * size of the forest (16, 32, 64 or 128; else ESHAPE). */
int prefix_tree_flatten(const hkv_node *nodes, int32_t n_nodes, const int32_t *node_pages,
                        int32_t n_node_pages, const int32_t *req_leaf, int32_t n_req, int32_t max_pages,
                        int32_t *block_table, int32_t *kv_len, int32_t *node_req_indptr,
                        int32_t *node_req_idx, int32_t *node_tok_start);
int prefix_tree_flatten_paged(const hkv_node *nodes, int32_t n_nodes, const int32_t *node_pages,
                              int32_t n_node_pages, const int32_t *req_leaf, int32_t n_req, int32_t page_size,
                              int32_t max_pages, int32_t *block_table, int32_t *kv_len, int32_t *node_req_indptr,
                              int32_t *node_req_idx, int32_t *node_tok_start);

/* Prefill token usage u_p of Section 5 for a sequence of calls on one worker: calls[0]
 * processes every token on path(root, calls[0]); calls[j] only the tokens on the path from the
 * lowest common ancestor of calls[j-1] and calls[j] (exclusive) down to calls[j].  Host-only.
 * u_p[j] is the number of new tokens attn_prefill_with_prefix has to be given for call j when
 * the previous call's pages are still cached. */
int prefix_tree_prefill_usage(const hkv_node *nodes, int32_t n_nodes, const int32_t *calls,
                              int32_t n_calls, int64_t *u_p);

/* ------------------------------------------------------------------------------------------
 * Log-sum-exp combine of partial attention results (natural logarithm).
 * Output row i owns the partials part_idx[row_indptr[i] .. row_indptr[i+1]):
 *   lse_i = ln sum_n exp(lse_parts[n]),   out_i = sum_n exp(lse_parts[n] - lse_i) * o_parts[n].
 * A partial with lse = -inf contributes nothing (its o may hold anything); a row with no
 * finite partial gives out = 0, lse = -inf.  Never produces NaN from finite inputs.
 *   o_parts [n_parts][128] float, lse_parts [n_parts] float, row_indptr [n_rows+1] int32,
 *   part_idx int32: all device.  out: device [n_rows][128] of out_dtype (HKV_BF16, rounded to
 *   nearest even, or HKV_FP32).  lse_out: device [n_rows] float, may be NULL.
 * The index arrays are trusted (they live on the device); only the arguments are validated. */
int lse_merge(const float *o_parts, const float *lse_parts, const int32_t *row_indptr,
              const int32_t *part_idx, int32_t n_rows, void *out, int32_t out_dtype, float *lse_out,
              void *stream);

/* The same combine for partials stored densely: output row i owns the partials i*max_parts + k,
 * k < part_count[i / rows_per_count] (part_count: device int32 [ceil(n_rows / rows_per_count)],
 * each entry in 0..max_parts).  This is the layout attn_decode_plan_run uses: the prefix above a
 * tree node is common to all requests below it, so a node's chunks take the same positions k in
 * every one of those requests' lists, and rows_per_count is the number of query heads.
 * o_parts and out must be 16-byte aligned. */
int lse_merge_dense(const float *o_parts, const float *lse_parts, const int32_t *part_count,
                    int32_t rows_per_count, int32_t max_parts, int32_t n_rows, void *out, int32_t out_dtype,
                    float *lse_out, void *stream);

/* ------------------------------------------------------------------------------------------
 * Batched decode over a prefix forest: one query token per request.  Every node's pages are
 * read from HBM once and applied to all requests below the node; the per-node partial results
 * (o, lse) are then combined along each request's path by the kernel behind lse_merge.
 *
 * A plan holds the flattened topology (work list, page ids, merge CSR) on host and device so
 * that a serving loop pays for the tree walk once per topology, not once per step.
 */
enum {
    HKV_PLAN_HOST_ONLY = 1, /* build and validate on the host, allocate nothing on the device */
    /* Decode plans over fp8 pools only (ESHAPE otherwise): both products run on the fp8 matrix
     * instruction.  K and V codes enter as they are; a query row is split into two e4m3 terms
     * (after a power-of-two scaling of the row; exact for every element down to 2^-10 of the
     * row's largest), a probability, scaled by its block's V scale relative to the largest V scale
     * of the 64-token step it belongs to, into two e4m3 terms that carry 8 significant bits, as the
     * bf16 value of the default path does.  Same speed and the same error bounds as the default
     * path, with one condition the default path does not have: a weight below about 2^-14 of the
     * step's largest weight-times-scale loses relative precision (e4m3 has no more range), which
     * shows only if the V scales of the four 16-token blocks of one step differ by more than about
     * 2^7 while the attention weight sits on the blocks with the small scales. */
    HKV_PLAN_FP8_MATRIX = 2,
    /* Decode plans: attn_decode_plan_run normally queues the kernel for nodes shared by many query rows on a
     * stream of the plan's own, beside the kernel that streams the other nodes on the caller's stream (one
     * event forks to it, one joins it before the merge; both are ordered after everything queued earlier on
     * the caller's stream, and the call is safe under stream capture).  With this flag everything is queued
     * on the caller's stream, one kernel after the other. */
    HKV_PLAN_ONE_STREAM = 4
};

/* nodes, node_pages, req_leaf: host.  Validates the forest (ETREE/ERANGE, page ids against the
 * pool), builds the work list and uploads it (blocking).  ESHAPE unless num_q_heads is a
 * multiple of the pool's num_kv_heads with a ratio of at most 16.
 * With bf16 and fp8 pools every node is read through its own page list, so any node may end inside
 * a page (its last page is then partly used and its children start on pages of their own).  That
 * makes the forest itself the attention mask of a tree of drafted tokens: one node per drafted
 * token (or run of tokens) under the request's context, one "request" per node to be verified,
 * and each such row sees the context, its ancestors and itself. */
int hkv_decode_plan_create(hkv_pool *pool, const hkv_node *nodes, int32_t n_nodes, const int32_t *node_pages,
                           int32_t n_node_pages, const int32_t *req_leaf, int32_t n_req, int32_t num_q_heads,
                           uint32_t flags, hkv_decode_plan **out);
/* The same for tokens_per_req (1..16) query tokens per request, e.g. the verification of a run of
 * drafted tokens: the request's T newest tokens (the last T of its path; they must all lie in its
 * leaf node, whose K/V are already in the pool) are queried together, token t of the T seeing every
 * key up to and including its own position.  q, out and lse_out of attn_decode_plan_run then hold
 * n_req * T rows, request-major ([n_req][T][num_q_heads][128]); all counts the introspection calls
 * return (requests of an item, part_counts) are in query rows, i.e. as for a plan over n_req * T
 * requests.  A query row that sees no token of some chunk of its leaf gets the empty partial there.
 * EINVAL if tokens_per_req is out of range or exceeds a request's leaf length. */
int hkv_decode_plan_create_multi(hkv_pool *pool, const hkv_node *nodes, int32_t n_nodes, const int32_t *node_pages,
                                 int32_t n_node_pages, const int32_t *req_leaf, int32_t n_req, int32_t tokens_per_req,
                                 int32_t num_q_heads, uint32_t flags, hkv_decode_plan **out);
/* Verification of a tree of drafted tokens per request (tree-structured speculative decoding): the
 * request's T = tokens_per_req (1..64) newest tokens, the last T of its leaf node, are drafted
 * tokens in any order; query row t of the request sees every key before them and drafted token j
 * iff bit j of visible[r * T + t] is set: its ancestors in the tree of drafts and itself (bit t
 * must be set, bits >= T must be clear; else EINVAL).  A causal run of T tokens is the mask with
 * bits 0..t, which is what hkv_decode_plan_create_multi builds.  Row layout and counts as there.
 * visible: host, [n_req * T].  ESHAPE for fp32 pools (they verify causal runs only). */
int hkv_decode_plan_create_tree(hkv_pool *pool, const hkv_node *nodes, int32_t n_nodes, const int32_t *node_pages,
                                int32_t n_node_pages, const int32_t *req_leaf, int32_t n_req, int32_t tokens_per_req,
                                const uint64_t *visible, int32_t num_q_heads, uint32_t flags, hkv_decode_plan **out);
/* A plan for a decode loop: as hkv_decode_plan_create, with room for every request's leaf to grow by
 * up to reserve_tokens tokens, so that generating a token does not cost a new plan (a tree walk, a
 * device allocation and a blocking upload) but one call of hkv_decode_plan_append.  Every request
 * needs a leaf of its own for that: a node without children, named by no other request, holding at
 * least one token (ETREE otherwise).  bf16 and fp8 pools (ESHAPE for fp32 pools).
 *
 * hkv_decode_plan_append: every request's leaf has grown by one token, whose K/V the caller stores
 * (kv_pool_append) before the next run.  new_page_ids: host, [n_req]; entry r is read only if the
 * token opens a new page (the leaf held a multiple of the page size), and is then the id of that
 * page; may be NULL if no request needs one.  Host work is a few microseconds; the device's copy
 * of the work list is updated by a small kernel queued on `stream` (beyond 256 requests: re-sent
 * from pinned memory by a copy kernel), which must be the stream of the runs before and after it
 * (the update is ordered between them).  ENOMEM once reserve_tokens appends are used up
 * (build a new plan then), EINVAL on a plan that was not created growing, ERANGE for a page id
 * outside the pool; nothing changes on error.  The chunking of the forest stays as planned at
 * creation: a leaf's last chunk simply gets longer. */
int hkv_decode_plan_create_growing(hkv_pool *pool, const hkv_node *nodes, int32_t n_nodes, const int32_t *node_pages,
                                   int32_t n_node_pages, const int32_t *req_leaf, int32_t n_req, int32_t num_q_heads,
                                   int32_t reserve_tokens, uint32_t flags, hkv_decode_plan **out);

/* Everything the four calls above can ask for, in one call, plus the planner's settings.  params may be NULL
 * (then this is hkv_decode_plan_create); every field left 0 keeps the library's own choice, so a caller sets
 * only what it needs (zero the struct first).  The settings change how the forest is cut into work items and
 * which of the library's kernels run them, never the result; they exist for sweeps and so that tests reach a
 * particular path at small sizes.  EINVAL for a value outside the range stated with its field. */
typedef struct {
    int32_t tokens_per_req;   /* query tokens per request, 1..64 (beyond 16 only with `visible`); 0 = 1 */
    const uint64_t *visible;  /* host [n_req * tokens_per_req]: as hkv_decode_plan_create_tree; NULL = causal run */
    int32_t reserve_tokens;   /* > 0: a growing plan, as hkv_decode_plan_create_growing */
    const int32_t *q_rows;    /* host [n_req * tokens_per_req] or NULL: row i of the plan (request i / T, token i % T)
                                 reads row q_rows[i] of q and writes row q_rows[i] of out and lse_out, so that a
                                 step's decode rows may lie anywhere among the rows of other work (a mixed
                                 step).  Entries >= 0 and all different (EINVAL); bf16 and fp8 pools (ESHAPE
                                 for fp32 pools).  NULL: row i */
    /* ---- planner settings */
    int32_t leaf_chunk;       /* tokens per item of nodes read by at most 16 query rows; multiple of 16 */
    int32_t shared_chunk;     /* tokens per item of nodes shared by more rows; multiple of 16, at most 2048 */
    int32_t max_rows;         /* query rows per item of such nodes: 16..64 */
    int32_t pack;             /* four short items per workgroup, one per wavefront: 1 never, 2 when the forest has
                                 more items than the chip holds at once (the default), 3 always */
    int32_t pack_tokens;      /* longest item of that mode, tokens */
    int32_t stages;           /* 16 KiB LDS stages a workgroup owns: 3..5 */
    int32_t interleave;       /* items shared by many rows and items of few rows are listed side by side in
                                 groups of this size (default 8); -1: one class after the other */
    int32_t tile_min_rows;    /* nodes shared by this many query rows or more may go to the 256-row tile kernel
                                 (default 128, at least 65) ... */
    int32_t tile_min_gflop;   /* ... if the forest holds this much such work (default 40); -1: whatever the amount */
    int32_t tile_workgroups;  /* persistent workgroups of the tile kernel (default: from the two amounts of work) */
    int32_t tile_chunk;       /* tokens per item of the tile kernel; multiple of 16, at most 8192 */
    int32_t large_batch_updates; /* growing plans: 1 = apply appends as for more than 256 requests (work list re-sent
                                 from pinned memory instead of a small kernel that carries the change in its arguments) */
    int32_t fused;            /* -1: never run the two kinds of items as one launch (then the tile kernel runs beside the
                                 other on a second stream, or in front of it with HKV_PLAN_ONE_STREAM); 0: one
                                 launch whenever no other item is shared by more than 16 query rows */
} hkv_decode_plan_params;
int hkv_decode_plan_create_ex(hkv_pool *pool, const hkv_node *nodes, int32_t n_nodes, const int32_t *node_pages,
                              int32_t n_node_pages, const int32_t *req_leaf, int32_t n_req, int32_t num_q_heads,
                              uint32_t flags, const hkv_decode_plan_params *params, hkv_decode_plan **out);
int hkv_decode_plan_append(hkv_decode_plan *plan, const int32_t *new_page_ids, void *stream);
/* The same together with the write: row r of k_src / v_src (device, [n_req][num_kv_heads][128] bf16)
 * is the new token of request r and is stored at the end of its leaf, as kv_pool_append would store
 * it (the plan knows the page and the slot).  For up to 256 requests the write and the plan's update
 * are one kernel launch.  Errors as hkv_decode_plan_append; EINVAL for null or unaligned k_src / v_src. */
int hkv_decode_plan_append_tokens(hkv_decode_plan *plan, const int32_t *new_page_ids, const void *k_src,
                                  const void *v_src, void *stream);
int hkv_decode_plan_destroy(hkv_decode_plan *plan);
/* Bytes of device workspace attn_decode_plan_run needs (per partial: o as 128 fp16 values times a power of two,
 * that power's reciprocal and lse as floats),
 * 0 on a null plan. */
size_t hkv_decode_plan_workspace_bytes(const hkv_decode_plan *plan);
/* Introspection for tests and tools (host copies).  Work item layout, 8 int32 each:
 * (page_off, n_tokens, kv_head, req_off, n_req, part_slot, tok_begin, node).  page_off indexes
 * the plan's list of 16-token blocks (= node_pages when the page size is 16; else every page p
 * of a node expanded to the blocks p*S + j it uses), req_off the node->request CSR values that
 * prefix_tree_flatten returns.  An item applies the tokens [tok_begin, tok_begin + n_tokens) of
 * `node` to n_req requests x (num_q_heads / num_kv_heads) heads of kv_head; row (request r, head
 * h) of the item writes partial (r*num_q_heads + h)*max_parts + part_slot. */
int32_t hkv_decode_plan_num_items(const hkv_decode_plan *plan);
/* Of these, the last hkv_decode_plan_num_tile_items are items of nodes shared by 128 query rows or more (up
 * to 256 / G requests each, at most 8192 tokens): they are run by code built like the prefill kernel (256-row
 * tiles) on hkv_decode_plan_tile_workgroups persistent workgroups.  hkv_decode_plan_is_fused: 1 if those
 * workgroups and the workgroups of the other items go out as one launch (possible when none of the other
 * items is shared by more than 16 query rows), 0 if they are two kernels on two streams. */
int32_t hkv_decode_plan_num_tile_items(const hkv_decode_plan *plan);
int32_t hkv_decode_plan_tile_workgroups(const hkv_decode_plan *plan);
int32_t hkv_decode_plan_is_fused(const hkv_decode_plan *plan);
/* Workgroups of the per-node kernel: one per item, except that in forests with more items than the
 * chip holds at once the short items of at most 16 query rows (listed last) share a workgroup four
 * at a time, one item per wavefront. */
int32_t hkv_decode_plan_num_workgroups(const hkv_decode_plan *plan);
int32_t hkv_decode_plan_num_parts(const hkv_decode_plan *plan); /* n_req*num_q_heads*max_parts */
int hkv_decode_plan_items(const hkv_decode_plan *plan, int32_t *items_out /* [n_items][8] */);
int32_t hkv_decode_plan_max_parts(const hkv_decode_plan *plan);
/* part_count [n_req]: number of partials each row of the request owns. */
int hkv_decode_plan_part_counts(const hkv_decode_plan *plan, int32_t *part_count);

/* Runs one decode step.  q: device [n_req][num_q_heads][128] bf16.  out: device, same shape,
 * bf16.  lse_out: device [n_req][num_q_heads] float or NULL.  workspace: device, at least
 * hkv_decode_plan_workspace_bytes(plan) bytes, 256-byte aligned; its contents are scratch.
 * A request whose path holds no token gets out = 0, lse = -inf.
 * EINVAL (null/unaligned), ENOMEM (workspace too small), EHIP. */
int attn_decode_plan_run(hkv_decode_plan *plan, const void *q, float scale, void *out, float *lse_out,
                         void *workspace, size_t workspace_bytes, void *stream);

/* attn_decode_plan_run for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the partial results go to a workspace the
 * library holds itself, a fixed array of hkv_static_workspace_bytes() = 32 MiB of device memory per
 * GPU that exists from the time the library is loaded until the process ends, so the call takes
 * neither a workspace nor allocates anything (no hipMalloc / hipFree, no allocating library routine);
 * it only queues the same two kernels on `stream`.  q, out, lse_out, scale: as attn_decode_plan_run.
 * ENOMEM if hkv_decode_plan_workspace_bytes(plan) exceeds the array (e.g. more than 127 000 partials of
 * 264 bytes: use attn_decode_plan_run with a workspace of the caller's then); nothing is queued on
 * error.  All calls on one GPU share the one array and it keeps the last call's contents (every slot
 * that is read is written first by the same call, so nothing has to be cleared): two such calls
 * that overlap in time on one GPU, on different streams or from different plans, race; queue them
 * on one stream or order them with events.  The plan must have been created on the GPU that is
 * current at the call. */
size_t hkv_static_workspace_bytes(void);
int attn_decode_plan_run_static(hkv_decode_plan *plan, const void *q, float scale, void *out, float *lse_out,
                                void *stream);

/* Profiling aid.  mode 0: off.  mode 1: attn_decode_plan_run attaches a begin and an end HIP event to
 * each of its two kernel dispatches on the stream it is given, so that an interval is the kernel's own
 * duration on the device, without the gap to its neighbours in the queue.
 * hkv_decode_plan_elapsed_ms waits for the most recent profiled run to finish and returns the GPU time
 * of the per-node kernel and of the merge kernel in milliseconds.
 * EINVAL if no profiled run has been queued. */
int hkv_decode_plan_set_profiling(hkv_decode_plan *plan, int32_t mode);
int hkv_decode_plan_elapsed_ms(hkv_decode_plan *plan, float *node_ms /* host */, float *merge_ms /* host */);
/* The same run's per-node phase by kernel: the kernel over the items of few rows and the tile kernel (0 for
 * one that did not run); node_ms above spans both, from the earlier begin to the later end. */
int hkv_decode_plan_elapsed_kernels_ms(hkv_decode_plan *plan, float *rows_kernel_ms /* host */,
                                       float *tile_kernel_ms /* host */);

/* One-shot form: plans (or reuses the plan cached in the pool when the forest is unchanged) and
 * runs.  Same arguments as the two calls above. */
int attn_decode_prefix_tree(hkv_pool *pool, const void *q, const hkv_node *nodes, int32_t n_nodes,
                            const int32_t *node_pages, int32_t n_node_pages, const int32_t *req_leaf,
                            int32_t n_req, int32_t num_q_heads, float scale, void *out, float *lse_out,
                            void *workspace, size_t workspace_bytes, void *stream);
/* Workspace bytes the one-shot call needs for this forest (0 on error; see hkv_last_error). */
size_t attn_decode_workspace_bytes(hkv_pool *pool, const hkv_node *nodes, int32_t n_nodes,
                                   const int32_t *node_pages, int32_t n_node_pages, const int32_t *req_leaf,
                                   int32_t n_req, int32_t num_q_heads);

/* ------------------------------------------------------------------------------------------
 * Prefill of the uncached suffix (Section 5, u_p): request r brings s_r = cu_q[r+1] - cu_q[r]
 * new tokens whose K/V have already been written to the pool (kv_pool_write) at positions
 * prefix_len_r .. kv_len_r - 1, prefix_len_r = kv_len_r - s_r >= 0.  New token i sits at
 * absolute position a = prefix_len_r + i and attends keys t <= a of the request's block table:
 * all cached prefix tokens plus the causal part of its own suffix, itself included.
 *   cu_q [n_req+1], block_table [n_req][max_pages], kv_len [n_req]: host.  Entries of
 *   block_table beyond ceil(kv_len/16) are ignored.  ERANGE if a used page id is outside the pool.
 * ESHAPE unless num_q_heads is a multiple of num_kv_heads with a ratio G of at most 16 (a
 * workgroup's 256 rows hold floor(256/G) tokens x G heads; at most G - 1 rows stay unused).
 */
int hkv_prefill_plan_create(hkv_pool *pool, const int32_t *cu_q, const int32_t *block_table, int32_t max_pages,
                            const int32_t *kv_len, int32_t n_req, int32_t num_q_heads, uint32_t flags,
                            hkv_prefill_plan **out);
/* The same for a step that mixes prefill with other work in one q / out / lse (Section 6, engine integration:
 * chunks of prompts run next to decode steps): request r's q_len[r] new tokens are rows q_row_begin[r] ..
 * q_row_begin[r] + q_len[r] - 1 of q, out and lse_out; rows no request names are neither read nor written.
 * q_row_begin, q_len: host [n_req], >= 0; EINVAL if two requests share a row.  bf16 and fp8 pools
 * (ESHAPE for fp32 pools).  Everything else as hkv_prefill_plan_create. */
int hkv_prefill_plan_create_rows(hkv_pool *pool, const int32_t *q_row_begin, const int32_t *q_len,
                                 const int32_t *block_table, int32_t max_pages, const int32_t *kv_len, int32_t n_req,
                                 int32_t num_q_heads, uint32_t flags, hkv_prefill_plan **out);
int hkv_prefill_plan_destroy(hkv_prefill_plan *plan);
/* Number of (request, query tile, kv head) workgroups the plan launches. */
int32_t hkv_prefill_plan_num_tiles(const hkv_prefill_plan *plan);
/* The prefill kernel keeps one softmax reference per row (the maximum of its first 32 scores); a tile in which a
 * later score exceeds it by more than the exponent range allows repeats with a running maximum, at about
 * twice the cost.  count (host): how many tiles did so over all runs of this plan so far (the call waits for
 * the device).  bf16 and fp8 pools; always 0 for fp32 pools. */
int hkv_prefill_plan_fallback_tiles(hkv_prefill_plan *plan, int64_t *count);
/* Tile layout for tests, 8 int32 each: (req, q_begin, n_q, kv_head, q_row0, prefix_len, kv_len, bt_off). */
int hkv_prefill_plan_tiles(const hkv_prefill_plan *plan, int32_t *tiles_out);

/* q: device [cu_q[n_req]][num_q_heads][128] bf16; out: device, same shape, bf16; lse_out: device
 * [cu_q[n_req]][num_q_heads] float or NULL. */
int attn_prefill_plan_run(hkv_prefill_plan *plan, const void *q, float scale, void *out, float *lse_out,
                          void *stream);
/* fp8 pools: the matrix-core kernel reads bf16, so the pages the batch reads (each once, however
 * many requests share it) are first dequantised (code * scale, rounded to bf16) into a scratch pool
 * in the caller's workspace: hkv_prefill_plan_workspace_bytes(plan) bytes (8 KiB per distinct page
 * and KV head; 0 for bf16 and fp32 pools), device memory, 256-byte aligned, scratch.  The pre-pass
 * moves 3 bytes per cached element against 512 flop per (query, key) pair: well below 1 % of the
 * kernel at the sizes prefill runs at.  attn_prefill_plan_run is the same call without a workspace.
 * EINVAL (fp8 pool and no / unaligned workspace), ENOMEM (too small). */
size_t hkv_prefill_plan_workspace_bytes(const hkv_prefill_plan *plan);
int attn_prefill_plan_run_ws(hkv_prefill_plan *plan, const void *q, float scale, void *out, float *lse_out,
                             void *workspace, size_t workspace_bytes, void *stream);

/* One-shot form; workspace may be NULL for bf16 and fp32 pools (a query tile reads its whole key
 * range itself; attn_prefill_workspace_bytes is 0); an fp8 pool needs what
 * hkv_prefill_plan_workspace_bytes reports for the same batch (the error text of a too small
 * workspace names the size). */
int attn_prefill_with_prefix(hkv_pool *pool, const void *q, const int32_t *cu_q, const int32_t *block_table,
                             int32_t max_pages, const int32_t *kv_len, int32_t n_req, int32_t num_q_heads,
                             float scale, void *out, float *lse_out, void *workspace, size_t workspace_bytes,
                             void *stream);
size_t attn_prefill_workspace_bytes(int32_t total_q, int32_t num_q_heads);

/* ------------------------------------------------------------------------------------------
 * Block-level prefix cache over a pool (host bookkeeping only; Section 6, "LLM Engine
 * Integration": prefixes are kept block by block, precomputed ones are pinned, blocks are evicted
 * least recently used first and a prefix never before its extensions, an evicted prefix is
 * recomputed by the next call that needs it).
 * A block is 16 tokens; its identity is (preceding block, its 16 token ids).  Only full blocks are
 * shared; a sequence's partial last block is private.  The cache takes its pages from the pool
 * (kv_pool_alloc: lowest free id first) and holds one pool reference per page it owns.
 * Evictable = no live sequence uses it, not pinned, no cached block extends it; among those the
 * oldest last use goes first, ties by lower page id; the clock ticks once per acquire / release. */
typedef struct hkv_cache hkv_cache;
int kv_cache_create(hkv_pool *pool, hkv_cache **out);
int kv_cache_destroy(hkv_cache *cache); /* returns every page it holds to the pool */
/* Looks up the longest cached prefix of tokens (host, n_tokens ids) in whole blocks, takes a
 * reference on each hit, and gives every remaining block a page (free list first, then by
 * eviction); new full blocks enter the cache at once, so the caller must fill them (kv_pool_write
 * of tokens n_cached_tokens .. n_tokens-1, then attn_prefill_with_prefix) before anyone else hits
 * them.  page_ids (host, ceil(n_tokens/16) entries) receives the sequence's block table;
 * n_cached_tokens the number of leading tokens whose KV is already there.  pin != 0 also pins all
 * full blocks of the sequence.  ENOMEM if no page is free and nothing can be evicted: then the call
 * gives back what it took and holds nothing. */
int kv_cache_acquire(hkv_cache *cache, const int32_t *tokens, int32_t n_tokens, int32_t pin, int32_t *page_ids,
                     int32_t *n_cached_tokens);
/* Ends a sequence's use of its pages (the list kv_cache_acquire returned): full blocks stay cached
 * and become evictable once nobody else uses them; the private partial page returns to the pool.
 * ERANGE if a page is not held by any sequence. */
int kv_cache_release(hkv_cache *cache, const int32_t *page_ids, int32_t n_pages);
/* Drops one pin from each listed page that is pinned (others are ignored). */
int kv_cache_unpin(hkv_cache *cache, const int32_t *page_ids, int32_t n_pages);
/* Counters since creation (any pointer may be NULL). */
int kv_cache_stats(const hkv_cache *cache, int64_t *cached_blocks, int64_t *hits, int64_t *misses,
                   int64_t *evictions);

/* ------------------------------------------------------------------------------------------
 * Scheduling layer (host only, integers only): templated radix tree, token-step cost model and
 * cache-aware scheduling (Section 5: "Modeling Prompt Structure with a Templated Radix Tree",
 * "Scheduling Problem Formulation" with its token-usage and precedence-delay equations, the
 * scheduling algorithm; appendix "Templated Radix Tree Construction").
 *
 * A call's prefix template is a list of int32 symbols: s >= 0 is a static token id, s < 0 stands
 * for the output of call -(s + 1) (a placeholder; it makes this call depend on that one).
 * omega(v) of a tree node = static tokens of its segment + len_out of every placeholder in it;
 * the root and the leaves (one per call, child of the node where its template ends) weigh 0.
 * Workers are identical, alpha = 1 / capacity; every time below is an integer scaled by the
 * capacity M:  U = len_out * u_p + len_out (len_out + 1) / 2  (= M u),  delay = M * len_out  (= M d).
 * A worker runs its calls one after another in schedule order.
 * Nodes are numbered in depth-first preorder from the root (node 0), children in order of
 * creation (a node created by a split takes the place of the node it was split from); this makes
 * `parent` a valid parent-first forest for the attention entry points, with omega as n_tokens. */
typedef struct hkv_trt hkv_trt;

/* Builds the tree: calls are inserted in topological order of their dependencies (smallest index
 * first among the ready ones) by radix-tree insertion with node splitting.
 * tmpl_indptr [n_calls+1], tmpl_syms, len_out [n_calls], worker [n_calls] (NULL: all on worker 0):
 * host.  ETREE if a placeholder names a missing call, the call itself, or the dependencies form a
 * cycle; ERANGE for negative len_out / worker; EINVAL; ENOMEM. */
int trt_build(const int32_t *tmpl_indptr, const int32_t *tmpl_syms, const int32_t *len_out,
              const int32_t *worker, int32_t n_calls, hkv_trt **out);
int trt_destroy(hkv_trt *tree);
int32_t trt_num_nodes(const hkv_trt *tree);
int32_t trt_num_syms(const hkv_trt *tree);  /* total length of all node segments */
int32_t trt_num_calls(const hkv_trt *tree);
/* Copies the flat tree out (host arrays; any pointer may be NULL): parent, omega (int64), the
 * call of a leaf (-1 for other nodes), each node's segment as [seg_begin, seg_begin + seg_len)
 * of syms, and the leaf of every call. */
int trt_nodes(const hkv_trt *tree, int32_t *parent, int64_t *weight, int32_t *call, int32_t *seg_begin,
              int32_t *seg_len, int32_t *syms, int32_t *leaf_of_call);
/* u_p of a sequence of calls run back to back on one worker: u_p[0] sums omega over path(root,
 * leaf of calls[0]], u_p[j] over the path from the lowest common ancestor of the leaves of
 * calls[j-1] and calls[j] (exclusive) down to the latter.  ERANGE for a call index out of range. */
int trt_prefill_usage(const hkv_trt *tree, const int32_t *calls, int32_t n, int64_t *u_p);
/* Start B and completion C of every call (indexed by call, may be NULL) and the total token step
 * T = max C under schedule sigma (worker i runs sigma[sigma_indptr[i] .. sigma_indptr[i+1])):
 * B = max(previous completion on the worker, C' + capacity * len_out' over the dependencies),
 * C = B + U.  ERANGE if sigma is no partition of the calls, ETREE if it contradicts the
 * dependencies (a worker's next call waits for one that can never run). */
int trt_evaluate(const hkv_trt *tree, const int32_t *sigma_indptr, const int32_t *sigma, int32_t n_workers,
                 int64_t capacity, int64_t *B, int64_t *C, int64_t *T);
/* Cache-aware scheduling: depth-first descent over the tree, at every node taking the remaining
 * children by greatest dependency depth (longest chain of dependents below any unscheduled leaf of
 * the subtree), then earliest schedulable step, then node number; a leaf is placed when its
 * dependencies are scheduled and it opens no idle gap on its worker; when a whole pass places
 * nothing more, a forced pass places the ready call with the earliest start.  Calls stay on the
 * worker given at trt_build.  Outputs: sigma_indptr [n_workers+1], sigma [n_calls], B, C (may be
 * NULL), T.  ERANGE if a call's worker is >= n_workers. */
int trt_schedule(const hkv_trt *tree, int32_t n_workers, int64_t capacity, int32_t *sigma_indptr,
                 int32_t *sigma, int64_t *B, int64_t *C, int64_t *T);

/* PartitionWorkflow (Section 5, first step of the scheduling algorithm: operators are partitioned across
 * the workers and replicated per assignment to balance load).  The calls of a batch fall into groups
 * connected by dependencies (one per input query); a group goes to one worker as a whole, so an operator is
 * replicated on every worker that received one of its queries and no dependency crosses workers.  Groups are
 * placed in order of decreasing estimated token usage (ties: smaller first call), each on the worker with
 * the least usage so far (ties: lower number); usage of a call = len_out * omega(prompt) + len_out
 * (len_out + 1) / 2 with a placeholder counted as the output length of its call.  Templates as for
 * trt_build; worker: host [n_calls], out (feed it to trt_build).  EINVAL / ERANGE as trt_build. */
int trt_partition(const int32_t *tmpl_indptr, const int32_t *tmpl_syms, const int32_t *len_out, int32_t n_calls,
                  int32_t n_workers, int32_t *worker);
/* Nested sequences (Section 5, paragraph below the scheduling algorithm): a worker's schedule as inner
 * sequences of the calls that share their static prompt (the first node below the root on their path), in
 * the order of sigma inside; the intermediate buffer releases an inner sequence when the last call of its
 * family on that worker has been emitted, so inner sequences appear in the order of their last call.
 * sigma as trt_schedule returns it.  Outputs (host): seq_indptr [n_workers + 1]: worker i owns the inner
 * sequences seq_indptr[i] .. seq_indptr[i+1] - 1; seq_begin [n_calls + 1] (the first n_seq + 1 entries are
 * written): sequence s is nested[seq_begin[s] .. seq_begin[s+1] - 1]; nested [n_calls].
 * EINVAL / ERANGE if sigma is no partition of the calls. */
int trt_nested(const hkv_trt *tree, const int32_t *sigma_indptr, const int32_t *sigma, int32_t n_workers,
               int32_t *seq_indptr, int32_t *seq_begin, int32_t *nested);
/* Best-effort execution of a soft schedule under the cost model of trt_evaluate (workers "execute
 * best-effort, buffering and issuing ready LLM calls ... while preserving cache-friendly ordering"): order
 * is one priority order per worker (e.g. the flattened nested sequences), which the dependencies may
 * contradict.  Repeatedly, every worker with calls left names the first call of its order whose dependencies
 * have all been issued; the worker whose candidate can start earliest (ties: lower number) issues it at that
 * step.  Outputs: sigma [n_calls] (worker i's realised order in the slots of order_indptr), B, C (may be
 * NULL), T.  On an order that respects the dependencies the result equals trt_evaluate's.  ETREE on a
 * dependency cycle. */
int trt_run_soft(const hkv_trt *tree, const int32_t *order_indptr, const int32_t *order, int32_t n_workers,
                 int64_t capacity, int32_t *sigma, int64_t *B, int64_t *C, int64_t *T);

#ifdef __cplusplus
}
#endif
#endif /* HELIUMKV_H */
