// Internal interface between the host side of the library (api.cpp) and its gfx950 kernels.
// Not part of the C ABI.
#pragma once

#include <hip/hip_runtime_api.h>
#include <stddef.h>
#include <stdint.h>

namespace hkv {

constexpr int kPage = 16;
constexpr int kHeadDim = 128;
constexpr int kBlockElems = kPage * kHeadDim;  // elements of one (page, head) K or V block

// One decode workgroup: the tokens [tok_begin, tok_begin + n_tokens) of one tree node, one KV
// head, applied to n_req of the requests below the node (n_req * G query rows, at most 64).
struct DecodeItem {
    int32_t page_off;   // index of the item's first page in the plan's page list
    int32_t n_tokens;   // tokens of this item; only the node's last item may end inside a page
    int32_t kv_head;
    int32_t req_off;    // index of the item's first request in the node->request CSR values
    int32_t n_req;
    int32_t part_slot;  // position of this item among the partials of every row below the node:
                        // row (request r, q head h) writes partial (r*Hq + h)*max_parts + part_slot
    int32_t tok_begin;  // first token within the node (multiple of 16)
    int32_t node;
};

// One prefill workgroup: n_q consecutive new tokens of one request, all G query heads of one KV head.
struct PrefillTile {
    int32_t req;
    int32_t q_begin;    // first new token of the tile within the request's suffix
    int32_t n_q;
    int32_t kv_head;
    int32_t q_row0;     // row of that token in q / out: cu_q[req] + q_begin
    int32_t prefix_len; // cached tokens in front of the request's suffix
    int32_t kv_len;
    int32_t bt_off;     // offset of the request's row in the uploaded block table
};

struct PoolView {
    const void *k_pages;
    const void *v_pages;
    const float *k_scale;
    const float *v_scale;
    int32_t num_kv_heads;
    int32_t dtype;
};

struct DecodeLaunch {
    PoolView pool;
    const void *q;               // [n_req][Hq][128] bf16
    const DecodeItem *items;     // device
    const int32_t *pages;        // device: the plan's page list
    const int32_t *node_req_idx; // device: node->request CSR values
    uint16_t *o_parts;           // [n_req*Hq*max_parts][128] fp16, each partial times a power of two of its own ...
    float *lse_parts;            // [n_req*Hq*max_parts]
    float *down_parts;           // [n_req*Hq*max_parts]: ... whose reciprocal is kept here
    int32_t n_items;
    int32_t num_q_heads;
    int32_t max_parts;
    float scale;
    // Several query tokens per request (null otherwise): row r of q is query token r % T of request
    // r / T; inside the node row_leaf[r] it sees the first row_limit[r] tokens (everything before the
    // request's T newest tokens) and, of the tokens behind them, number j iff bit j of row_mask[r] is
    // set (a causal run, or the ancestors in a tree of drafted tokens); every other node of its path
    // it sees whole.
    const int32_t *row_leaf;     // device [n_req * T]
    const int32_t *row_limit;    // device [n_req * T]
    const unsigned long long *row_mask;  // device [n_req * T]
    // Items [0, n_single) get a workgroup each; the items behind them (short, at most 16 rows) are run
    // four to a workgroup, one per wavefront.
    int32_t n_single;
    // LDS stages of 16 KiB a workgroup owns (3..5): items shared by more than 16 query rows keep
    // n_stages - 1 steps in flight.  The launch reserves n_stages * 16 KiB of LDS per workgroup.
    int32_t n_stages;
    // fp8 pools: run both products on the fp8 matrix instruction (codes of K and V as they are, query
    // and probabilities as two e4m3 terms each) instead of widening the codes to bf16.
    int32_t fp8_matrix;
    // Row r of the plan reads row q_rows[r] of q (device; null: row r).  Partials stay indexed by r.
    const int32_t *q_rows;
};

struct PrefillLaunch {
    PoolView pool;
    const void *q;
    const PrefillTile *tiles;    // device
    const int32_t *block_table;  // device
    void *out;
    float *lse_out;              // may be null
    int32_t n_tiles;
    int32_t num_q_heads;
    float scale;
    unsigned int *fallback_tiles;  // device, may be null: counts the tiles that had to repeat with a running maximum
};

struct PoolWriteLaunch {
    void *k_pages;
    void *v_pages;
    float *k_scale;
    float *v_scale;
    int32_t num_kv_heads;
    int32_t dtype;
    const int32_t *page_ids;     // device
    int32_t n_pages;
    int32_t first_slot;
    int32_t n_tokens;
    const void *k_src;
    const void *v_src;
    // One token for each of n_pages sequences instead of one run of tokens (null otherwise): workgroup
    // (i, head) stores source row i at slot slots[i] (0..15) of block page_ids[i]; first_slot and
    // n_tokens are not used.
    const int32_t *slots;        // device
};

// One token for each of up to kMaxInlineAppend sequences, ids and slots by value.
constexpr int kMaxInlineAppend = 256;
struct PoolAppendInline {
    PoolWriteLaunch base;        // page_ids / slots / first_slot / n_tokens unused; n_pages = number of tokens
    int32_t block[kMaxInlineAppend];
    uint8_t slot[kMaxInlineAppend];
};

// One decode step's change to an uploaded growing plan, for up to kMaxInlineAppend requests: the items
// listed in grow_items get one token more, and request r's new 16-token block (if it opens one) is
// entered at position block_pos[r] of the plan's block list.
struct PlanGrowInline {
    DecodeItem *items;           // device
    int32_t *pages;              // device
    const int32_t *grow_items;   // device, n_grow entries
    int32_t n_grow;
    int32_t n_req;
    int32_t new_block[kMaxInlineAppend];  // -1: none
    int32_t block_pos[kMaxInlineAppend];
};

// Whole-page copies inside one pool (copy-on-write of pages that several holders share).
constexpr int kMaxCopyPairs = 32;
struct PoolCopyLaunch {
    PoolView pool;
    int32_t blocks_per_page;     // a page is this many consecutive 16-token blocks
    int32_t n;
    int32_t src[kMaxCopyPairs];
    int32_t dst[kMaxCopyPairs];
};

// fp8 pages -> bf16 pages of a scratch pool (page i of the scratch = src_pages[i] of the pool), so that
// the matrix-core prefill kernel can read an fp8 pool.
struct PoolDequantLaunch {
    PoolView pool;               // the fp8 pool
    const int32_t *src_pages;    // device [n_pages]
    int32_t n_pages;
    void *k_dst;                 // device, n_pages * num_kv_heads * 2048 bf16, bf16 block format
    void *v_dst;
};

// fp32 pools: one wavefront per (query token, query head), no sharing (rows_fp32.hip).
struct RowsLaunch {
    PoolView pool;
    const float *q;              // [n_q_tokens][Hq][128] fp32
    const int32_t *block_table;  // device [n_rows_of_table][max_pages]
    const int32_t *row_req;      // device [n_q_tokens]: row of the block table
    const int32_t *row_len;      // device [n_q_tokens]: keys the token sees
    float *out;                  // [n_q_tokens][Hq][128] fp32
    float *lse_out;              // may be null
    int32_t n_q_tokens;
    int32_t num_q_heads;
    int32_t max_pages;
    float scale;
};

// Largest token count of a decode item that is shared by more than 16 query rows.
constexpr int kMaxSharedItemTokens = 2048;

// Decode items shared by more than kMinTileItemRows query rows are run by the 256-row tile kernel (the
// prefill kernel in its second role), on a stream of its own next to the kernel that streams the rest.
constexpr int kMinTileItemRows = 65;
constexpr int kMaxTileItemTokens = 8192;  // tokens per such item
constexpr int kScaleSlots = 512;          // pages whose fp8 scales the tile kernel keeps in LDS
struct DecodeTilesLaunch {
    PoolView pool;
    const void *q;               // [n_req][Hq][128] bf16
    const DecodeItem *items;     // device: the items of this kernel (at most 256 / G requests each)
    const int32_t *pages;        // device: the plan's block list
    const int32_t *node_req_idx; // device: node->request CSR values
    uint16_t *o_parts;           // as DecodeLaunch::o_parts
    float *lse_parts;
    float *down_parts;
    int32_t n_items;
    int32_t num_q_heads;
    int32_t max_parts;
    float scale;
    int32_t n_workgroups;        // persistent workgroups: workgroup w runs items w, w + n_workgroups, ...
    const int32_t *q_rows;       // device, may be null: as DecodeLaunch::q_rows
};

// Query tokens per prefill workgroup for a given group size G (rows per workgroup / G).
int prefill_tile_tokens(int group);
// Both kinds of decode items in one launch (no item of `a` may be shared by more than 16 query rows).
hipError_t launch_decode_fused(const DecodeLaunch &a, const DecodeTilesLaunch &d, hipStream_t s,
                               hipEvent_t ev_begin = nullptr, hipEvent_t ev_end = nullptr);

hipError_t launch_pool_write(const PoolWriteLaunch &a, hipStream_t s);
// src may be pinned host memory (its device-side address); bytes is rounded down to a multiple of 16
hipError_t launch_upload(const void *src, void *dst, size_t bytes, hipStream_t s);
hipError_t launch_pool_append_inline(const PoolAppendInline &a, hipStream_t s);
// both in one launch: workgroup (r, head) stores request r's token and lengthens the leaf's item of that head
hipError_t launch_decode_step_append(const PoolAppendInline &w, const PlanGrowInline &g, hipStream_t s);
hipError_t launch_plan_grow_inline(const PlanGrowInline &a, hipStream_t s);
hipError_t launch_pool_copy(const PoolCopyLaunch &a, hipStream_t s);
hipError_t launch_pool_dequant(const PoolDequantLaunch &a, hipStream_t s);
// Once per device (later calls only read the result), with that device current and outside graph capture:
// allows the decode kernels their LDS and looks up the device's static workspace (kStaticWorkspaceBytes
// bytes, 256-byte aligned), returned through static_ws unless that is null.  Safe from several threads.
constexpr size_t kStaticWorkspaceBytes = (size_t)32 << 20;
hipError_t prepare_decode_device(void **static_ws);
hipError_t launch_decode(const DecodeLaunch &a, hipStream_t s, hipEvent_t ev_begin = nullptr, hipEvent_t ev_end = nullptr);
hipError_t launch_rows_fp32(const RowsLaunch &a, hipStream_t s);
hipError_t launch_pool_write_fp32(const PoolWriteLaunch &a, hipStream_t s);
hipError_t launch_prefill(const PrefillLaunch &a, hipStream_t s);
hipError_t launch_decode_tiles(const DecodeTilesLaunch &a, hipStream_t s, hipEvent_t ev_begin = nullptr, hipEvent_t ev_end = nullptr);
hipError_t launch_lse_merge(const float *o_parts, const float *lse_parts, const int32_t *row_indptr,
                            const int32_t *part_idx, int32_t n_rows, void *out, int32_t out_dtype,
                            float *lse_out, hipStream_t s);
// out_rows (device, may be null): the rows of group g = row / rows_per_count are written to group out_rows[g]
// of out / lse_out instead of group g.
// down_parts (device, may be null): o_parts holds fp16 values, partial n to be multiplied by down_parts[n] (the
// decode plans' own partials), instead of floats.
hipError_t launch_lse_merge_dense(const void *o_parts, const float *lse_parts, const int32_t *part_count,
                                  int32_t rows_per_count, int32_t max_parts, int32_t n_rows, void *out,
                                  int32_t out_dtype, float *lse_out, hipStream_t s, hipEvent_t ev_begin = nullptr,
                                  hipEvent_t ev_end = nullptr, const int32_t *out_rows = nullptr,
                                  const float *down_parts = nullptr);

}  // namespace hkv
