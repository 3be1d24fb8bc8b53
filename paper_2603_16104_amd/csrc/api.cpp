// Host side of the heliumkv C ABI: pool bookkeeping, forest validation and flattening, work
// planning, argument checks, kernel launches.  All arithmetic on K/V/Q lives in the kernels.
#include "../../include/heliumkv.h"
#include "hkv_internal.h"

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <deque>
#include <new>
#include <numeric>
#include <string>
#include <unordered_map>
#include <vector>

using namespace hkv;

// ---------------------------------------------------------------------------------------------
// errors
namespace {
thread_local std::string g_err;
}

namespace hkv {
// records the thread-local message and returns the code (shared with the other host files)
int fail(int code, const char *fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}
}  // namespace hkv

namespace {

int fail_hip(hipError_t e, const char *what) {
    return fail(HKV_EHIP, "%s: %s", what, hipGetErrorString(e));
}

#define HKV_HIP(call)                                  \
    do {                                               \
        hipError_t e_ = (call);                        \
        if (e_ != hipSuccess) return fail_hip(e_, #call); \
    } while (0)

size_t elem_bytes(int dtype) { return dtype == HKV_BF16 ? 2 : dtype == HKV_FP8_E4M3 ? 1 : 4; }

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// What the planner needs to know of the chip: compute units, and how many workgroups of the per-node decode
// kernel one of them holds (three with bf16 pools, two with fp8 pools: registers).  Asked of the current device;
// plans built without a device (HKV_PLAN_HOST_ONLY on a machine without a GPU) assume an MI355X.
struct ChipShape {
    int n_cu = 256;
    int lds_per_cu = 160 * 1024;
};
ChipShape chip_shape() {
    ChipShape c;
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) {
        if (prop.multiProcessorCount > 0) c.n_cu = prop.multiProcessorCount;
        if (prop.maxSharedMemoryPerMultiProcessor > 0) c.lds_per_cu = (int)prop.maxSharedMemoryPerMultiProcessor;
    } else {
        (void)hipGetLastError();  // no device: not an error of the caller's
    }
    return c;
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// opaque objects
struct hkv_decode_plan {
    hkv_pool *pool = nullptr;
    int32_t n_req = 0, num_q_heads = 0, group = 0, n_parts = 0, max_parts = 1;
    std::vector<hkv_node> key_nodes;        // the caller's forest: key of the one-shot cache
    std::vector<int32_t> key_pages, req_leaf;
    std::vector<hkv_node> nodes;            // the same forest in 16-token blocks (page_begin, n_pages into node_pages)
    std::vector<int32_t> node_pages;
    std::vector<DecodeItem> items;
    // Items shared by kMinTileItemRows query rows or more (up to 256 / G requests each): run by the 256-row
    // tile kernel on tile_workgroups persistent workgroups, on a stream of the plan's own next to the kernel
    // that runs `items` (or in front of it on the caller's stream when concurrent is false).
    std::vector<DecodeItem> tile_items;
    int32_t tile_workgroups = 0;
    bool no_tiles = false, concurrent = true;
    bool fused = false;  // both kinds of items go out as one launch (no item of `items` has more than 16 rows)
    hipStream_t side = nullptr;
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    hipEvent_t ev_tile[2] = {nullptr, nullptr};  // profiling: begin/end of the tile kernel
    std::vector<int32_t> node_req_indptr, node_req_idx, part_count;
    // one device allocation holding items | pages | node_req_idx | part_count | tile_items
    void *dev = nullptr;
    DecodeItem *d_items = nullptr, *d_tile_items = nullptr;
    int32_t n_single = 0;  // items [0, n_single) run one per workgroup, the rest four per workgroup
    int32_t n_stages = 3;  // LDS stages of 16 KiB per workgroup of the per-node kernel
    bool fp8_matrix = false;  // fp8 pools: both products on the fp8 matrix instruction (HKV_PLAN_FP8_MATRIX)
    hkv_decode_plan_params opt{};  // the planner's settings (0 = the library's choice)
    int32_t *d_pages = nullptr, *d_node_req_idx = nullptr, *d_part_count = nullptr;
    std::vector<int32_t> q_rows;  // row of q / out / lse of every row of the plan (empty: row r is row r)
    int32_t *d_q_rows = nullptr;
    bool profiling = false, profiled_run = false;
    hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};  // begin/end of the node kernel, begin/end of the merge
    // several query tokens per request: n_req above counts query rows (requests x tokens_per_req)
    int32_t tokens_per_req = 1;
    // one allocation (d_row_mask), null when tokens_per_req == 1
    unsigned long long *d_row_mask = nullptr;
    int32_t *d_row_leaf = nullptr, *d_row_limit = nullptr;
    // fp32 pools: no work items; every query row walks its own block table (one allocation: d_bt)
    std::vector<int32_t> row_len;
    int32_t max_pages = 0;
    int32_t *d_bt = nullptr, *d_rows_req = nullptr, *d_rows_len = nullptr;
    // growing plans (hkv_decode_plan_create_growing): every request's leaf has block slots in node_pages
    // for reserve_tokens more tokens; grow_items holds, per request, the num_kv_heads items of the leaf's
    // last chunk.  Items and block list are re-sent after every append through a ring of pinned buffers.
    int32_t reserve_tokens = 0, appended = 0;
    std::vector<int32_t> grow_items;
    static constexpr int kGrowSlots = 4;
    char *h_grow = nullptr;  // pinned, kGrowSlots x grow_bytes
    char *d_grow = nullptr;  // the same memory as the device addresses it
    int32_t *d_grow_items = nullptr;  // device copy of grow_items (up to 256 requests: updates by a small kernel)
    size_t grow_bytes = 0;   // items + block list as laid out on the device, a multiple of 16
    hipEvent_t grow_free[kGrowSlots] = {};
    bool grow_in_flight[kGrowSlots] = {};
    int grow_next = 0;
};

struct hkv_prefill_plan {
    hkv_pool *pool = nullptr;
    int32_t n_req = 0, num_q_heads = 0, total_q = 0;
    int32_t key_max_pages = 0;   // row length of the caller's block table (pages)
    int32_t max_pages = 0;       // row length of the device table (16-token blocks)
    std::vector<int32_t> cu_q, block_table, kv_len;   // key of the one-shot cache
    std::vector<PrefillTile> tiles;
    void *dev = nullptr;
    PrefillTile *d_tiles = nullptr;
    int32_t *d_block_table = nullptr;
    int32_t *d_rows_req = nullptr, *d_rows_len = nullptr;  // fp32 pools: per new token (one allocation: d_rows_req)
    // fp8 pools: the pages the batch reads are first dequantised into a bf16 scratch pool in the caller's
    // workspace (page i of the scratch = src_pages[i]); the device block table then holds scratch indices.
    std::vector<int32_t> src_pages;
    int32_t *d_src_pages = nullptr;
    unsigned int *d_fallback = nullptr;  // tiles that repeated with a running maximum, over all runs of the plan
};

struct hkv_pool {
    hkv_pool_desc d{};
    // A page of page_size = 16 * S tokens is S consecutive 16-token blocks of the buffers: block
    // page * S + j holds tokens 16 j .. 16 j + 15 of the page.  Everything behind the entry points
    // (work lists, kernels) deals in 16-token blocks; page ids are translated where they come in.
    int32_t blocks_per_page = 1;
    std::vector<int32_t> refcnt;
    std::deque<int32_t> free_list;
    // Staging of page ids for kv_pool_write: a ring of slots (pinned host + device, one allocation
    // each), so that back-to-back writes on a stream do not wait for one another; a slot is reused
    // only after the event recorded behind its last write has completed.
    static constexpr int kMaxWritePages = 65536;
    static constexpr int kWriteSlots = 8;
    int32_t *h_ids = nullptr;  // pinned host, kWriteSlots x kMaxWritePages
    int32_t *hd_ids = nullptr; // the same memory as the device addresses it (source of the copy kernel)
    int32_t *d_ids = nullptr;  // device, same shape
    hipEvent_t slot_free[kWriteSlots] = {};
    bool slot_in_flight[kWriteSlots] = {};
    int next_slot = 0;
    hkv_decode_plan *cached_decode = nullptr;
    hkv_prefill_plan *cached_prefill = nullptr;
};

// ---------------------------------------------------------------------------------------------
extern "C" const char *hkv_last_error(void) { return g_err.c_str(); }

// ---------------------------------------------------------------------------------------------
// pool
extern "C" int kv_pool_create(const hkv_pool_desc *desc, hkv_pool **out) {
    if (!desc || !out) return fail(HKV_EINVAL, "kv_pool_create: null argument");
    *out = nullptr;
    if ((desc->page_size != 16 && desc->page_size != 32 && desc->page_size != 64 && desc->page_size != 128) ||
        desc->head_dim != HKV_HEAD_DIM)
        return fail(HKV_ESHAPE, "kv_pool_create: page_size must be 16, 32, 64 or 128 and head_dim 128 (got %d, %d)",
                    desc->page_size, desc->head_dim);
    if ((int64_t)desc->num_pages * (desc->page_size / HKV_PAGE_SIZE) > INT32_MAX)
        return fail(HKV_EINVAL, "kv_pool_create: too many 16-token blocks");
    if (desc->dtype != HKV_BF16 && desc->dtype != HKV_FP8_E4M3 && desc->dtype != HKV_FP32)
        return fail(HKV_ESHAPE, "kv_pool_create: pool dtype %d (bf16, fp8 e4m3 or fp32)", desc->dtype);
    if (desc->num_pages <= 0 || desc->num_kv_heads <= 0)
        return fail(HKV_EINVAL, "kv_pool_create: num_pages and num_kv_heads must be positive");
    if (!desc->k_pages || !desc->v_pages) return fail(HKV_EINVAL, "kv_pool_create: null page buffer");
    if (desc->dtype == HKV_FP8_E4M3 && (!desc->k_scale || !desc->v_scale))
        return fail(HKV_ESHAPE, "kv_pool_create: fp8 pools need k_scale and v_scale");
    if ((reinterpret_cast<uintptr_t>(desc->k_pages) | reinterpret_cast<uintptr_t>(desc->v_pages)) & 15)
        return fail(HKV_EINVAL, "kv_pool_create: page buffers must be 16-byte aligned");
    hkv_pool *p = new (std::nothrow) hkv_pool;
    if (!p) return fail(HKV_ENOMEM, "kv_pool_create: out of host memory");
    p->d = *desc;
    p->d.free_order = nullptr;
    p->blocks_per_page = desc->page_size / HKV_PAGE_SIZE;
    p->refcnt.assign(desc->num_pages, 0);
    if (desc->free_order) {
        std::vector<char> seen(desc->num_pages, 0);
        for (int i = 0; i < desc->num_pages; ++i) {
            int32_t id = desc->free_order[i];
            if (id < 0 || id >= desc->num_pages || seen[id]) {
                delete p;
                return fail(HKV_EINVAL, "kv_pool_create: free_order is not a permutation (entry %d = %d)", i, id);
            }
            seen[id] = 1;
            p->free_list.push_back(id);
        }
    } else {
        for (int i = 0; i < desc->num_pages; ++i) p->free_list.push_back(i);
    }
    *out = p;
    return HKV_OK;
}

extern "C" int kv_pool_destroy(hkv_pool *pool) {
    if (!pool) return HKV_OK;
    if (pool->cached_decode) hkv_decode_plan_destroy(pool->cached_decode);
    if (pool->cached_prefill) hkv_prefill_plan_destroy(pool->cached_prefill);
    for (hipEvent_t e : pool->slot_free)
        if (e) {
            (void)hipEventSynchronize(e);
            (void)hipEventDestroy(e);
        }
    if (pool->d_ids) (void)hipFree(pool->d_ids);
    if (pool->h_ids) (void)hipHostFree(pool->h_ids);
    delete pool;
    return HKV_OK;
}

extern "C" int kv_pool_alloc(hkv_pool *pool, int32_t n, int32_t *ids_out) {
    if (!pool || n < 0 || (n > 0 && !ids_out)) return fail(HKV_EINVAL, "kv_pool_alloc: bad argument");
    if ((size_t)n > pool->free_list.size())
        return fail(HKV_ENOMEM, "kv_pool_alloc: %d pages requested, %zu free", n, pool->free_list.size());
    for (int i = 0; i < n; ++i) {
        int32_t id = pool->free_list.front();
        pool->free_list.pop_front();
        pool->refcnt[id] = 1;
        ids_out[i] = id;
    }
    return HKV_OK;
}

static int check_held(const hkv_pool *pool, int32_t n, const int32_t *ids, const char *who) {
    if (!pool || n < 0 || (n > 0 && !ids)) return fail(HKV_EINVAL, "%s: bad argument", who);
    for (int i = 0; i < n; ++i) {
        if (ids[i] < 0 || ids[i] >= pool->d.num_pages)
            return fail(HKV_ERANGE, "%s: page id %d (entry %d) outside pool of %d pages", who, ids[i], i,
                        pool->d.num_pages);
    }
    // a page listed k times needs at least k references for a release; at least 1 for a retain
    return HKV_OK;
}

extern "C" int kv_pool_retain(hkv_pool *pool, int32_t n, const int32_t *ids) {
    if (int rc = check_held(pool, n, ids, "kv_pool_retain")) return rc;
    for (int i = 0; i < n; ++i)
        if (pool->refcnt[ids[i]] <= 0) return fail(HKV_EINVAL, "kv_pool_retain: page %d is not allocated", ids[i]);
    for (int i = 0; i < n; ++i) ++pool->refcnt[ids[i]];
    return HKV_OK;
}

extern "C" int kv_pool_release(hkv_pool *pool, int32_t n, const int32_t *ids) {
    if (int rc = check_held(pool, n, ids, "kv_pool_release")) return rc;
    std::vector<int32_t> sorted(ids, ids + n);  // a page may occur several times: count per page
    std::sort(sorted.begin(), sorted.end());
    for (int i = 0, run = 0; i < n; ++i) {
        run = (i > 0 && sorted[i] == sorted[i - 1]) ? run + 1 : 1;
        if (run > pool->refcnt[sorted[i]])
            return fail(HKV_EINVAL, "kv_pool_release: page %d released more often than it is held", sorted[i]);
    }
    for (int i = 0; i < n; ++i)
        if (--pool->refcnt[ids[i]] == 0) pool->free_list.push_back(ids[i]);
    return HKV_OK;
}

extern "C" int32_t kv_pool_num_free(const hkv_pool *pool) {
    if (!pool) return fail(HKV_EINVAL, "kv_pool_num_free: null pool");
    return (int32_t)pool->free_list.size();
}

extern "C" int32_t kv_pool_page_size(const hkv_pool *pool) {
    if (!pool) return fail(HKV_EINVAL, "kv_pool_page_size: null pool");
    return pool->d.page_size;
}

extern "C" int32_t kv_pool_refcount(const hkv_pool *pool, int32_t page_id) {
    if (!pool) return fail(HKV_EINVAL, "kv_pool_refcount: null pool");
    if (page_id < 0 || page_id >= pool->d.num_pages) return fail(HKV_ERANGE, "kv_pool_refcount: page id %d", page_id);
    return pool->refcnt[page_id];
}

static PoolView view_of(const hkv_pool *p) {
    return PoolView{p->d.k_pages, p->d.v_pages, p->d.k_scale, p->d.v_scale, p->d.num_kv_heads, p->d.dtype};
}

extern "C" int kv_pool_copy_on_write(hkv_pool *pool, int32_t n, int32_t *ids, void *stream) {
    if (int rc = check_held(pool, n, ids, "kv_pool_copy_on_write")) return rc;
    std::vector<int32_t> sorted(ids, ids + n);
    std::sort(sorted.begin(), sorted.end());
    size_t shared = 0;
    for (int i = 0; i < n; ++i) {
        if (i > 0 && sorted[i] == sorted[i - 1])
            return fail(HKV_EINVAL, "kv_pool_copy_on_write: page %d listed twice", sorted[i]);
        if (pool->refcnt[sorted[i]] <= 0)
            return fail(HKV_EINVAL, "kv_pool_copy_on_write: page %d is not allocated", sorted[i]);
        shared += pool->refcnt[sorted[i]] > 1;
    }
    if (shared > pool->free_list.size())
        return fail(HKV_ENOMEM, "kv_pool_copy_on_write: %zu private copies needed, %zu pages free", shared,
                    pool->free_list.size());
    PoolCopyLaunch a{};
    a.pool = view_of(pool);
    a.blocks_per_page = pool->blocks_per_page;
    for (int i = 0; i < n; ++i) {
        const int32_t old = ids[i];
        if (pool->refcnt[old] == 1) continue;  // sole holder: it may write in place
        const int32_t fresh = pool->free_list.front();
        pool->free_list.pop_front();
        pool->refcnt[fresh] = 1;
        --pool->refcnt[old];
        ids[i] = fresh;
        a.src[a.n] = old;
        a.dst[a.n] = fresh;
        if (++a.n == kMaxCopyPairs) {
            HKV_HIP(launch_pool_copy(a, static_cast<hipStream_t>(stream)));
            a.n = 0;
        }
    }
    HKV_HIP(launch_pool_copy(a, static_cast<hipStream_t>(stream)));
    return HKV_OK;
}

static int ensure_write_staging(hkv_pool *pool) {
    if (pool->h_ids) return HKV_OK;
    const size_t bytes = sizeof(int32_t) * hkv_pool::kMaxWritePages * hkv_pool::kWriteSlots;
    HKV_HIP(hipHostMalloc((void **)&pool->h_ids, bytes, hipHostMallocDefault));
    HKV_HIP(hipHostGetDevicePointer((void **)&pool->hd_ids, pool->h_ids, 0));
    HKV_HIP(hipMalloc((void **)&pool->d_ids, bytes));
    for (hipEvent_t &e : pool->slot_free) HKV_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
    return HKV_OK;
}

extern "C" int kv_pool_write(hkv_pool *pool, const int32_t *page_ids, int32_t first_slot, int32_t n_tokens,
                             const void *k_src, const void *v_src, void *stream) {
    if (!pool) return fail(HKV_EINVAL, "kv_pool_write: null pool");
    const int P = pool->d.page_size, S = pool->blocks_per_page;
    if (n_tokens < 0 || first_slot < 0 || first_slot >= P)
        return fail(HKV_EINVAL, "kv_pool_write: n_tokens %d, first_slot %d", n_tokens, first_slot);
    if (n_tokens == 0) return HKV_OK;
    if (!page_ids || !k_src || !v_src) return fail(HKV_EINVAL, "kv_pool_write: null argument");
    if ((reinterpret_cast<uintptr_t>(k_src) | reinterpret_cast<uintptr_t>(v_src)) & 15)
        return fail(HKV_EINVAL, "kv_pool_write: k_src and v_src must be 16-byte aligned");
    // 16-token blocks touched: b0 .. b1 of the listed pages' concatenated blocks
    const int64_t b0 = first_slot / HKV_PAGE_SIZE, b1 = ((int64_t)first_slot + n_tokens - 1) / HKV_PAGE_SIZE;
    const int64_t n_pg = b1 - b0 + 1;
    if (n_pg > hkv_pool::kMaxWritePages)
        return fail(HKV_EINVAL, "kv_pool_write: %lld pages in one call (limit %d)", (long long)n_pg,
                    hkv_pool::kMaxWritePages);
    for (int64_t i = 0; i <= b1 / S; ++i)
        if (page_ids[i] < 0 || page_ids[i] >= pool->d.num_pages)
            return fail(HKV_ERANGE, "kv_pool_write: page id %d (entry %lld) outside pool of %d pages", page_ids[i],
                        (long long)i, pool->d.num_pages);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (int rc = ensure_write_staging(pool)) return rc;
    const int slot = pool->next_slot;
    pool->next_slot = (slot + 1) % hkv_pool::kWriteSlots;
    if (pool->slot_in_flight[slot]) HKV_HIP(hipEventSynchronize(pool->slot_free[slot]));  // its last write is done
    int32_t *h = pool->h_ids + (size_t)slot * hkv_pool::kMaxWritePages;
    int32_t *d = pool->d_ids + (size_t)slot * hkv_pool::kMaxWritePages;
    for (int64_t b = b0; b <= b1; ++b) h[b - b0] = page_ids[b / S] * S + (int32_t)(b % S);
    // a copy kernel on the stream reads the pinned slot (a DMA copy between kernels of one stream costs more)
    HKV_HIP(launch_upload(pool->hd_ids + (size_t)slot * hkv_pool::kMaxWritePages, d, align_up(sizeof(int32_t) * (size_t)n_pg, 16), s));
    PoolWriteLaunch a{pool->d.k_pages, pool->d.v_pages, pool->d.k_scale, pool->d.v_scale, pool->d.num_kv_heads,
                      pool->d.dtype, d, (int32_t)n_pg, first_slot % HKV_PAGE_SIZE, n_tokens, k_src, v_src, nullptr};
    if (pool->d.dtype == HKV_FP32)
        HKV_HIP(launch_pool_write_fp32(a, s));
    else
        HKV_HIP(launch_pool_write(a, s));
    HKV_HIP(hipEventRecord(pool->slot_free[slot], s));
    pool->slot_in_flight[slot] = true;
    return HKV_OK;
}

extern "C" int kv_pool_append(hkv_pool *pool, const int32_t *page_ids, const int32_t *slots, int32_t n,
                              const void *k_src, const void *v_src, void *stream) {
    if (!pool) return fail(HKV_EINVAL, "kv_pool_append: null pool");
    if (n < 0) return fail(HKV_EINVAL, "kv_pool_append: n %d", n);
    if (n == 0) return HKV_OK;
    if (!page_ids || !slots || !k_src || !v_src) return fail(HKV_EINVAL, "kv_pool_append: null argument");
    if (pool->d.dtype == HKV_FP32) return fail(HKV_ESHAPE, "kv_pool_append: bf16 and fp8 pools only");
    if ((reinterpret_cast<uintptr_t>(k_src) | reinterpret_cast<uintptr_t>(v_src)) & 15)
        return fail(HKV_EINVAL, "kv_pool_append: k_src and v_src must be 16-byte aligned");
    if (n > hkv_pool::kMaxWritePages / 2) return fail(HKV_EINVAL, "kv_pool_append: %d tokens in one call (limit %d)", n, hkv_pool::kMaxWritePages / 2);
    const int P = pool->d.page_size, S = pool->blocks_per_page;
    for (int i = 0; i < n; ++i) {
        if (page_ids[i] < 0 || page_ids[i] >= pool->d.num_pages)
            return fail(HKV_ERANGE, "kv_pool_append: page id %d (entry %d) outside pool of %d pages", page_ids[i], i, pool->d.num_pages);
        if (slots[i] < 0 || slots[i] >= P) return fail(HKV_EINVAL, "kv_pool_append: slot %d (entry %d)", slots[i], i);
        if (pool->refcnt[page_ids[i]] > 1)
            return fail(HKV_EINVAL, "kv_pool_append: page %d (entry %d) has %d owners: kv_pool_copy_on_write first", page_ids[i], i,
                        pool->refcnt[page_ids[i]]);
    }
    if (n > 1) {  // two tokens of one call in one block would race on the block's scale and on its re-encoding
        std::vector<int32_t> blocks(n);
        for (int i = 0; i < n; ++i) blocks[i] = page_ids[i] * S + slots[i] / HKV_PAGE_SIZE;
        std::sort(blocks.begin(), blocks.end());
        auto dup = std::adjacent_find(blocks.begin(), blocks.end());
        if (dup != blocks.end())
            return fail(HKV_EINVAL, "kv_pool_append: two tokens go to block %d of page %d", *dup % S, *dup / S);
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (n <= kMaxInlineAppend) {  // the usual decode batch: everything travels in the kernel arguments
        PoolAppendInline a{};
        a.base = PoolWriteLaunch{pool->d.k_pages, pool->d.v_pages, pool->d.k_scale, pool->d.v_scale, pool->d.num_kv_heads,
                                 pool->d.dtype, nullptr, n, 0, n, k_src, v_src, nullptr};
        for (int i = 0; i < n; ++i) {
            a.block[i] = page_ids[i] * S + slots[i] / HKV_PAGE_SIZE;
            a.slot[i] = (uint8_t)(slots[i] % HKV_PAGE_SIZE);
        }
        HKV_HIP(launch_pool_append_inline(a, s));
        return HKV_OK;
    }
    if (int rc = ensure_write_staging(pool)) return rc;
    const int slot = pool->next_slot;
    pool->next_slot = (slot + 1) % hkv_pool::kWriteSlots;
    if (pool->slot_in_flight[slot]) HKV_HIP(hipEventSynchronize(pool->slot_free[slot]));
    int32_t *h = pool->h_ids + (size_t)slot * hkv_pool::kMaxWritePages;
    int32_t *d = pool->d_ids + (size_t)slot * hkv_pool::kMaxWritePages;
    for (int i = 0; i < n; ++i) {  // block ids, then the slots inside them
        h[i] = page_ids[i] * S + slots[i] / HKV_PAGE_SIZE;
        h[n + i] = slots[i] % HKV_PAGE_SIZE;
    }
    HKV_HIP(launch_upload(pool->hd_ids + (size_t)slot * hkv_pool::kMaxWritePages, d, align_up(sizeof(int32_t) * 2 * (size_t)n, 16), s));
    PoolWriteLaunch a{pool->d.k_pages, pool->d.v_pages, pool->d.k_scale, pool->d.v_scale, pool->d.num_kv_heads,
                      pool->d.dtype, d, n, 0, n, k_src, v_src, d + n};
    HKV_HIP(launch_pool_write(a, s));
    HKV_HIP(hipEventRecord(pool->slot_free[slot], s));
    pool->slot_in_flight[slot] = true;
    return HKV_OK;
}

// ---------------------------------------------------------------------------------------------
// forest
// whole_page_parents: a node with children must hold a multiple of 16 tokens (what a flat block table
// needs: positions along a path then map to pages without gaps); false for callers that walk the forest
// node by node.
static int validate_forest(const hkv_node *nodes, int32_t n_nodes, const int32_t *node_pages, int32_t n_node_pages,
                           const char *who, bool whole_page_parents = true, int page_size = HKV_PAGE_SIZE) {
    if (n_nodes < 0 || n_node_pages < 0 || (n_nodes > 0 && !nodes) || (n_node_pages > 0 && !node_pages))
        return fail(HKV_EINVAL, "%s: bad forest arguments", who);
    std::vector<char> has_child(n_nodes, 0);
    for (int v = 0; v < n_nodes; ++v) {
        const hkv_node &nd = nodes[v];
        if (nd.parent < -1 || nd.parent >= v)
            return fail(HKV_ETREE, "%s: node %d has parent %d (parents must come first)", who, v, nd.parent);
        if (nd.n_tokens < 0 || nd.n_pages != (nd.n_tokens + page_size - 1) / page_size)
            return fail(HKV_ETREE, "%s: node %d has %d tokens but %d pages", who, v, nd.n_tokens, nd.n_pages);
        if (nd.page_begin < 0 || (int64_t)nd.page_begin + nd.n_pages > n_node_pages)
            return fail(HKV_ERANGE, "%s: node %d pages [%d, %d) outside node_pages of %d", who, v, nd.page_begin,
                        nd.page_begin + nd.n_pages, n_node_pages);
        if (nd.parent >= 0) has_child[nd.parent] = 1;
    }
    if (whole_page_parents)
        for (int v = 0; v < n_nodes; ++v)
            if (has_child[v] && nodes[v].n_tokens % page_size)
                return fail(HKV_ETREE, "%s: node %d has children but %d tokens (not a multiple of %d)", who, v,
                            nodes[v].n_tokens, page_size);
    return HKV_OK;
}

static int build_node_req_csr(const hkv_node *nodes, int32_t n_nodes, const int32_t *req_leaf, int32_t n_req,
                              std::vector<int32_t> &indptr, std::vector<int32_t> &idx, const char *who) {
    if (n_req < 0 || (n_req > 0 && !req_leaf)) return fail(HKV_EINVAL, "%s: bad request list", who);
    indptr.assign((size_t)n_nodes + 1, 0);
    for (int r = 0; r < n_req; ++r) {
        if (req_leaf[r] < 0 || req_leaf[r] >= n_nodes)
            return fail(HKV_ERANGE, "%s: request %d ends at node %d of %d", who, r, req_leaf[r], n_nodes);
        for (int v = req_leaf[r]; v >= 0; v = nodes[v].parent) ++indptr[v + 1];
    }
    for (int v = 0; v < n_nodes; ++v) indptr[v + 1] += indptr[v];
    idx.assign((size_t)indptr[n_nodes], 0);
    std::vector<int32_t> fill(indptr.begin(), indptr.end() - 1);
    for (int r = 0; r < n_req; ++r)  // ascending r keeps every node's list sorted
        for (int v = req_leaf[r]; v >= 0; v = nodes[v].parent) idx[fill[v]++] = r;
    return HKV_OK;
}

extern "C" int prefix_tree_flatten(const hkv_node *nodes, int32_t n_nodes, const int32_t *node_pages,
                                   int32_t n_node_pages, const int32_t *req_leaf, int32_t n_req, int32_t max_pages,
                                   int32_t *block_table, int32_t *kv_len, int32_t *node_req_indptr,
                                   int32_t *node_req_idx, int32_t *node_tok_start) {
    return prefix_tree_flatten_paged(nodes, n_nodes, node_pages, n_node_pages, req_leaf, n_req, HKV_PAGE_SIZE, max_pages,
                                     block_table, kv_len, node_req_indptr, node_req_idx, node_tok_start);
}

extern "C" int prefix_tree_flatten_paged(const hkv_node *nodes, int32_t n_nodes, const int32_t *node_pages,
                                         int32_t n_node_pages, const int32_t *req_leaf, int32_t n_req,
                                         int32_t page_size, int32_t max_pages, int32_t *block_table, int32_t *kv_len,
                                         int32_t *node_req_indptr, int32_t *node_req_idx, int32_t *node_tok_start) {
    if (max_pages < 0) return fail(HKV_EINVAL, "prefix_tree_flatten: max_pages %d", max_pages);
    if (page_size != 16 && page_size != 32 && page_size != 64 && page_size != 128)
        return fail(HKV_ESHAPE, "prefix_tree_flatten: page_size %d (16, 32, 64 or 128)", page_size);
    if (int rc = validate_forest(nodes, n_nodes, node_pages, n_node_pages, "prefix_tree_flatten", true, page_size)) return rc;
    std::vector<int32_t> indptr, idx;
    if (int rc = build_node_req_csr(nodes, n_nodes, req_leaf, n_req, indptr, idx, "prefix_tree_flatten")) return rc;
    std::vector<int32_t> tok_start(n_nodes, 0), pages_before(n_nodes, 0);
    for (int v = 0; v < n_nodes; ++v) {
        int par = nodes[v].parent;
        if (par >= 0) {
            tok_start[v] = tok_start[par] + nodes[par].n_tokens;
            pages_before[v] = pages_before[par] + nodes[par].n_pages;
        }
    }
    for (int r = 0; r < n_req; ++r) {
        int leaf = req_leaf[r];
        int total_pages = pages_before[leaf] + nodes[leaf].n_pages;
        if (total_pages > max_pages)
            return fail(HKV_ENOMEM, "prefix_tree_flatten: request %d needs %d pages, max_pages is %d", r, total_pages,
                        max_pages);
    }
    for (int r = 0; r < n_req; ++r) {
        int leaf = req_leaf[r];
        if (kv_len) kv_len[r] = tok_start[leaf] + nodes[leaf].n_tokens;
        if (!block_table) continue;
        int32_t *row = block_table + (size_t)r * max_pages;
        int total_pages = pages_before[leaf] + nodes[leaf].n_pages;
        for (int i = total_pages; i < max_pages; ++i) row[i] = -1;
        for (int v = leaf; v >= 0; v = nodes[v].parent)
            for (int j = 0; j < nodes[v].n_pages; ++j) row[pages_before[v] + j] = node_pages[nodes[v].page_begin + j];
    }
    if (node_req_indptr) memcpy(node_req_indptr, indptr.data(), sizeof(int32_t) * indptr.size());
    if (node_req_idx && !idx.empty()) memcpy(node_req_idx, idx.data(), sizeof(int32_t) * idx.size());
    if (node_tok_start && n_nodes) memcpy(node_tok_start, tok_start.data(), sizeof(int32_t) * n_nodes);
    return HKV_OK;
}

extern "C" int prefix_tree_prefill_usage(const hkv_node *nodes, int32_t n_nodes, const int32_t *calls,
                                         int32_t n_calls, int64_t *u_p) {
    if (n_nodes < 0 || n_calls < 0 || (n_nodes > 0 && !nodes) || (n_calls > 0 && (!calls || !u_p)))
        return fail(HKV_EINVAL, "prefix_tree_prefill_usage: bad argument");
    for (int v = 0; v < n_nodes; ++v)
        if (nodes[v].parent < -1 || nodes[v].parent >= v || nodes[v].n_tokens < 0)
            return fail(HKV_ETREE, "prefix_tree_prefill_usage: node %d malformed", v);
    // depth and token count from the root let two leaves meet at their lowest common ancestor
    std::vector<int32_t> depth(n_nodes, 0);
    std::vector<int64_t> tok_end(n_nodes, 0);
    for (int v = 0; v < n_nodes; ++v) {
        int par = nodes[v].parent;
        depth[v] = par < 0 ? 0 : depth[par] + 1;
        tok_end[v] = (par < 0 ? 0 : tok_end[par]) + nodes[v].n_tokens;
    }
    for (int j = 0; j < n_calls; ++j) {
        if (calls[j] < 0 || calls[j] >= n_nodes)
            return fail(HKV_ERANGE, "prefix_tree_prefill_usage: call %d names node %d of %d", j, calls[j], n_nodes);
        int64_t shared = 0;
        if (j > 0) {
            int a = calls[j - 1], b = calls[j];
            while (a >= 0 && b >= 0 && a != b) {
                if (depth[a] >= depth[b]) a = nodes[a].parent; else b = nodes[b].parent;
            }
            if (a >= 0 && a == b) shared = tok_end[a];
        }
        u_p[j] = tok_end[calls[j]] - shared;
    }
    return HKV_OK;
}

// ---------------------------------------------------------------------------------------------
// lse_merge
extern "C" int lse_merge(const float *o_parts, const float *lse_parts, const int32_t *row_indptr,
                         const int32_t *part_idx, int32_t n_rows, void *out, int32_t out_dtype, float *lse_out,
                         void *stream) {
    if (n_rows < 0) return fail(HKV_EINVAL, "lse_merge: n_rows %d", n_rows);
    if (out_dtype != HKV_BF16 && out_dtype != HKV_FP32) return fail(HKV_ESHAPE, "lse_merge: out_dtype %d", out_dtype);
    if (n_rows == 0) return HKV_OK;
    if (!o_parts || !lse_parts || !row_indptr || !part_idx || !out) return fail(HKV_EINVAL, "lse_merge: null argument");
    if ((reinterpret_cast<uintptr_t>(o_parts) & 7) || (reinterpret_cast<uintptr_t>(out) & 7))
        return fail(HKV_EINVAL, "lse_merge: o_parts and out must be 8-byte aligned");
    HKV_HIP(launch_lse_merge(o_parts, lse_parts, row_indptr, part_idx, n_rows, out, out_dtype, lse_out,
                             static_cast<hipStream_t>(stream)));
    return HKV_OK;
}

extern "C" int lse_merge_dense(const float *o_parts, const float *lse_parts, const int32_t *part_count,
                               int32_t rows_per_count, int32_t max_parts, int32_t n_rows, void *out, int32_t out_dtype,
                               float *lse_out, void *stream) {
    if (n_rows < 0 || rows_per_count <= 0 || max_parts <= 0)
        return fail(HKV_EINVAL, "lse_merge_dense: n_rows %d, rows_per_count %d, max_parts %d", n_rows, rows_per_count,
                    max_parts);
    if (out_dtype != HKV_BF16 && out_dtype != HKV_FP32) return fail(HKV_ESHAPE, "lse_merge_dense: out_dtype %d", out_dtype);
    if (n_rows == 0) return HKV_OK;
    if (!o_parts || !lse_parts || !part_count || !out) return fail(HKV_EINVAL, "lse_merge_dense: null argument");
    if ((reinterpret_cast<uintptr_t>(o_parts) | reinterpret_cast<uintptr_t>(out)) & 15)
        return fail(HKV_EINVAL, "lse_merge_dense: o_parts and out must be 16-byte aligned");
    HKV_HIP(launch_lse_merge_dense(o_parts, lse_parts, part_count, rows_per_count, max_parts, n_rows, out, out_dtype,
                                   lse_out, static_cast<hipStream_t>(stream)));
    return HKV_OK;
}

// ---------------------------------------------------------------------------------------------
// decode planning
//
// A node with T tokens that R requests pass through is cut into work items of at most 64 query
// rows (R_item * G) and a token chunk each.  Every item yields one partial result per row, so the
// chunk length trades parallelism (more items) against partial-result traffic (516 B per row and
// item, written once and read once).
//
// Partials are stored densely: the path above a node is common to every request below it, so the
// chunks of a node get the same positions k in the partial lists of all those requests, and row
// (r, h) keeps its partials at (r*Hq + h)*max_parts + k.  The merge then needs no index lists,
// only the number of partials per request.
static void plan_items(hkv_decode_plan &pl) {
    const int G = pl.group;
    const int Hkv = pl.pool->d.num_kv_heads;
    const int n_nodes = (int)pl.nodes.size();
    const hkv_decode_plan_params &opt = pl.opt;
    auto or_default = [](int32_t v, int dflt) { return v != 0 ? (int)v : dflt; };
    const ChipShape chip = chip_shape();
    const int max_req_per_item = std::max(1, or_default(opt.max_rows, 64) / G);
    // Chunk lengths.  Nodes read by at most 16 rows ("leaf type") stay whole unless the forest has
    // fewer (node, head) units than workgroups fit on the chip at once; then they are cut, but not
    // below 256 tokens.  Nodes shared by more rows run one row tile per wavefront over all tokens
    // of the item, so their chunks are kept near the typical leaf-type item to finish together.
    const int kResidentGroups = chip.n_cu * (pl.pool->d.dtype == HKV_FP8_E4M3 ? 2 : 3);  // workgroups the chip holds at once
    // Nodes shared by many rows go to the 256-row tile kernel (not with per-row visibility, which that kernel
    // does not know, and not when the caller asked for the fp8 matrix instruction).
    const int tile_min_rows = or_default(opt.tile_min_rows, 128);
    // The second kernel, its stream and the two events pay only when that share of the step is large (measured:
    // c2 and c3, 2 and 9 GFLOP of such work in steps of 30 to 50 us, lose; c5, 137 GFLOP in 0.5 ms, gains 11 %).
    bool tiles_pay = false;
    {
        double flop = 0;
        for (int v = 0; v < n_nodes; ++v) {
            const int R = pl.node_req_indptr[v + 1] - pl.node_req_indptr[v];
            if (R * G >= std::max(tile_min_rows, kMinTileItemRows))
                flop += 4.0 * HKV_HEAD_DIM * pl.nodes[v].n_tokens * (double)R * pl.num_q_heads;
        }
        tiles_pay = opt.tile_min_gflop < 0 || flop >= 1e9 * or_default(opt.tile_min_gflop, 40);
    }
    auto tiled = [&](int v) {
        const int R = pl.node_req_indptr[v + 1] - pl.node_req_indptr[v];
        return tiles_pay && !pl.no_tiles && !pl.fp8_matrix && pl.nodes[v].n_tokens > 0 &&
               R * G >= std::max(tile_min_rows, kMinTileItemRows);
    };
    int64_t leaf_units = 0, leaf_tokens = 0, shared_units = 0;
    for (int v = 0; v < n_nodes; ++v) {
        int R = pl.node_req_indptr[v + 1] - pl.node_req_indptr[v];
        if (pl.nodes[v].n_tokens == 0 || R == 0 || tiled(v)) continue;
        if (R * G > 16) {  // counted at the smallest chunk length used for such nodes
            shared_units += (int64_t)((R + max_req_per_item - 1) / max_req_per_item) * Hkv *
                            ((pl.nodes[v].n_tokens + 511) / 512);
        } else {
            leaf_units += Hkv;
            leaf_tokens += pl.nodes[v].n_tokens;
        }
    }
    int leaf_split = 1;
    if (leaf_units > 0 && leaf_units + shared_units < kResidentGroups / 2)
        leaf_split = (int)((kResidentGroups / 2 + leaf_units - 1) / leaf_units);
    const int mean_leaf = leaf_units ? (int)(leaf_tokens * Hkv / leaf_units) : 512;
    int leaf_chunk = std::max(256, (mean_leaf / leaf_split + 15) / 16 * 16);
    if (leaf_split == 1) leaf_chunk = 1 << 30;  // whole nodes
    int shared_chunk = std::min(kMaxSharedItemTokens, std::max(512, std::min(mean_leaf, leaf_chunk) / 16 * 16));
    // Long shared paths: every chunk costs each row below it one partial (written once, read once) and
    // every item a start-up, while a long item is the last to finish; measured on forests with 2k to 9k
    // shared tokens the best chunk is about a sixth of the path, between 512 and 1024 tokens.  Beyond
    // 16k shared tokens the chunks grow further so that a row collects about 16 partials at most.
    {
        std::vector<int64_t> shared_above(n_nodes, 0);
        int64_t longest = 0;
        for (int v = 0; v < n_nodes; ++v) {
            const int R = pl.node_req_indptr[v + 1] - pl.node_req_indptr[v];
            const int64_t up = pl.nodes[v].parent >= 0 ? shared_above[pl.nodes[v].parent] : 0;
            shared_above[v] = up + (R * G > 16 && !tiled(v) ? pl.nodes[v].n_tokens : 0);
            longest = std::max(longest, shared_above[v]);
        }
        int64_t by_path = std::min<int64_t>(1024, (longest / 6 + 128) / 256 * 256);
        if (longest > 16 * by_path) by_path = std::min<int64_t>(kMaxSharedItemTokens, (longest / 16 + 255) / 256 * 256);
        shared_chunk = std::max(shared_chunk, (int)by_path);
    }
    leaf_chunk = or_default(opt.leaf_chunk, leaf_chunk) / 16 * 16;
    shared_chunk = std::min(kMaxSharedItemTokens, or_default(opt.shared_chunk, shared_chunk)) / 16 * 16;
    // Few-row nodes a little longer than what one wavefront takes alone (pack_tokens): run whole, their
    // four wavefronts get only a few steps each and pay a start-up and a combine through LDS for them.
    // When cutting them into pieces of at most pack_tokens makes the forest large enough for the
    // four-items-per-workgroup mode, each wavefront streams a piece of 8 to 12 steps on its own instead
    // (c2: 512-token leaves as 2 x 256, per-node kernel 31.7 -> 30.0 us).  Nodes of 8 / 3 pack_tokens and
    // more keep their four wavefronts: those already get that many steps each.
    const int step_tokens = pl.pool->d.dtype == HKV_FP8_E4M3 ? 64 : 32;
    const int pack_tokens = or_default(opt.pack_tokens, 12 * step_tokens);
    const int pack_mode = or_default(opt.pack, 2);  // 1: never, 2: when the items exceed the resident workgroups, 3: always
    auto cut_for_packing = [&](int n_tokens) { return n_tokens > pack_tokens && 3 * n_tokens < 8 * pack_tokens; };
    bool cut_leaves = false;
    if (leaf_split == 1 && pack_mode != 1 && opt.leaf_chunk == 0) {
        int64_t units = shared_units;
        bool any = false;
        for (int v = 0; v < n_nodes; ++v) {
            const int R = pl.node_req_indptr[v + 1] - pl.node_req_indptr[v];
            const int T = pl.nodes[v].n_tokens;
            if (T == 0 || R == 0 || R * G > 16) continue;
            any |= cut_for_packing(T);
            units += (int64_t)Hkv * (cut_for_packing(T) ? (T + pack_tokens - 1) / pack_tokens : 1);
        }
        cut_leaves = any && (pack_mode == 3 || units > kResidentGroups);
    }
    // The tile kernel's share of the chip: its persistent workgroups hold one compute unit each for as long as
    // the other kernel streams its bytes, so their number follows from the two amounts of work (matrix
    // arithmetic at about 3.5 TFLOP/s per compute unit against bytes at about 5.5 TB/s for the chip).
    const int req_per_tile = std::max(1, 256 / G);
    pl.tile_items.clear();
    pl.tile_workgroups = 0;
    int tile_chunk = kMaxTileItemTokens;
    double step_seconds = 0;  // what streaming all the bytes of the step takes
    {
        double tile_flop = 0, other_bytes = 0, tile_bytes = 0;
        int64_t tile_units = 0, tile_tokens_max = 0;
        const double bytes_per_token = 2.0 * HKV_HEAD_DIM * (pl.pool->d.dtype == HKV_FP8_E4M3 ? 1 : 2);
        for (int v = 0; v < n_nodes; ++v) {
            const int R = pl.node_req_indptr[v + 1] - pl.node_req_indptr[v];
            if (pl.nodes[v].n_tokens == 0 || R == 0) continue;
            if (tiled(v)) {
                tile_flop += 4.0 * HKV_HEAD_DIM * pl.nodes[v].n_tokens * (double)R * pl.num_q_heads;
                tile_units += (int64_t)((R + req_per_tile - 1) / req_per_tile) * Hkv;
                tile_tokens_max = std::max<int64_t>(tile_tokens_max, pl.nodes[v].n_tokens);
                tile_bytes += bytes_per_token * pl.nodes[v].n_tokens * Hkv;
            } else {
                other_bytes += bytes_per_token * pl.nodes[v].n_tokens * Hkv;
            }
        }
        step_seconds = (other_bytes + tile_bytes) / 5.6e12;
        if (tile_units > 0) {
            const int n_cu = chip.n_cu;
            int wgs = n_cu;
            if (other_bytes > 0) {
                const double t_other = other_bytes / 5.5e12;
                wgs = (int)(tile_flop / (3.5e12 * t_other) + 0.999);
                wgs = std::min(n_cu - 64, std::max(8, (wgs + 7) / 8 * 8));  // whole groups of 8: one per XCD
            }
            wgs = std::min(n_cu, or_default(opt.tile_workgroups, wgs));
            pl.tile_workgroups = wgs;
            // chunks: about one item per workgroup (a workgroup that is done gives its compute unit to the other
            // items, and every chunk costs every row below the node a partial), more where the nodes are few
            const int64_t n_chunks = std::max<int64_t>(1, std::min<int64_t>((wgs + tile_units / 2) / tile_units, tile_tokens_max / 256));
            int64_t ch = ((tile_tokens_max + n_chunks - 1) / n_chunks + 63) / 64 * 64;
            tile_chunk = (int)std::min<int64_t>(kMaxTileItemTokens, std::max<int64_t>(256, ch));
            tile_chunk = std::min(kMaxTileItemTokens, or_default(opt.tile_chunk, tile_chunk)) / 16 * 16;
        }
    }
    struct Proto { DecodeItem it; int64_t cost; };
    std::vector<Proto> protos;
    std::vector<int32_t> node_chunks(n_nodes, 0), slot_base(n_nodes, 0);
    for (int v = 0; v < n_nodes; ++v) {
        const hkv_node &nd = pl.nodes[v];
        if (nd.parent >= 0) slot_base[v] = slot_base[nd.parent] + node_chunks[nd.parent];
        int R = pl.node_req_indptr[v + 1] - pl.node_req_indptr[v];
        if (nd.n_tokens == 0 || R == 0) continue;
        if (tiled(v)) {  // equal chunks of whole pages x equal request groups x KV heads, longest chunks first below
            const int n_chunks = (nd.n_tokens + tile_chunk - 1) / tile_chunk;
            const int pages_per_chunk = (nd.n_pages + n_chunks - 1) / n_chunks;
            node_chunks[v] = (nd.n_pages + pages_per_chunk - 1) / pages_per_chunk;
            const int n_groups = (R + req_per_tile - 1) / req_per_tile;
            const int req_per_group = (R + n_groups - 1) / n_groups;
            for (int pg = 0, ci = 0; pg < nd.n_pages; pg += pages_per_chunk, ++ci) {
                const int tb = pg * 16;
                const int nt = std::min(pages_per_chunk * 16, nd.n_tokens - tb);
                for (int r0 = 0; r0 < R; r0 += req_per_group)
                    for (int h = 0; h < Hkv; ++h)
                        pl.tile_items.push_back(DecodeItem{nd.page_begin + pg, nt, h, pl.node_req_indptr[v] + r0,
                                                           std::min(req_per_group, R - r0), slot_base[v] + ci, tb, v});
            }
            continue;
        }
        int chunk = std::max(16, R * G > 16 ? shared_chunk : leaf_chunk);
        if (R * G <= 16 && cut_leaves && cut_for_packing(nd.n_tokens)) chunk = pack_tokens;  // equal pieces below
        // equal chunks of whole pages
        int n_chunks = (nd.n_tokens + chunk - 1) / chunk;
        int pages_per_chunk = (nd.n_pages + n_chunks - 1) / n_chunks;
        node_chunks[v] = (nd.n_pages + pages_per_chunk - 1) / pages_per_chunk;
        for (int r0 = 0; r0 < R; r0 += max_req_per_item) {
            int nr = std::min(max_req_per_item, R - r0);
            for (int pg = 0, ci = 0; pg < nd.n_pages; pg += pages_per_chunk, ++ci) {
                int tb = pg * 16;
                int nt = std::min(pages_per_chunk * 16, nd.n_tokens - tb);
                for (int h = 0; h < Hkv; ++h) {
                    DecodeItem it{nd.page_begin + pg, nt, h, pl.node_req_indptr[v] + r0, nr, slot_base[v] + ci, tb, v};
                    int rows = nr * G;
                    protos.push_back({it, (int64_t)nt * std::max(16, (rows + 15) / 16 * 16)});
                }
            }
        }
    }
    // Forests with more items than the chip holds at once: the short items of at most 16 rows are run four
    // to a workgroup, one per wavefront (a workgroup's start-up then serves four items, and such a
    // wavefront streams its whole item with one step in flight); they are listed behind the others.
    const bool pack = pack_mode == 3 || (pack_mode == 2 && (int64_t)protos.size() > kResidentGroups);
    auto packable = [&](const Proto &p) { return pack && p.it.n_req * G <= 16 && p.it.n_tokens <= pack_tokens; };
    // one item per workgroup first, heavy before light in both classes: a single integer key per item
    for (Proto &p : protos) p.cost = (packable(p) ? 0 : (int64_t)1 << 56) + p.cost;
    std::stable_sort(protos.begin(), protos.end(), [](const Proto &a, const Proto &b) { return a.cost > b.cost; });
    // Among the one-item workgroups, items shared by more than 16 query rows are bound by their instruction
    // stream and items of few rows by memory: the two classes are dispatched side by side, each spread evenly
    // over the list (groups of 8 = one workgroup per XCD), so that both are resident on every CU throughout
    // instead of one class after the other.  Within a class the order stays heavy before light.
    if (const int group = or_default(opt.interleave, 8); group > 0) {
        std::vector<Proto> many, few, rest, merged;
        for (auto &p : protos) (packable(p) ? rest : p.it.n_req * G > 16 ? many : few).push_back(p);
        if (!many.empty() && !few.empty()) {
            merged.reserve(protos.size());
            size_t a = 0, b = 0;
            while (a < many.size()) {
                for (int i = 0; i < group && a < many.size(); ++i) merged.push_back(many[a++]);
                const size_t target = (size_t)((double)a * few.size() / many.size() + 0.5);
                while (b < target && b < few.size()) merged.push_back(few[b++]);
            }
            while (b < few.size()) merged.push_back(few[b++]);
            merged.insert(merged.end(), rest.begin(), rest.end());
            protos.swap(merged);
        }
    }
    std::stable_sort(pl.tile_items.begin(), pl.tile_items.end(),
                     [](const DecodeItem &x, const DecodeItem &y) { return x.n_tokens > y.n_tokens; });
    // While the items leave a quarter of the chip to the other items' first workgroups: as few persistent
    // workgroups as finish their chain of items within the step (a tile item runs at about 5.5 TFLOP/s on its
    // compute unit), in whole groups of 8 (one per XCD).  The items then hold few compute units for the whole
    // step instead of many for a part of it, which the streaming items use better (c5: 64 workgroups of two
    // items against 128 of one, step -2 %); a chain that outlasts the step would lengthen it, hence the margin.
    if (opt.tile_workgroups == 0 && !pl.tile_items.empty() && (int)pl.tile_items.size() <= chip.n_cu - 64) {
        const int n_items = (int)pl.tile_items.size();
        double item_seconds = 0;
        for (const DecodeItem &it : pl.tile_items)
            item_seconds = std::max(item_seconds, 4.0 * HKV_HEAD_DIM * it.n_tokens * (double)it.n_req * G / 5.5e12);
        const int chain = std::max(1, (int)(step_seconds / item_seconds - 0.1));
        pl.tile_workgroups = std::min(n_items, ((n_items + chain - 1) / chain + 7) / 8 * 8);
    }
    pl.tile_workgroups = std::min<int32_t>(pl.tile_workgroups, (int32_t)pl.tile_items.size());
    pl.items.clear();
    pl.n_single = 0;
    for (auto &p : protos) {
        pl.items.push_back(p.it);
        pl.n_single += !packable(p);
    }
    // LDS stages per workgroup.  The fp8 kernel runs two workgroups per CU (registers), so each may own
    // half of the CU's 160 KiB: five stages, four steps of a shared item in flight instead of two.
    pl.n_stages = or_default(opt.stages, pl.pool->d.dtype == HKV_FP8_E4M3 ? 5 : 3);
    pl.part_count.assign(pl.n_req, 0);
    pl.max_parts = 1;
    for (int r = 0; r < pl.n_req; ++r) {
        int leaf = pl.req_leaf[r];
        pl.part_count[r] = slot_base[leaf] + node_chunks[leaf];
        pl.max_parts = std::max(pl.max_parts, pl.part_count[r]);
    }
    pl.n_parts = pl.n_req * pl.num_q_heads * pl.max_parts;
    // One launch for both kinds of items where the kernel allows it: its workgroups of the other items run two
    // blocks side by side, which works as long as no item synchronises per step (more than 16 query rows).
    pl.fused = !pl.tile_items.empty() && !pl.items.empty() && opt.fused >= 0 && !pl.fp8_matrix;
    for (const DecodeItem &it : pl.items) pl.fused = pl.fused && it.n_req * G <= 16;
}

static int upload_decode_plan(hkv_decode_plan &pl) {
    size_t off_items = 0;
    size_t off_pages = align_up(off_items + sizeof(DecodeItem) * pl.items.size(), 256);
    size_t off_nri = align_up(off_pages + sizeof(int32_t) * pl.node_pages.size(), 256);
    size_t off_cnt = align_up(off_nri + sizeof(int32_t) * pl.node_req_idx.size(), 256);
    size_t off_tiles = align_up(off_cnt + sizeof(int32_t) * pl.part_count.size(), 256);
    size_t off_qrows = align_up(off_tiles + sizeof(DecodeItem) * pl.tile_items.size(), 256);
    size_t total = align_up(off_qrows + sizeof(int32_t) * pl.q_rows.size(), 256) + 256;
    HKV_HIP(hipMalloc(&pl.dev, total));
    char *base = static_cast<char *>(pl.dev);
    pl.d_items = reinterpret_cast<DecodeItem *>(base + off_items);
    pl.d_pages = reinterpret_cast<int32_t *>(base + off_pages);
    pl.d_node_req_idx = reinterpret_cast<int32_t *>(base + off_nri);
    pl.d_part_count = reinterpret_cast<int32_t *>(base + off_cnt);
    pl.d_tile_items = reinterpret_cast<DecodeItem *>(base + off_tiles);
    pl.d_q_rows = pl.q_rows.empty() ? nullptr : reinterpret_cast<int32_t *>(base + off_qrows);
    // one host image, one copy
    std::vector<char> image(total, 0);
    auto put = [&](size_t off, const void *src, size_t n) {
        if (n) memcpy(image.data() + off, src, n);
    };
    put(off_items, pl.items.data(), sizeof(DecodeItem) * pl.items.size());
    put(off_pages, pl.node_pages.data(), sizeof(int32_t) * pl.node_pages.size());
    put(off_nri, pl.node_req_idx.data(), sizeof(int32_t) * pl.node_req_idx.size());
    put(off_cnt, pl.part_count.data(), sizeof(int32_t) * pl.part_count.size());
    put(off_tiles, pl.tile_items.data(), sizeof(DecodeItem) * pl.tile_items.size());
    put(off_qrows, pl.q_rows.data(), sizeof(int32_t) * pl.q_rows.size());
    HKV_HIP(hipMemcpy(pl.dev, image.data(), total, hipMemcpyHostToDevice));
    if (pl.reserve_tokens > 0 && pl.n_req <= kMaxInlineAppend && !pl.grow_items.empty() && !pl.opt.large_batch_updates) {
        HKV_HIP(hipMalloc((void **)&pl.d_grow_items, sizeof(int32_t) * pl.grow_items.size()));
        HKV_HIP(hipMemcpy(pl.d_grow_items, pl.grow_items.data(), sizeof(int32_t) * pl.grow_items.size(), hipMemcpyHostToDevice));
    } else if (pl.reserve_tokens > 0) {
        pl.grow_bytes = align_up(off_pages + sizeof(int32_t) * pl.node_pages.size(), 16);  // inside the allocation: off_nri is 256-aligned
        HKV_HIP(hipHostMalloc((void **)&pl.h_grow, pl.grow_bytes * hkv_decode_plan::kGrowSlots, hipHostMallocDefault));
        HKV_HIP(hipHostGetDevicePointer((void **)&pl.d_grow, pl.h_grow, 0));
        memset(pl.h_grow, 0, pl.grow_bytes * hkv_decode_plan::kGrowSlots);
        for (hipEvent_t &e : pl.grow_free) HKV_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
    }
    if (!pl.tile_items.empty() && !pl.fused) {  // the tile kernel's own stream and the two events that fork to it and join it
        HKV_HIP(hipStreamCreateWithFlags(&pl.side, hipStreamNonBlocking));
        HKV_HIP(hipEventCreateWithFlags(&pl.ev_fork, hipEventDisableTiming));
        HKV_HIP(hipEventCreateWithFlags(&pl.ev_join, hipEventDisableTiming));
    }
    // here, so that the first run may already be under graph capture
    HKV_HIP(prepare_decode_device(nullptr));
    return HKV_OK;
}

// fp32 pools: per-row block tables (root-to-leaf page lists) and lengths instead of work items
static int build_fp32_rows(hkv_decode_plan &pl, bool upload) {
    const int n = pl.n_req;
    std::vector<std::vector<int32_t>> paths(n);
    pl.row_len.assign(n, 0);
    pl.max_pages = 1;
    for (int r = 0; r < n; ++r) {
        std::vector<int32_t> chain;
        for (int v = pl.req_leaf[r]; v >= 0; v = pl.nodes[v].parent) chain.push_back(v);
        for (auto it = chain.rbegin(); it != chain.rend(); ++it) {
            const hkv_node &nd = pl.nodes[*it];
            paths[r].insert(paths[r].end(), pl.node_pages.begin() + nd.page_begin, pl.node_pages.begin() + nd.page_begin + nd.n_pages);
            pl.row_len[r] += nd.n_tokens;
        }
        pl.max_pages = std::max<int32_t>(pl.max_pages, (int32_t)paths[r].size());
    }
    if (!upload || n == 0) return HKV_OK;
    std::vector<int32_t> bt((size_t)n * pl.max_pages, 0), req(n);
    for (int r = 0; r < n; ++r) {
        std::copy(paths[r].begin(), paths[r].end(), bt.begin() + (size_t)r * pl.max_pages);
        req[r] = r;
    }
    const size_t b_bt = align_up(sizeof(int32_t) * bt.size(), 256), b_n = align_up(sizeof(int32_t) * n, 256);
    HKV_HIP(hipMalloc((void **)&pl.d_bt, b_bt + 2 * b_n));
    pl.d_rows_req = reinterpret_cast<int32_t *>(reinterpret_cast<char *>(pl.d_bt) + b_bt);
    pl.d_rows_len = reinterpret_cast<int32_t *>(reinterpret_cast<char *>(pl.d_bt) + b_bt + b_n);
    HKV_HIP(hipMemcpy(pl.d_bt, bt.data(), sizeof(int32_t) * bt.size(), hipMemcpyHostToDevice));
    HKV_HIP(hipMemcpy(pl.d_rows_req, req.data(), sizeof(int32_t) * n, hipMemcpyHostToDevice));
    HKV_HIP(hipMemcpy(pl.d_rows_len, pl.row_len.data(), sizeof(int32_t) * n, hipMemcpyHostToDevice));
    return HKV_OK;
}

// internal flag: no item may go to the 256-row tile kernel (plans with per-row visibility)
constexpr uint32_t kPlanNoTiles = 0x40000000u;

// the planner's settings, each 0 (the library's choice) or inside its documented range
static int check_plan_settings(const hkv_decode_plan_params *o) {
    if (!o) return HKV_OK;
    auto bad = [](const char *name, int32_t v) { return fail(HKV_EINVAL, "hkv_decode_plan_create_ex: %s = %d is out of range", name, v); };
    if (o->leaf_chunk < 0 || o->leaf_chunk % 16) return bad("leaf_chunk", o->leaf_chunk);
    if (o->shared_chunk < 0 || o->shared_chunk % 16 || o->shared_chunk > kMaxSharedItemTokens) return bad("shared_chunk", o->shared_chunk);
    if (o->max_rows != 0 && (o->max_rows < 16 || o->max_rows > 64)) return bad("max_rows", o->max_rows);
    if (o->pack < 0 || o->pack > 3) return bad("pack", o->pack);
    if (o->pack_tokens < 0) return bad("pack_tokens", o->pack_tokens);
    if (o->stages != 0 && (o->stages < 3 || o->stages > 5)) return bad("stages", o->stages);
    if (o->interleave < -1) return bad("interleave", o->interleave);
    if (o->tile_min_rows != 0 && o->tile_min_rows < kMinTileItemRows) return bad("tile_min_rows", o->tile_min_rows);
    if (o->tile_min_gflop < -1) return bad("tile_min_gflop", o->tile_min_gflop);
    if (o->tile_workgroups < 0) return bad("tile_workgroups", o->tile_workgroups);
    if (o->tile_chunk < 0 || o->tile_chunk % 16 || o->tile_chunk > kMaxTileItemTokens) return bad("tile_chunk", o->tile_chunk);
    if (o->large_batch_updates < 0 || o->large_batch_updates > 1) return bad("large_batch_updates", o->large_batch_updates);
    if (o->fused < -1 || o->fused > 0) return bad("fused", o->fused);
    return HKV_OK;
}

static int create_decode_plan(hkv_pool *pool, const hkv_node *nodes, int32_t n_nodes, const int32_t *node_pages,
                              int32_t n_node_pages, const int32_t *req_leaf, int32_t n_req, int32_t num_q_heads,
                              uint32_t flags, int32_t reserve_tokens, const hkv_decode_plan_params *opt,
                              hkv_decode_plan **out) {
    if (!pool || !out) return fail(HKV_EINVAL, "hkv_decode_plan_create: null argument");
    *out = nullptr;
    if (int rc = check_plan_settings(opt)) return rc;
    const int Hkv = pool->d.num_kv_heads;
    if (num_q_heads <= 0 || num_q_heads % Hkv || num_q_heads / Hkv > 16)
        return fail(HKV_ESHAPE, "hkv_decode_plan_create: %d query heads over %d KV heads", num_q_heads, Hkv);
    if ((flags & HKV_PLAN_FP8_MATRIX) && pool->d.dtype != HKV_FP8_E4M3)
        return fail(HKV_ESHAPE, "hkv_decode_plan_create: HKV_PLAN_FP8_MATRIX needs an fp8 pool");
    // The per-node kernels read every node through its own page list, so nodes may end inside a page
    // anywhere; the full-precision path walks flat block tables and keeps the whole-page rule.
    if (int rc = validate_forest(nodes, n_nodes, node_pages, n_node_pages, "hkv_decode_plan_create",
                                 pool->d.dtype == HKV_FP32, pool->d.page_size))
        return rc;
    for (int v = 0; v < n_nodes; ++v)
        for (int j = 0; j < nodes[v].n_pages; ++j) {
            int32_t id = node_pages[nodes[v].page_begin + j];
            if (id < 0 || id >= pool->d.num_pages)
                return fail(HKV_ERANGE, "hkv_decode_plan_create: node %d page %d has id %d outside pool of %d", v, j,
                            id, pool->d.num_pages);
        }
    hkv_decode_plan *pl = new (std::nothrow) hkv_decode_plan;
    if (!pl) return fail(HKV_ENOMEM, "hkv_decode_plan_create: out of host memory");
    pl->pool = pool;
    pl->n_req = n_req;
    pl->num_q_heads = num_q_heads;
    pl->group = num_q_heads / Hkv;
    pl->fp8_matrix = pool->d.dtype == HKV_FP8_E4M3 && (flags & HKV_PLAN_FP8_MATRIX);
    if (opt) pl->opt = *opt;
    if (opt && opt->q_rows) {
        if (pool->d.dtype == HKV_FP32) {
            delete pl;
            return fail(HKV_ESHAPE, "hkv_decode_plan_create_ex: q_rows with an fp32 pool");
        }
        pl->q_rows.assign(opt->q_rows, opt->q_rows + n_req);
        std::vector<int32_t> sorted(pl->q_rows);
        std::sort(sorted.begin(), sorted.end());
        if (!sorted.empty() && (sorted.front() < 0 || std::adjacent_find(sorted.begin(), sorted.end()) != sorted.end())) {
            delete pl;
            return fail(HKV_EINVAL, "hkv_decode_plan_create_ex: q_rows must be non-negative and all different");
        }
        pl->opt.q_rows = nullptr;  // the caller's array is not kept
    }
    pl->opt.visible = nullptr;
    pl->no_tiles = (flags & kPlanNoTiles) != 0;
    pl->concurrent = !(flags & HKV_PLAN_ONE_STREAM);
    if (int rc = build_node_req_csr(nodes, n_nodes, req_leaf, n_req, pl->node_req_indptr, pl->node_req_idx,
                                    "hkv_decode_plan_create")) {
        delete pl;
        return rc;
    }
    pl->key_nodes.assign(nodes, nodes + n_nodes);
    pl->key_pages.assign(node_pages, node_pages + n_node_pages);
    pl->req_leaf.assign(req_leaf, req_leaf + n_req);
    // the plan itself works on 16-token blocks: block j of page p is block p * S + j of the buffers
    pl->nodes.assign(nodes, nodes + n_nodes);
    pl->node_pages.clear();
    const int S = pool->blocks_per_page;
    pl->node_pages.reserve((size_t)n_node_pages * S + (reserve_tokens > 0 ? (size_t)n_req * (reserve_tokens / HKV_PAGE_SIZE + 2) : 0));
    std::vector<char> grows(n_nodes, 0);
    if (reserve_tokens > 0)
        for (int r = 0; r < n_req; ++r) grows[req_leaf[r]] = 1;
    pl->reserve_tokens = reserve_tokens;
    for (int v = 0; v < n_nodes; ++v) {
        hkv_node &nd = pl->nodes[v];
        const int n_blocks = (nd.n_tokens + HKV_PAGE_SIZE - 1) / HKV_PAGE_SIZE;
        const int first = (int)pl->node_pages.size();
        for (int b = 0; b < n_blocks; ++b) pl->node_pages.push_back(node_pages[nodes[v].page_begin + b / S] * S + b % S);
        if (grows[v]) {  // slots for the blocks the leaf may grow into; until then they repeat its last block (in bounds)
            const int cap = (nd.n_tokens + reserve_tokens + HKV_PAGE_SIZE - 1) / HKV_PAGE_SIZE;
            for (int b = n_blocks; b < cap; ++b) pl->node_pages.push_back(pl->node_pages.back());
        }
        nd.page_begin = first;
        nd.n_pages = n_blocks;
    }
    if (pool->d.dtype == HKV_FP32) {  // full-precision path: no work items, no partials
        if (int rc = build_fp32_rows(*pl, !(flags & HKV_PLAN_HOST_ONLY))) {
            if (pl->d_bt) (void)hipFree(pl->d_bt);
            delete pl;
            return rc;
        }
        pl->part_count.assign(n_req, 0);
        *out = pl;
        return HKV_OK;
    }
    plan_items(*pl);
    if (reserve_tokens > 0) {  // the items that grow with each request: the leaf's last chunk, one per KV head
        pl->grow_items.assign((size_t)n_req * Hkv, -1);
        for (int r = 0; r < n_req; ++r) {
            const int v = req_leaf[r];
            int last_begin = -1;
            for (const DecodeItem &it : pl->items)
                if (it.node == v) last_begin = std::max(last_begin, it.tok_begin);
            for (size_t i = 0; i < pl->items.size(); ++i)
                if (pl->items[i].node == v && pl->items[i].tok_begin == last_begin)
                    pl->grow_items[(size_t)r * Hkv + pl->items[i].kv_head] = (int32_t)i;
        }
        for (int32_t gi : pl->grow_items)
            if (gi < 0) {
                delete pl;
                return fail(HKV_EINVAL, "hkv_decode_plan_create_growing: a leaf without work items");
            }
        pl->key_nodes.clear();  // never the pool's cached one-shot plan
        pl->key_pages.clear();
    }
    if (!(flags & HKV_PLAN_HOST_ONLY)) {
        if (int rc = upload_decode_plan(*pl)) {
            hkv_decode_plan_destroy(pl);
            return rc;
        }
    }
    *out = pl;
    return HKV_OK;
}

extern "C" int hkv_decode_plan_create(hkv_pool *pool, const hkv_node *nodes, int32_t n_nodes,
                                      const int32_t *node_pages, int32_t n_node_pages, const int32_t *req_leaf,
                                      int32_t n_req, int32_t num_q_heads, uint32_t flags, hkv_decode_plan **out) {
    return create_decode_plan(pool, nodes, n_nodes, node_pages, n_node_pages, req_leaf, n_req, num_q_heads,
                              flags & ~kPlanNoTiles, 0, nullptr, out);
}

static int create_growing_plan(hkv_pool *pool, const hkv_node *nodes, int32_t n_nodes, const int32_t *node_pages,
                               int32_t n_node_pages, const int32_t *req_leaf, int32_t n_req, int32_t num_q_heads,
                               int32_t reserve_tokens, uint32_t flags, const hkv_decode_plan_params *opt,
                               hkv_decode_plan **out) {
    if (!pool || !out) return fail(HKV_EINVAL, "hkv_decode_plan_create_growing: null argument");
    *out = nullptr;
    if (pool->d.dtype == HKV_FP32) return fail(HKV_ESHAPE, "hkv_decode_plan_create_growing: bf16 and fp8 pools only");
    if (reserve_tokens < 1 || reserve_tokens > (1 << 20))
        return fail(HKV_EINVAL, "hkv_decode_plan_create_growing: reserve_tokens %d", reserve_tokens);
    if (n_nodes < 0 || n_req < 0 || (n_nodes > 0 && !nodes) || (n_req > 0 && !req_leaf))
        return fail(HKV_EINVAL, "hkv_decode_plan_create_growing: bad forest arguments");
    // every request needs a leaf of its own to grow: no other request on it, no children, at least one token
    std::vector<int32_t> users(n_nodes, 0);
    for (int r = 0; r < n_req; ++r) {
        if (req_leaf[r] < 0 || req_leaf[r] >= n_nodes)
            return fail(HKV_ERANGE, "hkv_decode_plan_create_growing: request %d names node %d of %d", r, req_leaf[r], n_nodes);
        ++users[req_leaf[r]];
    }
    for (int v = 0; v < n_nodes; ++v)
        if (nodes[v].parent >= 0 && nodes[v].parent < n_nodes && users[nodes[v].parent])
            return fail(HKV_ETREE, "hkv_decode_plan_create_growing: node %d, the leaf of a request, has children", nodes[v].parent);
    for (int r = 0; r < n_req; ++r) {
        if (users[req_leaf[r]] != 1)
            return fail(HKV_ETREE, "hkv_decode_plan_create_growing: node %d is the leaf of %d requests", req_leaf[r], users[req_leaf[r]]);
        if (nodes[req_leaf[r]].n_tokens < 1)
            return fail(HKV_ETREE, "hkv_decode_plan_create_growing: the leaf of request %d holds no token", r);
    }
    return create_decode_plan(pool, nodes, n_nodes, node_pages, n_node_pages, req_leaf, n_req, num_q_heads,
                              flags & ~kPlanNoTiles, reserve_tokens, opt, out);
}

extern "C" int hkv_decode_plan_create_growing(hkv_pool *pool, const hkv_node *nodes, int32_t n_nodes,
                                              const int32_t *node_pages, int32_t n_node_pages,
                                              const int32_t *req_leaf, int32_t n_req, int32_t num_q_heads,
                                              int32_t reserve_tokens, uint32_t flags, hkv_decode_plan **out) {
    return create_growing_plan(pool, nodes, n_nodes, node_pages, n_node_pages, req_leaf, n_req, num_q_heads,
                               reserve_tokens, flags, nullptr, out);
}

// k_src / v_src: null (the caller stores the tokens itself), or the new token of every request, stored here
// at the end of its leaf, in the same launch as the plan's update where that runs as a kernel.
static int plan_append(hkv_decode_plan *plan, const int32_t *new_page_ids, const void *k_src, const void *v_src,
                       void *stream) {
    if (!plan) return fail(HKV_EINVAL, "hkv_decode_plan_append: null plan");
    if (plan->reserve_tokens <= 0) return fail(HKV_EINVAL, "hkv_decode_plan_append: not a growing plan");
    if (plan->appended >= plan->reserve_tokens)
        return fail(HKV_ENOMEM, "hkv_decode_plan_append: the %d reserved tokens are used up", plan->reserve_tokens);
    hkv_pool *pool = plan->pool;
    const int P = pool->d.page_size, S = pool->blocks_per_page, Hkv = pool->d.num_kv_heads;
    // check everything before anything changes
    for (int r = 0; r < plan->n_req; ++r) {
        const hkv_node &nd = plan->nodes[plan->req_leaf[r]];
        if (nd.n_tokens % P) continue;  // the new token goes into the leaf's last page
        if (!new_page_ids) return fail(HKV_EINVAL, "hkv_decode_plan_append: request %d needs a new page, none given", r);
        if (new_page_ids[r] < 0 || new_page_ids[r] >= pool->d.num_pages)
            return fail(HKV_ERANGE, "hkv_decode_plan_append: page id %d for request %d outside pool of %d pages",
                        new_page_ids[r], r, pool->d.num_pages);
    }
    const bool with_tokens = k_src != nullptr;
    if (with_tokens && (!v_src || ((reinterpret_cast<uintptr_t>(k_src) | reinterpret_cast<uintptr_t>(v_src)) & 15)))
        return fail(HKV_EINVAL, "hkv_decode_plan_append_tokens: k_src and v_src must be non-null and 16-byte aligned");
    const bool inline_update = plan->dev && plan->d_grow_items;
    PlanGrowInline g{};
    PoolAppendInline w{};
    std::vector<int32_t> w_page, w_slot;  // the tokens' places, for the path of larger batches
    if (with_tokens && !inline_update) {
        w_page.resize(plan->n_req);
        w_slot.resize(plan->n_req);
    }
    for (int r = 0; r < plan->n_req; ++r) {
        hkv_node &nd = plan->nodes[plan->req_leaf[r]];
        if (inline_update) g.new_block[r] = -1;
        if (with_tokens) {  // where the new token goes: slot n_tokens % P of the leaf's last (or new) page
            const int32_t page = nd.n_tokens % P == 0 ? new_page_ids[r] : plan->node_pages[nd.page_begin + nd.n_pages - 1] / S;
            if (inline_update) {
                w.block[r] = page * S + (nd.n_tokens % P) / HKV_PAGE_SIZE;
                w.slot[r] = (uint8_t)(nd.n_tokens % HKV_PAGE_SIZE);
            } else {
                w_page[r] = page;
                w_slot[r] = nd.n_tokens % P;
            }
        }
        if (nd.n_tokens % HKV_PAGE_SIZE == 0) {  // a new 16-token block: of a new page, or the next one of the last page
            const int32_t block = nd.n_tokens % P == 0 ? new_page_ids[r] * S
                                                      : plan->node_pages[nd.page_begin + nd.n_pages - 1] + 1;
            plan->node_pages[nd.page_begin + nd.n_pages] = block;
            if (inline_update) {
                g.new_block[r] = block;
                g.block_pos[r] = nd.page_begin + nd.n_pages;
            }
            ++nd.n_pages;
        }
        ++nd.n_tokens;
        for (int h = 0; h < Hkv; ++h) ++plan->items[plan->grow_items[(size_t)r * Hkv + h]].n_tokens;
    }
    ++plan->appended;
    if (!plan->dev) return HKV_OK;  // host-only plan
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (inline_update) {  // the usual batch: the change travels in the arguments of a small kernel
        g.items = plan->d_items;
        g.pages = plan->d_pages;
        g.grow_items = plan->d_grow_items;
        g.n_grow = (int32_t)plan->grow_items.size();
        g.n_req = plan->n_req;
        if (with_tokens) {  // the same launch stores the tokens
            w.base = PoolWriteLaunch{pool->d.k_pages, pool->d.v_pages, pool->d.k_scale, pool->d.v_scale, Hkv, pool->d.dtype,
                                     nullptr, plan->n_req, 0, plan->n_req, k_src, v_src, nullptr};
            HKV_HIP(launch_decode_step_append(w, g, s));
        } else {
            HKV_HIP(launch_plan_grow_inline(g, s));
        }
        return HKV_OK;
    }
    if (with_tokens)
        if (int rc = kv_pool_append(pool, w_page.data(), w_slot.data(), plan->n_req, k_src, v_src, stream)) return rc;
    const int slot = plan->grow_next;
    plan->grow_next = (slot + 1) % hkv_decode_plan::kGrowSlots;
    if (plan->grow_in_flight[slot]) HKV_HIP(hipEventSynchronize(plan->grow_free[slot]));  // its last copy is done
    char *h = plan->h_grow + (size_t)slot * plan->grow_bytes;
    const size_t off_pages = reinterpret_cast<char *>(plan->d_pages) - static_cast<char *>(plan->dev);
    memcpy(h, plan->items.data(), sizeof(DecodeItem) * plan->items.size());
    memcpy(h + off_pages, plan->node_pages.data(), sizeof(int32_t) * plan->node_pages.size());
    // a copy kernel on the stream reads the pinned buffer (a DMA copy between two kernels of one stream
    // costs far more than it moves here)
    HKV_HIP(launch_upload(plan->d_grow + (size_t)slot * plan->grow_bytes, plan->dev, plan->grow_bytes, s));
    HKV_HIP(hipEventRecord(plan->grow_free[slot], s));
    plan->grow_in_flight[slot] = true;
    return HKV_OK;
}

extern "C" int hkv_decode_plan_append(hkv_decode_plan *plan, const int32_t *new_page_ids, void *stream) {
    return plan_append(plan, new_page_ids, nullptr, nullptr, stream);
}

extern "C" int hkv_decode_plan_append_tokens(hkv_decode_plan *plan, const int32_t *new_page_ids, const void *k_src,
                                             const void *v_src, void *stream) {
    if (!k_src || !v_src) return fail(HKV_EINVAL, "hkv_decode_plan_append_tokens: null k_src / v_src");
    return plan_append(plan, new_page_ids, k_src, v_src, stream);
}

// Plan over n_req * T query rows: the T newest tokens of every request (the last T of its leaf node) are
// queried together; row t sees everything before them and, of them, token j iff bit j of masks[r * T + t]
// is set (masks == nullptr: the causal run, bits 0..t).
static int create_rows_plan(hkv_pool *pool, const hkv_node *nodes, int32_t n_nodes, const int32_t *node_pages,
                            int32_t n_node_pages, const int32_t *req_leaf, int32_t n_req, int32_t T,
                            const uint64_t *masks, int32_t num_q_heads, uint32_t flags,
                            const hkv_decode_plan_params *opt, hkv_decode_plan **out, const char *who) {
    if (n_req < 0 || (n_req > 0 && !req_leaf)) return fail(HKV_EINVAL, "%s: bad request list", who);
    if ((int64_t)n_req * T > INT32_MAX / 2) return fail(HKV_EINVAL, "%s: too many query rows", who);
    if (masks && pool && pool->d.dtype == HKV_FP32)
        return fail(HKV_ESHAPE, "%s: the full-precision path verifies causal runs only", who);
    std::vector<int32_t> rows((size_t)n_req * T);
    for (int r = 0; r < n_req; ++r)
        for (int t = 0; t < T; ++t) rows[(size_t)r * T + t] = req_leaf[r];
    hkv_decode_plan *pl = nullptr;
    const uint32_t rows_flags = (flags & ~kPlanNoTiles) | ((T > 1 || masks) ? kPlanNoTiles : 0u);
    if (int rc = create_decode_plan(pool, nodes, n_nodes, node_pages, n_node_pages, rows.data(), n_req * T, num_q_heads,
                                    rows_flags, 0, opt, &pl))
        return rc;
    pl->tokens_per_req = T;
    if (T > 1 || masks) {
        std::vector<int32_t> lim((size_t)n_req * T);
        std::vector<unsigned long long> vis((size_t)n_req * T);
        for (int r = 0; r < n_req; ++r) {
            const int n_leaf = nodes[req_leaf[r]].n_tokens;  // validated by hkv_decode_plan_create
            if (n_leaf < T) {
                hkv_decode_plan_destroy(pl);
                return fail(HKV_EINVAL, "%s: request %d has %d query tokens but its leaf holds only %d tokens (the "
                            "newest tokens must lie in the leaf)", who, r, T, n_leaf);
            }
            for (int t = 0; t < T; ++t) {
                const size_t i = (size_t)r * T + t;
                lim[i] = n_leaf - T;
                vis[i] = masks ? masks[i] : (t == 63 ? ~0ull : (1ull << (t + 1)) - 1);
                if (!(vis[i] >> t & 1) || (T < 64 && vis[i] >> T)) {
                    hkv_decode_plan_destroy(pl);
                    return fail(HKV_EINVAL, "%s: request %d token %d: a token must see itself and nothing beyond the %d "
                                "newest tokens (mask %llx)", who, r, t, T, vis[i]);
                }
            }
        }
        if (pool->d.dtype == HKV_FP32) {  // query token t of a request sees all but the T-1-t newest keys
            for (int r = 0; r < n_req; ++r)
                for (int t = 0; t < T; ++t) pl->row_len[(size_t)r * T + t] -= T - 1 - t;
            if (pl->d_rows_len) {
                hipError_t e = hipMemcpy(pl->d_rows_len, pl->row_len.data(), sizeof(int32_t) * pl->row_len.size(), hipMemcpyHostToDevice);
                if (e != hipSuccess) {
                    hkv_decode_plan_destroy(pl);
                    return fail_hip(e, who);
                }
            }
        } else if (pl->dev && n_req > 0) {
            const size_t n = rows.size();
            hipError_t e = hipMalloc((void **)&pl->d_row_mask, n * (sizeof(unsigned long long) + 2 * sizeof(int32_t)));
            if (e == hipSuccess) {
                pl->d_row_leaf = reinterpret_cast<int32_t *>(pl->d_row_mask + n);
                pl->d_row_limit = pl->d_row_leaf + n;
                e = hipMemcpy(pl->d_row_mask, vis.data(), n * sizeof(unsigned long long), hipMemcpyHostToDevice);
            }
            if (e == hipSuccess) e = hipMemcpy(pl->d_row_leaf, rows.data(), n * sizeof(int32_t), hipMemcpyHostToDevice);
            if (e == hipSuccess) e = hipMemcpy(pl->d_row_limit, lim.data(), n * sizeof(int32_t), hipMemcpyHostToDevice);
            if (e != hipSuccess) {
                hkv_decode_plan_destroy(pl);
                return fail_hip(e, who);
            }
        }
    }
    *out = pl;
    return HKV_OK;
}

extern "C" int hkv_decode_plan_create_multi(hkv_pool *pool, const hkv_node *nodes, int32_t n_nodes,
                                            const int32_t *node_pages, int32_t n_node_pages, const int32_t *req_leaf,
                                            int32_t n_req, int32_t tokens_per_req, int32_t num_q_heads, uint32_t flags,
                                            hkv_decode_plan **out) {
    if (!out) return fail(HKV_EINVAL, "hkv_decode_plan_create_multi: null out");
    *out = nullptr;
    if (tokens_per_req < 1 || tokens_per_req > 16)
        return fail(HKV_EINVAL, "hkv_decode_plan_create_multi: %d query tokens per request (1..16)", tokens_per_req);
    return create_rows_plan(pool, nodes, n_nodes, node_pages, n_node_pages, req_leaf, n_req, tokens_per_req, nullptr,
                            num_q_heads, flags, nullptr, out, "hkv_decode_plan_create_multi");
}

extern "C" int hkv_decode_plan_create_tree(hkv_pool *pool, const hkv_node *nodes, int32_t n_nodes,
                                           const int32_t *node_pages, int32_t n_node_pages, const int32_t *req_leaf,
                                           int32_t n_req, int32_t tokens_per_req, const uint64_t *visible,
                                           int32_t num_q_heads, uint32_t flags, hkv_decode_plan **out) {
    if (!out) return fail(HKV_EINVAL, "hkv_decode_plan_create_tree: null out");
    *out = nullptr;
    if (tokens_per_req < 1 || tokens_per_req > 64)
        return fail(HKV_EINVAL, "hkv_decode_plan_create_tree: %d drafted tokens per request (1..64)", tokens_per_req);
    if (n_req > 0 && !visible) return fail(HKV_EINVAL, "hkv_decode_plan_create_tree: null visibility masks");
    return create_rows_plan(pool, nodes, n_nodes, node_pages, n_node_pages, req_leaf, n_req, tokens_per_req, visible,
                            num_q_heads, flags, nullptr, out, "hkv_decode_plan_create_tree");
}

extern "C" int hkv_decode_plan_create_ex(hkv_pool *pool, const hkv_node *nodes, int32_t n_nodes,
                                         const int32_t *node_pages, int32_t n_node_pages, const int32_t *req_leaf,
                                         int32_t n_req, int32_t num_q_heads, uint32_t flags,
                                         const hkv_decode_plan_params *params, hkv_decode_plan **out) {
    if (!out) return fail(HKV_EINVAL, "hkv_decode_plan_create_ex: null out");
    *out = nullptr;
    const int32_t T = params && params->tokens_per_req ? params->tokens_per_req : 1;
    const uint64_t *visible = params ? params->visible : nullptr;
    const int32_t reserve = params ? params->reserve_tokens : 0;
    if (T < 1 || T > 64 || (T > 16 && !visible))
        return fail(HKV_EINVAL, "hkv_decode_plan_create_ex: %d query tokens per request (1..16, up to 64 with visibility masks)", T);
    if (reserve < 0) return fail(HKV_EINVAL, "hkv_decode_plan_create_ex: reserve_tokens %d", reserve);
    if (reserve > 0 && (T > 1 || visible))
        return fail(HKV_EINVAL, "hkv_decode_plan_create_ex: a growing plan has one query token per request");
    if (T > 1 || visible)
        return create_rows_plan(pool, nodes, n_nodes, node_pages, n_node_pages, req_leaf, n_req, T, visible, num_q_heads,
                                flags, params, out, "hkv_decode_plan_create_ex");
    if (reserve > 0)
        return create_growing_plan(pool, nodes, n_nodes, node_pages, n_node_pages, req_leaf, n_req, num_q_heads, reserve,
                                   flags, params, out);
    return create_decode_plan(pool, nodes, n_nodes, node_pages, n_node_pages, req_leaf, n_req, num_q_heads,
                              flags & ~kPlanNoTiles, 0, params, out);
}

extern "C" int hkv_decode_plan_destroy(hkv_decode_plan *plan) {
    if (!plan) return HKV_OK;
    if (plan->dev) (void)hipFree(plan->dev);  // hipFree waits for work that may still read it
    if (plan->d_row_mask) (void)hipFree(plan->d_row_mask);
    if (plan->d_bt) (void)hipFree(plan->d_bt);
    for (hipEvent_t e : plan->ev)
        if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : {plan->ev_fork, plan->ev_join, plan->ev_tile[0], plan->ev_tile[1]})
        if (e) (void)hipEventDestroy(e);
    if (plan->side) (void)hipStreamDestroy(plan->side);
    if (plan->h_grow) (void)hipHostFree(plan->h_grow);
    if (plan->d_grow_items) (void)hipFree(plan->d_grow_items);
    for (hipEvent_t e : plan->grow_free)
        if (e) (void)hipEventDestroy(e);
    delete plan;
    return HKV_OK;
}

extern "C" size_t hkv_decode_plan_workspace_bytes(const hkv_decode_plan *plan) {
    if (!plan || plan->pool->d.dtype == HKV_FP32) return 0;
    return align_up((size_t)plan->n_parts * HKV_HEAD_DIM * sizeof(uint16_t), 256) +
           2 * align_up((size_t)plan->n_parts * sizeof(float), 256);
}

extern "C" int32_t hkv_decode_plan_num_items(const hkv_decode_plan *plan) {
    return plan ? (int32_t)(plan->items.size() + plan->tile_items.size()) : fail(HKV_EINVAL, "null plan");
}
extern "C" int32_t hkv_decode_plan_num_tile_items(const hkv_decode_plan *plan) {
    return plan ? (int32_t)plan->tile_items.size() : fail(HKV_EINVAL, "null plan");
}
extern "C" int32_t hkv_decode_plan_is_fused(const hkv_decode_plan *plan) {
    return plan ? (plan->fused ? 1 : 0) : fail(HKV_EINVAL, "null plan");
}
extern "C" int32_t hkv_decode_plan_tile_workgroups(const hkv_decode_plan *plan) {
    return plan ? plan->tile_workgroups : fail(HKV_EINVAL, "null plan");
}
extern "C" int32_t hkv_decode_plan_num_parts(const hkv_decode_plan *plan) {
    return plan ? plan->n_parts : fail(HKV_EINVAL, "null plan");
}
extern "C" int hkv_decode_plan_items(const hkv_decode_plan *plan, int32_t *items_out) {
    if (!plan || !items_out) return fail(HKV_EINVAL, "hkv_decode_plan_items: null argument");
    static_assert(sizeof(DecodeItem) == 32, "item layout is part of the introspection contract");
    if (!plan->items.empty()) memcpy(items_out, plan->items.data(), sizeof(DecodeItem) * plan->items.size());
    if (!plan->tile_items.empty())
        memcpy(items_out + 8 * plan->items.size(), plan->tile_items.data(), sizeof(DecodeItem) * plan->tile_items.size());
    return HKV_OK;
}
extern "C" int32_t hkv_decode_plan_num_workgroups(const hkv_decode_plan *plan) {
    if (!plan) return fail(HKV_EINVAL, "null plan");
    return plan->n_single + ((int32_t)plan->items.size() - plan->n_single + 3) / 4;  // (the tile kernel's are counted apart)
}
extern "C" int32_t hkv_decode_plan_max_parts(const hkv_decode_plan *plan) {
    return plan ? plan->max_parts : fail(HKV_EINVAL, "null plan");
}
extern "C" int hkv_decode_plan_part_counts(const hkv_decode_plan *plan, int32_t *part_count) {
    if (!plan || (plan->n_req > 0 && !part_count)) return fail(HKV_EINVAL, "hkv_decode_plan_part_counts: null argument");
    if (plan->n_req) memcpy(part_count, plan->part_count.data(), sizeof(int32_t) * plan->n_req);
    return HKV_OK;
}

// The common part of the two run calls; arguments are checked by the callers.  workspace holds at least
// hkv_decode_plan_workspace_bytes(plan) bytes (unused for fp32 pools).
static int run_decode_plan(hkv_decode_plan *plan, const void *q, float scale, void *out, float *lse_out,
                           void *workspace, void *stream) {
    if (plan->pool->d.dtype == HKV_FP32) {
        RowsLaunch a{view_of(plan->pool), static_cast<const float *>(q), plan->d_bt, plan->d_rows_req, plan->d_rows_len,
                     static_cast<float *>(out), lse_out, plan->n_req, plan->num_q_heads, plan->max_pages, scale};
        HKV_HIP(launch_rows_fp32(a, static_cast<hipStream_t>(stream)));
        return HKV_OK;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    // per partial: o as fp16 times a power of two, lse, and the reciprocal of that power
    uint16_t *o_parts = static_cast<uint16_t *>(workspace);
    float *lse_parts = reinterpret_cast<float *>(static_cast<char *>(workspace) +
                                                 align_up((size_t)plan->n_parts * HKV_HEAD_DIM * sizeof(uint16_t), 256));
    float *down_parts = lse_parts + align_up((size_t)plan->n_parts * sizeof(float), 256) / sizeof(float);
    const bool prof = plan->profiling;
    const bool tiles = !plan->tile_items.empty();
    const bool fork = tiles && plan->concurrent && !plan->items.empty() && !plan->fused;
    // The tile kernel goes first and stays on the caller's stream, so that its persistent workgroups, which need
    // a whole compute unit each, take theirs before the other kernel's many small workgroups fill the chip; that
    // kernel follows on the plan's own stream (behind an event that marks the same point of the caller's stream)
    // and is joined again before the merge.
    if (fork) {
        HKV_HIP(hipEventRecord(plan->ev_fork, s));
        HKV_HIP(hipStreamWaitEvent(plan->side, plan->ev_fork, 0));
    }
    const DecodeTilesLaunch t{view_of(plan->pool), q, plan->d_tile_items, plan->d_pages, plan->d_node_req_idx, o_parts, lse_parts,
                              down_parts, (int32_t)plan->tile_items.size(), plan->num_q_heads, plan->max_parts, scale,
                              plan->tile_workgroups, plan->d_q_rows};
    const DecodeLaunch a{view_of(plan->pool), q, plan->d_items, plan->d_pages, plan->d_node_req_idx, o_parts, lse_parts,
                         down_parts, (int32_t)plan->items.size(), plan->num_q_heads, plan->max_parts, scale,
                         plan->d_row_leaf, plan->d_row_limit, plan->d_row_mask, plan->n_single, plan->n_stages,
                         plan->fp8_matrix ? 1 : 0, plan->d_q_rows};
    if (plan->fused) {
        HKV_HIP(launch_decode_fused(a, t, s, prof ? plan->ev[0] : nullptr, prof ? plan->ev[1] : nullptr));
    } else if (tiles) {
        HKV_HIP(launch_decode_tiles(t, s, prof ? plan->ev_tile[0] : nullptr, prof ? plan->ev_tile[1] : nullptr));
    }
    if (!plan->items.empty() && !plan->fused) {
        hipStream_t rs = fork ? plan->side : s;
        HKV_HIP(launch_decode(a, rs, prof ? plan->ev[0] : nullptr, prof ? plan->ev[1] : nullptr));
        if (fork) {
            HKV_HIP(hipEventRecord(plan->ev_join, plan->side));
            HKV_HIP(hipStreamWaitEvent(s, plan->ev_join, 0));
        }
    }
    HKV_HIP(launch_lse_merge_dense(o_parts, lse_parts, plan->d_part_count, plan->num_q_heads, plan->max_parts,
                                   plan->n_req * plan->num_q_heads, out, HKV_BF16, lse_out, s,
                                   prof ? plan->ev[2] : nullptr, prof ? plan->ev[3] : nullptr, plan->d_q_rows, down_parts));
    if (prof) plan->profiled_run = !plan->items.empty() || tiles;
    return HKV_OK;
}

static int check_decode_run(const hkv_decode_plan *plan, const void *q, const void *out, const char *who) {
    if (!q || !out) return fail(HKV_EINVAL, "%s: null q or out", who);
    if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(out)) & 15)
        return fail(HKV_EINVAL, "%s: q and out must be 16-byte aligned", who);
    if (plan->pool->d.dtype == HKV_FP32 ? !plan->d_bt : !plan->dev)
        return fail(HKV_EINVAL, "%s: plan was built host-only", who);
    return HKV_OK;
}

extern "C" int attn_decode_plan_run(hkv_decode_plan *plan, const void *q, float scale, void *out, float *lse_out,
                                    void *workspace, size_t workspace_bytes, void *stream) {
    if (!plan) return fail(HKV_EINVAL, "attn_decode_plan_run: null plan");
    if (plan->n_req == 0) return HKV_OK;
    if (int rc = check_decode_run(plan, q, out, "attn_decode_plan_run")) return rc;
    const size_t need = hkv_decode_plan_workspace_bytes(plan);
    if (need && (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255)))
        return fail(HKV_EINVAL, "attn_decode_plan_run: workspace must be non-null and 256-byte aligned");
    if (workspace_bytes < need)
        return fail(HKV_ENOMEM, "attn_decode_plan_run: workspace has %zu bytes, %zu needed", workspace_bytes, need);
    return run_decode_plan(plan, q, scale, out, lse_out, workspace, stream);
}

extern "C" size_t hkv_static_workspace_bytes(void) { return kStaticWorkspaceBytes; }

extern "C" int attn_decode_plan_run_static(hkv_decode_plan *plan, const void *q, float scale, void *out,
                                           float *lse_out, void *stream) {
    if (!plan) return fail(HKV_EINVAL, "attn_decode_plan_run_static: null plan");
    if (plan->n_req == 0) return HKV_OK;
    if (int rc = check_decode_run(plan, q, out, "attn_decode_plan_run_static")) return rc;
    const size_t need = hkv_decode_plan_workspace_bytes(plan);
    if (need > kStaticWorkspaceBytes)
        return fail(HKV_ENOMEM, "attn_decode_plan_run_static: the plan needs %zu bytes of workspace, the static "
                    "workspace holds %zu (use attn_decode_plan_run with a workspace of the caller's)", need,
                    (size_t)kStaticWorkspaceBytes);
    void *ws = nullptr;  // this device's copy of the static array (looked up when the plan was created)
    HKV_HIP(prepare_decode_device(&ws));
    return run_decode_plan(plan, q, scale, out, lse_out, ws, stream);
}

extern "C" int hkv_decode_plan_set_profiling(hkv_decode_plan *plan, int32_t mode) {
    if (!plan) return fail(HKV_EINVAL, "hkv_decode_plan_set_profiling: null plan");
    if (mode < 0 || mode > 1) return fail(HKV_EINVAL, "hkv_decode_plan_set_profiling: mode %d", mode);
    if (mode == 1 && !plan->ev[0]) {
        for (hipEvent_t &e : plan->ev) HKV_HIP(hipEventCreate(&e));
        for (hipEvent_t &e : plan->ev_tile) HKV_HIP(hipEventCreate(&e));
    }
    plan->profiling = mode == 1;
    return HKV_OK;
}

// GPU time of the node phase of the most recent profiled run: from the earlier begin to the later end of the
// kernel over `items` and the tile kernel (either may be absent), and each of the two on its own.
static int node_phase_ms(hkv_decode_plan *plan, float *span, float *rows_ms, float *tile_ms) {
    const bool rows = !plan->items.empty(), tiles = !plan->tile_items.empty() && !plan->fused;  // (one launch: its events are ev[0..1])
    *span = *rows_ms = *tile_ms = 0.f;
    if (rows) HKV_HIP(hipEventElapsedTime(rows_ms, plan->ev[0], plan->ev[1]));
    if (tiles) HKV_HIP(hipEventElapsedTime(tile_ms, plan->ev_tile[0], plan->ev_tile[1]));
    if (rows && tiles) {  // on the time line of the tile kernel's begin
        float rows_begin = 0.f, rows_end = 0.f;
        HKV_HIP(hipEventElapsedTime(&rows_begin, plan->ev_tile[0], plan->ev[0]));
        HKV_HIP(hipEventElapsedTime(&rows_end, plan->ev_tile[0], plan->ev[1]));
        *span = std::max(*tile_ms, rows_end) - std::min(0.f, rows_begin);
    } else {
        *span = rows ? *rows_ms : *tile_ms;
    }
    return HKV_OK;
}

extern "C" int hkv_decode_plan_elapsed_ms(hkv_decode_plan *plan, float *node_ms, float *merge_ms) {
    if (!plan || !node_ms || !merge_ms) return fail(HKV_EINVAL, "hkv_decode_plan_elapsed_ms: null argument");
    if (!plan->profiled_run) return fail(HKV_EINVAL, "hkv_decode_plan_elapsed_ms: no profiled run has been queued");
    HKV_HIP(hipEventSynchronize(plan->ev[3]));
    float rows_ms = 0.f, tile_ms = 0.f;
    if (int rc = node_phase_ms(plan, node_ms, &rows_ms, &tile_ms)) return rc;
    HKV_HIP(hipEventElapsedTime(merge_ms, plan->ev[2], plan->ev[3]));
    return HKV_OK;
}

extern "C" int hkv_decode_plan_elapsed_kernels_ms(hkv_decode_plan *plan, float *rows_kernel_ms, float *tile_kernel_ms) {
    if (!plan || !rows_kernel_ms || !tile_kernel_ms) return fail(HKV_EINVAL, "hkv_decode_plan_elapsed_kernels_ms: null argument");
    if (!plan->profiled_run) return fail(HKV_EINVAL, "hkv_decode_plan_elapsed_kernels_ms: no profiled run has been queued");
    HKV_HIP(hipEventSynchronize(plan->ev[3]));
    float span = 0.f;
    return node_phase_ms(plan, &span, rows_kernel_ms, tile_kernel_ms);
}

static bool same_forest(const hkv_decode_plan *pl, const hkv_node *nodes, int32_t n_nodes, const int32_t *node_pages,
                        int32_t n_node_pages, const int32_t *req_leaf, int32_t n_req, int32_t num_q_heads) {
    return pl && pl->num_q_heads == num_q_heads && (int32_t)pl->key_nodes.size() == n_nodes &&
           (int32_t)pl->key_pages.size() == n_node_pages && (int32_t)pl->req_leaf.size() == n_req &&
           (n_nodes == 0 || !memcmp(pl->key_nodes.data(), nodes, sizeof(hkv_node) * n_nodes)) &&
           (n_node_pages == 0 || !memcmp(pl->key_pages.data(), node_pages, sizeof(int32_t) * n_node_pages)) &&
           (n_req == 0 || !memcmp(pl->req_leaf.data(), req_leaf, sizeof(int32_t) * n_req));
}

static int cached_decode_plan(hkv_pool *pool, const hkv_node *nodes, int32_t n_nodes, const int32_t *node_pages,
                              int32_t n_node_pages, const int32_t *req_leaf, int32_t n_req, int32_t num_q_heads,
                              uint32_t flags, hkv_decode_plan **out) {
    if (!pool) return fail(HKV_EINVAL, "null pool");
    if (n_nodes < 0 || n_node_pages < 0 || n_req < 0 || (n_nodes > 0 && !nodes) || (n_node_pages > 0 && !node_pages) ||
        (n_req > 0 && !req_leaf))
        return fail(HKV_EINVAL, "bad forest arguments");
    hkv_decode_plan *c = pool->cached_decode;
    if (same_forest(c, nodes, n_nodes, node_pages, n_node_pages, req_leaf, n_req, num_q_heads) &&
        (c->dev || (flags & HKV_PLAN_HOST_ONLY))) {
        *out = c;
        return HKV_OK;
    }
    hkv_decode_plan *fresh = nullptr;
    if (int rc = hkv_decode_plan_create(pool, nodes, n_nodes, node_pages, n_node_pages, req_leaf, n_req, num_q_heads,
                                        flags, &fresh))
        return rc;
    if (c) hkv_decode_plan_destroy(c);
    pool->cached_decode = fresh;
    *out = fresh;
    return HKV_OK;
}

extern "C" int attn_decode_prefix_tree(hkv_pool *pool, const void *q, const hkv_node *nodes, int32_t n_nodes,
                                       const int32_t *node_pages, int32_t n_node_pages, const int32_t *req_leaf,
                                       int32_t n_req, int32_t num_q_heads, float scale, void *out, float *lse_out,
                                       void *workspace, size_t workspace_bytes, void *stream) {
    hkv_decode_plan *pl = nullptr;
    // validate everything that does not need the device before touching it
    if (n_req > 0 && (!q || !out)) return fail(HKV_EINVAL, "attn_decode_prefix_tree: null q or out");
    if (int rc = cached_decode_plan(pool, nodes, n_nodes, node_pages, n_node_pages, req_leaf, n_req, num_q_heads, 0,
                                    &pl))
        return rc;
    return attn_decode_plan_run(pl, q, scale, out, lse_out, workspace, workspace_bytes, stream);
}

extern "C" size_t attn_decode_workspace_bytes(hkv_pool *pool, const hkv_node *nodes, int32_t n_nodes,
                                              const int32_t *node_pages, int32_t n_node_pages, const int32_t *req_leaf,
                                              int32_t n_req, int32_t num_q_heads) {
    hkv_decode_plan *pl = nullptr;
    uint32_t flags = (pool && pool->cached_decode && pool->cached_decode->dev) ? 0u : (uint32_t)HKV_PLAN_HOST_ONLY;
    if (cached_decode_plan(pool, nodes, n_nodes, node_pages, n_node_pages, req_leaf, n_req, num_q_heads, flags, &pl))
        return 0;
    return hkv_decode_plan_workspace_bytes(pl);
}

// ---------------------------------------------------------------------------------------------
// prefill planning
// cu_q: request r's new tokens are rows cu_q[r] .. cu_q[r + 1] - 1 of q / out / lse.  q_row_begin (may be null):
// they are rows q_row_begin[r] .. q_row_begin[r] + (cu_q[r + 1] - cu_q[r]) - 1 instead.
static int create_prefill_plan(hkv_pool *pool, const int32_t *cu_q, const int32_t *q_row_begin, const int32_t *block_table,
                               int32_t max_pages, const int32_t *kv_len, int32_t n_req, int32_t num_q_heads,
                               uint32_t flags, hkv_prefill_plan **out) {
    if (!pool || !out) return fail(HKV_EINVAL, "hkv_prefill_plan_create: null argument");
    *out = nullptr;
    const int Hkv = pool->d.num_kv_heads;
    if (num_q_heads <= 0 || num_q_heads % Hkv) return fail(HKV_ESHAPE, "hkv_prefill_plan_create: %d query heads over %d KV heads", num_q_heads, Hkv);
    const int G = num_q_heads / Hkv;
    if (G > 16) return fail(HKV_ESHAPE, "hkv_prefill_plan_create: query/KV head ratio %d (supported: 1..16)", G);
    if (n_req < 0 || max_pages < 0 || (n_req > 0 && (!cu_q || !kv_len || (max_pages > 0 && !block_table))))
        return fail(HKV_EINVAL, "hkv_prefill_plan_create: bad argument");
    if (n_req > 0 && cu_q[0] != 0) return fail(HKV_EINVAL, "hkv_prefill_plan_create: cu_q[0] must be 0");
    for (int r = 0; r < n_req; ++r) {
        int64_t s = (int64_t)cu_q[r + 1] - cu_q[r];
        if (s < 0) return fail(HKV_EINVAL, "hkv_prefill_plan_create: cu_q decreases at request %d", r);
        if (kv_len[r] < s) return fail(HKV_EINVAL, "hkv_prefill_plan_create: request %d has kv_len %d < %lld new tokens", r, kv_len[r], (long long)s);
        int64_t need = ((int64_t)kv_len[r] + pool->d.page_size - 1) / pool->d.page_size;
        if (need > max_pages) return fail(HKV_ENOMEM, "hkv_prefill_plan_create: request %d needs %lld pages, max_pages is %d", r, (long long)need, max_pages);
        if (s == 0) continue;  // nothing of this request is read
        for (int64_t i = 0; i < need; ++i) {
            int32_t id = block_table[(size_t)r * max_pages + i];
            if (id < 0 || id >= pool->d.num_pages)
                return fail(HKV_ERANGE, "hkv_prefill_plan_create: request %d page %lld has id %d outside pool of %d", r, (long long)i, id, pool->d.num_pages);
        }
    }
    hkv_prefill_plan *pl = new (std::nothrow) hkv_prefill_plan;
    if (!pl) return fail(HKV_ENOMEM, "hkv_prefill_plan_create: out of host memory");
    pl->pool = pool;
    pl->n_req = n_req;
    pl->num_q_heads = num_q_heads;
    pl->key_max_pages = max_pages;
    pl->total_q = n_req ? cu_q[n_req] : 0;
    pl->cu_q.assign(cu_q, cu_q + (n_req ? n_req + 1 : 0));
    pl->kv_len.assign(kv_len, kv_len + n_req);
    if (n_req && max_pages) pl->block_table.assign(block_table, block_table + (size_t)n_req * max_pages);
    // the kernels index 16-token blocks: block j of page p is block p * S + j of the buffers
    const int S = pool->blocks_per_page;
    const int max_blocks = max_pages * S;
    pl->max_pages = max_blocks;
    std::vector<int32_t> blocks((size_t)n_req * max_blocks, 0);
    for (int r = 0; r < n_req; ++r) {
        if (cu_q[r + 1] == cu_q[r]) continue;
        const int64_t nb = ((int64_t)kv_len[r] + HKV_PAGE_SIZE - 1) / HKV_PAGE_SIZE;
        for (int64_t b = 0; b < nb; ++b)
            blocks[(size_t)r * max_blocks + b] = block_table[(size_t)r * max_pages + b / S] * S + (int32_t)(b % S);
    }
    const int TQ = prefill_tile_tokens(G);
    struct Proto { int32_t req, q_begin, n_q; int64_t extent; };
    std::vector<Proto> protos;
    for (int r = 0; r < n_req; ++r) {
        int s = cu_q[r + 1] - cu_q[r];
        int prefix = kv_len[r] - s;
        for (int q0 = 0; q0 < s; q0 += TQ) {
            int nq = std::min(TQ, s - q0);
            protos.push_back({r, q0, nq, (int64_t)prefix + q0 + nq});
        }
    }
    // longest key range first; the KV heads of one query tile sit next to each other so that
    // workgroup index mod num_kv_heads is the KV head (one head per XCD when there are 8)
    std::stable_sort(protos.begin(), protos.end(), [](const Proto &a, const Proto &b) { return a.extent > b.extent; });
    for (const Proto &p : protos)
        for (int h = 0; h < Hkv; ++h) {
            int s = cu_q[p.req + 1] - cu_q[p.req];
            pl->tiles.push_back(PrefillTile{p.req, p.q_begin, p.n_q, h, (q_row_begin ? q_row_begin[p.req] : cu_q[p.req]) + p.q_begin, kv_len[p.req] - s,
                                            kv_len[p.req], p.req * max_blocks});
        }
    // fp8 pools: number the pages this batch reads (first use first) and point the device table at them
    std::vector<int32_t> remapped;
    if (pool->d.dtype == HKV_FP8_E4M3) {
        std::unordered_map<int32_t, int32_t> index;
        remapped.assign(blocks.size(), 0);
        for (int r = 0; r < n_req; ++r) {
            if (cu_q[r + 1] == cu_q[r]) continue;
            const int64_t need = ((int64_t)kv_len[r] + HKV_PAGE_SIZE - 1) / HKV_PAGE_SIZE;
            for (int64_t i = 0; i < need; ++i) {
                const int32_t id = blocks[(size_t)r * max_blocks + i];
                auto it = index.find(id);
                if (it == index.end()) {
                    it = index.emplace(id, (int32_t)pl->src_pages.size()).first;
                    pl->src_pages.push_back(id);
                }
                remapped[(size_t)r * max_blocks + i] = it->second;
            }
        }
    }
    const std::vector<int32_t> &dev_table = pool->d.dtype == HKV_FP8_E4M3 ? remapped : blocks;
    if (!(flags & HKV_PLAN_HOST_ONLY) && !pl->tiles.empty()) {
        size_t off_bt = align_up(sizeof(PrefillTile) * pl->tiles.size(), 256);
        size_t off_src = off_bt + align_up(sizeof(int32_t) * dev_table.size(), 256);
        size_t off_fb = off_src + align_up(sizeof(int32_t) * pl->src_pages.size(), 256);
        size_t total = off_fb + 256;
        hipError_t e = hipMalloc(&pl->dev, total);
        if (e == hipSuccess) {
            pl->d_fallback = reinterpret_cast<unsigned int *>(static_cast<char *>(pl->dev) + off_fb);
            e = hipMemset(pl->d_fallback, 0, 256);
        }
        if (e == hipSuccess) {
            pl->d_tiles = static_cast<PrefillTile *>(pl->dev);
            pl->d_block_table = reinterpret_cast<int32_t *>(static_cast<char *>(pl->dev) + off_bt);
            pl->d_src_pages = reinterpret_cast<int32_t *>(static_cast<char *>(pl->dev) + off_src);
            e = hipMemcpy(pl->d_tiles, pl->tiles.data(), sizeof(PrefillTile) * pl->tiles.size(), hipMemcpyHostToDevice);
        }
        if (e == hipSuccess)
            e = hipMemcpy(pl->d_block_table, dev_table.data(), sizeof(int32_t) * dev_table.size(), hipMemcpyHostToDevice);
        if (e == hipSuccess && !pl->src_pages.empty())
            e = hipMemcpy(pl->d_src_pages, pl->src_pages.data(), sizeof(int32_t) * pl->src_pages.size(), hipMemcpyHostToDevice);
        if (e == hipSuccess && pool->d.dtype == HKV_FP32 && pl->total_q > 0) {
            std::vector<int32_t> rr(2 * (size_t)pl->total_q);
            for (int r = 0; r < n_req; ++r)
                for (int i = cu_q[r]; i < cu_q[r + 1]; ++i) {
                    rr[i] = r;
                    rr[(size_t)pl->total_q + i] = kv_len[r] - (cu_q[r + 1] - cu_q[r]) + (i - cu_q[r]) + 1;
                }
            e = hipMalloc((void **)&pl->d_rows_req, sizeof(int32_t) * rr.size());
            if (e == hipSuccess) {
                pl->d_rows_len = pl->d_rows_req + pl->total_q;
                e = hipMemcpy(pl->d_rows_req, rr.data(), sizeof(int32_t) * rr.size(), hipMemcpyHostToDevice);
            }
        }
        if (e != hipSuccess) {
            if (pl->dev) (void)hipFree(pl->dev);
            if (pl->d_rows_req) (void)hipFree(pl->d_rows_req);
            delete pl;
            return fail_hip(e, "hkv_prefill_plan_create: device upload");
        }
    }
    *out = pl;
    return HKV_OK;
}

extern "C" int hkv_prefill_plan_create(hkv_pool *pool, const int32_t *cu_q, const int32_t *block_table,
                                       int32_t max_pages, const int32_t *kv_len, int32_t n_req, int32_t num_q_heads,
                                       uint32_t flags, hkv_prefill_plan **out) {
    return create_prefill_plan(pool, cu_q, nullptr, block_table, max_pages, kv_len, n_req, num_q_heads, flags, out);
}

extern "C" int hkv_prefill_plan_create_rows(hkv_pool *pool, const int32_t *q_row_begin, const int32_t *q_len,
                                            const int32_t *block_table, int32_t max_pages, const int32_t *kv_len,
                                            int32_t n_req, int32_t num_q_heads, uint32_t flags, hkv_prefill_plan **out) {
    if (!pool || !out) return fail(HKV_EINVAL, "hkv_prefill_plan_create_rows: null argument");
    *out = nullptr;
    if (pool->d.dtype == HKV_FP32) return fail(HKV_ESHAPE, "hkv_prefill_plan_create_rows: bf16 and fp8 pools only");
    if (n_req < 0 || (n_req > 0 && (!q_row_begin || !q_len))) return fail(HKV_EINVAL, "hkv_prefill_plan_create_rows: bad argument");
    std::vector<int32_t> cu((size_t)n_req + 1, 0);
    std::vector<std::pair<int64_t, int64_t>> spans;
    for (int r = 0; r < n_req; ++r) {
        if (q_len[r] < 0 || q_row_begin[r] < 0 || (int64_t)q_row_begin[r] + q_len[r] > INT32_MAX || (int64_t)cu[r] + q_len[r] > INT32_MAX)
            return fail(HKV_EINVAL, "hkv_prefill_plan_create_rows: request %d: rows %d .. + %d", r, q_row_begin[r], q_len[r]);
        cu[r + 1] = cu[r] + q_len[r];
        if (q_len[r] > 0) spans.push_back({q_row_begin[r], (int64_t)q_row_begin[r] + q_len[r]});
    }
    std::sort(spans.begin(), spans.end());
    for (size_t i = 1; i < spans.size(); ++i)
        if (spans[i].first < spans[i - 1].second)
            return fail(HKV_EINVAL, "hkv_prefill_plan_create_rows: two requests share row %lld", (long long)spans[i].first);
    return create_prefill_plan(pool, cu.data(), q_row_begin, block_table, max_pages, kv_len, n_req, num_q_heads, flags, out);
}

extern "C" int hkv_prefill_plan_destroy(hkv_prefill_plan *plan) {
    if (!plan) return HKV_OK;
    if (plan->dev) (void)hipFree(plan->dev);
    if (plan->d_rows_req) (void)hipFree(plan->d_rows_req);
    delete plan;
    return HKV_OK;
}

extern "C" int32_t hkv_prefill_plan_num_tiles(const hkv_prefill_plan *plan) {
    return plan ? (int32_t)plan->tiles.size() : fail(HKV_EINVAL, "null plan");
}

extern "C" int hkv_prefill_plan_tiles(const hkv_prefill_plan *plan, int32_t *tiles_out) {
    if (!plan || !tiles_out) return fail(HKV_EINVAL, "hkv_prefill_plan_tiles: null argument");
    static_assert(sizeof(PrefillTile) == 32, "tile layout is part of the introspection contract");
    if (!plan->tiles.empty()) memcpy(tiles_out, plan->tiles.data(), sizeof(PrefillTile) * plan->tiles.size());
    return HKV_OK;
}

extern "C" int hkv_prefill_plan_fallback_tiles(hkv_prefill_plan *plan, int64_t *count) {
    if (!plan || !count) return fail(HKV_EINVAL, "hkv_prefill_plan_fallback_tiles: null argument");
    *count = 0;
    if (!plan->d_fallback) return HKV_OK;  // host-only plan, or a plan without tiles
    unsigned int n = 0;
    HKV_HIP(hipMemcpy(&n, plan->d_fallback, sizeof(n), hipMemcpyDeviceToHost));
    *count = n;
    return HKV_OK;
}

extern "C" size_t hkv_prefill_plan_workspace_bytes(const hkv_prefill_plan *plan) {
    if (!plan) return 0;
    return 2 * plan->src_pages.size() * (size_t)plan->pool->d.num_kv_heads * HKV_PAGE_SIZE * HKV_HEAD_DIM * sizeof(uint16_t);
}

extern "C" int attn_prefill_plan_run(hkv_prefill_plan *plan, const void *q, float scale, void *out, float *lse_out,
                                     void *stream) {
    return attn_prefill_plan_run_ws(plan, q, scale, out, lse_out, nullptr, 0, stream);
}

extern "C" int attn_prefill_plan_run_ws(hkv_prefill_plan *plan, const void *q, float scale, void *out, float *lse_out,
                                        void *workspace, size_t workspace_bytes, void *stream) {
    if (!plan) return fail(HKV_EINVAL, "attn_prefill_plan_run: null plan");
    if (plan->tiles.empty()) return HKV_OK;
    if (!q || !out) return fail(HKV_EINVAL, "attn_prefill_plan_run: null q or out");
    if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(out)) & 15)
        return fail(HKV_EINVAL, "attn_prefill_plan_run: q and out must be 16-byte aligned");
    if (!plan->dev) return fail(HKV_EINVAL, "attn_prefill_plan_run: plan was built host-only");
    if (plan->pool->d.dtype == HKV_FP32) {  // full-precision path: one wavefront per (new token, head)
        RowsLaunch r{view_of(plan->pool), static_cast<const float *>(q), plan->d_block_table, plan->d_rows_req, plan->d_rows_len,
                     static_cast<float *>(out), lse_out, plan->total_q, plan->num_q_heads, plan->max_pages, scale};
        HKV_HIP(launch_rows_fp32(r, static_cast<hipStream_t>(stream)));
        return HKV_OK;
    }
    PoolView view = view_of(plan->pool);
    if (plan->pool->d.dtype == HKV_FP8_E4M3) {  // dequantise the pages of this batch, then read the scratch pool
        const size_t need = hkv_prefill_plan_workspace_bytes(plan);
        if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255))
            return fail(HKV_EINVAL, "attn_prefill_plan_run: an fp8 pool needs a 256-byte aligned workspace of %zu bytes", need);
        if (workspace_bytes < need)
            return fail(HKV_ENOMEM, "attn_prefill_plan_run: workspace has %zu bytes, %zu needed", workspace_bytes, need);
        void *k_dst = workspace, *v_dst = static_cast<char *>(workspace) + need / 2;
        PoolDequantLaunch d{view, plan->d_src_pages, (int32_t)plan->src_pages.size(), k_dst, v_dst};
        HKV_HIP(launch_pool_dequant(d, static_cast<hipStream_t>(stream)));
        view = PoolView{k_dst, v_dst, nullptr, nullptr, view.num_kv_heads, HKV_BF16};
    }
    PrefillLaunch a{view, q, plan->d_tiles, plan->d_block_table, out, lse_out,
                    (int32_t)plan->tiles.size(), plan->num_q_heads, scale, plan->d_fallback};
    HKV_HIP(launch_prefill(a, static_cast<hipStream_t>(stream)));
    return HKV_OK;
}

extern "C" int attn_prefill_with_prefix(hkv_pool *pool, const void *q, const int32_t *cu_q, const int32_t *block_table,
                                        int32_t max_pages, const int32_t *kv_len, int32_t n_req, int32_t num_q_heads,
                                        float scale, void *out, float *lse_out, void *workspace, size_t workspace_bytes,
                                        void *stream) {
    if (!pool) return fail(HKV_EINVAL, "attn_prefill_with_prefix: null pool");
    hkv_prefill_plan *c = pool->cached_prefill;
    bool same = c && c->dev && c->n_req == n_req && c->num_q_heads == num_q_heads && c->key_max_pages == max_pages &&
                n_req > 0 && cu_q && kv_len && block_table &&
                !memcmp(c->cu_q.data(), cu_q, sizeof(int32_t) * (n_req + 1)) &&
                !memcmp(c->kv_len.data(), kv_len, sizeof(int32_t) * n_req) &&
                !memcmp(c->block_table.data(), block_table, sizeof(int32_t) * (size_t)n_req * max_pages);
    if (!same) {
        hkv_prefill_plan *fresh = nullptr;
        if (int rc = hkv_prefill_plan_create(pool, cu_q, block_table, max_pages, kv_len, n_req, num_q_heads, 0, &fresh))
            return rc;
        if (c) hkv_prefill_plan_destroy(c);
        pool->cached_prefill = c = fresh;
    }
    return attn_prefill_plan_run_ws(c, q, scale, out, lse_out, workspace, workspace_bytes, stream);
}

extern "C" size_t attn_prefill_workspace_bytes(int32_t total_q, int32_t num_q_heads) {
    (void)total_q;
    (void)num_q_heads;
    return 0;
}
