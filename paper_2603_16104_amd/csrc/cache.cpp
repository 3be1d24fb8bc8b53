// Block-level prefix cache on top of the page pool (host bookkeeping only): which pages hold the
// KV of which token prefix, who uses them, which may be evicted.  (Section 6, "LLM Engine
// Integration": precomputed prefixes are pinned; under memory pressure blocks are evicted least
// recently used first and a prefix never before its extensions; an evicted prefix is recomputed.)
//
// A block is one page of tokens (16 unless the pool says otherwise); its identity is (preceding block,
// its token ids), so two sequences share
// a block exactly when they agree on everything up to its end.  Only full blocks are shared; a
// sequence's partial last block is private.  Evictable = no live user, not pinned, nothing cached
// extends it; among those the oldest last use goes first, ties by lower page id; the clock ticks
// once per acquire / release call.
#include <cstdint>
#include <cstring>
#include <map>
#include <new>
#include <set>
#include <unordered_map>
#include <vector>

#include "../../include/heliumkv.h"

namespace hkv {
int fail(int code, const char *fmt, ...);
}
using hkv::fail;

namespace {

struct Block {
    Block *parent = nullptr;
    std::vector<int32_t> key;
    int32_t page = -1;
    std::map<std::vector<int32_t>, Block *> children;
    int32_t ref = 0, pin = 0;
    int64_t last_use = 0;
};

}  // namespace

struct hkv_cache {
    hkv_pool *pool = nullptr;
    int32_t block = HKV_PAGE_SIZE;  // tokens per cached block = the pool's page size
    Block root;
    std::unordered_map<int32_t, Block *> by_page;      // cached full blocks
    std::unordered_map<int32_t, int> private_pages;    // partial last blocks in use
    std::set<std::pair<int64_t, int32_t>> evictable;   // (last use, page) of blocks that may go
    int64_t clock = 0;
    int64_t hits = 0, misses = 0, evictions = 0;

    static bool can_go(const Block *b) { return b->ref == 0 && b->pin == 0 && b->children.empty(); }
    // call around every change of ref / pin / children / last_use of b
    void drop(Block *b) {
        if (b != &root && can_go(b)) evictable.erase({b->last_use, b->page});
    }
    void add(Block *b) {
        if (b != &root && can_go(b)) evictable.insert({b->last_use, b->page});
    }
    // a page for a new block: the pool's next free one, else the best eviction victim; -1 if none
    int32_t take_page() {
        int32_t id = -1;
        if (kv_pool_num_free(pool) > 0) {
            if (kv_pool_alloc(pool, 1, &id) != HKV_OK) return -1;
            return id;
        }
        if (evictable.empty()) return -1;
        auto it = evictable.begin();
        Block *b = by_page[it->second];
        evictable.erase(it);
        Block *par = b->parent;
        drop(par);
        par->children.erase(b->key);
        add(par);
        by_page.erase(b->page);
        id = b->page;
        delete b;
        ++evictions;
        return id;  // the page keeps its pool reference: it goes straight to its next owner
    }
    void release_pages(const int32_t *pages, int32_t n) {
        ++clock;
        for (int i = 0; i < n; ++i) {
            auto pv = private_pages.find(pages[i]);
            if (pv != private_pages.end()) {
                private_pages.erase(pv);
                (void)kv_pool_release(pool, 1, &pages[i]);
                continue;
            }
            auto it = by_page.find(pages[i]);
            if (it == by_page.end() || it->second->ref <= 0) continue;  // validated by the caller
            Block *b = it->second;
            drop(b);
            --b->ref;
            b->last_use = clock;
            add(b);
        }
    }
    void free_tree(Block *b) {
        for (auto &kv : b->children) {
            free_tree(kv.second);
            delete kv.second;
        }
        b->children.clear();
    }
};

extern "C" int kv_cache_create(hkv_pool *pool, hkv_cache **out) {
    if (!pool || !out) return fail(HKV_EINVAL, "kv_cache_create: null argument");
    hkv_cache *c = new (std::nothrow) hkv_cache;
    if (!c) return fail(HKV_ENOMEM, "kv_cache_create: out of host memory");
    c->pool = pool;
    c->block = kv_pool_page_size(pool);
    *out = c;
    return HKV_OK;
}

extern "C" int kv_cache_destroy(hkv_cache *c) {
    if (!c) return HKV_OK;
    for (auto &kv : c->by_page) (void)kv_pool_release(c->pool, 1, &kv.first);
    for (auto &kv : c->private_pages) (void)kv_pool_release(c->pool, 1, &kv.first);
    c->free_tree(&c->root);
    delete c;
    return HKV_OK;
}

extern "C" int kv_cache_acquire(hkv_cache *c, const int32_t *tokens, int32_t n_tokens, int32_t pin, int32_t *page_ids,
                                int32_t *n_cached_tokens) {
    if (!c || n_tokens < 0 || (n_tokens > 0 && (!tokens || !page_ids)) || !n_cached_tokens)
        return fail(HKV_EINVAL, "kv_cache_acquire: bad argument");
    ++c->clock;
    const int P = c->block;
    const int n_full = n_tokens / P;
    Block *node = &c->root;
    std::vector<Block *> taken;
    int j = 0, n_pages = 0;
    for (; j < n_full; ++j) {  // hits
        std::vector<int32_t> key(tokens + j * P, tokens + (j + 1) * P);
        auto it = node->children.find(key);
        if (it == node->children.end()) break;
        Block *b = it->second;
        c->drop(b);
        ++b->ref;
        b->last_use = c->clock;
        c->add(b);
        taken.push_back(b);
        page_ids[n_pages++] = b->page;
        node = b;
        ++c->hits;
    }
    *n_cached_tokens = j * P;
    const int n_hit = j;
    bool ok = true;
    for (; j < n_full && ok; ++j) {  // misses: new full blocks enter the cache at once
        const int32_t page = c->take_page();
        if (page < 0) {
            ok = false;
            break;
        }
        Block *b = new (std::nothrow) Block;
        if (!b) {
            (void)kv_pool_release(c->pool, 1, &page);
            ok = false;
            break;
        }
        b->parent = node;
        b->key.assign(tokens + j * P, tokens + (j + 1) * P);
        b->page = page;
        b->ref = 1;
        b->last_use = c->clock;
        c->drop(node);  // it gains a child: no longer a candidate
        node->children[b->key] = b;
        c->by_page[page] = b;
        taken.push_back(b);
        page_ids[n_pages++] = page;
        node = b;
        ++c->misses;
    }
    if (ok && n_tokens % P) {  // private partial block
        const int32_t page = c->take_page();
        if (page < 0) {
            ok = false;
        } else {
            c->private_pages[page] = 1;
            page_ids[n_pages++] = page;
        }
    }
    if (!ok) {  // the call fails as a whole
        c->release_pages(page_ids, n_hit);  // the hits: as a release (the clock ticks once more)
        for (size_t i = taken.size(); i-- > (size_t)n_hit;) {
            // a block created here never held KV: it leaves the cache again (deepest first), so that no later
            // call finds it as a hit; its page goes back to the pool
            Block *b = taken[i], *par = b->parent;
            par->children.erase(b->key);
            c->add(par);  // it may have lost its last child
            c->by_page.erase(b->page);
            (void)kv_pool_release(c->pool, 1, &b->page);
            delete b;
        }
        c->hits -= n_hit;
        c->misses -= (int64_t)taken.size() - n_hit;
        *n_cached_tokens = 0;
        return fail(HKV_ENOMEM, "kv_cache_acquire: no page free and nothing evictable (%d tokens)", n_tokens);
    }
    if (pin)
        for (Block *b : taken) {
            c->drop(b);
            ++b->pin;
        }
    return HKV_OK;
}

extern "C" int kv_cache_release(hkv_cache *c, const int32_t *page_ids, int32_t n_pages) {
    if (!c || n_pages < 0 || (n_pages > 0 && !page_ids)) return fail(HKV_EINVAL, "kv_cache_release: bad argument");
    for (int i = 0; i < n_pages; ++i) {
        if (c->private_pages.count(page_ids[i])) continue;
        auto it = c->by_page.find(page_ids[i]);
        if (it == c->by_page.end() || it->second->ref <= 0)
            return fail(HKV_ERANGE, "kv_cache_release: page %d (entry %d) is not held by a sequence", page_ids[i], i);
    }
    c->release_pages(page_ids, n_pages);
    return HKV_OK;
}

extern "C" int kv_cache_unpin(hkv_cache *c, const int32_t *page_ids, int32_t n_pages) {
    if (!c || n_pages < 0 || (n_pages > 0 && !page_ids)) return fail(HKV_EINVAL, "kv_cache_unpin: bad argument");
    for (int i = 0; i < n_pages; ++i) {
        auto it = c->by_page.find(page_ids[i]);
        if (it == c->by_page.end() || it->second->pin <= 0) continue;
        Block *b = it->second;
        --b->pin;
        c->add(b);
    }
    return HKV_OK;
}

extern "C" int kv_cache_stats(const hkv_cache *c, int64_t *cached_blocks, int64_t *hits, int64_t *misses, int64_t *evictions) {
    if (!c) return fail(HKV_EINVAL, "kv_cache_stats: null cache");
    if (cached_blocks) *cached_blocks = (int64_t)c->by_page.size();
    if (hits) *hits = c->hits;
    if (misses) *misses = c->misses;
    if (evictions) *evictions = c->evictions;
    return HKV_OK;
}
