"""Plain-Python oracle of the block-level prefix cache that sits on top of the page pool.

TEST INFRASTRUCTURE ONLY (imported by tests/ and by nothing in the product package).

What follows the paper (Section 6, "LLM Engine Integration"): the KV cache of a prompt prefix is
kept in GPU memory block by block and reused by later calls; blocks of precomputed prefixes can be
pinned; under memory pressure unpinned blocks are evicted at block level, least recently used first
and never a prefix before its extensions (the longest match goes first); an evicted prefix is simply
recomputed by the next call that needs it.

Readings where the paper is silent (the library takes the same ones)
  C1  A block is one page of consecutive tokens (16, or the pool's page size); its identity is
      (identity of the preceding block, its token ids): two sequences share a block exactly when they agree on everything up to its end.
      Only full blocks are shared; a sequence's last, partial block is private to it.
  C2  acquire(tokens): walk the full blocks from the front while they are cached (hits), then give
      every remaining block a page: from the pool's free list (lowest id first, as kv_pool_alloc
      does) or, when that is empty, by evicting.  New full blocks enter the cache at once.
      A call that runs out of pages fails as a whole: its hits are released, the blocks it had created
      leave the cache again (deepest first, pages back to the pool in that order; they never held KV,
      so a later call must not count them as cached) and its hit/miss counts are taken back.  Blocks it
      evicted on the way stay evicted.
  C3  Evictable = not referenced by a live sequence, not pinned, and no cached block extends it.
      Among those the one with the oldest last-use time goes first; ties by lower page id.  Last-use
      time is a logical clock that ticks once per acquire / release call.
  C4  release(pages): drops the sequence's references; its private partial page returns to the pool.
  C5  pin / unpin count per block; a pinned block is never evicted (nor, then, anything it extends).
PARITY UNPINNED against any external system: the paper names the policy, not its corner cases.
The tests pin the invariants the policy must satisfy and the library's bit-exact agreement."""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple

BLOCK = 16


class _Block:
    def __init__(self, parent: Optional["_Block"], key: Tuple[int, ...], page: int):
        self.parent, self.key, self.page = parent, key, page
        self.children: Dict[Tuple[int, ...], "_Block"] = {}
        self.ref = 0
        self.pin = 0
        self.last_use = 0


class PrefixCache:
    def __init__(self, num_pages: int, free_order: Optional[Sequence[int]] = None, block: int = BLOCK):
        self.block = block                       # tokens per cached block = the pool's page size
        self.free: List[int] = list(free_order) if free_order is not None else list(range(num_pages))
        self.root = _Block(None, (), -1)
        self.by_page: Dict[int, _Block] = {}     # cached full blocks
        self.private: Dict[int, int] = {}        # page -> 1 for partial last blocks in use
        self.clock = 0
        self.hits = self.misses = self.evictions = 0
        self.evicted_pages: List[int] = []       # in eviction order (for the tests)

    # ---- internals
    def _evict_one(self) -> int:
        best = None
        for b in self.by_page.values():
            if b.ref == 0 and b.pin == 0 and not b.children:
                if best is None or (b.last_use, b.page) < (best.last_use, best.page):
                    best = b
        if best is None:
            raise MemoryError("no page free and nothing evictable")
        del best.parent.children[best.key]
        del self.by_page[best.page]
        self.evictions += 1
        self.evicted_pages.append(best.page)
        return best.page

    def _page(self) -> int:
        if self.free:
            return self.free.pop(0)
        return self._evict_one()

    # ---- interface
    def acquire(self, tokens: Sequence[int], pin: bool = False) -> Tuple[List[int], int]:
        """Returns (page ids of all ceil(n/block) blocks, number of cached tokens at the front)."""
        self.clock += 1
        n = len(tokens)
        n_full = n // self.block
        pages: List[int] = []
        node, j = self.root, 0
        taken: List[_Block] = []
        while j < n_full:                                   # hits
            key = tuple(int(t) for t in tokens[j * self.block:(j + 1) * self.block])
            nxt = node.children.get(key)
            if nxt is None:
                break
            nxt.ref += 1
            nxt.last_use = self.clock
            taken.append(nxt)
            pages.append(nxt.page)
            node, j = nxt, j + 1
            self.hits += 1
        cached = j * self.block
        n_hit = j
        try:
            while j < n_full:                               # misses: new full blocks
                key = tuple(int(t) for t in tokens[j * self.block:(j + 1) * self.block])
                b = _Block(node, key, self._page())
                b.ref, b.last_use = 1, self.clock
                node.children[key] = b
                self.by_page[b.page] = b
                taken.append(b)
                pages.append(b.page)
                node, j = b, j + 1
                self.misses += 1
            if n % self.block:                                   # private partial block
                p = self._page()
                self.private[p] = 1
                pages.append(p)
        except MemoryError:
            self.release(pages[:n_hit])                     # the hits: as a release
            for b in reversed(taken[n_hit:]):               # the blocks created here never held KV: out again
                del b.parent.children[b.key]
                del self.by_page[b.page]
                self.free.append(b.page)
            self.hits -= n_hit
            self.misses -= len(taken) - n_hit
            raise
        if pin:
            for b in taken:
                b.pin += 1
        return pages, cached

    def release(self, pages: Sequence[int]) -> None:
        self.clock += 1
        for p in pages:
            if p in self.private:
                del self.private[p]
                self.free.append(p)
                continue
            b = self.by_page[p]
            assert b.ref > 0
            b.ref -= 1
            b.last_use = self.clock

    def unpin(self, pages: Sequence[int]) -> None:
        for p in pages:
            b = self.by_page.get(p)
            if b is not None and b.pin > 0:
                b.pin -= 1

    def num_cached_blocks(self) -> int:
        return len(self.by_page)
