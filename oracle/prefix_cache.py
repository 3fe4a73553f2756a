"""Oracle of the cross-model prefix-cache manager: the block bookkeeping written as its definition.

TEST INFRASTRUCTURE ONLY: imported by tests/ and by bench.py's cpu_baseline leg, never by the product.

What the paper fixes (Sec. 1, Sec. 3.2, Sec. 4.3, App. A.2): in ICaRus the K/V of a token sequence is
produced by the frozen base model, so it is the same whichever adapter decodes; a cached prefix can
therefore be reused by a request of ANY model ("cross-model prefix caching").  In the conventional
multi-LoRA system the cache of a prefix belongs to the adapter that computed it and only requests of that
adapter can reuse it; N adapters working on one context hold N copies (Table 1: O(M + N L_t) against
O(M + L_t)) and, when memory is full, evict and recompute.

The paper runs inside a serving stack and does not specify the bookkeeping; this is the policy both
implementations follow (each reading where the paper is silent is spelled out below):

  * The pool has `num_blocks` blocks of `block_size` tokens.  A block is FREE, LIVE (referenced by
    ref >= 1 sequences) or CACHED (published, ref == 0, evictable).
  * A full block is PUBLISHED under the key (model if key_by_model else none, all tokens of the
    sequence up to and including this block): here literally that tuple.
  * acquire(tokens, model, reserve): hits = the longest run of leading blocks i = 0, 1, ... that are
    published under the key of tokens[0 : (i+1) B], at most (n-1) // B of them (one token is always left
    to compute, so that the request produces logits).  The hit blocks are referenced; then
    ceil((n + reserve) / B) - hits fresh blocks are taken.  If the free and cached-unreferenced blocks
    (not counting the hits) do not cover that, nothing changes and the call fails.
  * A fresh block comes from the front of the free queue (initially 0, 1, 2, ...); if that is empty, the
    least recently released cached block is evicted (unpublished) and reused.
  * commit(tokens, model, blocks): every full block of the sequence that is not published yet is
    published under its key, unless another block already holds that key (then this one stays private).
  * release(blocks): from the last block to the first, ref -= 1; at zero a published block goes to the
    most-recent end of the eviction queue, an unpublished one to the back of the free queue.  (Tails are
    released before heads, so a chain is evicted from its tail.)
"""
from __future__ import annotations

from collections import OrderedDict, deque


class CacheFull(RuntimeError):
    pass


class OraclePrefixCache:
    def __init__(self, num_blocks: int, block_size: int, key_by_model: bool):
        assert num_blocks > 0 and block_size > 0
        self.N, self.B, self.key_by_model = num_blocks, block_size, bool(key_by_model)
        self.free = deque(range(num_blocks))
        self.ref = [0] * num_blocks
        self.key_of = [None] * num_blocks          # published key of a block, or None
        self.block_of = {}                         # key -> block
        self.lru = OrderedDict()                   # cached (published, unreferenced) blocks, oldest first
        self.stats = dict(lookups=0, hit_tokens=0, miss_tokens=0, evictions=0, peak_live=0)

    # -- helpers ---------------------------------------------------------------------------
    def _key(self, tokens, n_blocks, model):
        return (int(model) if self.key_by_model else -1, tuple(int(t) for t in tokens[: n_blocks * self.B]))

    def _live(self):
        return sum(1 for r in self.ref if r > 0)

    def _take(self):
        if self.free:
            return self.free.popleft()
        b, _ = self.lru.popitem(last=False)
        del self.block_of[self.key_of[b]]
        self.key_of[b] = None
        self.stats["evictions"] += 1
        return b

    def _grow(self, need):
        out = []
        for _ in range(need):
            b = self._take()
            self.ref[b] = 1
            out.append(b)
        self.stats["peak_live"] = max(self.stats["peak_live"], self._live())
        return out

    # -- the four operations -----------------------------------------------------------------
    def acquire(self, tokens, model, reserve=0):
        """-> (blocks, n_cached_tokens)"""
        n = len(tokens)
        assert n >= 1 and reserve >= 0
        hits = []
        for i in range((n - 1) // self.B):
            b = self.block_of.get(self._key(tokens, i + 1, model))
            if b is None:
                break
            hits.append(b)
        need = -(-(n + reserve) // self.B) - len(hits)
        in_lru = sum(1 for b in hits if self.ref[b] == 0)
        if len(self.free) + len(self.lru) - in_lru < need:
            raise CacheFull(f"need {need} blocks, {len(self.free)} free + {len(self.lru) - in_lru} evictable")
        for b in hits:
            if self.ref[b] == 0:
                del self.lru[b]
            self.ref[b] += 1
        blocks = hits + self._grow(need)
        self.stats["lookups"] += 1
        self.stats["hit_tokens"] += len(hits) * self.B
        self.stats["miss_tokens"] += n - len(hits) * self.B
        return blocks, len(hits) * self.B

    def extend(self, blocks, n_tokens_total):
        """More blocks for a live sequence that grows to n_tokens_total tokens: -> the longer block list."""
        need = -(-n_tokens_total // self.B) - len(blocks)
        if need <= 0:
            return list(blocks)
        if len(self.free) + len(self.lru) < need:
            raise CacheFull(f"need {need} blocks")
        return list(blocks) + self._grow(need)

    def commit(self, tokens, model, blocks):
        for i in range(min(len(tokens) // self.B, len(blocks))):
            b = blocks[i]
            if self.key_of[b] is not None:
                continue
            k = self._key(tokens, i + 1, model)
            if k in self.block_of:
                continue
            self.block_of[k] = b
            self.key_of[b] = k

    def release(self, blocks):
        for b in reversed(list(blocks)):
            assert self.ref[b] > 0
            self.ref[b] -= 1
            if self.ref[b] == 0:
                if self.key_of[b] is not None:
                    self.lru[b] = True
                else:
                    self.free.append(b)

    def counts(self):
        return dict(self.stats, live=self._live(), cached=len(self.lru), free=len(self.free))
