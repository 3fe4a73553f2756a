/*
 * icarus_cache.h -- C ABI of the cross-model prefix-cache manager (host side, no GPU work).
 *
 * In ICaRus the K/V of a token sequence is written by the frozen base model, so it is the same whichever
 * adapter decodes: a cached prefix can serve a request of ANY model (Sec. 1; Sec. 3.2; Sec. 4.3,
 * "reuse identical prefix caches across models").  In the conventional multi-LoRA system a cached prefix
 * belongs to the adapter that computed it (App. A.2): N adapters on one context keep N copies
 * (Table 1, memory O(M + N L_t) against O(M + L_t)) and evict and recompute once memory is full (Sec. 4.3).
 * This manager hands out the blocks of the paged KV pool that icarus.h's calls read and write: it owns the
 * block ids, their reference counts, a map from token prefixes to published blocks, and the eviction
 * order.  key_by_model = 0 is ICaRus (keys carry no adapter id); key_by_model = 1 is the baseline system.
 *
 * Policy (the paper leaves it to the serving stack):
 *  - A block is FREE, LIVE (referenced by >= 1 sequences) or CACHED (published, unreferenced, evictable).
 *  - A full block is published under (adapter id if key_by_model, all tokens of its sequence up to and
 *    including the block).  Lookups compare tokens exactly; the hash only finds candidates.
 *  - A fresh block is the front of the free queue (initially 0, 1, 2, ...); if that is empty, the least
 *    recently released cached block is evicted and reused.
 *  - Releasing a sequence walks its blocks from the last to the first, so a chain is evicted tail first.
 *
 * All pointers are HOST pointers.  Calls on one manager are serialised by an internal mutex.  Every call
 * returns an icarus_status; on failure nothing has changed and icarus_cache_last_error() has the message.
 */
#ifndef ICARUS_CACHE_H
#define ICARUS_CACHE_H

#include "icarus.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct icarus_cache icarus_cache;

typedef struct icarus_cache_config {
    int32_t num_blocks;    /* blocks of the KV pool this manager hands out, >= 1 */
    int32_t block_size;    /* tokens per block, >= 1 (the layer's block_size) */
    int32_t key_by_model;  /* 0: prefixes are shared by all adapters (ICaRus); 1: per adapter (baseline) */
} icarus_cache_config;

typedef struct icarus_cache_stats {
    int64_t lookups;       /* acquire calls that succeeded */
    int64_t hit_tokens;    /* tokens found cached by them */
    int64_t miss_tokens;   /* tokens of their contexts that were not */
    int64_t evictions;     /* cached blocks unpublished to make room */
    int32_t live, cached, free_blocks; /* blocks in each state now */
    int32_t peak_live;     /* most blocks ever live at once */
} icarus_cache_stats;

icarus_status icarus_cache_create(const icarus_cache_config *cfg, icarus_cache **out);
void icarus_cache_destroy(icarus_cache *c);
const char *icarus_cache_last_error(const icarus_cache *c);

/* Start a sequence whose context is tokens[0, n_tokens), to be decoded by adapter `model`.
 * The longest run of leading full blocks that are published is reused (at most (n_tokens - 1) / block_size
 * of them: one token is always left to compute, so that the request produces logits) and referenced; fresh
 * blocks are taken for the rest of n_tokens + reserve_tokens tokens.
 * blocks [max_blocks] receives the sequence's block ids in order (a row of the block table), *n_blocks their
 * number, *n_cached_tokens how many leading tokens already have their K/V in those blocks (a multiple of
 * block_size): the caller prefills tokens [n_cached_tokens, n_tokens) with ctx_len = n_cached_tokens.
 * ICARUS_ERR_CAPACITY: max_blocks too small, or not enough free + evictable blocks. */
icarus_status icarus_cache_acquire(icarus_cache *c, const int32_t *tokens, int32_t n_tokens, int32_t model,
                                   int32_t reserve_tokens, int32_t *blocks, int32_t max_blocks, int32_t *n_blocks,
                                   int32_t *n_cached_tokens);

/* A live sequence grows to n_tokens_total tokens: blocks [max_blocks] holds its *n_blocks ids and receives
 * the fresh ones behind them.  ICARUS_ERR_CAPACITY as above. */
icarus_status icarus_cache_extend(icarus_cache *c, int32_t *blocks, int32_t max_blocks, int32_t *n_blocks,
                                  int32_t n_tokens_total);

/* The K/V of tokens[0, n_tokens) of a live sequence is in its blocks now: publish every full block that is
 * not published yet, unless another block already holds the same prefix (then this one stays private to
 * the sequence and returns to the free queue on release). */
icarus_status icarus_cache_commit(icarus_cache *c, const int32_t *tokens, int32_t n_tokens, int32_t model,
                                  const int32_t *blocks, int32_t n_blocks);

/* The sequence is finished: drop its references, last block first.  Published blocks stay cached. */
icarus_status icarus_cache_release(icarus_cache *c, const int32_t *blocks, int32_t n_blocks);

icarus_status icarus_cache_get_stats(icarus_cache *c, icarus_cache_stats *out);

#ifdef __cplusplus
}
#endif
#endif /* ICARUS_CACHE_H */
