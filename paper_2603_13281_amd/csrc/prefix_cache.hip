// Cross-model prefix-cache manager: host-side bookkeeping of the paged KV pool's blocks
// (Sec. 3.2 and Sec. 4.3: one cache for all adapters; Table 1: memory O(M + L_t) against O(M + N L_t)).
// No GPU work here: the file sits with the kernels because it is part of the same C-ABI library.
//
// Published prefixes form a trie: a node stands for one token prefix that is a whole number of blocks
// (its key: the node of the prefix one block shorter, the adapter id or -1 at the first level, the last
// block's tokens, compared exactly; the hash only finds candidates), and holds the id of the block that
// is published for it, or none once that block has been evicted while longer prefixes are still cached.
// By induction a node names its whole prefix, so one block of tokens is compared per step of a lookup.
#include "../../include/icarus_cache.h"

#include <algorithm>
#include <cstring>
#include <deque>
#include <mutex>
#include <string>
#include <unordered_map>
#include <vector>

namespace {

struct Block {
    int32_t ref = 0;
    int32_t node = -1;                     // trie node it is published for, or -1
    int32_t lru_prev = -1, lru_next = -1;  // intrusive list of cached blocks, oldest at the head
};

struct Node {
    int32_t parent = -1;   // node of the prefix one block shorter (-1: first block)
    int32_t model = -1;    // adapter id (first level of per-adapter caches), else -1
    int32_t block = -1;    // published block, or -1
    int32_t children = 0;
    uint64_t hash = 0;
    bool used = false;
};

uint64_t mix64(uint64_t x) {
    x ^= x >> 30; x *= 0xbf58476d1ce4e5b9ull;
    x ^= x >> 27; x *= 0x94d049bb133111ebull;
    x ^= x >> 31;
    return x;
}

}  // namespace

struct icarus_cache {
    icarus_cache_config cfg{};
    std::vector<Block> blk;
    std::vector<Node> node;
    std::vector<int32_t> node_tok;                   // [nodes][block_size]
    std::vector<int32_t> node_free;
    std::deque<int32_t> free_q;
    int32_t lru_head = -1, lru_tail = -1, n_lru = 0;
    std::unordered_multimap<uint64_t, int32_t> map;  // key hash -> node
    icarus_cache_stats st{};
    int32_t n_live = 0;
    std::string err;
    std::mutex mu;

    uint64_t key_hash(int32_t parent, int32_t model, const int32_t *t) const {
        uint64_t h = mix64(((uint64_t)(uint32_t)parent << 32) ^ (uint32_t)model);
        for (int i = 0; i < cfg.block_size; ++i) h = mix64(h ^ (uint32_t)t[i]) + 0x632be59bd9b4e019ull;
        return h;
    }
    int32_t find_node(int32_t parent, int32_t model, const int32_t *t, uint64_t *hash_out = nullptr) const {
        uint64_t h = key_hash(parent, model, t);
        if (hash_out) *hash_out = h;
        auto range = map.equal_range(h);
        for (auto it = range.first; it != range.second; ++it) {
            const Node &n = node[it->second];
            if (n.parent == parent && n.model == model && !memcmp(&node_tok[(size_t)it->second * cfg.block_size], t, sizeof(int32_t) * cfg.block_size))
                return it->second;
        }
        return -1;
    }
    int32_t new_node(int32_t parent, int32_t model, const int32_t *t, uint64_t h) {
        int32_t id;
        if (!node_free.empty()) {
            id = node_free.back();
            node_free.pop_back();
        } else {
            id = (int32_t)node.size();
            node.emplace_back();
            node_tok.resize(node_tok.size() + cfg.block_size);
        }
        Node &n = node[id];
        n = Node();
        n.parent = parent; n.model = model; n.hash = h; n.used = true;
        memcpy(&node_tok[(size_t)id * cfg.block_size], t, sizeof(int32_t) * cfg.block_size);
        if (parent >= 0) ++node[parent].children;
        map.emplace(h, id);
        return id;
    }
    void drop_if_empty(int32_t id) {  // nodes without a block and without longer prefixes below them go, upwards
        while (id >= 0 && node[id].block < 0 && node[id].children == 0) {
            Node &n = node[id];
            auto range = map.equal_range(n.hash);
            for (auto it = range.first; it != range.second; ++it)
                if (it->second == id) { map.erase(it); break; }
            int32_t up = n.parent;
            n.used = false;
            node_free.push_back(id);
            if (up >= 0) --node[up].children;
            id = up;
        }
    }
    void lru_remove(int32_t b) {
        Block &x = blk[b];
        if (x.lru_prev >= 0) blk[x.lru_prev].lru_next = x.lru_next; else lru_head = x.lru_next;
        if (x.lru_next >= 0) blk[x.lru_next].lru_prev = x.lru_prev; else lru_tail = x.lru_prev;
        x.lru_prev = x.lru_next = -1;
        --n_lru;
    }
    void lru_push_back(int32_t b) {
        Block &x = blk[b];
        x.lru_prev = lru_tail; x.lru_next = -1;
        if (lru_tail >= 0) blk[lru_tail].lru_next = b; else lru_head = b;
        lru_tail = b;
        ++n_lru;
    }
    int32_t take() {  // caller has checked that a block is available
        int32_t b;
        if (!free_q.empty()) {
            b = free_q.front();
            free_q.pop_front();
        } else {
            b = lru_head;
            lru_remove(b);
            int32_t n = blk[b].node;
            node[n].block = -1;
            blk[b].node = -1;
            drop_if_empty(n);
            ++st.evictions;
        }
        blk[b].ref = 1;
        ++n_live;
        if (n_live > st.peak_live) st.peak_live = n_live;
        return b;
    }
    int model_key(int32_t model) const { return cfg.key_by_model ? model : -1; }
    icarus_status fail(icarus_status s, const std::string &m) { err = m; return s; }
};

static std::string g_cache_create_error;

extern "C" {

icarus_status icarus_cache_create(const icarus_cache_config *cfg, icarus_cache **out) {
    if (!cfg || !out) { g_cache_create_error = "null argument"; return ICARUS_ERR_INVALID_ARG; }
    if (cfg->num_blocks < 1 || cfg->block_size < 1) { g_cache_create_error = "num_blocks and block_size must be >= 1"; return ICARUS_ERR_SHAPE; }
    icarus_cache *c = new icarus_cache;
    c->cfg = *cfg;
    c->blk.resize(cfg->num_blocks);
    for (int32_t b = 0; b < cfg->num_blocks; ++b) c->free_q.push_back(b);
    *out = c;
    return ICARUS_OK;
}

void icarus_cache_destroy(icarus_cache *c) { delete c; }

const char *icarus_cache_last_error(const icarus_cache *c) { return c ? c->err.c_str() : g_cache_create_error.c_str(); }

icarus_status icarus_cache_acquire(icarus_cache *c, const int32_t *tokens, int32_t n_tokens, int32_t model,
                                   int32_t reserve_tokens, int32_t *blocks, int32_t max_blocks, int32_t *n_blocks,
                                   int32_t *n_cached_tokens) {
    if (!c) return ICARUS_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lk(c->mu);
    if (!tokens || !blocks || !n_blocks || !n_cached_tokens || n_tokens < 1 || reserve_tokens < 0 || max_blocks < 0)
        return c->fail(ICARUS_ERR_INVALID_ARG, "acquire: null pointer, empty context or negative size");
    if (c->cfg.key_by_model && model < 0) return c->fail(ICARUS_ERR_MODEL_ID, "acquire: adapter id must be >= 0 when keys carry it");
    const int B = c->cfg.block_size, mk = c->model_key(model);
    const int64_t total = ((int64_t)n_tokens + reserve_tokens + B - 1) / B;
    if (total > max_blocks) return c->fail(ICARUS_ERR_CAPACITY, "acquire: the sequence needs " + std::to_string(total) + " blocks, max_blocks is " + std::to_string(max_blocks));
    int32_t hits = 0, parent = -1, hits_in_lru = 0;
    for (int i = 0; i < (n_tokens - 1) / B; ++i) {
        int32_t n = c->find_node(parent, parent < 0 ? mk : -1, tokens + (size_t)i * B);
        if (n < 0 || c->node[n].block < 0) break;
        int32_t b = c->node[n].block;
        blocks[hits++] = b;
        if (c->blk[b].ref == 0) ++hits_in_lru;
        parent = n;
    }
    const int64_t need = total - hits;
    if ((int64_t)c->free_q.size() + c->n_lru - hits_in_lru < need)
        return c->fail(ICARUS_ERR_CAPACITY, "acquire: " + std::to_string(need) + " fresh blocks needed, " + std::to_string(c->free_q.size()) +
                                                " free and " + std::to_string(c->n_lru - hits_in_lru) + " evictable");
    for (int i = 0; i < hits; ++i) {
        Block &x = c->blk[blocks[i]];
        if (x.ref == 0) { c->lru_remove(blocks[i]); ++c->n_live; }
        ++x.ref;
    }
    if (c->n_live > c->st.peak_live) c->st.peak_live = c->n_live;
    for (int64_t i = 0; i < need; ++i) blocks[hits + i] = c->take();
    *n_blocks = (int32_t)total;
    *n_cached_tokens = hits * B;
    ++c->st.lookups;
    c->st.hit_tokens += (int64_t)hits * B;
    c->st.miss_tokens += n_tokens - (int64_t)hits * B;
    return ICARUS_OK;
}

icarus_status icarus_cache_extend(icarus_cache *c, int32_t *blocks, int32_t max_blocks, int32_t *n_blocks, int32_t n_tokens_total) {
    if (!c) return ICARUS_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lk(c->mu);
    if (!blocks || !n_blocks || *n_blocks < 0 || n_tokens_total < 0 || max_blocks < *n_blocks)
        return c->fail(ICARUS_ERR_INVALID_ARG, "extend: null pointer or negative size");
    const int B = c->cfg.block_size;
    const int64_t total = ((int64_t)n_tokens_total + B - 1) / B, need = total - *n_blocks;
    if (need <= 0) return ICARUS_OK;
    if (total > max_blocks) return c->fail(ICARUS_ERR_CAPACITY, "extend: the sequence needs " + std::to_string(total) + " blocks, max_blocks is " + std::to_string(max_blocks));
    if ((int64_t)c->free_q.size() + c->n_lru < need)
        return c->fail(ICARUS_ERR_CAPACITY, "extend: " + std::to_string(need) + " fresh blocks needed, " + std::to_string(c->free_q.size() + c->n_lru) + " available");
    for (int64_t i = 0; i < need; ++i) blocks[*n_blocks + i] = c->take();
    *n_blocks = (int32_t)total;
    return ICARUS_OK;
}

icarus_status icarus_cache_commit(icarus_cache *c, const int32_t *tokens, int32_t n_tokens, int32_t model, const int32_t *blocks,
                                  int32_t n_blocks) {
    if (!c) return ICARUS_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lk(c->mu);
    if (!tokens || !blocks || n_tokens < 0 || n_blocks < 0) return c->fail(ICARUS_ERR_INVALID_ARG, "commit: null pointer or negative size");
    if (c->cfg.key_by_model && model < 0) return c->fail(ICARUS_ERR_MODEL_ID, "commit: adapter id must be >= 0 when keys carry it");
    const int B = c->cfg.block_size, mk = c->model_key(model);
    const int full = std::min(n_tokens / B, n_blocks);
    for (int i = 0; i < full; ++i)
        if (blocks[i] < 0 || blocks[i] >= c->cfg.num_blocks || c->blk[blocks[i]].ref < 1)
            return c->fail(ICARUS_ERR_INVALID_ARG, "commit: block " + std::to_string(i) + " of the sequence is not live");
    int32_t parent = -1;  // node of the prefix before block i
    for (int i = 0; i < full; ++i) {
        const int32_t b = blocks[i];
        if (c->blk[b].node >= 0) {  // published already (a hit block, or an earlier commit)
            parent = c->blk[b].node;
            continue;
        }
        const int32_t *t = tokens + (size_t)i * B;
        uint64_t h;
        int32_t n = c->find_node(parent, parent < 0 ? mk : -1, t, &h);
        if (n < 0) n = c->new_node(parent, parent < 0 ? mk : -1, t, h);
        if (c->node[n].block < 0) {
            c->node[n].block = b;
            c->blk[b].node = n;
        }  // else another block holds this prefix: b stays private
        parent = n;
    }
    return ICARUS_OK;
}

icarus_status icarus_cache_release(icarus_cache *c, const int32_t *blocks, int32_t n_blocks) {
    if (!c) return ICARUS_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lk(c->mu);
    if ((!blocks && n_blocks) || n_blocks < 0) return c->fail(ICARUS_ERR_INVALID_ARG, "release: null pointer or negative size");
    {   // every id valid, and no block released more often than it is referenced
        std::unordered_map<int32_t, int32_t> cnt;
        for (int i = 0; i < n_blocks; ++i) {
            if (blocks[i] < 0 || blocks[i] >= c->cfg.num_blocks) return c->fail(ICARUS_ERR_INVALID_ARG, "release: block id out of range");
            if (++cnt[blocks[i]] > c->blk[blocks[i]].ref) return c->fail(ICARUS_ERR_INVALID_ARG, "release: block " + std::to_string(blocks[i]) + " is not referenced that often");
        }
    }
    for (int i = n_blocks - 1; i >= 0; --i) {
        Block &x = c->blk[blocks[i]];
        if (--x.ref == 0) {
            --c->n_live;
            if (x.node >= 0) c->lru_push_back(blocks[i]);
            else c->free_q.push_back(blocks[i]);
        }
    }
    return ICARUS_OK;
}

icarus_status icarus_cache_get_stats(icarus_cache *c, icarus_cache_stats *out) {
    if (!c || !out) return ICARUS_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lk(c->mu);
    *out = c->st;
    out->live = c->n_live;
    out->cached = c->n_lru;
    out->free_blocks = (int32_t)c->free_q.size();
    return ICARUS_OK;
}

}  // extern "C"
