"""Pins of the prefix-cache oracle (oracle/prefix_cache.py) against what the paper and the policy fix:
hand-worked cases, the memory argument of Table 1 as a closed form, invariants under random schedules."""
import numpy as np
import pytest

from oracle.prefix_cache import CacheFull, OraclePrefixCache
from paper_2603_13281_amd import cache_sim, synth


def toks(*ranges):
    return np.concatenate([np.arange(a, b, dtype=np.int32) for a, b in ranges])


def test_hand_worked_cross_model_hit_and_lru():
    """Block size 4, 6 blocks.  Worked by hand from the policy."""
    c = OraclePrefixCache(6, 4, key_by_model=False)
    p = toks((100, 110))                                     # 10 tokens: 2 full blocks + 2
    b, hit = c.acquire(p, model=0)
    assert (b, hit) == ([0, 1, 2], 0)                        # nothing cached; fresh blocks in id order
    c.commit(p, 0, b)                                        # publishes blocks 0, 1 (block 2 is not full)
    c.release(b)                                             # 2 -> free queue (back); then 1, 0 -> eviction queue
    assert list(c.lru) == [1, 0] and list(c.free) == [3, 4, 5, 2]
    # another model, same prompt + 3 more tokens: both full blocks hit (13 tokens: at most 12 // 4 = 3 blocks may hit)
    q = np.concatenate([p, toks((200, 203))])
    b2, hit2 = c.acquire(q, model=5)
    assert hit2 == 8 and b2 == [0, 1, 3, 4]
    c.commit(q, 5, b2)                                       # publishes block 3 (tokens 8..11); block 4 holds 1 token
    c.release(b2)
    assert list(c.lru) == [3, 1, 0] and list(c.free) == [5, 2, 4]
    # a prompt that is exactly 2 blocks long: one token must be left to compute, so only 1 block may hit
    b3, hit3 = c.acquire(p[:8], model=1)
    assert hit3 == 4 and b3 == [0, 5]
    c.release(b3)                                            # block 5 unpublished -> free; block 0 -> most recent
    assert list(c.lru) == [3, 1, 0] and list(c.free) == [2, 4, 5]
    # fill the pool: 5 fresh blocks needed, 3 free -> evicts the two least recently released: 3, then 1
    z = toks((900, 920))
    b4, hit4 = c.acquire(z, model=0)
    assert hit4 == 0 and b4 == [2, 4, 5, 3, 1] and c.stats["evictions"] == 2
    # block 1 is gone, so the old prompt hits only its first block now; and nothing is left to allocate from
    with pytest.raises(CacheFull):
        c.acquire(q, model=0)
    assert c.ref[0] == 0 and list(c.lru) == [0]              # the failed call changed nothing
    c.release(b4)


def test_per_model_keys_do_not_cross():
    c = OraclePrefixCache(16, 4, key_by_model=True)
    p = toks((0, 13))
    b, _ = c.acquire(p, 0); c.commit(p, 0, b); c.release(b)
    assert c.acquire(p, 1)[1] == 0                           # another adapter: no reuse (baseline system)
    c2 = OraclePrefixCache(16, 4, key_by_model=True)
    b, _ = c2.acquire(p, 0); c2.commit(p, 0, b); c2.release(b)
    assert c2.acquire(p, 0)[1] == 12                         # the same adapter: 3 full blocks


def test_duplicate_content_is_published_once():
    c = OraclePrefixCache(16, 4, key_by_model=False)
    p = toks((0, 9))
    a, _ = c.acquire(p, 0)
    b, hb = c.acquire(p, 1)                                  # concurrent: nothing published yet
    assert hb == 0 and set(a).isdisjoint(b)
    c.commit(p, 0, a); c.commit(p, 1, b)                     # second commit finds the keys taken
    c.release(b)
    assert len(c.lru) == 0 and len(c.free) == 16 - 3         # b's blocks were private: straight back to free
    c.release(a)
    assert list(c.lru) == [a[1], a[0]]


@pytest.mark.parametrize("n_models", [2, 4, 8])
def test_table1_memory_closed_form(n_models):
    """Table 1: one context of L_t tokens served by N adapters in turn occupies ceil-blocks(L_t) blocks when the
    cache is shared and N times as many (each adapter its own copy) in the baseline; the baseline prefills every
    token once per adapter, the shared cache once."""
    B, L0, grow, rounds = 16, 640, 64, 3
    rng = np.random.default_rng(3)
    text = rng.integers(0, 1000, size=L0 + grow * n_models * rounds + 1).astype(np.int32)
    res = {}
    for per_model in (False, True):
        c = OraclePrefixCache(4096, B, key_by_model=per_model)
        n, prefilled = L0, 0
        for turn in range(n_models * rounds):
            m = turn % n_models
            blocks, hit = c.acquire(text[:n], m)
            prefilled += n - hit
            n += grow                                         # the agent and its tool add `grow` tokens
            blocks = c.extend(blocks, n)
            c.commit(text[:n], m, blocks)
            c.release(blocks)
        res[per_model] = (c.counts()["cached"], prefilled, n)
    (shared_blocks, shared_prefill, n), (base_blocks, base_prefill, _) = res[False], res[True]
    assert shared_blocks == n // B                            # one copy of the context
    # baseline: adapter m last saw the context at its last turn: n - grow * (N - 1 - m') tokens
    assert base_blocks == sum((n - grow * k) // B for k in range(n_models))
    assert base_blocks > (n_models - 1) * shared_blocks
    # shared: the prompt once; afterwards everything is cached except the one block a hit must leave (L0, grow
    # are multiples of B, so that is exactly B tokens per turn): what the agents generate is cached as they decode
    turns = n_models * rounds
    assert shared_prefill == L0 + (turns - 1) * B
    # baseline: adapter m first sees L0 + m grow tokens and has none of them; at each later turn the other N - 1
    # adapters have added (N - 1) grow tokens that it must prefill itself
    assert base_prefill == sum(L0 + m * grow for m in range(n_models)) + (rounds - 1) * n_models * (n_models - 1) * grow


@pytest.mark.parametrize("pattern", ["round_robin", "skewed"])
@pytest.mark.parametrize("per_model", [False, True])
def test_invariants_on_agent_schedules(pattern, per_model):
    sched = synth.make_agent_schedule(12, 4, 5, seed=2, pattern=pattern, prompt_len=(300, 700), concurrency=3)
    c = OraclePrefixCache(260, 16, key_by_model=per_model)      # small pool: evictions happen
    rec = []
    out = cache_sim.run_schedule(c, sched, record=rec)
    assert out["evictions"] > 0
    assert out["live"] == 0 and out["cached"] + out["free"] == 260
    assert all(r == 0 for r in c.ref)
    # a block is in exactly one of: free queue, eviction queue
    assert sorted(list(c.free) + list(c.lru)) == list(range(260))
    # published keys and blocks are a bijection
    assert len(c.block_of) == sum(k is not None for k in c.key_of)
    for k, b in c.block_of.items():
        assert c.key_of[b] == k
    # a hit never exceeds the context, is whole blocks, and leaves a token to compute
    for t, (blocks, hit) in zip(sched, rec[::2]):
        assert hit % 16 == 0 and hit <= len(t.context) - 1 and len(blocks) == -(-len(t.context) // 16)
        assert len(set(blocks)) == len(blocks)
    assert out["prefill_tokens"] + out["hit_tokens_total"] == out["context_tokens"]


def test_shared_cache_never_prefills_more_than_per_model():
    for pattern in ("round_robin", "skewed"):
        sched = synth.make_agent_schedule(10, 8, 6, seed=5, pattern=pattern, prompt_len=(300, 700))
        r = {}
        for per_model in (False, True):
            r[per_model] = cache_sim.run_schedule(OraclePrefixCache(100000, 16, per_model), sched)
        assert r[False]["prefill_tokens"] < r[True]["prefill_tokens"]
        assert r[False]["cached"] < r[True]["cached"]
