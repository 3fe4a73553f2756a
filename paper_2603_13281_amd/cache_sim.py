"""Drive a prefix-cache manager through a schedule of agent turns and count what it had to do.

Works on any object with acquire / extend / commit / release / counts (the library's manager through
binding.PrefixCache in the product, the oracle's in tests): it holds none of the bookkeeping itself.
"""
from __future__ import annotations

import numpy as np


def run_schedule(cache, schedule, record=None):
    """Every turn: acquire the context (a prefix of it may be cached), "prefill" the rest, "decode" the
    agent's tokens (the sequence grows block by block), publish what is now cached, release.
    The observation that follows is text: it is prefilled by whoever is invoked next.
    Returns totals; `record`, a list, receives (blocks, n_cached) of every acquire for comparisons."""
    prefill_tokens = hit_tokens = context_tokens = 0
    for t in schedule:
        ctx = t.context
        blocks, n_cached = cache.acquire(ctx, t.model, reserve=0)
        if record is not None:
            record.append((list(blocks), int(n_cached)))
        prefill_tokens += len(ctx) - n_cached
        hit_tokens += n_cached
        context_tokens += len(ctx)
        seq = np.concatenate([ctx, t.new_tokens[: t.n_generated]])
        blocks = cache.extend(blocks, len(seq))
        if record is not None:
            record.append((list(blocks), -1))
        cache.commit(seq, t.model, blocks)
        cache.release(blocks)
    out = dict(cache.counts())
    out.update(prefill_tokens=prefill_tokens, hit_tokens_total=hit_tokens, context_tokens=context_tokens, turns=len(schedule))
    return out
