"""Cross-model prefix reuse end to end: the manager's block tables drive the layer stack on the GPU.

Agent 0 works on a prompt; agent 2 is then invoked on the same context plus new text.  With ICaRus keys the
manager returns the blocks agent 0's request filled, only the new tokens are prefilled, and the result must
be what the stack oracle computes from scratch for the whole context (Sec. 3.2: the cache is the base
model's, whichever adapter decodes).  With per-adapter keys (the baseline system) nothing may be reused."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_second_model_reuses_first_models_blocks():
    from test_gpu_stack import _build, _check_tokens
    from paper_2603_13281_amd import binding, synth

    shape, n_layers, vocab, tol = synth.LLAMA_SMALL, 3, 1024, 2e-2
    Bk = shape.block_size
    num_blocks, max_blocks = 40, 8
    wts, orc, stack, pools = _build(shape, n_layers, vocab, num_blocks, seed=21)
    for p in pools:                       # stale data everywhere: a wrong block would show
        p.normal_()
    cache = binding.PrefixCache(num_blocks, Bk, key_by_model=False)
    baseline = binding.PrefixCache(num_blocks, Bk, key_by_model=True)
    rng = np.random.default_rng(8)
    prompt = rng.integers(0, vocab, size=75).astype(np.int32)

    def table(blocks):
        bt = np.zeros((1, max_blocks), dtype=np.int32)
        bt[0, :len(blocks)] = blocks
        return bt, torch.from_numpy(bt).to("cuda:0")

    # ---- agent 0: whole prompt, three greedy tokens --------------------------------------------------
    blocks, hit = cache.acquire(prompt, model=0, reserve=3)
    assert hit == 0
    bt, dbt = table(blocks)
    nxt, _ = stack.prefill(pools, dbt, [0], [len(prompt)], prompt)
    seq = list(prompt)
    tok = nxt.clone()
    for t in range(3):
        seq.append(int(tok.cpu()[0]))
        stack.decode(pools, dbt, [len(seq) - 1], np.int32([0, 0]), np.int32([-1, 0]), tok, seq_next=tok)
    torch.cuda.synchronize()
    seq_a = np.array(seq, dtype=np.int32)                    # 78 tokens: 4 full blocks hold K/V
    cache.commit(seq_a, 0, blocks)
    cache.release(blocks)
    b0, _ = baseline.acquire(prompt, 0, reserve=3); baseline.commit(seq_a, 0, b0); baseline.release(b0)

    # ---- agent 2 on the same context + an observation --------------------------------------------------
    ctx_b = np.concatenate([seq_a, rng.integers(0, vocab, size=11).astype(np.int32)])     # 89 tokens
    assert baseline.acquire(ctx_b, model=2)[1] == 0          # per-adapter keys: recompute everything
    blocks_b, hit_b = cache.acquire(ctx_b, model=2, reserve=2)
    assert hit_b == 64 and blocks_b[:4] == blocks[:4]        # 4 of agent 0's blocks, whatever the adapter
    bt_b, dbt_b = table(blocks_b)
    nxt_b, lg_b = stack.prefill(pools, dbt_b, [hit_b], [len(ctx_b) - hit_b], ctx_b[hit_b:], want_logits=True)
    # oracle: the whole context from scratch in its own pools
    opools = orc.new_pools()
    obt = np.arange(max_blocks, dtype=np.int32)[None]
    want_lg, want_tok = orc.prefill(opools, obt, [0], [len(ctx_b)], ctx_b)
    torch.cuda.synchronize()
    _check_tokens(nxt_b.cpu().numpy(), lg_b.cpu().numpy().astype(np.float64), want_lg, tol, "prefill over reused blocks")
    # one token step of agent 2 (encoder row + its decoder row) over the shared blocks
    cur = want_tok.astype(np.int32)
    row_next, lg = stack.decode(pools, dbt_b, [len(ctx_b)], np.int32([0, 0]), np.int32([-1, 2]), torch.from_numpy(cur).to("cuda:0"),
                                want_logits=True)
    want_lg2, want_rows, _ = orc.decode(opools, obt, [len(ctx_b)], np.int32([0, 0]), np.int32([-1, 2]), cur)
    torch.cuda.synchronize()
    _check_tokens(row_next.cpu().numpy(), lg.cpu().numpy().astype(np.float64), want_lg2, tol, "decode over reused blocks")
    cache.release(blocks_b)
