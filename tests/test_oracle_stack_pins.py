"""Pins of the layer-stack oracle (Alg. 3 outer loop, Alg. 1 for the prompt): multi-layer loop with
per-layer caches, final norm, LM head, greedy token.  Checked against a textbook decoder-only
transformer written with torch library routines in float64 that sees the whole token sequence at
once (no cache, full causal attention), and against the invariants the method states."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_13281_amd import synth
from helpers import oracle_config

SHAPE = synth.TINY.replace(d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ffn=96, n_models=2, lora_rank=4)
QSHAPE = synth.QWEN_SMALL.replace(d_model=96, n_q_heads=6, n_kv_heads=2, head_dim=16, d_ffn=128, lora_rank=4, bf16=False)
VOCAB, LAYERS = 97, 3


def _stack(shape, wts, num_blocks):
    cfg = oracle_config(shape, num_blocks)
    layers = [oracle.Oracle(cfg, b, l) for b, l in zip(wts["bases"], wts["loras"])]
    return oracle.OracleStack(layers, wts["embed"], wts["final_norm"], wts["lm_head"])


def _textbook_logits(shape, wts, tokens, lora_model=None):
    """Whole-sequence decoder-only transformer, float64, torch library routines.  lora_model = j merges
    model j's adapters into every projection except k and v (what a plain fine-tuned decoder on a
    cache it does not write would compute is NOT this; used only with B = 0 or base weights)."""
    F = torch.nn.functional
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    d, Hq, Hkv, D = shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    n = len(tokens)
    x = t(wts["embed"])[torch.as_tensor(tokens, dtype=torch.long)]          # [n, d]
    pos = torch.arange(n, dtype=torch.float64)
    w = torch.tensor(shape.rope_theta, dtype=torch.float64) ** (-torch.arange(D // 2, dtype=torch.float64) * 2 / D)
    rot = torch.polar(torch.ones(n, D // 2, dtype=torch.float64), pos[:, None] * w[None])   # [n, D/2]

    def rope(z):   # [n, H, D]
        c = torch.complex(z[..., :D // 2], z[..., D // 2:]) * rot[:, None, :]
        return torch.cat([c.real, c.imag], dim=-1)
    for base in wts["bases"]:
        xn = F.rms_norm(x, (d,), t(base["norm_attn"]), shape.rms_eps)
        q = F.linear(xn, t(base["q"])).view(n, Hq, D)
        k = F.linear(xn, t(base["k"])).view(n, Hkv, D)
        v = F.linear(xn, t(base["v"])).view(n, Hkv, D)
        if shape.qk_norm:
            q = F.rms_norm(q, (D,), t(base["q_norm"]), shape.rms_eps)
            k = F.rms_norm(k, (D,), t(base["k_norm"]), shape.rms_eps)
        q, k = rope(q), rope(k)
        k, v = k.to(torch.float32).to(torch.float64), v.to(torch.float32).to(torch.float64)   # the cache holds fp32
        g = Hq // Hkv
        a = F.scaled_dot_product_attention(q.permute(1, 0, 2), k.permute(1, 0, 2).repeat_interleave(g, dim=0),
                                           v.permute(1, 0, 2).repeat_interleave(g, dim=0), is_causal=True)
        z = x + F.linear(a.permute(1, 0, 2).reshape(n, Hq * D), t(base["o"]))
        zn = F.rms_norm(z, (d,), t(base["norm_ffn"]), shape.rms_eps)
        x = z + F.linear(F.silu(F.linear(zn, t(base["gate"]))) * F.linear(zn, t(base["up"])), t(base["down"]))
        x = x.to(torch.float32).to(torch.float64)       # layer outputs are stored in fp32
    xn = F.rms_norm(x, (d,), t(wts["final_norm"]), shape.rms_eps)
    return F.linear(xn, t(wts["lm_head"])).numpy()       # [n, vocab]


@pytest.mark.parametrize("shape", [SHAPE, QSHAPE], ids=lambda s: s.name)
def test_stack_equals_textbook_transformer(shape):
    """Prompt through prefill, then teacher-forced decode steps: the base stream's logits at every
    position equal those of a cache-free whole-sequence transformer (Sec. 3.1: with identical
    encoder and decoder the scheme is the ordinary decoder-only model)."""
    wts = synth.make_stack(shape, LAYERS, VOCAB, seed=5, zero_b=True)
    rng = np.random.default_rng(1)
    tokens = rng.integers(0, VOCAB, size=11)
    P = 7
    Bk = shape.block_size
    nb = (len(tokens) + Bk - 1) // Bk + 1
    st = _stack(shape, wts, nb)
    pools = st.new_pools()
    bt = np.arange(nb, dtype=np.int32)[::-1].copy()[None]
    want = _textbook_logits(shape, wts, tokens)
    logits, first = st.prefill(pools, bt, [0], [P], tokens[:P])
    np.testing.assert_allclose(logits[0], want[P - 1], rtol=0, atol=2e-6 * np.abs(want).max())
    assert first[0] == int(np.argmax(want[P - 1]))
    for i in range(P, len(tokens)):
        lg, tok, slots = st.decode(pools, bt, [i], [0, 0], [-1, 1], [tokens[i]])
        np.testing.assert_allclose(lg[0], want[i], rtol=0, atol=2e-6 * np.abs(want).max())
        np.testing.assert_array_equal(lg[1], lg[0])      # B = 0: the decoder stream is the base model
        assert tok[0] == tok[1] == int(np.argmax(want[i]))
        assert slots[0] == int(bt[0, i // Bk]) * Bk + i % Bk


def test_first_token_comes_from_the_base_model_and_caches_ignore_adapters():
    """Alg. 1: the prompt runs through the frozen encoder only, so its caches and the first token do
    not depend on the adapters; later tokens (decoder stream) do."""
    a = synth.make_stack(SHAPE, LAYERS, VOCAB, seed=6, lora_std=0.3)
    b = dict(a, loras=synth.make_stack(SHAPE, LAYERS, VOCAB, seed=7, lora_std=0.3)["loras"])
    tokens = np.random.default_rng(2).integers(0, VOCAB, size=9)
    Bk = SHAPE.block_size
    nb = 2
    bt = np.arange(nb, dtype=np.int32)[None]
    outs = []
    for wts in (a, b):
        st = _stack(SHAPE, wts, nb)
        pools = st.new_pools()
        lg0, first = st.prefill(pools, bt, [0], [len(tokens)], tokens)
        lg1, tok, _ = st.decode(pools, bt, [len(tokens)], [0, 0], [-1, 0], [int(first[0])])
        outs.append((lg0, first, lg1, [p.copy() for p in pools]))
    np.testing.assert_array_equal(outs[0][0], outs[1][0])
    np.testing.assert_array_equal(outs[0][1], outs[1][1])
    for pa, pb in zip(outs[0][3], outs[1][3]):
        np.testing.assert_array_equal(pa, pb)                         # every layer's cache, after prefill and one decode step
    np.testing.assert_array_equal(outs[0][2][0], outs[1][2][0])        # base stream of the decode step
    assert np.abs(outs[0][2][1] - outs[1][2][1]).max() > 1e-3           # decoder stream sees its own adapter


def test_prefill_in_two_chunks_equals_one_chunk():
    wts = synth.make_stack(SHAPE, LAYERS, VOCAB, seed=8)
    tokens = np.random.default_rng(3).integers(0, VOCAB, size=10)
    nb = 2
    bt = np.arange(nb, dtype=np.int32)[None]
    st = _stack(SHAPE, wts, nb)
    p1, p2 = st.new_pools(), st.new_pools()
    lg_a, tok_a = st.prefill(p1, bt, [0], [10], tokens)
    st.prefill(p2, bt, [0], [6], tokens[:6])
    lg_b, tok_b = st.prefill(p2, bt, [6], [4], tokens[6:])
    np.testing.assert_array_equal(lg_a, lg_b)
    np.testing.assert_array_equal(tok_a, tok_b)
    for a, b in zip(p1, p2):
        np.testing.assert_array_equal(a, b)


def test_greedy_token_is_first_maximum():
    """Ties: the first index of the largest logit (two identical LM-head rows)."""
    wts = synth.make_stack(SHAPE, 1, VOCAB, seed=9)
    lm = wts["lm_head"].copy()
    st0 = _stack(SHAPE, wts, 2)
    pools = st0.new_pools()
    bt = np.arange(2, dtype=np.int32)[None]
    lg, tok = st0.prefill(pools, bt, [0], [3], [1, 2, 3])
    best = int(tok[0])
    other = (best + 5) % VOCAB
    lm[other] = lm[best]
    st1 = _stack(SHAPE, dict(wts, lm_head=lm), 2)
    lg1, tok1 = st1.prefill(st1.new_pools(), bt, [0], [3], [1, 2, 3])
    assert lg1[0, other] == lg1[0, best]
    assert int(tok1[0]) == min(best, other)
