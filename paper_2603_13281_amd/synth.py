"""Seeded synthetic inputs for the ICaRus shared-KV layer step.

Serves the tests, the benchmark and the smoke check.  Holds none of the method's
arithmetic: only shapes, seeded random draws, storage-precision rounding of the
*inputs* (through torch's bfloat16 cast) and the bookkeeping of a paged batch
(lengths, active model sets, permuted block tables, row lists).

Workload recipe (stands in for the paper's agent-serving traffic, Sec. 4.3 and
App. A.2, whose datasets are not available): base weights N(0, 0.02), LoRA A and
B N(0, 0.02) with scale 2.0 (the paper's alpha/r = 256/128), norm weights 1,
hidden rows N(0, 1), directly filled caches K, V ~ N(0, 1); eight adapters on
one GPU, long shared contexts, a subset of agents active per sequence.
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass

import numpy as np
import torch

PROJ = ("q", "k", "v", "o", "gate", "up", "down")
ALL_TARGETS = 0x7F
QVO_TARGETS = 0b0001101  # q, v, o


@dataclass(frozen=True)
class LayerShape:
    name: str
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    n_models: int
    lora_rank: int
    lora_target_mask: int = ALL_TARGETS
    qk_norm: bool = False
    bf16: bool = True
    rope_theta: float = 5e5
    rms_eps: float = 1e-5
    lora_scale: float = 2.0
    block_size: int = 16

    def proj_in(self, p: str) -> int:
        return {"q": self.d_model, "k": self.d_model, "v": self.d_model, "gate": self.d_model,
                "up": self.d_model, "o": self.n_q_heads * self.head_dim, "down": self.d_ffn}[p]

    def proj_out(self, p: str) -> int:
        return {"q": self.n_q_heads * self.head_dim, "k": self.n_kv_heads * self.head_dim,
                "v": self.n_kv_heads * self.head_dim, "gate": self.d_ffn, "up": self.d_ffn,
                "o": self.d_model, "down": self.d_model}[p]

    def replace(self, **kw) -> "LayerShape":
        return dataclasses.replace(self, **kw)


# The five benchmark configurations' layer shapes.
TINY = LayerShape("tiny-fp32", 256, 4, 4, 64, 688, 2, 8, QVO_TARGETS, False, False, 1e4, 1e-5)
LLAMA8B = LayerShape("llama3-8b-layer", 4096, 32, 8, 128, 14336, 8, 16, ALL_TARGETS, False, True, 5e5, 1e-5)
QWEN32B = LayerShape("qwen3-32b-layer", 5120, 64, 8, 128, 25600, 8, 32, ALL_TARGETS, True, True, 1e6, 1e-6)
# Reduced shapes with the same structure (GQA group, head_dim, rank) for fast parity cases.
LLAMA_SMALL = LayerShape("llama-small", 512, 8, 2, 128, 1024, 4, 16, ALL_TARGETS, False, True, 5e5, 1e-5)
QWEN_SMALL = LayerShape("qwen-small", 512, 16, 2, 128, 768, 3, 32, ALL_TARGETS, True, True, 1e6, 1e-6)


def _rng(seed: int, stream: str) -> np.random.Generator:
    names = ("weights", "lora", "hidden", "kv", "lens", "active", "perm", "norm", "misc")
    return np.random.default_rng(np.random.SeedSequence([seed, names.index(stream)]))


def to_storage(a: np.ndarray, bf16: bool) -> np.ndarray:
    """Round float32 values to what the storage dtype can hold (returned as float32)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if not bf16:
        return a
    return torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()


def make_base(shape: LayerShape, seed: int = 0, norm_ones: bool = True) -> dict:
    rng = _rng(seed, "weights")
    base = {}
    for p in PROJ:
        w = rng.standard_normal((shape.proj_out(p), shape.proj_in(p)), dtype=np.float32) * np.float32(0.02)
        base[p] = to_storage(w, shape.bf16)
    nr = _rng(seed, "norm")
    def norm(n):
        if norm_ones:
            return np.ones(n, dtype=np.float32)
        return to_storage(1.0 + 0.1 * nr.standard_normal(n, dtype=np.float32), shape.bf16)
    base["norm_attn"] = norm(shape.d_model)
    base["norm_ffn"] = norm(shape.d_model)
    if shape.qk_norm:
        base["q_norm"] = norm(shape.head_dim)
        base["k_norm"] = norm(shape.head_dim)
    return base


def make_lora(shape: LayerShape, seed: int = 0, zero_b: bool = False, std: float = 0.02) -> dict:
    """Adapters for every projection (k and v included: the path must never read them)."""
    rng = _rng(seed, "lora")
    lora = {}
    M, r = shape.n_models, shape.lora_rank
    for p in PROJ:
        A = rng.standard_normal((M, r, shape.proj_in(p)), dtype=np.float32) * np.float32(std)
        B = rng.standard_normal((M, shape.proj_out(p), r), dtype=np.float32) * np.float32(std)
        if zero_b:
            B[:] = 0
        lora[p] = (to_storage(A, shape.bf16), to_storage(B, shape.bf16))
    return lora


def make_stack(shape: LayerShape, n_layers: int, vocab: int, seed: int = 0, zero_b: bool = False, lora_std: float = 0.02,
               norm_ones: bool = False) -> dict:
    """Weights of a stack of layers with token embedding, final norm and LM head (all seeded):
    {"bases": [...], "loras": [...], "embed" [vocab, d], "final_norm" [d], "lm_head" [vocab, d]}."""
    bases = [make_base(shape, seed=seed * 1000 + l, norm_ones=norm_ones) for l in range(n_layers)]
    loras = [make_lora(shape, seed=seed * 1000 + l, zero_b=zero_b, std=lora_std) for l in range(n_layers)]
    rng = np.random.default_rng(np.random.SeedSequence([seed, 9, n_layers, vocab]))
    embed = to_storage(rng.standard_normal((vocab, shape.d_model), dtype=np.float32), shape.bf16)
    lm_head = to_storage(rng.standard_normal((vocab, shape.d_model), dtype=np.float32) * np.float32(0.05), shape.bf16)
    fn = np.ones(shape.d_model, dtype=np.float32) if norm_ones else \
        to_storage(1.0 + 0.1 * rng.standard_normal(shape.d_model, dtype=np.float32), shape.bf16)
    return {"bases": bases, "loras": loras, "embed": embed, "final_norm": fn, "lm_head": lm_head}


def make_hidden(shape: LayerShape, n_rows: int, seed: int = 0, tag: int = 0) -> np.ndarray:
    rng = np.random.default_rng(np.random.SeedSequence([seed, 2, tag]))
    return to_storage(rng.standard_normal((n_rows, shape.d_model), dtype=np.float32), shape.bf16)


@dataclass
class Batch:
    """A paged decode batch: bookkeeping only."""
    ctx_lens: np.ndarray      # [S] tokens cached before the step
    block_tables: np.ndarray  # [S, max_blocks] int32
    num_blocks: int
    row_seq: np.ndarray       # [R]
    row_model: np.ndarray     # [R], -1 = encoder row
    active: list              # per sequence: sorted model ids

    @property
    def S(self) -> int:
        return len(self.ctx_lens)

    @property
    def R(self) -> int:
        return len(self.row_seq)

    @property
    def n_decoder_rows(self) -> int:
        return int((self.row_model >= 0).sum())


def make_batch(shape: LayerShape, ctx_lens, n_active, seed: int = 0, headroom: int = 1,
               pool_factor: float = 1.5, permute: bool = True, shuffle_models: bool = True) -> Batch:
    """ctx_lens [S]; n_active [S] models active per sequence (0..M).

    Every sequence gets blocks for ctx_len + headroom tokens out of a pool
    pool_factor times larger, drawn as a random permutation of the pool.
    """
    ctx_lens = np.asarray(ctx_lens, dtype=np.int32)
    n_active = np.asarray(n_active, dtype=np.int32)
    S = len(ctx_lens)
    Bk = shape.block_size
    need = [(int(L) + headroom + Bk - 1) // Bk for L in ctx_lens]
    max_blocks = max(need) if need else 1
    num_blocks = max(int(np.ceil(sum(need) * pool_factor)), sum(need), 1)
    perm_rng = _rng(seed, "perm")
    ids = perm_rng.permutation(num_blocks) if permute else np.arange(num_blocks)
    bt = np.zeros((S, max_blocks), dtype=np.int32)
    k = 0
    for s in range(S):
        bt[s, :need[s]] = ids[k:k + need[s]]
        k += need[s]
    act_rng = _rng(seed, "active")
    row_seq, row_model, active = [], [], []
    for s in range(S):
        m = int(n_active[s])
        chosen = act_rng.choice(shape.n_models, size=m, replace=False) if m > 0 else np.zeros(0, dtype=np.int64)
        if not shuffle_models:
            chosen = np.sort(chosen)
        active.append([int(j) for j in chosen])
        row_seq.append(s)
        row_model.append(-1)
        for j in chosen:
            row_seq.append(s)
            row_model.append(int(j))
    return Batch(ctx_lens, bt, num_blocks, np.asarray(row_seq, dtype=np.int32),
                 np.asarray(row_model, dtype=np.int32), active)


def draw_lens(seed: int, S: int, lo: int, hi: int) -> np.ndarray:
    return _rng(seed, "lens").integers(lo, hi + 1, size=S).astype(np.int32)


def draw_active_counts(seed: int, S: int, lo: int, hi: int) -> np.ndarray:
    return np.random.default_rng(np.random.SeedSequence([seed, 5, 1])).integers(lo, hi + 1, size=S).astype(np.int32)


def make_kv_tokens(shape: LayerShape, n_tokens: int, seed: int = 0, tag: int = 0):
    """K, V [n_tokens, Hkv, D] ~ N(0,1) in storage precision, for directly filled caches."""
    rng = np.random.default_rng(np.random.SeedSequence([seed, 3, tag]))
    K = rng.standard_normal((n_tokens, shape.n_kv_heads, shape.head_dim), dtype=np.float32)
    V = rng.standard_normal((n_tokens, shape.n_kv_heads, shape.head_dim), dtype=np.float32)
    return to_storage(K, shape.bf16), to_storage(V, shape.bf16)


# ---- multi-agent conversations for the prefix-cache manager -----------------------------------
@dataclass
class AgentTurn:
    conversation: int
    model: int
    context: np.ndarray      # int32: every token the agent sees when it is invoked (prompt + all earlier turns)
    new_tokens: np.ndarray   # int32: what this turn appends (the agent's output, then the tool observation)
    n_generated: int         # how many of new_tokens the agent generates itself (the rest is observation text)


def make_agent_schedule(n_conversations: int, n_models: int, turns: int, seed: int = 0, pattern: str = "round_robin",
                        prompt_len=(600, 1400), out_len=(40, 160), obs_len=(60, 400), shared_system_prompt: int = 256,
                        concurrency: int = 4, vocab: int = 32000):
    """Seeded stand-in for the paper's agentic workload (Sec. 4.3, App. A.2: a ReAct-style loop in which a
    controller hands one shared, growing context to one of N task agents per turn; App. F: `skewed` = one
    agent is chosen with probability 1/2, the others share the rest at random; `round_robin` = fixed order).
    Conversations start with a system prompt common to all of them, then their own question; every turn
    appends the agent's output and an observation.  `concurrency` conversations are in progress at a time and
    take turns in rotation.  Returns the list of AgentTurn in service order."""
    rng = np.random.default_rng(np.random.SeedSequence([seed, 1009, n_conversations, n_models, turns, 0 if pattern == "round_robin" else 1]))
    system = rng.integers(0, vocab, size=shared_system_prompt, dtype=np.int32)
    ctx, done, model_next = {}, {}, {}
    for c in range(n_conversations):
        n = int(rng.integers(prompt_len[0], prompt_len[1] + 1))
        ctx[c] = np.concatenate([system, rng.integers(0, vocab, size=max(1, n - shared_system_prompt), dtype=np.int32)])
        done[c] = 0
        model_next[c] = int(rng.integers(0, n_models))
    out = []
    active, waiting = [], list(range(n_conversations))
    while active or waiting:
        while waiting and len(active) < concurrency:
            active.append(waiting.pop(0))
        c = active.pop(0)
        if pattern == "round_robin":
            m = model_next[c]
            model_next[c] = (m + 1) % n_models
        elif pattern == "skewed":
            m = 0 if (n_models == 1 or rng.random() < 0.5) else int(rng.integers(1, n_models))
        else:
            raise ValueError(pattern)
        n_out = int(rng.integers(out_len[0], out_len[1] + 1))
        n_obs = int(rng.integers(obs_len[0], obs_len[1] + 1))
        new = rng.integers(0, vocab, size=n_out + n_obs, dtype=np.int32)
        out.append(AgentTurn(c, m, ctx[c].copy(), new, n_out))
        ctx[c] = np.concatenate([ctx[c], new])
        done[c] += 1
        if done[c] < turns:
            active.append(c)
    return out


def make_full_decoders(shape: LayerShape, base: dict, seed: int = 0, std: float = 0.01) -> dict:
    """Private full weights of every decoder (full fine-tuning, or adapters merged into the weights): the base
    weight plus an independent N(0, std) perturbation per model, in storage precision.  p -> [M, out_p, in_p]
    for the projections a decoder owns (q, o, gate, up, down; K and V stay the encoder's)."""
    out = {}
    for k, p in enumerate(("q", "o", "gate", "up", "down")):
        rng = np.random.default_rng(np.random.SeedSequence([seed, 2027, k]))
        w = base[p].astype(np.float32)
        out[p] = to_storage(w[None] + rng.standard_normal((shape.n_models,) + w.shape).astype(np.float32) * std, shape.bf16)
    return out
