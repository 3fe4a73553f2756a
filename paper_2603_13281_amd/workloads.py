"""The benchmark configurations as device-resident workloads (seeded, synthetic).

Builds what bench.py times and what the full-size parity tests sample: layer weights, adapters,
a paged KV pool filled directly with N(0,1) keys and values, permuted block tables, row lists and
hidden rows.  Bookkeeping and uploads only: the layer itself runs in the library.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
import torch

from . import binding, synth


@dataclass
class DecodeWorkload:
    name: str
    description: str
    shape: synth.LayerShape
    batch: synth.Batch
    base: dict            # host float32 (storage-representable) -- the oracle reads these
    lora: dict
    layer: binding.IcarusLayer
    pool: torch.Tensor    # device, library layout
    block_tables: torch.Tensor
    x: list               # rotating device inputs [R, d]
    x_host: list
    headroom: int
    kv_scales: tuple = None   # (k_scale, v_scale) when the pool holds FP8 codes
    full: dict = None         # host float32 private decoder weights p -> [M, out, in] (instead of adapters)

    def ctx_lens(self, step: int) -> np.ndarray:
        return (self.batch.ctx_lens + step).astype(np.int32)

    def kv_bytes(self, step: int) -> int:
        """Algorithmic KV bytes one attention launch reads: each cached token once per sequence."""
        s = self.shape
        es = 1 if self.kv_scales else (2 if s.bf16 else 4)
        return int((self.ctx_lens(step).astype(np.int64) + 1).sum()) * s.n_kv_heads * s.head_dim * 2 * es

    def qo_bytes(self) -> int:
        s = self.shape
        return 2 * self.batch.R * s.n_q_heads * s.head_dim * (2 if s.bf16 else 4)


SPECS = {
    # name: (shape, S, (len_lo, len_hi), (act_lo, act_hi), description)
    "c2": (synth.LLAMA8B, 1, (4096, 4096), (8, 8),
           "config 2: Llama-3-8B-shaped layer, M=8 rank-16 adapters, 1 sequence, 4096-token shared prefix"),
    "c3": (synth.LLAMA8B, 64, (1024, 16384), (1, 8),
           "config 3: multi-agent decode batch, Llama-3-8B-shaped layer, M=8, 64 sequences, shared contexts "
           "U[1024,16384], 1-8 models active per sequence, permuted block tables"),
    "c5": (synth.QWEN32B, 16, (32768, 32768), (8, 8),
           "config 5: Qwen3-32B-shaped layer (QK-RMSNorm), M=8 rank-32 adapters, 16 sequences, 32768-token "
           "shared contexts, all models active"),
    # reduced stand-ins for quick runs and tests
    "c3-small": (synth.LLAMA_SMALL.replace(n_models=8), 16, (100, 3000), (1, 8), "reduced config 3"),
}
SPECS["c3-fp8"] = SPECS["c3"][:4] + (SPECS["c3"][4] + "; KV cache in FP8 E4M3 (static scales)",)
SPECS["c3-small-fp8"] = SPECS["c3-small"][:4] + ("reduced config 3, FP8 KV cache",)
SPECS["c3-full"] = SPECS["c3"][:4] + (SPECS["c3"][4] + "; decoders with private full weights instead of adapters",)
SPECS["c3-small-full"] = SPECS["c3-small"][:4] + ("reduced config 3, private decoder weights",)
SPECS["c5-fp8"] = SPECS["c5"][:4] + (SPECS["c5"][4] + "; KV cache in FP8 E4M3 (static scales)",)
FP8_POOL_SCALE = 4.0 / 448.0   # the synthetic cache is N(0,1) clipped at 4 sigma: 4 sigma -> the largest code


def upload(a: np.ndarray, bf16: bool, device) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.to(device=device, dtype=torch.bfloat16 if bf16 else torch.float32).contiguous()


def layer_config(shape: synth.LayerShape, num_blocks: int, max_position: int) -> binding.LayerConfig:
    return binding.LayerConfig(
        d_model=shape.d_model, n_q_heads=shape.n_q_heads, n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim,
        d_ffn=shape.d_ffn, block_size=shape.block_size, num_blocks=num_blocks, n_models=shape.n_models,
        lora_rank=shape.lora_rank, lora_target_mask=shape.lora_target_mask, bf16=shape.bf16, qk_norm=shape.qk_norm,
        max_position=max_position, rope_theta=shape.rope_theta, rms_eps=shape.rms_eps, lora_scale=shape.lora_scale)


def build_decode_workload(name: str, device="cuda:0", headroom: int = 128, seed: int = 0, n_x: int = 4,
                          verbose: bool = False) -> DecodeWorkload:
    shape, S, (lo, hi), (alo, ahi), desc = SPECS[name]
    import sys
    say = (lambda *a: print(*a, file=sys.stderr, flush=True)) if verbose else (lambda *a: None)
    say(f"[workload {name}] weights")
    base = synth.make_base(shape, seed=seed)
    lora = synth.make_lora(shape, seed=seed)
    lens = synth.draw_lens(seed, S, lo, hi) if lo != hi else np.full(S, lo, dtype=np.int32)
    nact = synth.draw_active_counts(seed, S, alo, ahi) if alo != ahi else np.full(S, alo, dtype=np.int32)
    batch = synth.make_batch(shape, lens, nact, seed=seed, headroom=headroom)
    cfg = layer_config(shape, batch.num_blocks, int(lens.max()) + headroom + 1)
    fp8 = name.endswith("-fp8")
    if fp8:
        cfg.kv_fp8, cfg.k_scale, cfg.v_scale = True, FP8_POOL_SCALE, FP8_POOL_SCALE
    dbase = {k: upload(v, shape.bf16, device) for k, v in base.items()}
    dlora = {p: (upload(A, shape.bf16, device), upload(B, shape.bf16, device)) for p, (A, B) in lora.items()}
    layer = binding.IcarusLayer(cfg, dbase, dlora)
    say(f"[workload {name}] pool: {batch.num_blocks} blocks")
    gen = torch.Generator(device=device)
    gen.manual_seed(1000 + seed)
    pool = torch.empty(cfg.pool_shape(), dtype=cfg.pool_dtype, device=device)
    step_blocks = max(1, (1 << 28) // (pool[0].numel()))
    for b0 in range(0, batch.num_blocks, step_blocks):        # fill in slabs: bounded temporaries
        sl = pool[b0:b0 + step_blocks]
        r = torch.randn(sl.shape, generator=gen, device=device, dtype=torch.float32)
        if fp8:   # the same N(0,1) cache, as codes (the cast rounds to nearest even; values are clipped below 448)
            sl.copy_((r.clamp_(-4.0, 4.0) / FP8_POOL_SCALE).to(torch.float8_e4m3fn).view(torch.uint8))
        else:
            sl.copy_(r)
    bt = torch.from_numpy(batch.block_tables).to(device)
    xs_host = [synth.make_hidden(shape, batch.R, seed=seed, tag=10 + i) for i in range(n_x)]
    xs = [upload(x, shape.bf16, device) for x in xs_host]
    full_host = None
    if name.endswith("-full"):   # every decoder its own weights: base + N(0, 0.01), made on the device, copied back for the oracle
        say(f"[workload {name}] private decoder weights")
        g2 = torch.Generator(device=device)
        g2.manual_seed(5000 + seed)
        full_dev, full_host = {}, {}
        for p in ("q", "o", "gate", "up", "down"):
            w = dbase[p]
            t = torch.empty((shape.n_models,) + tuple(w.shape), dtype=w.dtype, device=device)
            for j in range(shape.n_models):
                t[j] = (w.float() + 0.01 * torch.randn(w.shape, generator=g2, device=device)).to(w.dtype)
            full_dev[p] = t
            full_host[p] = t.float().cpu().numpy()
        layer.set_full_decoders(full_dev)
        lora = None
    return DecodeWorkload(name, desc, shape, batch, base, lora, layer, pool, bt, xs, xs_host, headroom,
                          (FP8_POOL_SCALE, FP8_POOL_SCALE) if fp8 else None, full_host)


def build_private_kv_baseline(wl: DecodeWorkload, device="cuda:0", seed: int = 0, n_x: int = 4) -> DecodeWorkload:
    """The same traffic served the conventional way, on the same kernels: every active (sequence, model)
    pair keeps a private KV cache (what per-model K/V weights force), so each of the R_d decoder rows is
    a sequence of its own that appends its own K/V and attends with a group of g query heads; there is
    no encoder row.  Adapter deltas are left out (they would only add time to this baseline)."""
    shape, b = wl.shape, wl.batch
    m = np.bincount(b.row_seq[b.row_model >= 0], minlength=b.S)
    lens = np.repeat(b.ctx_lens, m).astype(np.int32)
    batch = synth.make_batch(shape, lens, np.zeros(len(lens), dtype=np.int32), seed=seed + 1, headroom=wl.headroom)
    cfg = layer_config(shape, batch.num_blocks, int(lens.max()) + wl.headroom + 1)
    cfg.n_models, cfg.lora_rank, cfg.lora_target_mask = 0, 0, 0
    dbase = {k: upload(v, shape.bf16, device) for k, v in wl.base.items()}
    layer = binding.IcarusLayer(cfg, dbase, None)
    gen = torch.Generator(device=device)
    gen.manual_seed(3000 + seed)
    pool = torch.empty(cfg.pool_shape(), dtype=cfg.torch_dtype, device=device)
    step_blocks = max(1, (1 << 28) // (pool[0].numel()))
    for b0 in range(0, batch.num_blocks, step_blocks):
        sl = pool[b0:b0 + step_blocks]
        sl.copy_(torch.randn(sl.shape, generator=gen, device=device, dtype=torch.float32))
    bt = torch.from_numpy(batch.block_tables).to(device)
    xs_host = [synth.make_hidden(shape, batch.R, seed=seed, tag=40 + i) for i in range(n_x)]
    xs = [upload(x, shape.bf16, device) for x in xs_host]
    return DecodeWorkload(wl.name + "-private-kv", "per-model KV baseline of " + wl.description, shape, batch, wl.base, None,
                          layer, pool, bt, xs, xs_host, wl.headroom)


def sequence_kv_to_host(wl: DecodeWorkload, s: int, n_tokens: int):
    """Copy sequence s's first n_tokens cached K, V from the device pool: float32 [n, Hkv, D] each."""
    sh = wl.shape
    Bk, D = sh.block_size, sh.head_dim
    nb = (n_tokens + Bk - 1) // Bk
    ids = torch.from_numpy(wl.batch.block_tables[s, :nb].astype(np.int64)).to(wl.pool.device)
    blk = wl.pool.index_select(0, ids).to(torch.float32).cpu().numpy()      # [nb, Hkv, 2, Bk*D]
    K = blk[:, :, 0].reshape(nb, sh.n_kv_heads, Bk, D).transpose(0, 2, 1, 3).reshape(nb * Bk, sh.n_kv_heads, D)
    V = blk[:, :, 1].reshape(nb, sh.n_kv_heads, D, Bk).transpose(0, 3, 1, 2).reshape(nb * Bk, sh.n_kv_heads, D)
    return np.ascontiguousarray(K[:n_tokens]), np.ascontiguousarray(V[:n_tokens])


@dataclass
class PrefillWorkload:
    name: str
    description: str
    shape: synth.LayerShape
    batch: synth.Batch          # ctx_lens = cached prefix lengths; rows unused
    chunk_lens: np.ndarray
    base: dict
    layer: binding.IcarusLayer
    pool: torch.Tensor
    block_tables: torch.Tensor
    x: torch.Tensor             # [sum chunk, d]
    x_host: np.ndarray
    kv_scales: tuple = None     # (k_scale, v_scale) when the pool holds FP8 codes

    @property
    def n_tokens(self) -> int:
        return int(self.chunk_lens.sum())


PREFILL_SPECS = {
    "c4": (synth.LLAMA8B, 32, 8192, 512,
           "config 4: cross-model prefill reuse, Llama-3-8B-shaped layer, 32 sequences with 8192-token cached "
           "prefixes, each appends a 512-token chunk through the frozen encoder"),
    "c4-small": (synth.LLAMA_SMALL, 4, 300, 70, "reduced config 4"),
}
PREFILL_SPECS["c4-fp8"] = PREFILL_SPECS["c4"][:4] + (PREFILL_SPECS["c4"][4] + "; KV cache in FP8 E4M3 (static scales)",)
PREFILL_SPECS["c4-small-fp8"] = PREFILL_SPECS["c4-small"][:4] + ("reduced config 4, FP8 KV cache",)


def build_prefill_workload(name: str, device="cuda:0", seed: int = 0, verbose: bool = False) -> PrefillWorkload:
    import sys
    shape, S, prefix, chunk, desc = PREFILL_SPECS[name]
    say = (lambda *a: print(*a, file=sys.stderr, flush=True)) if verbose else (lambda *a: None)
    say(f"[workload {name}] weights")
    base = synth.make_base(shape, seed=seed)
    lens = np.full(S, prefix, dtype=np.int32)
    batch = synth.make_batch(shape, lens, np.zeros(S, dtype=np.int32), seed=seed, headroom=chunk + 16)
    cfg = layer_config(shape, batch.num_blocks, prefix + chunk + 17)
    cfg.n_models, cfg.lora_rank, cfg.lora_target_mask = 0, 0, 0      # prefill uses the frozen encoder only
    fp8 = name.endswith("-fp8")
    if fp8:
        cfg.kv_fp8, cfg.k_scale, cfg.v_scale = True, FP8_POOL_SCALE, FP8_POOL_SCALE
    dbase = {k: upload(v, shape.bf16, device) for k, v in base.items()}
    layer = binding.IcarusLayer(cfg, dbase, None)
    say(f"[workload {name}] pool: {batch.num_blocks} blocks")
    gen = torch.Generator(device=device)
    gen.manual_seed(2000 + seed)
    pool = torch.empty(cfg.pool_shape(), dtype=cfg.pool_dtype, device=device)
    step_blocks = max(1, (1 << 28) // (pool[0].numel()))
    for b0 in range(0, batch.num_blocks, step_blocks):
        sl = pool[b0:b0 + step_blocks]
        r = torch.randn(sl.shape, generator=gen, device=device, dtype=torch.float32)
        if fp8:
            sl.copy_((r.clamp_(-4.0, 4.0) / FP8_POOL_SCALE).to(torch.float8_e4m3fn).view(torch.uint8))
        else:
            sl.copy_(r)
    bt = torch.from_numpy(batch.block_tables).to(device)
    chunk_lens = np.full(S, chunk, dtype=np.int32)
    x_host = synth.make_hidden(shape, int(chunk_lens.sum()), seed=seed, tag=20)
    x = upload(x_host, shape.bf16, device)
    return PrefillWorkload(name, desc, shape, batch, chunk_lens, base, layer, pool, bt, x, x_host,
                           (FP8_POOL_SCALE, FP8_POOL_SCALE) if fp8 else None)


@dataclass
class StackWorkload:
    name: str
    description: str
    shape: synth.LayerShape
    n_layers: int
    vocab: int
    batch: synth.Batch
    weights: dict            # host float32 (storage-representable): the oracle reads these
    stack: binding.IcarusStack
    pools: list              # per layer, device, library layout
    block_tables: torch.Tensor
    seq_token: torch.Tensor  # device int32 [S]
    headroom: int

    def ctx_lens(self, step: int) -> np.ndarray:
        return (self.batch.ctx_lens + step).astype(np.int32)


STACK_SPECS = {
    # name: (shape, layers, vocab, S, (len_lo, len_hi), description)
    "stack": (synth.LLAMA8B, 8, 128256, 32, (1024, 8192),
              "layer stack: 8 Llama-3-8B-shaped layers, vocabulary 128256, 32 sequences with shared contexts U[1024,8192], "
              "one encoder row and one decoder row (its own adapter of 8) per sequence, greedy token fed back on the device"),
    "stack-small": (synth.LLAMA_SMALL.replace(n_models=8), 3, 2048, 6, (40, 600), "reduced layer stack"),
}


def build_stack_workload(name: str, device="cuda:0", headroom: int = 128, seed: int = 0, verbose: bool = False) -> StackWorkload:
    import sys
    shape, n_layers, vocab, S, (lo, hi), desc = STACK_SPECS[name]
    say = (lambda *a: print(*a, file=sys.stderr, flush=True)) if verbose else (lambda *a: None)
    say(f"[workload {name}] weights of {n_layers} layers")
    wts = synth.make_stack(shape, n_layers, vocab, seed=seed, norm_ones=True)
    lens = synth.draw_lens(seed, S, lo, hi)
    batch = synth.make_batch(shape, lens, np.ones(S, dtype=np.int32), seed=seed, headroom=headroom)
    cfg = layer_config(shape, batch.num_blocks, int(lens.max()) + headroom + 1)
    layers = []
    for b, l in zip(wts["bases"], wts["loras"]):
        dbase = {k: upload(v, shape.bf16, device) for k, v in b.items()}
        dlora = {p: (upload(A, shape.bf16, device), upload(B, shape.bf16, device)) for p, (A, B) in l.items()}
        layers.append(binding.IcarusLayer(cfg, dbase, dlora))
    stack = binding.IcarusStack(layers, upload(wts["embed"], shape.bf16, device), upload(wts["final_norm"], shape.bf16, device),
                                upload(wts["lm_head"], shape.bf16, device))
    say(f"[workload {name}] {n_layers} pools of {batch.num_blocks} blocks")
    gen = torch.Generator(device=device)
    gen.manual_seed(4000 + seed)
    pools = []
    for _ in range(n_layers):
        pool = torch.empty(cfg.pool_shape(), dtype=cfg.torch_dtype, device=device)
        step_blocks = max(1, (1 << 28) // (pool[0].numel()))
        for b0 in range(0, batch.num_blocks, step_blocks):
            sl = pool[b0:b0 + step_blocks]
            sl.copy_(torch.randn(sl.shape, generator=gen, device=device, dtype=torch.float32))
        pools.append(pool)
    bt = torch.from_numpy(batch.block_tables).to(device)
    rng = np.random.default_rng(np.random.SeedSequence([seed, 77]))
    seq_token = torch.from_numpy(rng.integers(0, vocab, size=S).astype(np.int32)).to(device)
    return StackWorkload(name, desc, shape, n_layers, vocab, batch, wts, stack, pools, bt, seq_token, headroom)
