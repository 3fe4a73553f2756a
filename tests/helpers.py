"""Test-side glue: layout moves between the oracle's pool and flat per-token K/V, error metrics."""
import numpy as np

import oracle
from paper_2603_13281_amd import synth


def oracle_config(shape: synth.LayerShape, num_blocks: int) -> oracle.LayerConfig:
    return oracle.LayerConfig(
        d_model=shape.d_model, n_q_heads=shape.n_q_heads, n_kv_heads=shape.n_kv_heads,
        head_dim=shape.head_dim, d_ffn=shape.d_ffn, block_size=shape.block_size, num_blocks=num_blocks,
        n_models=shape.n_models, lora_rank=shape.lora_rank, lora_target_mask=shape.lora_target_mask,
        qk_norm=shape.qk_norm, bf16=shape.bf16, rope_theta=shape.rope_theta, rms_eps=shape.rms_eps,
        lora_scale=shape.lora_scale)


def fill_pool(pool: np.ndarray, bt_row: np.ndarray, K: np.ndarray, V: np.ndarray) -> None:
    """Place K, V [n, Hkv, D] at logical positions 0..n-1 of one sequence.
    pool: oracle layout [num_blocks, 2, Hkv, Bk, D]."""
    Bk = pool.shape[3]
    t = np.arange(K.shape[0])
    b, o = np.asarray(bt_row)[t // Bk].astype(np.int64), t % Bk
    pool[b, 0, :, o, :] = K          # advanced indices (b, o) first: [n, Hkv, D]
    pool[b, 1, :, o, :] = V


def read_pool(pool: np.ndarray, bt_row: np.ndarray, n: int):
    Bk = pool.shape[3]
    K = np.stack([pool[int(bt_row[t // Bk]), 0, :, t % Bk, :] for t in range(n)]) if n else np.zeros((0,) + pool.shape[2:3] + pool.shape[4:])
    V = np.stack([pool[int(bt_row[t // Bk]), 1, :, t % Bk, :] for t in range(n)]) if n else K.copy()
    return K, V


def filled_batch(shape, batch, seed=0):
    """Oracle pool with every sequence's prefix directly filled with N(0,1) K/V."""
    pool = np.zeros((batch.num_blocks, 2, shape.n_kv_heads, shape.block_size, shape.head_dim), dtype=np.float32)
    for s in range(batch.S):
        K, V = synth.make_kv_tokens(shape, int(batch.ctx_lens[s]), seed, tag=s)
        fill_pool(pool, batch.block_tables[s], K, V)
    return pool


def rel_err(got: np.ndarray, want: np.ndarray) -> float:
    """max|g - o| / max|o| -- the per-tensor gate."""
    want = np.asarray(want, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    den = np.max(np.abs(want)) if want.size else 1.0
    return float(np.max(np.abs(got - want)) / den) if want.size else 0.0


def assert_close(got, want, tol, what=""):
    """Gate: max|g-o|/max|o| <= tol and |g-o| <= tol*|o| + tol*rms(o) elementwise."""
    want = np.asarray(want, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    if want.size == 0:
        return
    assert np.all(np.isfinite(got)), f"{what}: non-finite values"
    e = rel_err(got, want)
    assert e <= tol, f"{what}: max|g-o|/max|o| = {e:.3e} > {tol}"
    rms = float(np.sqrt(np.mean(want ** 2)))
    bad = np.abs(got - want) > tol * np.abs(want) + tol * rms
    assert not bad.any(), f"{what}: {int(bad.sum())} elements outside rtol={tol}, atol={tol}*rms"
