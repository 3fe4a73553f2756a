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


def mark_unwritten(shape, batch, pool, value) -> None:
    """Set every slot of the pool that no sequence of the batch has written to `value` (by position, not by
    content: a written entry that happens to be exactly 0 stays as it is)."""
    written = np.zeros(pool.shape, dtype=bool)
    for s in range(batch.S):
        n = int(batch.ctx_lens[s])
        one = np.ones((n, shape.n_kv_heads, shape.head_dim), dtype=bool)
        fill_pool(written, batch.block_tables[s], one, one)
    pool[~written] = value


# Cache gate, bf16 storage: |got - want| <= one bf16 ulp of the oracle's value (the entry's own rounding) +
# CACHE_SLACK_BF16 * rms of the written entries.  The slack is 1.5 x the worst deviation that rounding the normed
# row to bf16 (what the matrix cores are fed) causes over 10^6 entries: 8.07e-3 rms, sigma 1.66e-3 rms
# (tests/test_cache_gate_model.py measures both on the CPU and ties this constant to them).
CACHE_SLACK_BF16 = 1.2e-2


def bf16_spacing(x: np.ndarray) -> np.ndarray:
    """Spacing of bfloat16 at |x| (8 significant bits)."""
    ax = np.maximum(np.abs(np.asarray(x, dtype=np.float64)), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(ax)) - 7)


def assert_cache_close(got, want, bf16: bool, what: str, rms=None):
    """Cache entries against the oracle's rounded values (see CACHE_SLACK_BF16).  fp32 storage: one ulp plus the
    fp32 accumulation allowance (1e-5 of the largest entry).  rms: of the written entries; by default of the
    entries that differ at all."""
    want = np.asarray(want, dtype=np.float64)
    diff = np.abs(np.asarray(got, dtype=np.float64) - want)
    if bf16:
        if rms is None:
            written = want[diff > 0]
            rms = float(np.sqrt(np.mean(written ** 2))) if written.size else 0.0
        ok = diff <= bf16_spacing(want) * 1.0001 + CACHE_SLACK_BF16 * rms
    else:
        ok = diff <= np.abs(want) * 2.0 ** -23 + 1e-5 * float(np.max(np.abs(want)))
    assert ok.all(), f"{what}: {int((~ok).sum())} cache elements outside the gate, worst {float(diff.max()):.3e}"


def e4m3_spacing(x: np.ndarray, scale: float) -> np.ndarray:
    """Spacing of the FP8 E4M3 grid (times scale) at |x|."""
    a = np.maximum(np.abs(np.asarray(x, dtype=np.float64)) / scale, 2.0 ** -6)
    return 2.0 ** (np.floor(np.log2(a)) - 3) * scale


def assert_fp8_cache_close(got, want, scale: float, bf16: bool, what: str):
    """FP8 cache entries (values = code * scale) against the oracle's.  A float decides the code on both sides:
    the device rounds its fp32 K/V, the oracle its float64 K/V, which differ by the bf16 arithmetic upstream
    (2^-7 of the tensor's rms covers it); on top of that the rounding may fall one grid step apart."""
    got, want = np.asarray(got, dtype=np.float64), np.asarray(want, dtype=np.float64)
    assert np.isfinite(got).all(), f"{what}: non-finite cache values"
    slack = (2.0 ** -7 if bf16 else 2.0 ** -16) * np.sqrt(np.mean(want ** 2))
    ratio = (np.abs(got - want) - slack) / e4m3_spacing(np.maximum(np.abs(got), np.abs(want)), scale)
    assert ratio.max() <= 1.001, f"{what}: {ratio.max():.3f} grid steps apart; {(ratio > 1.001).sum()} of {ratio.size}"


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
