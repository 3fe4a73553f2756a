"""Pins of the oracle's FP8 (E4M3) KV cache: the rounding against the format's definition and a library
cast, and the cache semantics (stored value = code * scale; attention reads what is stored)."""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from paper_2603_13281_amd import synth
from helpers import oracle_config, read_pool


def e4m3_values():
    """All finite values of the OCP FP8 E4M3 format, from its definition: sign, 4 exponent bits (bias 7),
    3 mantissa bits; exponent field 0 = subnormal; the all-ones exponent with all-ones mantissa is NaN."""
    vals = []
    for code in range(256):
        s, e, m = code >> 7, (code >> 3) & 15, code & 7
        if e == 15 and m == 7:
            continue
        v = (m / 8.0) * 2.0 ** -6 if e == 0 else (1 + m / 8.0) * 2.0 ** (e - 7)
        vals.append(-v if s else v)
    return np.array(vals)


def test_e4m3_fixed_points_and_range():
    v = e4m3_values()
    assert len(v) == 254 and v.max() == 448.0 and np.min(np.abs(v[v != 0])) == 2.0 ** -9
    assert np.array_equal(oracle.round_e4m3(v), v)                       # every value of the format is a fixed point
    assert np.array_equal(oracle.round_e4m3([449.0, 1e9, -1e30]), [448.0, 448.0, -448.0])   # saturation


def test_e4m3_is_nearest_with_ties_to_even():
    v = np.unique(np.abs(e4m3_values()))
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.uniform(0, 448, 20000), rng.uniform(0, 0.05, 5000), 10.0 ** rng.uniform(-6, 2.6, 5000)])
    r = oracle.round_e4m3(x)
    # nearest: no value of the format is closer
    nearest = np.abs(x[:, None] - v[None, :]).min(axis=1)
    assert np.allclose(np.abs(r - x), nearest, rtol=0, atol=1e-15)
    # ties: midpoints between neighbours go to the one with even mantissa (even multiple of the quantum)
    mid = (v[:-1] + v[1:]) / 2
    rm = oracle.round_e4m3(mid)
    for lo, hi, got in zip(v[:-1], v[1:], rm):
        quantum = hi - lo
        want = lo if round(lo / quantum) % 2 == 0 else hi
        assert got == want, (lo, hi, got)
    assert np.array_equal(oracle.round_e4m3(-mid), -rm)


def test_e4m3_matches_library_cast():
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.standard_normal(20000) * s for s in (1e-2, 1.0, 100.0)]).astype(np.float32)
    x = x[np.abs(x) <= 448]
    want = torch.from_numpy(x).to(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(oracle.round_e4m3(x.astype(np.float64)), want)


@pytest.fixture(scope="module")
def cached():
    shape = synth.LLAMA_SMALL
    base, lora = synth.make_base(shape, seed=4), synth.make_lora(shape, seed=4)
    batch = synth.make_batch(shape, [45, 20], [2, 1], seed=4)
    x = synth.make_hidden(shape, 65, seed=4, tag=2)
    cfg = oracle_config(shape, batch.num_blocks)
    plain = oracle.Oracle(cfg, base, lora)
    pool = plain.new_pool()
    plain.prefill(pool, batch.block_tables, [0, 0], [45, 20], x, want_out=False)
    K, V = read_pool(pool, batch.block_tables[0], 45)
    ks, vs = float(np.abs(K).max()) / 300.0, float(np.abs(V).max()) / 300.0
    cfg8 = dataclasses.replace(cfg, kv_fp8=True, k_scale=ks, v_scale=vs)
    q8 = oracle.Oracle(cfg8, base, lora)
    pool8 = q8.new_pool()
    q8.prefill(pool8, batch.block_tables, [0, 0], [45, 20], x, want_out=False)
    return dict(shape=shape, base=base, lora=lora, batch=batch, plain=plain, q8=q8, pool=pool, pool8=pool8, ks=ks, vs=vs, cfg8=cfg8)


def test_cache_holds_codes_times_scale_within_half_a_step(cached):
    """Every cached value is (an E4M3 value) x scale and lies within half a quantisation step of the value
    the unquantised cache of the same layer input holds (first layer: the inputs of K and V are identical)."""
    c = cached
    K8, V8 = read_pool(c["pool8"], c["batch"].block_tables[0], 45)
    K, V = read_pool(c["pool"], c["batch"].block_tables[0], 45)
    for got, ref, s in ((K8, K, c["ks"]), (V8, V, c["vs"])):
        codes = got.astype(np.float64) / s
        assert np.allclose(oracle.round_e4m3(codes), codes, rtol=1e-6, atol=0)      # float32 pool: 2^-24 slack
        # half a step: 2^-4 relative for normals, 2^-10 (in code units) for subnormals; the reference was itself
        # rounded to bf16 (2^-9 relative)
        bound = np.maximum(2.0 ** -4 * np.abs(ref), 2.0 ** -10 * s) + 2.0 ** -8 * np.abs(ref)
        assert (np.abs(got - ref) <= bound).all()
    assert np.abs(K8 - K).max() > 0                                               # and it did quantise


def test_attention_reads_the_stored_values(cached):
    """The output over the FP8 cache equals softmax attention written with numpy over the values read back
    from that cache: nothing of the unquantised K/V takes part."""
    c = cached
    shape, batch = c["shape"], c["batch"]
    rng = np.random.default_rng(5)
    R = 3
    q = rng.standard_normal((R, shape.n_q_heads, shape.head_dim)).astype(np.float32)
    row_seq = np.int32([0, 0, 1])
    kv_lens = np.int32([45, 20])
    got = c["q8"].attn_shared_kv(q, c["pool8"], batch.block_tables, kv_lens, row_seq)
    g = shape.n_q_heads // shape.n_kv_heads
    for r in range(R):
        s = row_seq[r]
        K, V = read_pool(c["pool8"], batch.block_tables[s], int(kv_lens[s]))
        for h in range(shape.n_q_heads):
            kk, vv = K[:, h // g, :].astype(np.float64), V[:, h // g, :].astype(np.float64)
            sc = kk @ q[r, h].astype(np.float64) / np.sqrt(shape.head_dim)
            p = np.exp(sc - sc.max()); p /= p.sum()
            assert np.allclose(np.asarray(got)[r].reshape(shape.n_q_heads, -1)[h], p @ vv, rtol=1e-9, atol=1e-12)


def test_fp8_cache_is_the_same_whichever_adapter_decodes_and_close_to_bf16(cached):
    c = cached
    shape, batch = c["shape"], c["batch"]
    x = synth.make_hidden(shape, batch.R, seed=4)
    outs = {}
    for name, orc, pool in (("fp8", c["q8"], c["pool8"]), ("bf16", c["plain"], c["pool"])):
        pools = []
        for models in ([0, 1, 2], [3, 1, 0]):          # different adapters on the same sequences
            p = pool.copy()
            rm = batch.row_model.copy()
            rm[rm >= 0] = [models[i % 3] for i in range(int((rm >= 0).sum()))]
            y, _ = orc.decode_step(p, batch.block_tables, batch.ctx_lens, batch.row_seq, rm, x)
            pools.append(p)
        assert np.array_equal(pools[0], pools[1])      # Eq. 4: the encoder alone writes the cache
        outs[name] = y
    err = np.abs(outs["fp8"] - outs["bf16"]).max() / np.abs(outs["bf16"]).max()
    assert 0 < err < 0.05, err
