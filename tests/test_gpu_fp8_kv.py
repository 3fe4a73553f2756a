"""FP8 (E4M3) shared KV cache on the GPU against the oracle with the same cache format.

The cache holds quantised codes, so a float decides an integer: both sides round x / scale to the nearest
E4M3 value, the device from its fp32 K/V (computed from bf16 GEMMs), the oracle from float64.  Where
x / scale lies near a rounding boundary the codes differ by one step; cached values are compared to within
the arithmetic's slack plus one step of the grid, outputs to the layer tolerance."""
import dataclasses

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

TOL = {True: 2e-2, False: 1e-4}


def _setup(shape, lens, nact, seed, chunk):
    import oracle
    from gpu_util import make_layer
    from helpers import oracle_config, read_pool
    from paper_2603_13281_amd import synth
    base, lora = synth.make_base(shape, seed=seed), synth.make_lora(shape, seed=seed)
    batch = synth.make_batch(shape, lens, nact, seed=seed, headroom=4)
    S = len(lens)
    n_pre = int(np.sum(chunk))
    xp = synth.make_hidden(shape, n_pre, seed=seed, tag=3)
    cfg = oracle_config(shape, batch.num_blocks)
    # the caller's calibration: static scales from an unquantised pass over the same prompt
    plain = oracle.Oracle(cfg, base, lora)
    pool = plain.new_pool()
    plain.prefill(pool, batch.block_tables, np.zeros(S, np.int32), chunk, xp, want_out=False)
    amax_k = max(np.abs(read_pool(pool, batch.block_tables[s], int(chunk[s]))[0]).max() for s in range(S))
    amax_v = max(np.abs(read_pool(pool, batch.block_tables[s], int(chunk[s]))[1]).max() for s in range(S))
    ks, vs = float(amax_k) / 240.0, float(amax_v) / 240.0
    orc = oracle.Oracle(dataclasses.replace(cfg, kv_fp8=True, k_scale=ks, v_scale=vs), base, lora)
    layer = make_layer(shape, base, lora, batch.num_blocks, kv_fp8=True, k_scale=ks, v_scale=vs)
    return base, lora, batch, xp, orc, layer, ks, vs


@pytest.mark.parametrize("kind", ["llama-small", "qwen-small", "tiny-fp32"])
def test_prefill_then_decode_with_fp8_cache(kind):
    from gpu_util import dev, e4m3_step, fp8_pool_to_float, host, pool_from_device_layout
    from helpers import assert_close, read_pool
    from paper_2603_13281_amd import synth
    shape = {"llama-small": synth.LLAMA_SMALL, "qwen-small": synth.QWEN_SMALL, "tiny-fp32": synth.TINY}[kind]
    n_models = shape.n_models
    lens = np.int32([700, 45, 333, 64])                       # several pieces, tails of 28, 13 and 13 tokens, one exact
    nact = np.int32([min(3, n_models), 1, 2, 0])              # up to 1 + 3 streams x g heads: 1-3 query tiles at g = 4 / 8
    base, lora, batch, xp, orc, layer, ks, vs = _setup(shape, lens, nact, seed=6, chunk=lens)
    S = len(lens)
    zeros = np.zeros(S, np.int32)
    opool = orc.new_pool()
    want_p, _ = orc.prefill(opool, batch.block_tables, zeros, lens, xp)
    dpool = torch.full(layer.cfg.pool_shape(), 0x7f, dtype=torch.uint8, device="cuda:0")     # every byte a NaN code
    bt = torch.from_numpy(batch.block_tables).cuda()
    got_p = layer.prefill_kv(dpool, bt, zeros, lens, dev(xp, shape.bf16))
    torch.cuda.synchronize()
    assert_close(host(got_p), want_p, TOL[shape.bf16], f"{kind} prefill over an fp8 cache")
    # the cache: every written value within one grid step of the oracle's, most of them equal
    gp = pool_from_device_layout(fp8_pool_to_float(dpool, ks, vs), shape.block_size, shape.head_dim)
    n_diff = n_all = 0
    for s in range(S):
        Kd, Vd = read_pool(gp, batch.block_tables[s], int(lens[s]))
        Ko, Vo = read_pool(opool, batch.block_tables[s], int(lens[s]))
        for got, want, sc in ((Kd, Ko, ks), (Vd, Vo, vs)):
            assert np.isfinite(got).all()
            # the device's K/V before rounding differ from the oracle's by the bf16 arithmetic upstream (2^-7 of the
            # tensor's rms covers it, as for the bf16 cache); on top of that the rounding may fall one grid step apart
            slack = (2.0 ** -7 if shape.bf16 else 2.0 ** -16) * np.sqrt(np.mean(want.astype(np.float64) ** 2))
            ratio = (np.abs(got - want) - slack) / e4m3_step(np.maximum(np.abs(got), np.abs(want)), sc)
            worst = np.unravel_index(np.argmax(ratio), ratio.shape)
            assert ratio.max() <= 1.001, (f"{kind} cache of sequence {s}: {ratio.max():.3f} steps at {worst}: got "
                                          f"{got[worst] / sc} want {want[worst] / sc} (code units); {(ratio > 1.001).sum()} of {ratio.size}")
            n_diff += int((np.abs(got - want) > 1e-3 * e4m3_step(want, sc)).sum())      # a different code
            n_all += got.size
    assert n_diff <= 0.12 * n_all, (n_diff, n_all)
    # decode step over the device's own cache (matrix-core attention for the bf16 shapes)
    x = synth.make_hidden(shape, batch.R, seed=6)
    want, want_slots = orc.decode_step(opool, batch.block_tables, batch.ctx_lens, batch.row_seq, batch.row_model, x)
    slots = torch.zeros(S, dtype=torch.int64, device="cuda:0")
    got = layer.decode_step(dpool, bt, batch.ctx_lens, batch.row_seq, batch.row_model, dev(x, shape.bf16), slot_out=slots)
    torch.cuda.synchronize()
    assert np.array_equal(slots.cpu().numpy(), want_slots)
    assert_close(host(got), want, TOL[shape.bf16] if shape.bf16 else 2e-3, f"{kind} decode over an fp8 cache")
    # unwritten bytes are untouched
    touched = np.zeros(batch.num_blocks, dtype=bool)
    for s in range(S):
        touched[batch.block_tables[s, : (int(lens[s]) + 1 + shape.block_size - 1) // shape.block_size]] = True
    assert (dpool.cpu().numpy()[~touched] == 0x7f).all()


def test_matrix_core_and_vector_attention_match_the_oracle_on_the_same_codes():
    """icarus_attn_shared_kv over one FP8 pool of random codes: the MFMA kernel and the library's plain vector
    kernel, each against the oracle reading the same codes times the scales (the GQA line of Alg. 3), with 1 to 5
    query tiles (up to 10 rows x 8 heads per kv-head; 4 and 5 tiles walk the cache through the LDS ring in wave
    pairs), cut and uncut sequences, ragged tails."""
    import oracle
    from gpu_util import dev, fp8_pool_to_float, host, make_layer, pool_from_device_layout
    from helpers import assert_close, oracle_config
    from paper_2603_13281_amd import synth
    shape = synth.QWEN_SMALL
    ks, vs = 0.02, 0.013
    base, lora = synth.make_base(shape, seed=2), synth.make_lora(shape, seed=2)
    for rows_per_seq, lens in (([6, 1, 3, 5, 2], [1500, 31, 32, 33, 257]), ([2, 2], [4000, 15]), ([1], [700]),
                               ([10, 7, 1], [900, 2100, 40]), ([8, 2], [3000, 77]), ([9, 10, 8], [33, 1025, 160])):
        print("case: fp8 attention rows", rows_per_seq, "lens", lens, flush=True)
        lens = np.int32(lens)
        batch = synth.make_batch(shape, lens, np.zeros(len(lens), np.int32), seed=2, headroom=1)
        layer = make_layer(shape, base, lora, batch.num_blocks, kv_fp8=True, k_scale=ks, v_scale=vs)
        gen = torch.Generator(device="cuda:0"); gen.manual_seed(5)
        codes = torch.randint(0, 256, layer.cfg.pool_shape(), generator=gen, device="cuda:0", dtype=torch.uint8)
        codes[(codes & 0x7f) == 0x7f] = 0x38                      # no NaN codes inside the contexts
        codes[(codes & 0x78) == 0x78] &= 0xbf                     # |code value| < 32: scores stay in a sane range
        bt = torch.from_numpy(batch.block_tables).cuda()
        row_seq = np.repeat(np.arange(len(lens), dtype=np.int32), rows_per_seq)
        qh = synth.to_storage((np.random.default_rng(3).standard_normal((len(row_seq), shape.n_q_heads, shape.head_dim)) * 0.3).astype(np.float32), True)
        # the oracle reads the values the codes stand for
        opool = pool_from_device_layout(fp8_pool_to_float(codes, ks, vs), shape.block_size, shape.head_dim)
        orc = oracle.Oracle(dataclasses.replace(oracle_config(shape, batch.num_blocks), kv_fp8=True, k_scale=ks, v_scale=vs), base, None)
        want = orc.attn_shared_kv(qh, opool, batch.block_tables, lens, row_seq)
        q = dev(qh.reshape(len(row_seq), -1), True)
        layer.set_kernel_mode(0)
        a = layer.attn_shared_kv(q, codes, bt, lens, row_seq)
        layer.set_kernel_mode(1)
        b = layer.attn_shared_kv(q, codes, bt, lens, row_seq)
        torch.cuda.synchronize()
        a, b = host(a).reshape(want.shape), host(b).reshape(want.shape)
        assert_close(a, want, 2e-2, f"fp8 matrix-core attention, rows {rows_per_seq}")
        assert_close(b, want, 2e-2, f"fp8 vector attention, rows {rows_per_seq}")
        assert np.abs(a - b).max() > 0                            # two different kernels did run
        layer.close()


def test_create_rejects_bad_fp8_config():
    from gpu_util import layer_config
    from paper_2603_13281_amd import binding, synth
    from test_abi_host import _weights
    cfg = layer_config(synth.LLAMA_SMALL, 8)
    cfg.kv_fp8, cfg.k_scale = True, 0.0
    base, lora = _weights()
    with pytest.raises(binding.IcarusError) as e:
        binding.IcarusLayer(cfg, base, lora)
    assert e.value.status_name == "INVALID_ARG"
