"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element, on the same
seeded inputs.  Tolerances (per output tensor): max|g-o|/max|o| <= 2e-2 for bf16 storage, 1e-4 for fp32,
plus an elementwise rtol/atol gate (helpers.assert_close); cache entries within one storage ulp plus the slack that
the bf16 rounding of the normed row causes (helpers.CACHE_SLACK_BF16, measured in tests/test_cache_gate_model.py);
slots, and everything the call must not touch, bit-exact."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_13281_amd import synth
from helpers import assert_cache_close, assert_close, fill_pool, filled_batch, mark_unwritten, oracle_config, read_pool
from gpu_util import bf16_ulp, dev, host, make_layer, pool_from_device_layout, pool_to_device_layout

pytestmark = pytest.mark.gpu

TOL = {True: 2e-2, False: 1e-4}
MODES = [0, 1]  # 0: automatic kernel choice, 1: generic vector kernels


def _say(*a):
    print(*a, flush=True)


def _cache_close(shape, got_pool, want_pool, what):
    # pools in the oracle's layout [blocks, 2, Hkv, Bk, D]; K and V are different tensors (with QK-norm K has unit
    # rms per head, V the scale of the weights), so each plane is gated against the rms of its own written entries
    for plane, nm in ((0, "K"), (1, "V")):
        assert_cache_close(got_pool[:, plane], want_pool[:, plane], shape.bf16, f"{what} {nm}")


def _decode_case(shape, ctx, n_active, seed, mode, norm_ones=False):
    base = synth.make_base(shape, seed=seed, norm_ones=norm_ones)
    lora = synth.make_lora(shape, seed=seed)
    batch = synth.make_batch(shape, ctx, n_active, seed=seed)
    pool = filled_batch(shape, batch, seed=seed)
    pool[pool == 0] = -3.0                                   # sentinel in unfilled slots
    x = synth.make_hidden(shape, batch.R, seed=seed)
    orc = oracle.Oracle(oracle_config(shape, batch.num_blocks), base, lora)
    want_pool = pool.copy()
    want, want_slots = orc.decode_step(want_pool, batch.block_tables, batch.ctx_lens, batch.row_seq, batch.row_model, x)

    layer = make_layer(shape, base, lora, batch.num_blocks)
    layer.set_kernel_mode(mode)
    dpool = dev(pool_to_device_layout(pool), shape.bf16)
    bt = torch.from_numpy(batch.block_tables).cuda()
    slots = torch.full((batch.S,), -1, dtype=torch.int64, device="cuda")
    got = layer.decode_step(dpool, bt, batch.ctx_lens, batch.row_seq, batch.row_model, dev(x, shape.bf16), slot_out=slots)
    torch.cuda.synchronize()
    got_pool = pool_from_device_layout(host(dpool), shape.block_size, shape.head_dim)
    return batch, want, want_slots, want_pool, pool, host(got), slots.cpu().numpy(), got_pool


def _check_decode(shape, ctx, n_active, seed, mode, **kw):
    batch, want, want_slots, want_pool, pool0, got, slots, got_pool = _decode_case(shape, ctx, n_active, seed, mode, **kw)
    assert np.array_equal(slots, want_slots)
    # only the appended slots changed, and they match the oracle's entries
    changed = np.argwhere((got_pool != pool0).any(axis=(1, 2, 4)))
    assert sorted(int(b) * shape.block_size + int(o) for b, o in changed) == sorted(int(s) for s in want_slots)
    _cache_close(shape, got_pool, want_pool, "kv cache")
    assert_close(got, want, TOL[shape.bf16], "x_out")


@pytest.mark.parametrize("mode", MODES)
def test_config1_tiny_fp32_prefill_then_decode(mode):
    # Config 1: d 256, 4 heads of 64, FFN 688, M = 2 rank-8 adapters on q/v/o, one sequence, 128-token shared
    # prefix built by the frozen encoder's prefill, then one decode step with both models active.
    _say("case: config 1 tiny fp32, mode", mode)
    shape = synth.TINY
    base = synth.make_base(shape, seed=0)
    lora = synth.make_lora(shape, seed=0)
    batch = synth.make_batch(shape, [128], [2], seed=0)
    orc = oracle.Oracle(oracle_config(shape, batch.num_blocks), base, lora)
    xp = synth.make_hidden(shape, 128, seed=0, tag=1)
    want_pool = orc.new_pool()
    want_y, want_s = orc.prefill(want_pool, batch.block_tables, [0], [128], xp)

    layer = make_layer(shape, base, lora, batch.num_blocks)
    layer.set_kernel_mode(mode)
    dpool = torch.zeros(layer.cfg.pool_shape(), dtype=torch.float32, device="cuda")
    bt = torch.from_numpy(batch.block_tables).cuda()
    slots = torch.zeros(128, dtype=torch.int64, device="cuda")
    got_y = layer.prefill_kv(dpool, bt, [0], [128], dev(xp, False), slot_out=slots)
    torch.cuda.synchronize()
    assert np.array_equal(slots.cpu().numpy(), want_s)
    assert_close(host(got_y), want_y, 1e-4, "prefill x_out")
    _cache_close(shape, pool_from_device_layout(host(dpool), 16, 64), want_pool, "prefill cache")

    x = synth.make_hidden(shape, batch.R, seed=0)
    want, ws = orc.decode_step(want_pool, batch.block_tables, batch.ctx_lens, batch.row_seq, batch.row_model, x)
    s1 = torch.zeros(1, dtype=torch.int64, device="cuda")
    got = layer.decode_step(dpool, bt, batch.ctx_lens, batch.row_seq, batch.row_model, dev(x, False), slot_out=s1)
    torch.cuda.synchronize()
    assert int(s1[0]) == int(ws[0])
    assert_close(host(got), want, 1e-4, "decode x_out")
    _cache_close(shape, pool_from_device_layout(host(dpool), 16, 64), want_pool, "decode cache")


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("shape", [synth.LLAMA_SMALL, synth.QWEN_SMALL], ids=lambda s: s.name)
def test_decode_ragged_batch(shape, mode):
    # several tiles and ragged tails: lengths around block boundaries, empty context, 0..M active models
    _say("case: ragged decode", shape.name, "mode", mode)
    ctx = [0, 1, 15, 16, 17, 300, 1030, 47]
    M = shape.n_models
    n_active = [1, 0, M, 2, 1, M, min(3, M), 0]
    _check_decode(shape, ctx, n_active, seed=11, mode=mode)


@pytest.mark.parametrize("rows", [100, 129, 230, 300, 385])
def test_decode_row_counts_of_every_gemm_tile(rows):
    # The GEMM launcher picks its tile from the stacked row count: up to 64, up to 128, 193-256 (fused gate/up),
    # up to 384, more.  The other cases of this file stay below 64 rows; these reach the other tiles, each with a
    # ragged last row tile, and the first row count past a boundary (129, 385).  More than 256 rows also take the
    # row and RoPE kernels with one workgroup per row instead of several.
    _say("case: decode with", rows, "stacked rows")
    shape = synth.LLAMA_SMALL
    S = rows // 5
    ctx = [(7 * i) % 45 for i in range(S)]
    n_active = [4] * S
    extra = rows - 5 * S                       # one shorter sequence makes up the exact count
    if extra:
        ctx.append(33)
        n_active.append(extra - 1)
    _check_decode(shape, ctx, n_active, seed=21, mode=MODES[0])


@pytest.mark.parametrize("rows,d_ffn", [(330, 10304), (150, 20608), (131, 20608), (160, 20608), (161, 20608)])
def test_decode_wide_ffn_takes_the_wide_projection_gemm(rows, d_ffn):
    # A fused gate/up projection wide enough for 160 tiles of 192 x 256 goes to the register-staged GEMM kernel
    # (two row tiles of 192 at 330 rows; at most 160 rows: the 160 x 256 tile with three slabs of loads in flight,
    # partly filled at 131 and 150 rows, full at 160; 161 rows: one 192-row tile again; the last column tile is
    # ragged: d_ffn is not a multiple of 128).  Element by element against the oracle; the down projection then
    # contracts over the same odd width.
    _say("case: wide ffn", rows, "rows, d_ffn", d_ffn)
    # d_model 512: eight 64-wide slabs of base weights, so the kernel's steady-state loop runs as well as its tail
    shape = synth.QWEN_SMALL.replace(d_model=512, n_q_heads=2, n_kv_heads=2, d_ffn=d_ffn)
    S = rows // 4
    ctx = [(5 * i) % 40 for i in range(S)]
    n_active = [3] * S
    extra = rows - 4 * S
    if extra:
        ctx.append(17)
        n_active.append(extra - 1)
    _check_decode(shape, ctx, n_active, seed=23, mode=MODES[0])


@pytest.mark.parametrize("mode", MODES)
def test_decode_long_context_many_models(mode):
    _say("case: long context decode mode", mode)
    shape = synth.LLAMA_SMALL.replace(n_models=8)
    _check_decode(shape, [5000, 2049], [8, 5], seed=5, mode=mode)


def test_config2_llama8b_layer_decode():
    # Config 2 whole: Llama-3-8B-shaped layer, M = 8 rank-16 adapters on all seven projections, one sequence
    # with a 4096-token shared prefix (directly filled), one decode step, all eight models active.
    _say("case: config 2 llama-8b layer")
    _check_decode(synth.LLAMA8B, [4096], [8], seed=0, mode=0, norm_ones=True)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("shape", [synth.TINY, synth.LLAMA_SMALL, synth.QWEN_SMALL], ids=lambda s: s.name)
def test_attn_shared_kv(shape, mode):
    _say("case: attention only", shape.name, "mode", mode)
    lens = [1, 16, 33, 700, 2500]
    rows_per_seq = [1, 3, 1 + shape.n_models, 2, 1 + shape.n_models]
    batch = synth.make_batch(shape, lens, [0] * len(lens), seed=3, headroom=0)
    pool = filled_batch(shape, batch, seed=3)
    row_seq = np.repeat(np.arange(len(lens)), rows_per_seq).astype(np.int32)
    R = len(row_seq)
    rng = np.random.default_rng(7)
    q = synth.to_storage(rng.standard_normal((R, shape.n_q_heads, shape.head_dim)).astype(np.float32), shape.bf16)
    orc = oracle.Oracle(oracle_config(shape, batch.num_blocks), synth.make_base(shape), None)
    want = orc.attn_shared_kv(q, pool, batch.block_tables, lens, row_seq)
    layer = make_layer(shape, synth.make_base(shape), None, batch.num_blocks)
    layer.set_kernel_mode(mode)
    dpool = dev(pool_to_device_layout(pool), shape.bf16)
    got = layer.attn_shared_kv(dev(q, shape.bf16), dpool, torch.from_numpy(batch.block_tables).cuda(), lens, row_seq)
    torch.cuda.synchronize()
    assert_close(host(got), want, TOL[shape.bf16], "attention out")
    assert np.array_equal(host(dpool), pool_to_device_layout(pool))     # read-only


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("shape", [synth.LLAMA_SMALL, synth.QWEN_SMALL], ids=lambda s: s.name)
def test_prefill_chunk_over_paged_prefix_then_decode(shape, mode):
    # Config 4's structure at reduced size: cached prefixes, a chunk appended by the frozen encoder (starting
    # mid-block, spanning blocks), then a decode step by a model that never ran on the sequence: no recompute.
    _say("case: prefill chunk", shape.name, "mode", mode)
    pre = [37, 0, 160]
    chunk = [45, 20, 0]
    base = synth.make_base(shape, seed=2, norm_ones=False)
    lora = synth.make_lora(shape, seed=2)
    batch = synth.make_batch(shape, pre, [1, 2, 1], seed=2, headroom=64)
    pool = filled_batch(shape, batch, seed=2)
    pool[pool == 0] = 5.0
    x = synth.make_hidden(shape, sum(chunk), seed=2, tag=3)
    orc = oracle.Oracle(oracle_config(shape, batch.num_blocks), base, lora)
    want_pool = pool.copy()
    want, want_slots = orc.prefill(want_pool, batch.block_tables, pre, chunk, x)

    layer = make_layer(shape, base, lora, batch.num_blocks)
    layer.set_kernel_mode(mode)
    dpool = dev(pool_to_device_layout(pool), shape.bf16)
    bt = torch.from_numpy(batch.block_tables).cuda()
    slots = torch.zeros(sum(chunk), dtype=torch.int64, device="cuda")
    got = layer.prefill_kv(dpool, bt, pre, chunk, dev(x, shape.bf16), slot_out=slots)
    torch.cuda.synchronize()
    assert np.array_equal(slots.cpu().numpy(), want_slots)
    got_pool = pool_from_device_layout(host(dpool), shape.block_size, shape.head_dim)
    changed = np.argwhere((got_pool != pool).any(axis=(1, 2, 4)))
    assert sorted(int(b) * shape.block_size + int(o) for b, o in changed) == sorted(int(s) for s in want_slots)
    _cache_close(shape, got_pool, want_pool, "prefill cache")
    assert_close(host(got), want, TOL[shape.bf16], "prefill x_out")

    # cache-only prefill writes the same bytes
    dpool2 = dev(pool_to_device_layout(pool), shape.bf16)
    layer.prefill_kv(dpool2, bt, pre, chunk, dev(x, shape.bf16), want_out=False)
    torch.cuda.synchronize()
    assert torch.equal(dpool2, dpool)

    # decode on top of the GPU-written cache, against the oracle on the oracle-written cache
    ctx2 = [p + c for p, c in zip(pre, chunk)]
    b2 = synth.make_batch(shape, ctx2, [1, 2, 1], seed=2, headroom=1)
    xd = synth.make_hidden(shape, b2.R, seed=2, tag=4)
    wd, _ = orc.decode_step(want_pool, batch.block_tables, ctx2, b2.row_seq, b2.row_model, xd)
    gd = layer.decode_step(dpool, bt, ctx2, b2.row_seq, b2.row_model, dev(xd, shape.bf16))
    torch.cuda.synchronize()
    assert_close(host(gd), wd, TOL[shape.bf16], "decode after prefill")


@pytest.mark.parametrize("mode", MODES)
def test_cache_bits_do_not_depend_on_adapters(mode):
    # Sec. 3.2 / 3.3: the cache is written by the frozen encoder alone -> bit-identical on the GPU whatever
    # adapter weights are loaded and whichever models are active; K/V adapters are never read.
    _say("case: adapter independence mode", mode)
    shape = synth.LLAMA_SMALL
    base = synth.make_base(shape, seed=4)
    ctx = [33, 250]
    pools, outs = [], []
    for lora_seed, n_act, scale_kv in ((4, [2, 4], 1.0), (9, [2, 4], 1.0), (4, [0, 1], 1.0), (4, [2, 4], 50.0)):
        lora = synth.make_lora(shape, seed=lora_seed)
        lora["k"] = (lora["k"][0] * scale_kv, lora["k"][1])
        lora["v"] = (lora["v"][0], lora["v"][1] * scale_kv)
        batch = synth.make_batch(shape, ctx, n_act, seed=4)
        pool = filled_batch(shape, batch, seed=4)
        x_seq = synth.make_hidden(shape, 2, seed=4)
        layer = make_layer(shape, base, lora, batch.num_blocks)
        layer.set_kernel_mode(mode)
        dpool = dev(pool_to_device_layout(pool), True)
        y = layer.decode_step(dpool, torch.from_numpy(batch.block_tables).cuda(), ctx, batch.row_seq, batch.row_model,
                              dev(x_seq[batch.row_seq], True))
        torch.cuda.synchronize()
        pools.append(dpool.cpu())
        outs.append(y.cpu())
    assert all(torch.equal(pools[0], p) for p in pools[1:])
    assert torch.equal(outs[0], outs[3])            # K/V adapter perturbation is a no-op on outputs too
    assert not torch.equal(outs[0], outs[1])


@pytest.mark.parametrize("mode", MODES)
def test_zero_B_rows_equal_encoder_row_and_runs_are_deterministic(mode):
    _say("case: zero B, determinism, mode", mode)
    shape = synth.LLAMA_SMALL
    base = synth.make_base(shape, seed=6)
    lora = synth.make_lora(shape, seed=6, zero_b=True)
    batch = synth.make_batch(shape, [129, 64], [4, 2], seed=6)
    pool = filled_batch(shape, batch, seed=6)
    x = synth.make_hidden(shape, 2, seed=6)[batch.row_seq]
    layer = make_layer(shape, base, lora, batch.num_blocks)
    layer.set_kernel_mode(mode)
    bt = torch.from_numpy(batch.block_tables).cuda()
    ys = []
    for _ in range(2):
        dpool = dev(pool_to_device_layout(pool), True)
        ys.append(layer.decode_step(dpool, bt, batch.ctx_lens, batch.row_seq, batch.row_model, dev(x, True)).cpu())
    assert torch.equal(ys[0], ys[1])
    y = ys[0].float().numpy()
    orc = oracle.Oracle(oracle_config(shape, batch.num_blocks), base, lora)
    want, _ = orc.decode_step(pool.copy(), batch.block_tables, batch.ctx_lens, batch.row_seq, batch.row_model, x)
    assert_close(y, want, 2e-2, "zero-B x_out")
    # Sec. 3.2: with B = 0 a decoder is the base model.  On the device too, bit for bit: a row's arithmetic does not
    # depend on its place in a tile, the adapter's K-steps add exact zeros, and equal queries of one sequence see
    # equal scores, so every step of a decoder row repeats the encoder row's.
    for r in range(batch.R):
        enc = int(np.flatnonzero((batch.row_seq == batch.row_seq[r]) & (batch.row_model == -1))[0])
        assert torch.equal(ys[0][r], ys[0][enc]), f"row {r} differs from its sequence's encoder row {enc}"


def test_errors_surface_through_the_binding():
    from paper_2603_13281_amd.binding import IcarusError
    shape = synth.LLAMA_SMALL
    batch = synth.make_batch(shape, [20], [1], seed=0)
    layer = make_layer(shape, synth.make_base(shape), synth.make_lora(shape), batch.num_blocks)
    dpool = torch.zeros(layer.cfg.pool_shape(), dtype=torch.bfloat16, device="cuda")
    bt = torch.from_numpy(batch.block_tables).cuda()
    x = torch.zeros(2, shape.d_model, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(IcarusError) as e:
        layer.decode_step(dpool, bt, [20], [0, 0], [-1, 99], x)
    assert e.value.status_name == "MODEL_ID"
    with pytest.raises(IcarusError) as e:
        layer.decode_step(dpool, bt, [20], [0, 0], [-1, 0], x, workspace=torch.zeros(64, dtype=torch.uint8, device="cuda"))
    assert e.value.status_name == "CAPACITY"
    with pytest.raises(IcarusError) as e:
        layer.decode_step(dpool, bt, [10_000], [0, 0], [-1, 0], x)
    assert e.value.status_name == "CAPACITY"


@pytest.mark.parametrize("chunk", [0, 128, 256])
@pytest.mark.parametrize("g,rows", [(4, 1), (4, 4), (4, 9), (8, 2), (8, 7), (8, 9), (1, 3)])
def test_attn_mfma_tiles_splits_and_tails(g, rows, chunk):
    # matrix-core attention: every query-tile count (1..5 tiles of 16 stacked queries), single-chunk and
    # split sequences, lengths around the 16-token block, 32-token group and 128-token chunk boundaries
    _say("case: mfma attention g", g, "rows", rows, "chunk", chunk)
    shape = synth.LLAMA_SMALL.replace(n_q_heads=2 * g, n_kv_heads=2, d_model=256, n_models=8)
    lens = [1, 15, 16, 17, 31, 32, 33, 127, 128, 129, 255, 257, 1000, 3001]
    rows_per_seq = [rows if i % 3 else max(1, rows - 1) for i in range(len(lens))]
    batch = synth.make_batch(shape, lens, [0] * len(lens), seed=8, headroom=0)
    pool = filled_batch(shape, batch, seed=8)
    mark_unwritten(shape, batch, pool, np.nan)   # unwritten slots hold NaN: masked positions must not leak
    row_seq = np.repeat(np.arange(len(lens)), rows_per_seq).astype(np.int32)
    R = len(row_seq)
    rng = np.random.default_rng(9)
    q = synth.to_storage(rng.standard_normal((R, shape.n_q_heads, shape.head_dim)).astype(np.float32) * 2, True)
    orc = oracle.Oracle(oracle_config(shape, batch.num_blocks), synth.make_base(shape), None)
    want = orc.attn_shared_kv(q, pool, batch.block_tables, lens, row_seq)
    layer = make_layer(shape, synth.make_base(shape), None, batch.num_blocks)
    layer.set_attn_piece_limit(chunk)          # 0: automatic; else sequences longer than this are cut into pieces
    dpool = dev(pool_to_device_layout(pool), True)
    got = layer.attn_shared_kv(dev(q, True), dpool, torch.from_numpy(batch.block_tables).cuda(), lens, row_seq)
    torch.cuda.synchronize()
    assert_close(host(got), want, 2e-2, "attention out")


@pytest.mark.parametrize("shape", [synth.LLAMA_SMALL, synth.QWEN_SMALL], ids=lambda s: s.name)
def test_prefill_causal_groups_and_boundaries(shape):
    # prefill attention on the matrix cores: chunks cut into groups of consecutive tokens with a causal
    # stagger; prefixes and chunk lengths around the 16-token block, 32-token group and group-size boundaries
    _say("case: prefill causal boundaries", shape.name)
    pre = [0, 1, 20, 31, 32, 33, 63, 64, 500, 27]
    chunk = [1, 5, 12, 13, 25, 7, 66, 3, 130, 40]
    base = synth.make_base(shape, seed=13, norm_ones=False)
    batch = synth.make_batch(shape, pre, [0] * len(pre), seed=13, headroom=140)
    pool = filled_batch(shape, batch, seed=13)
    mark_unwritten(shape, batch, pool, np.nan)    # never-written slots hold NaN: masked positions must not leak
    x = synth.make_hidden(shape, sum(chunk), seed=13, tag=5)
    orc = oracle.Oracle(oracle_config(shape, batch.num_blocks), base, None)
    want_pool = pool.copy()
    want, want_slots = orc.prefill(want_pool, batch.block_tables, pre, chunk, x)
    layer = make_layer(shape, base, None, batch.num_blocks)
    dpool = dev(pool_to_device_layout(pool), True)
    bt = torch.from_numpy(batch.block_tables).cuda()
    slots = torch.zeros(sum(chunk), dtype=torch.int64, device="cuda")
    got = layer.prefill_kv(dpool, bt, pre, chunk, dev(x, True), slot_out=slots)
    torch.cuda.synchronize()
    assert np.array_equal(slots.cpu().numpy(), want_slots)
    assert_close(host(got), want, 2e-2, "prefill x_out")
    # generic kernels give the same answer (GPU vs GPU, to tolerance)
    layer.set_kernel_mode(1)
    dpool2 = dev(pool_to_device_layout(pool), True)
    got2 = layer.prefill_kv(dpool2, bt, pre, chunk, dev(x, True))
    torch.cuda.synchronize()
    assert_close(host(got2), want, 2e-2, "prefill x_out (generic kernels)")
