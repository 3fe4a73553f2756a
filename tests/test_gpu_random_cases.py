"""GPU parity on drawn shapes: decode steps, prefill chunks and attention calls whose sequence counts, context
lengths, active-model counts, chunk lengths, rows per sequence and piece limits are drawn from a seeded
generator (one stream per case), so that the combinations are not the hand-picked ones of the other files:
mixed query-tile counts in one call, pieces of several sequences in one workgroup's share, prefixes and chunks
that end on and next to the 16-token block, the 32-token group and the 128-token round.  Same gates as
tests/test_gpu_parity.py; every case prints its draw before it runs."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_13281_amd import synth
from helpers import assert_close, filled_batch, mark_unwritten, oracle_config
from gpu_util import dev, host, make_layer, pool_to_device_layout
from test_gpu_parity import _check_decode

pytestmark = pytest.mark.gpu

LENS = [0, 1, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257, 511, 700, 1500, 2500, 4100]
CHUNKS = [1, 2, 5, 16, 31, 33, 64, 70, 129, 200]


def _rng(case):
    return np.random.default_rng([2603, 13281, case])


@pytest.mark.parametrize("case", range(8))
def test_drawn_decode_step(case):
    rng = _rng(case)
    M = int(rng.choice([3, 4, 8]))
    shape = (synth.LLAMA_SMALL if rng.integers(2) else synth.QWEN_SMALL).replace(n_models=M)
    S = int(rng.choice([1, 2, 5, 12, 40, 70]))
    lens = [int(x) for x in rng.choice(LENS[:18] if S > 12 else LENS, size=S)]
    n_active = [int(rng.integers(0, M + 1)) for _ in range(S)]
    print(f"case: drawn decode {case}: {shape.name} M {M} S {S} rows {S + sum(n_active)} lens {lens} active {n_active}", flush=True)
    _check_decode(shape, lens, n_active, seed=300 + case, mode=0)


@pytest.mark.parametrize("case", range(8))
def test_drawn_prefill_chunks(case):
    rng = _rng(100 + case)
    shape = synth.LLAMA_SMALL if rng.integers(2) else synth.QWEN_SMALL
    S = int(rng.integers(1, 6))
    pre = [int(x) for x in rng.choice(LENS[:19], size=S)]
    chunk = [int(x) for x in rng.choice(CHUNKS, size=S)]
    print(f"case: drawn prefill {case}: {shape.name} prefix {pre} chunk {chunk}", flush=True)
    seed = 400 + case
    base = synth.make_base(shape, seed=seed, norm_ones=False)
    batch = synth.make_batch(shape, pre, [0] * S, seed=seed, headroom=max(chunk) + 16)
    pool = filled_batch(shape, batch, seed=seed)
    mark_unwritten(shape, batch, pool, np.nan)      # masked and not yet written positions must not leak
    x = synth.make_hidden(shape, sum(chunk), seed=seed, tag=5)
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


@pytest.mark.parametrize("case", range(12))
def test_drawn_attention_call(case):
    rng = _rng(200 + case)
    g = (8, 4, 8, 1)[case % 4]
    most = (9, 7, 3)[case // 4]                     # rows of the fullest sequence: 5, 4 and 2 query tiles at g = 8
    shape = synth.LLAMA_SMALL.replace(n_q_heads=2 * g, n_kv_heads=2, d_model=256, n_models=8)
    S = int(rng.integers(1, 9))
    lens = [max(1, int(x)) for x in rng.choice(LENS, size=S)]
    rows = [int(rng.integers(1, most + 1)) for _ in range(S)]
    rows[int(rng.integers(S))] = most
    limit = int(rng.choice([0, 64, 128, 512]))
    print(f"case: drawn attention {case}: g {g} lens {lens} rows {rows} piece limit {limit}", flush=True)
    seed = 500 + case
    batch = synth.make_batch(shape, lens, [0] * S, seed=seed, headroom=0)
    pool = filled_batch(shape, batch, seed=seed)
    mark_unwritten(shape, batch, pool, np.nan)      # masked positions must not leak
    row_seq = np.repeat(np.arange(S), rows).astype(np.int32)
    q = synth.to_storage(rng.standard_normal((len(row_seq), shape.n_q_heads, shape.head_dim)).astype(np.float32) * 2, True)
    base = synth.make_base(shape)
    want = oracle.Oracle(oracle_config(shape, batch.num_blocks), base, None).attn_shared_kv(q, pool, batch.block_tables, lens, row_seq)
    layer = make_layer(shape, base, None, batch.num_blocks)
    layer.set_attn_piece_limit(limit)               # 0: automatic; else sequences longer than this are cut into pieces
    got = layer.attn_shared_kv(dev(q, True), dev(pool_to_device_layout(pool), True), torch.from_numpy(batch.block_tables).cuda(),
                               lens, row_seq)
    torch.cuda.synchronize()
    assert_close(host(got), want, 2e-2, "attention out")


@pytest.mark.parametrize("case", range(6))
def test_drawn_fp8_attention_call(case):
    """The same over an FP8 pool of drawn codes (g = 8): the oracle reads the values the codes stand for."""
    import dataclasses
    from gpu_util import fp8_pool_to_float, pool_from_device_layout
    rng = _rng(300 + case)
    shape = synth.QWEN_SMALL
    ks, vs = 0.02, 0.013
    most = (10, 7, 3)[case % 3]                     # 5, 4 and 2 query tiles
    S = int(rng.integers(1, 7))
    lens = np.int32([max(1, int(x)) for x in rng.choice(LENS, size=S)])
    rows = [int(rng.integers(1, most + 1)) for _ in range(S)]
    rows[int(rng.integers(S))] = most
    limit = int(rng.choice([0, 128, 512]))
    print(f"case: drawn fp8 attention {case}: lens {lens.tolist()} rows {rows} piece limit {limit}", flush=True)
    seed = 600 + case
    base = synth.make_base(shape, seed=seed)
    batch = synth.make_batch(shape, lens, np.zeros(S, np.int32), seed=seed, headroom=1)
    layer = make_layer(shape, base, None, batch.num_blocks, kv_fp8=True, k_scale=ks, v_scale=vs)
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(seed)
    codes = torch.randint(0, 256, layer.cfg.pool_shape(), generator=gen, device="cuda:0", dtype=torch.uint8)
    codes[(codes & 0x7f) == 0x7f] = 0x38            # no NaN codes inside the contexts
    codes[(codes & 0x78) == 0x78] &= 0xbf           # |code value| < 32: scores stay in a sane range
    row_seq = np.repeat(np.arange(S, dtype=np.int32), rows)
    qh = synth.to_storage((rng.standard_normal((len(row_seq), shape.n_q_heads, shape.head_dim)) * 0.3).astype(np.float32), True)
    opool = pool_from_device_layout(fp8_pool_to_float(codes, ks, vs), shape.block_size, shape.head_dim)
    orc = oracle.Oracle(dataclasses.replace(oracle_config(shape, batch.num_blocks), kv_fp8=True, k_scale=ks, v_scale=vs), base, None)
    want = orc.attn_shared_kv(qh, opool, batch.block_tables, lens, row_seq)
    layer.set_attn_piece_limit(limit)
    got = layer.attn_shared_kv(dev(qh.reshape(len(row_seq), -1), True), codes, torch.from_numpy(batch.block_tables).cuda(), lens, row_seq)
    torch.cuda.synchronize()
    assert_close(host(got).reshape(want.shape), want, 2e-2, "fp8 attention out")
    layer.close()
