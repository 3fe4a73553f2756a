"""icarus_attn_shared_kv_static -- the entry point that allocates nothing -- against icarus_attn_shared_kv.

Both run the same kernels over the same plan; only the home of the scratch (the library's static device array
instead of the caller's workspace) and the way the metadata travels differ, so the outputs must be identical bit
for bit, and both must match the oracle to the attention tolerance.  Two calls in a row, the second smaller: the
array keeps the first call's contents and nothing of it may leak into the second."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _case(shape, lens, rows_per_seq, seed, limit):
    import oracle
    from gpu_util import dev, host, make_layer, pool_to_device_layout
    from helpers import assert_close, filled_batch, mark_unwritten, oracle_config
    from paper_2603_13281_amd import synth
    print("case: static attention", shape.name, "lens", lens, "rows", rows_per_seq, "piece limit", limit, flush=True)
    batch = synth.make_batch(shape, lens, [0] * len(lens), seed=seed, headroom=0)
    pool = filled_batch(shape, batch, seed=seed)
    mark_unwritten(shape, batch, pool, np.nan)                   # unwritten slots must not leak
    row_seq = np.repeat(np.arange(len(lens)), rows_per_seq).astype(np.int32)
    q = synth.to_storage(np.random.default_rng(seed).standard_normal((len(row_seq), shape.n_q_heads, shape.head_dim)).astype(np.float32),
                         shape.bf16)
    base = synth.make_base(shape)
    want = oracle.Oracle(oracle_config(shape, batch.num_blocks), base, None).attn_shared_kv(q, pool, batch.block_tables, lens, row_seq)
    layer = make_layer(shape, base, None, batch.num_blocks)
    layer.set_attn_piece_limit(limit)
    dpool = dev(pool_to_device_layout(pool), shape.bf16)
    bt = torch.from_numpy(batch.block_tables).cuda()
    dq = dev(q, shape.bf16)
    ref = layer.attn_shared_kv(dq, dpool, bt, lens, row_seq)
    out = torch.full_like(ref, float("nan"))
    layer.attn_shared_kv_static(dq, dpool, bt, lens, row_seq, out)
    torch.cuda.synchronize()
    assert torch.equal(out, ref), "static entry point differs from icarus_attn_shared_kv"
    assert_close(host(out), want, 2e-2 if shape.bf16 else 1e-4, "static attention vs oracle")
    layer.close()


def test_static_attention_twice_in_a_row_second_call_smaller():
    from paper_2603_13281_amd import synth
    sh = synth.LLAMA_SMALL.replace(n_models=8)
    # cut sequences (partial results in the array), several query tiles, ragged tails
    _case(sh, [3001, 700, 33, 1500], [9, 2, 1, 5], seed=31, limit=256)
    # smaller: fewer sequences, fewer rows, shorter contexts, fewer pieces
    _case(sh, [257, 31], [2, 1], seed=32, limit=128)
    # the vector kernels (fp32 shape) use the array for their row metadata only
    _case(synth.TINY, [130, 16], [3, 1], seed=33, limit=0)


def test_static_attention_refuses_what_does_not_fit():
    from gpu_util import make_layer
    from paper_2603_13281_amd import binding, synth
    sh = synth.LLAMA_SMALL.replace(n_models=8)
    # 200 sequences x 9 rows with a 32-token piece limit: ~6400 pieces x 2 kv-heads x 36 stacked queries x 130 floats
    # = 240 MB of partial results, far beyond the 32 MiB array: refused on the host, nothing launched
    S, L = 200, 1000
    batch = synth.make_batch(sh, [L] * S, [0] * S, seed=1, headroom=0)
    layer = make_layer(sh, synth.make_base(sh), None, batch.num_blocks)
    layer.set_attn_piece_limit(32)
    row_seq = np.repeat(np.arange(S), 9).astype(np.int32)
    q = torch.zeros((len(row_seq), sh.n_q_heads * sh.head_dim), dtype=torch.bfloat16, device="cuda:0")
    pool = torch.zeros(layer.cfg.pool_shape(), dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(binding.IcarusError) as e:
        layer.attn_shared_kv_static(q, pool, torch.from_numpy(batch.block_tables).cuda(), [L] * S, row_seq, torch.empty_like(q))
    assert e.value.status_name == "CAPACITY", str(e.value)
    layer.close()
