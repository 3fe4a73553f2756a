"""Decoders with private full weights on the GPU (grouped GEMMs over regrouped rows) against the oracle,
and against the library's own LoRA path on merged weights."""
import dataclasses

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

PROJ5 = ("q", "o", "gate", "up", "down")


def _oracle_cfg(shape, num_blocks):
    from helpers import oracle_config
    return dataclasses.replace(oracle_config(shape, num_blocks), lora_target_mask=0b1111001)


@pytest.mark.parametrize("kind", ["llama-small", "qwen-small"])
def test_decode_step_with_private_decoder_weights(kind):
    import oracle
    from gpu_util import dev, host, make_layer, pool_to_device_layout
    from helpers import assert_close, filled_batch
    from paper_2603_13281_amd import synth
    shape = {"llama-small": synth.LLAMA_SMALL, "qwen-small": synth.QWEN_SMALL}[kind]
    M = shape.n_models
    base = synth.make_base(shape, seed=12, norm_ones=False)
    full = synth.make_full_decoders(shape, base, seed=12, std=0.02)
    # rows of several models interleaved over the sequences; one model unused, one sequence without decoders
    lens = np.int32([300, 17, 96, 1200, 45])
    nact = np.int32([min(3, M), 1, 0, 2, min(3, M)])
    batch = synth.make_batch(shape, lens, nact, seed=12, headroom=2)
    orc = oracle.Oracle(_oracle_cfg(shape, batch.num_blocks), base, None, full=full)
    layer2 = make_layer(shape, base, synth.make_lora(shape, seed=1), batch.num_blocks)       # a context with n_models = M
    layer2.set_full_decoders({p: dev(full[p], True) for p in PROJ5})
    opool = filled_batch(shape, batch, seed=12)
    dpool = dev(pool_to_device_layout(opool), True)
    bt = torch.from_numpy(batch.block_tables).cuda()
    x = synth.make_hidden(shape, batch.R, seed=12)
    want, want_slots = orc.decode_step(opool, batch.block_tables, batch.ctx_lens, batch.row_seq, batch.row_model, x)
    slots = torch.zeros(batch.S, dtype=torch.int64, device="cuda:0")
    got = layer2.decode_step(dpool, bt, batch.ctx_lens, batch.row_seq, batch.row_model, dev(x, True), slot_out=slots)
    torch.cuda.synchronize()
    assert np.array_equal(slots.cpu().numpy(), want_slots)
    assert_close(host(got), want, 2e-2, f"{kind} private decoder weights")
    # back to the adapters: the same context runs its LoRA decoders again
    layer2.set_full_decoders(None)
    got_lora = layer2.decode_step(dpool.clone(), bt, batch.ctx_lens, batch.row_seq, batch.row_model, dev(x, True))
    torch.cuda.synchronize()
    dec = batch.row_model >= 0
    assert np.abs(host(got_lora)[dec] - host(got)[dec]).max() > 1e-3


def test_merged_lora_as_private_weights_matches_the_lora_path():
    """GPU against GPU: decoder j with the private weight W + s B_j A_j against the stacked LoRA GEMM."""
    from gpu_util import dev, host, make_layer, pool_to_device_layout
    from helpers import filled_batch
    from paper_2603_13281_amd import synth
    shape = synth.LLAMA_SMALL
    base, lora = synth.make_base(shape, seed=5), synth.make_lora(shape, seed=5, std=0.05)
    batch = synth.make_batch(shape, np.int32([500, 60, 33]), np.int32([4, 2, 1]), seed=5, headroom=2)
    merged = {p: synth.to_storage((base[p].astype(np.float64)[None] + shape.lora_scale * np.einsum(
        "mor,mri->moi", lora[p][1].astype(np.float64), lora[p][0].astype(np.float64))).astype(np.float32), True) for p in PROJ5}
    layer = make_layer(shape, base, lora, batch.num_blocks)
    pool = dev(pool_to_device_layout(filled_batch(shape, batch, seed=5)), True)
    bt = torch.from_numpy(batch.block_tables).cuda()
    x = dev(synth.make_hidden(shape, batch.R, seed=5), True)
    a_pool, b_pool = pool.clone(), pool.clone()
    a = layer.decode_step(a_pool, bt, batch.ctx_lens, batch.row_seq, batch.row_model, x)
    layer.set_full_decoders({p: dev(merged[p], True) for p in PROJ5})
    b = layer.decode_step(b_pool, bt, batch.ctx_lens, batch.row_seq, batch.row_model, x)
    torch.cuda.synchronize()
    a, b = host(a), host(b)
    assert np.abs(a - b).max() <= 2e-2 * np.abs(a).max()          # merged weights were rounded to bf16
    assert torch.equal(a_pool, b_pool)                            # the cache is the encoder's either way (Eq. 4)
    enc = batch.row_model < 0
    assert np.abs(a[enc] - b[enc]).max() <= 2.0 ** -7 * np.abs(a).max()   # same weights; another tile shape sums in another order


def test_private_weights_are_rejected_where_unsupported():
    from gpu_util import dev, make_layer
    from paper_2603_13281_amd import binding, synth
    shape = synth.TINY                                           # fp32: no matrix-core path
    base = synth.make_base(shape, seed=1)
    layer = make_layer(shape, base, synth.make_lora(shape, seed=1), 8)
    full = synth.make_full_decoders(shape, base, seed=1)
    with pytest.raises(binding.IcarusError) as e:
        layer.set_full_decoders({p: dev(full[p], False) for p in PROJ5})
    assert e.value.status_name == "UNSUPPORTED"
    shape = synth.LLAMA_SMALL
    base = synth.make_base(shape, seed=1)
    layer = make_layer(shape, base, synth.make_lora(shape, seed=1), 8)
    full = synth.make_full_decoders(shape, base, seed=1)
    d = {p: dev(full[p], True) for p in PROJ5}
    d.pop("down")
    with pytest.raises(binding.IcarusError) as e:
        layer.set_full_decoders(d)
    assert e.value.status_name == "INVALID_ARG"
