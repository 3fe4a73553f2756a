"""Pins of the oracle's private-weight decoders (Sec. 3.2: the decoder may be adapted by full fine-tuning or
by other adapters; at inference every such decoder is a full weight matrix of its own)."""
import dataclasses

import numpy as np

import oracle
from paper_2603_13281_amd import synth
from helpers import filled_batch, oracle_config

PROJ5 = ("q", "o", "gate", "up", "down")


def _case(bf16=False):
    shape = synth.TINY if not bf16 else synth.LLAMA_SMALL
    base, lora = synth.make_base(shape, seed=9), synth.make_lora(shape, seed=9)
    batch = synth.make_batch(shape, [21, 40, 7], [2, 1, 0], seed=9)
    cfg = dataclasses.replace(oracle_config(shape, batch.num_blocks), lora_target_mask=0b1111001)   # q, o, gate, up, down
    lora = {p: lora[p] for p in PROJ5 if p in lora}
    x = synth.make_hidden(shape, batch.R, seed=9)
    return shape, base, lora, batch, cfg, x


def test_private_weights_equal_to_the_base_give_the_base_model():
    shape, base, lora, batch, cfg, x = _case()
    full = {p: np.repeat(base[p][None], shape.n_models, axis=0) for p in PROJ5}
    a = oracle.Oracle(cfg, base, None, full=full)
    b = oracle.Oracle(dataclasses.replace(cfg, n_models=0, lora_rank=0, lora_target_mask=0), base, None)
    pa, pb = filled_batch(shape, batch, seed=9), filled_batch(shape, batch, seed=9)
    ya, sa = a.decode_step(pa, batch.block_tables, batch.ctx_lens, batch.row_seq, batch.row_model, x)
    yb, sb = b.decode_step(pb, batch.block_tables, batch.ctx_lens, batch.row_seq, batch.row_model, x)
    assert np.array_equal(ya, yb) and np.array_equal(pa, pb) and np.array_equal(sa, sb)


def test_merged_lora_weights_reproduce_the_lora_decoder():
    """W + s B_j A_j as decoder j's private weight is the LoRA decoder (the textbook merge)."""
    shape, base, lora, batch, cfg, x = _case()
    full = {p: (base[p].astype(np.float64)[None] + cfg.lora_scale * np.einsum("mor,mri->moi", lora[p][1].astype(np.float64),
                                                                              lora[p][0].astype(np.float64))).astype(np.float32)
            for p in PROJ5}
    a = oracle.Oracle(cfg, base, None, full=full)
    b = oracle.Oracle(cfg, base, lora)
    pa, pb = filled_batch(shape, batch, seed=9), filled_batch(shape, batch, seed=9)
    ya, _ = a.decode_step(pa, batch.block_tables, batch.ctx_lens, batch.row_seq, batch.row_model, x)
    yb, _ = b.decode_step(pb, batch.block_tables, batch.ctx_lens, batch.row_seq, batch.row_model, x)
    assert np.abs(yb).max() > 0 and np.abs(ya - yb).max() <= 2e-5 * np.abs(yb).max()    # the merged weight was cast to float32
    enc = batch.row_model < 0
    assert np.array_equal(ya[enc], yb[enc])                                           # encoder rows never see decoder weights
    assert np.array_equal(pa, pb)


def test_cache_is_the_encoders_whichever_private_decoder_runs():
    shape, base, lora, batch, cfg, x = _case()
    full = synth.make_full_decoders(shape, base, seed=3, std=0.05)
    orc = oracle.Oracle(cfg, base, None, full=full)
    pools, outs = [], []
    for shift in (0, 1):
        rm = batch.row_model.copy()
        rm[rm >= 0] = (rm[rm >= 0] + shift) % shape.n_models
        p = filled_batch(shape, batch, seed=9)
        y, _ = orc.decode_step(p, batch.block_tables, batch.ctx_lens, batch.row_seq, rm, x)
        pools.append(p); outs.append(y)
    assert np.array_equal(pools[0], pools[1])                       # Eq. 4
    dec = batch.row_model >= 0
    assert np.abs(outs[0][dec] - outs[1][dec]).max() > 1e-3         # the decoders do differ
    assert np.array_equal(outs[0][~dec], outs[1][~dec])
