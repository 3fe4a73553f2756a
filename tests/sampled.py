"""Sampled parity at full benchmark sizes: the oracle recomputes some sequences (all their rows)
of a large device-resident workload from what the device pool held before the call.

Test infrastructure: used by the full-size GPU tests and by bench.py's cpu_baseline leg.
"""
from __future__ import annotations

import time

import numpy as np

import oracle
from helpers import assert_cache_close, assert_close, assert_fp8_cache_close, fill_pool, read_pool


def kv_to_host(shape, pool_dev, block_table_row, n_tokens, kv_scales=None):
    """First n_tokens cached K, V of one sequence from the device pool (library layout
    [blocks][Hkv][2][Bk*D], V transposed): float32 [n, Hkv, D] each.  kv_scales = (k_scale, v_scale): the pool
    holds FP8 E4M3 codes (uint8) and the values are code * scale."""
    import torch
    Bk, D, Hkv = shape.block_size, shape.head_dim, shape.n_kv_heads
    nb = (n_tokens + Bk - 1) // Bk
    if nb == 0:
        z = np.zeros((0, Hkv, D), dtype=np.float32)
        return z, z.copy()
    ids = torch.from_numpy(np.asarray(block_table_row[:nb], dtype=np.int64)).to(pool_dev.device)
    blk = pool_dev.index_select(0, ids)                                      # [nb, Hkv, 2, Bk*D]
    if kv_scales is not None:
        blk = blk.cpu().view(torch.float8_e4m3fn).to(torch.float32).numpy()
        blk[:, :, 0] *= np.float32(kv_scales[0])
        blk[:, :, 1] *= np.float32(kv_scales[1])
    else:
        blk = blk.to(torch.float32).cpu().numpy()
    K = blk[:, :, 0].reshape(nb, Hkv, Bk, D).transpose(0, 2, 1, 3).reshape(nb * Bk, Hkv, D)
    V = blk[:, :, 1].reshape(nb, Hkv, D, Bk).transpose(0, 3, 1, 2).reshape(nb * Bk, Hkv, D)
    return np.ascontiguousarray(K[:n_tokens]), np.ascontiguousarray(V[:n_tokens])


def oracle_config(shape, num_blocks, with_lora=True, kv_scales=None):
    return oracle.LayerConfig(
        kv_fp8=kv_scales is not None, k_scale=kv_scales[0] if kv_scales else 1.0, v_scale=kv_scales[1] if kv_scales else 1.0,
        d_model=shape.d_model, n_q_heads=shape.n_q_heads, n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim,
        d_ffn=shape.d_ffn, block_size=shape.block_size, num_blocks=num_blocks,
        n_models=shape.n_models if with_lora else 0, lora_rank=shape.lora_rank if with_lora else 0,
        lora_target_mask=shape.lora_target_mask if with_lora else 0, qk_norm=shape.qk_norm, bf16=shape.bf16,
        rope_theta=shape.rope_theta, rms_eps=shape.rms_eps, lora_scale=shape.lora_scale)


def snapshot_prefixes(shape, pool_dev, block_tables, ctx_lens, sample, kv_scales=None):
    """K, V of the sampled sequences as cached BEFORE the call under test."""
    return {int(s): kv_to_host(shape, pool_dev, block_tables[s], int(ctx_lens[s]), kv_scales) for s in sample}


def decode_sample_check(shape, base, lora, prefixes, ctx_lens, row_seq, row_model, x_host, x_dev_out, tol, what,
                        slots_dev=None, block_tables=None, kv_scales=None, full=None, pool_dev_after=None):
    """Oracle decode step of the sequences in `prefixes` (their K/V before the call), compared with
    the device output rows of those sequences.  pool_dev_after (with block_tables): the device pool after the
    call; the K/V entry the call appended for each sampled sequence is compared with the oracle's.
    Returns timing and sizes of the sample."""
    import torch
    sample = sorted(prefixes)
    Bk = shape.block_size
    need = [(int(ctx_lens[s]) + 1 + Bk - 1) // Bk for s in sample]
    orc = oracle.Oracle(oracle_config(shape, sum(need), lora is not None or full is not None, kv_scales), base, lora, full=full)
    pool = orc.new_pool()
    bt = np.zeros((len(sample), max(need)), dtype=np.int32)
    k = 0
    rs, rmod, xs, rows_all = [], [], [], []
    for i, s in enumerate(sample):
        bt[i, :need[i]] = np.arange(k, k + need[i])
        k += need[i]
        K, V = prefixes[s]
        fill_pool(pool, bt[i], K, V)
        for r in np.flatnonzero(row_seq == s):
            rs.append(i)
            rmod.append(int(row_model[r]))
            xs.append(x_host[r])
            rows_all.append(int(r))
    t0 = time.perf_counter()
    want, slots = orc.decode_step(pool, bt, np.int32([ctx_lens[s] for s in sample]), np.int32(rs), np.int32(rmod), np.stack(xs))
    dt = time.perf_counter() - t0
    got = x_dev_out[torch.from_numpy(np.int64(rows_all)).to(x_dev_out.device)].to(torch.float32).cpu().numpy()
    assert_close(got, want, tol, what)
    if slots_dev is not None:      # slot indices are integers: exact, through the device block table
        got_slots = slots_dev.cpu().numpy()
        for i, s in enumerate(sample):
            p = int(ctx_lens[s])
            assert int(got_slots[s]) == int(block_tables[s, p // Bk]) * Bk + p % Bk, f"{what}: slot of sequence {s}"
    if pool_dev_after is not None:   # the values of the appended entries
        gk, gv, wk, wv = [], [], [], []
        for i, s in enumerate(sample):
            p = int(ctx_lens[s])
            # the block that holds position p, read from the device through the table
            Kd, Vd = kv_to_host(shape, pool_dev_after, block_tables[s][p // Bk:p // Bk + 1], p % Bk + 1, kv_scales)
            Ko, Vo = read_pool(pool, bt[i], p + 1)
            gk.append(Kd[-1]); gv.append(Vd[-1]); wk.append(Ko[-1]); wv.append(Vo[-1])
        for got_e, want_e, nm, sc in ((np.stack(gk), np.stack(wk), "K", kv_scales[0] if kv_scales else None),
                                      (np.stack(gv), np.stack(wv), "V", kv_scales[1] if kv_scales else None)):
            if kv_scales is not None:
                assert_fp8_cache_close(got_e, want_e, sc, shape.bf16, f"{what}: appended {nm}")
            else:
                assert_cache_close(got_e, want_e, shape.bf16, f"{what}: appended {nm}",
                                   rms=float(np.sqrt(np.mean(want_e.astype(np.float64) ** 2))))
    n_dec = sum(1 for m in rmod if m >= 0)
    return {"seconds": dt, "rows": len(rs), "decoder_rows": n_dec, "cached_tokens": int(sum(int(ctx_lens[s]) + 1 for s in sample)),
            "sample": sample}


def prefill_sample_check(shape, base, prefix_kv, L, T, x_host_chunk, x_dev_out_chunk, picks, tol, what, kv_scales=None):
    """Oracle prefill of one sequence's chunk over its cached prefix: K/V of all T tokens, the full
    layer for the tokens in `picks`; compares those rows with the device output."""
    import torch
    Bk = shape.block_size
    nb = (L + T + Bk - 1) // Bk
    orc = oracle.Oracle(oracle_config(shape, nb, False, kv_scales), base, None)
    pool = orc.new_pool()
    bt = np.arange(nb, dtype=np.int32)[None]
    fill_pool(pool, bt[0], *prefix_kv)
    sel = np.zeros(T, dtype=np.uint8)
    sel[picks] = 1
    t0 = time.perf_counter()
    want, _ = orc.prefill(pool, bt, [L], [T], x_host_chunk, select=sel)
    dt = time.perf_counter() - t0
    got = x_dev_out_chunk.to(torch.float32).cpu().numpy()
    assert_close(got[picks], want[picks], tol, what)
    return {"seconds": dt, "pool": pool, "block_table": bt[0]}
