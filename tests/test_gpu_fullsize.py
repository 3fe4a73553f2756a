"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

The oracle cannot run a whole benchmark batch in seconds, so it recomputes a sample: all rows of a
few sequences (decode) or selected chunk tokens of one sequence (prefill), from the K/V the device
pool held before the call.  What holds at any size is checked on everything: slot indices, cache
bytes outside the written slots, finiteness.  Workloads are the seeded synthetic ones of bench.py.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2      # max |got - want| / max |want| per output tensor, bf16 storage


def _sample_sequences(batch, ctx, n_random, seed):
    """Longest and shortest context, most and fewest active models, plus seeded random picks."""
    rows_per_seq = np.bincount(batch.row_seq, minlength=batch.S)
    picks = {int(np.argmax(ctx)), int(np.argmin(ctx)), int(np.argmax(rows_per_seq)), int(np.argmin(rows_per_seq))}
    rng = np.random.default_rng(seed)
    for s in rng.permutation(batch.S):
        if len(picks) >= 4 + n_random or len(picks) == batch.S:
            break
        picks.add(int(s))
    return sorted(picks)


@pytest.mark.parametrize("name,n_random", [("c3", 1), ("c5", 0), ("c2", 0), ("c3-fp8", 1), ("c5-fp8", 0), ("c3-full", 0)])
def test_decode_full_size_sampled(name, n_random):
    import sampled
    from paper_2603_13281_amd import workloads

    wl = workloads.build_decode_workload(name, "cuda:0")
    sh, b, step = wl.shape, wl.batch, 0
    ctx = wl.ctx_lens(step)
    sample = _sample_sequences(b, ctx, n_random, seed=11)
    if name.startswith("c5"):
        sample = [0, b.S - 1]                    # 32768-token contexts with 72 stacked heads: a sequence is ~10 s of oracle
    prefixes = sampled.snapshot_prefixes(sh, wl.pool, b.block_tables, ctx, sample, wl.kv_scales)
    pool_before = wl.pool.clone()
    x_out = torch.empty_like(wl.x[0])
    slots = torch.full((b.S,), -1, dtype=torch.int64, device="cuda:0")
    wl.layer.decode_step(wl.pool, wl.block_tables, ctx, b.row_seq, b.row_model, wl.x[0], x_out=x_out, slot_out=slots)
    torch.cuda.synchronize()
    assert torch.isfinite(x_out.to(torch.float32)).all()
    info = sampled.decode_sample_check(sh, wl.base, wl.lora, prefixes, ctx, b.row_seq, b.row_model, wl.x_host[0], x_out, TOL_BF16,
                                       f"{name} full-size sample", slots_dev=slots, block_tables=b.block_tables, kv_scales=wl.kv_scales, full=wl.full,
                                       pool_dev_after=wl.pool)
    assert info["rows"] >= len(sample)
    # every slot index, exactly; and no cache byte changed outside the S written slots
    Bk = sh.block_size
    want_slots = np.array([int(b.block_tables[s, int(ctx[s]) // Bk]) * Bk + int(ctx[s]) % Bk for s in range(b.S)], dtype=np.int64)
    assert np.array_equal(slots.cpu().numpy(), want_slots)
    changed = (wl.pool != pool_before).reshape(wl.pool.shape[0], -1).any(dim=1).nonzero().flatten().cpu().numpy()
    assert set(changed.tolist()) <= set((want_slots // Bk).tolist())
    blk = torch.from_numpy(want_slots // Bk).to("cuda:0")
    D, Hkv = sh.head_dim, sh.n_kv_heads
    diff = (wl.pool[blk] != pool_before[blk])                       # [S, Hkv, 2, Bk*D]
    k_changed = diff[:, :, 0].reshape(b.S, Hkv, Bk, D).any(dim=3).any(dim=1)      # [S, Bk] token slots of K
    v_changed = diff[:, :, 1].reshape(b.S, Hkv, D, Bk).any(dim=2).any(dim=1)      # V is stored transposed
    allowed = torch.zeros_like(k_changed)
    allowed[torch.arange(b.S, device="cuda:0"), torch.from_numpy(want_slots % Bk).to("cuda:0")] = True
    assert not (k_changed & ~allowed).any() and not (v_changed & ~allowed).any()


@pytest.mark.parametrize("name", ["c4", "c4-fp8"])
def test_prefill_full_size_sampled_then_decode_with_unseen_model(name):
    """Config 4: the chunk through the frozen encoder at full size -- three sequences (first, middle, last), chunk
    tokens on both sides of the attention kernel's 64-token workgroup tiles, against the oracle -- then one decode
    step of a model that never touched these sequences: it must read the cache the encoder wrote, change nothing
    but the S new slots, and match the oracle on sampled sequences."""
    import helpers
    import sampled
    from paper_2603_13281_amd import binding, synth, workloads

    print("case:", name, "prefill at full size", flush=True)
    wl = workloads.build_prefill_workload(name, "cuda:0")
    sh, S = wl.shape, len(wl.chunk_lens)
    pre, T = wl.batch.ctx_lens, int(wl.chunk_lens[0])
    bt = wl.batch.block_tables
    seqs = [0, S // 2, S - 1]
    prefix = {s: sampled.kv_to_host(sh, wl.pool, bt[s], int(pre[s]), wl.kv_scales) for s in seqs}
    pool_before = wl.pool.clone()
    x_out = torch.empty_like(wl.x)
    slots = torch.full((wl.n_tokens,), -1, dtype=torch.int64, device="cuda:0")
    wl.layer.prefill_kv(wl.pool, wl.block_tables, pre, wl.chunk_lens, wl.x, x_out=x_out, slot_out=slots)
    torch.cuda.synchronize()
    assert torch.isfinite(x_out.to(torch.float32)).all()
    picks = sorted({0, 63, 64, 255, 256, T - 1} & set(range(T)))
    for s0 in seqs:
        print("  sequence", s0, "picks", picks, flush=True)
        L = int(pre[s0])
        r0 = int(wl.chunk_lens[:s0].sum())
        res = sampled.prefill_sample_check(sh, wl.base, prefix[s0], L, T, wl.x_host[r0:r0 + T], x_out[r0:r0 + T], picks, TOL_BF16,
                                           f"{name} full-size prefill, sequence {s0}", kv_scales=wl.kv_scales)
        # the cache the device wrote for this sequence against the oracle's, every chunk token
        Kd, Vd = sampled.kv_to_host(sh, wl.pool, bt[s0], L + T, wl.kv_scales)
        Ko, Vo = helpers.read_pool(res["pool"], res["block_table"], L + T)
        for got, want, nm, sc in ((Kd[L:], Ko[L:], "K", 0), (Vd[L:], Vo[L:], "V", 1)):
            if wl.kv_scales is not None:
                helpers.assert_fp8_cache_close(got, want, wl.kv_scales[sc], True, f"{name} cache {nm} of sequence {s0}")
            else:
                helpers.assert_cache_close(got, want, True, f"{name} cache {nm} of sequence {s0}",
                                           rms=float(np.sqrt(np.mean(want.astype(np.float64) ** 2))))
    # slots: exact for every token of every sequence
    Bk = sh.block_size
    want_slots = np.concatenate([[int(bt[s, (int(pre[s]) + i) // Bk]) * Bk + (int(pre[s]) + i) % Bk for i in range(int(wl.chunk_lens[s]))]
                                 for s in range(S)]).astype(np.int64)
    assert np.array_equal(slots.cpu().numpy(), want_slots)
    changed = (wl.pool != pool_before).reshape(wl.pool.shape[0], -1).any(dim=1).nonzero().flatten().cpu().numpy()
    assert set(changed.tolist()) <= set((want_slots // Bk).tolist())
    del pool_before

    # a decoder that has never run on these sequences: one encoder row + one decoder row per sequence
    shl = sh.replace(n_models=8)
    lora = synth.make_lora(shl, seed=3)
    cfg = workloads.layer_config(shl, wl.pool.shape[0], int(pre.max()) + T + 2)
    if wl.kv_scales is not None:
        cfg.kv_fp8, cfg.k_scale, cfg.v_scale = True, wl.kv_scales[0], wl.kv_scales[1]
    dbase = {k: workloads.upload(v, True, "cuda:0") for k, v in wl.base.items()}
    dlora = {p: (workloads.upload(A, True, "cuda:0"), workloads.upload(B, True, "cuda:0")) for p, (A, B) in lora.items()}
    dec = binding.IcarusLayer(cfg, dbase, dlora)
    ctx = (pre + wl.chunk_lens).astype(np.int32)
    row_seq = np.repeat(np.arange(S, dtype=np.int32), 2)
    row_model = np.tile(np.int32([-1, 5]), S)
    xh = synth.make_hidden(shl, 2 * S, seed=3, tag=31)
    xd = workloads.upload(xh, True, "cuda:0")
    sample = [0, S - 1]
    prefixes = sampled.snapshot_prefixes(sh, wl.pool, bt, ctx, sample, wl.kv_scales)
    pool_mid = wl.pool.clone()
    y = torch.empty_like(xd)
    dslots = torch.full((S,), -1, dtype=torch.int64, device="cuda:0")
    dec.decode_step(wl.pool, wl.block_tables, ctx, row_seq, row_model, xd, x_out=y, slot_out=dslots)
    torch.cuda.synchronize()
    sampled.decode_sample_check(shl, wl.base, lora, prefixes, ctx, row_seq, row_model, xh, y, TOL_BF16,
                                f"{name} decode after prefill", slots_dev=dslots, block_tables=bt, kv_scales=wl.kv_scales,
                                pool_dev_after=wl.pool)
    want_d = np.array([int(bt[s, int(ctx[s]) // Bk]) * Bk + int(ctx[s]) % Bk for s in range(S)], dtype=np.int64)
    assert np.array_equal(dslots.cpu().numpy(), want_d)
    changed = (wl.pool != pool_mid).reshape(wl.pool.shape[0], -1).any(dim=1).nonzero().flatten().cpu().numpy()
    assert set(changed.tolist()) <= set((want_d // Bk).tolist())
