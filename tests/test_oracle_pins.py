"""Pins for the CPU oracle: closed forms, brute force on tiny shapes, library cross-checks of
the adapter-free special case, and the paper's structural invariants.

Each test names the passage or the mathematics that fixes the expected value.  None of them
calls the GPU path.
"""
import math
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2603_13281_amd import synth
from helpers import fill_pool, filled_batch, oracle_config, read_pool

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# --------------------------------------------------------------------------- primitives

def test_round_bf16_matches_library_cast():
    # float32 -> bfloat16 round-to-nearest-even as torch implements it (library routine).
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.standard_normal(4000).astype(np.float32) * s for s in (1e-3, 1.0, 300.0)])
    x = np.concatenate([x, np.float32([1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, -1.0 - 2 ** -8, 0.0, 2 ** -130])])
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    got = oracle.round_bf16(x.astype(np.float64))
    assert np.array_equal(got, want)


def test_round_bf16_is_direct_from_double():
    # 1 + 2^-8 + 2^-40 lies above the tie: direct rounding goes up; via float32 it would tie to even.
    assert oracle.round_bf16([1.0 + 2.0 ** -8 + 2.0 ** -40])[0] == 1.0 + 2.0 ** -7


def test_slot_closed_form():
    # physical slot = block_table[p // Bk] * Bk + p % Bk  (paged concat_sequence, Alg. 3)
    bt = np.array([7, 3, 11, 0], dtype=np.int32)
    for p in range(64):
        assert oracle.slot(bt, p, 16) == int(bt[p // 16]) * 16 + p % 16
    assert oracle.slot(bt, 16, 16) == 48 and oracle.slot(bt, 15, 16) == 127


def test_rmsnorm_closed_forms():
    # x = (3, 4): mean square 12.5 -> y = x / sqrt(12.5) * w
    y = oracle.rmsnorm([3.0, 4.0], [1.0, 2.0], 0.0)
    assert np.allclose(y, [3 / math.sqrt(12.5), 8 / math.sqrt(12.5)], rtol=1e-15)
    rng = np.random.default_rng(0)
    x = rng.standard_normal(257)
    y = oracle.rmsnorm(x, np.ones(257), 0.0)
    assert abs(np.mean(y ** 2) - 1.0) < 1e-12                     # unit mean square
    assert np.allclose(oracle.rmsnorm(5 * x, np.ones(257), 0.0), y, rtol=1e-12)  # scale invariant
    lib = torch.nn.functional.rms_norm(torch.from_numpy(x), (257,), torch.ones(257, dtype=torch.float64), 1e-5)
    assert np.allclose(oracle.rmsnorm(x, np.ones(257), 1e-5), lib.numpy(), rtol=1e-12)


def test_linear_is_matvec():
    rng = np.random.default_rng(2)
    W = rng.standard_normal((37, 53)).astype(np.float32)
    x = rng.standard_normal(53)
    assert np.allclose(oracle.linear(W, x), W.astype(np.float64) @ x, rtol=1e-13)
    # a transposed operand would fail this: W = e_2 e_5^T picks x[5] into y[2]
    E = np.zeros((4, 7), dtype=np.float32)
    E[2, 5] = 1
    assert np.array_equal(oracle.linear(E, np.arange(7.0)), [0, 0, 5, 0])


def test_lora_equals_merged_dense():
    # W x + s B (A x) == (W + s B A) x  (LoRA; Alg. 2 read as input-side adapter)
    rng = np.random.default_rng(3)
    A = rng.standard_normal((4, 19)).astype(np.float32)
    B = rng.standard_normal((11, 4)).astype(np.float32)
    x = rng.standard_normal(19)
    want = 2.5 * (B.astype(np.float64) @ A.astype(np.float64)) @ x
    assert np.allclose(oracle.adaptive_linear(A, B, 2.5, x), want, rtol=1e-12)
    assert np.all(oracle.adaptive_linear(A, np.zeros_like(B), 2.5, x) == 0.0)


def test_rope_closed_forms():
    # D = 2: one pair (0, 1), inv_freq = 1 -> plane rotation by the angle p
    v = oracle.rope([[1.0, 0.0]], 3, 10000.0)
    assert np.allclose(v, [[math.cos(3), math.sin(3)]], atol=1e-15)
    # D = 4: pairs (0,2) and (1,3); angles p and p * theta^(-1/2)
    th = 100.0
    v = oracle.rope([[1.0, 1.0, 0.0, 0.0]], 5, th)
    assert np.allclose(v, [[math.cos(5), math.cos(0.5), math.sin(5), math.sin(0.5)]], atol=1e-15)
    rng = np.random.default_rng(4)
    q, k = rng.standard_normal((2, 64)), rng.standard_normal((2, 64))
    assert np.array_equal(oracle.rope(q, 0, 5e5), q)                       # position 0 is the identity
    assert np.allclose(np.linalg.norm(oracle.rope(q, 777, 5e5), axis=1), np.linalg.norm(q, axis=1), rtol=1e-13)
    a = np.sum(oracle.rope(q, 100, 5e5) * oracle.rope(k, 37, 5e5), axis=1)
    b = np.sum(oracle.rope(q, 1100, 5e5) * oracle.rope(k, 1037, 5e5), axis=1)
    assert np.allclose(a, b, rtol=1e-9, atol=1e-10)                        # depends on m - n only
    # independent formulation: complex multiplication by exp(i p w)
    D = 64
    w = 5e5 ** (-np.arange(D // 2) * 2.0 / D)
    z = (q[:, :D // 2] + 1j * q[:, D // 2:]) * np.exp(1j * 12345 * w)
    assert np.allclose(oracle.rope(q, 12345, 5e5), np.concatenate([z.real, z.imag], axis=1), rtol=1e-10, atol=1e-12)


def _brute_attention(q, K, V, kv_of):
    U, D = q.shape
    n = K.shape[0]
    out = [[0.0] * D for _ in range(U)]
    for u in range(U):
        c = kv_of[u]
        s = [sum(float(q[u][i]) * float(K[t][c][i]) for i in range(D)) / math.sqrt(D) for t in range(n)]
        m = max(s)
        e = [math.exp(v - m) for v in s]
        z = sum(e)
        for i in range(D):
            out[u][i] = sum(e[t] * float(V[t][c][i]) for t in range(n)) / z
    return np.array(out)


@pytest.mark.parametrize("D,n,Hkv,g", [(2, 1, 1, 1), (2, 5, 1, 3), (4, 3, 2, 2), (4, 5, 2, 1)])
def test_attention_brute_force(D, n, Hkv, g):
    rng = np.random.default_rng(10 * D + n)
    Hq = Hkv * g
    q = rng.standard_normal((2 * Hq, D))
    K = rng.standard_normal((n, Hkv, D)).astype(np.float32)
    V = rng.standard_normal((n, Hkv, D)).astype(np.float32)
    kv_of = [(u % Hq) // g for u in range(2 * Hq)]
    assert np.allclose(oracle.attention(q, K, V, kv_of), _brute_attention(q, K, V, kv_of), rtol=1e-12, atol=1e-14)


def test_attention_closed_forms():
    rng = np.random.default_rng(5)
    D, n, Hkv = 8, 6, 2
    q = rng.standard_normal((4, D))
    K = rng.standard_normal((n, Hkv, D)).astype(np.float32)
    V = rng.standard_normal((n, Hkv, D)).astype(np.float32)
    kv_of = [0, 0, 1, 1]
    # all V rows equal -> the output is that row, whatever the scores
    Vc = np.broadcast_to(V[:1], V.shape).copy()
    o = oracle.attention(q, K, Vc, kv_of)
    assert np.allclose(o[0], Vc[0, 0], rtol=1e-14) and np.allclose(o[3], Vc[0, 1], rtol=1e-14)
    # q = 0 -> uniform average of V over positions
    o = oracle.attention(np.zeros((4, D)), K, V, kv_of)
    assert np.allclose(o[1], V[:, 0].mean(0), rtol=1e-6) and np.allclose(o[2], V[:, 1].mean(0), rtol=1e-6)
    # one overwhelming logit -> that position's V row
    Kh = K.copy()
    Kh[4, 0] = 0
    Kh[4, 0, 0] = 1000.0
    qh = np.zeros((4, D))
    qh[:, 0] = 50.0
    o = oracle.attention(qh, Kh, V, [0, 0, 0, 0])
    assert np.allclose(o[0], V[4, 0], rtol=1e-12)
    # a single cached position -> its V row
    o = oracle.attention(q, K[:1], V[:1], kv_of)
    assert np.allclose(o[2], V[0, 1], rtol=1e-14)


def test_attention_golden_weights():
    # scores ln1, ln2, ln3 (after the 1/sqrt(D) scale) give weights 1/6, 2/6, 3/6: hand-computed fixture.
    rows = [l.split() for l in open(os.path.join(GOLDEN, "attention_closed_form.txt")) if l.strip() and not l.startswith("#")]
    D = 4
    q = np.array([[2.0, 0, 0, 0]])           # q.k / sqrt(4) = k[0]
    K = np.zeros((3, 1, D), dtype=np.float64)
    K[:, 0, 0] = [math.log(1), math.log(2), math.log(3)]
    V = np.array([[float(v) for v in r[:D]] for r in rows[:3]]).reshape(3, 1, D)
    want = np.array([float(v) for v in rows[3][:D]])
    # K holds logs that float32 cannot represent exactly: compare at float32 resolution
    o = oracle.attention(q, K.astype(np.float32), V.astype(np.float32), [0])
    assert np.allclose(o[0], want, rtol=2e-7)


# --------------------------------------------------------------------------- whole layer vs library

def _torch_layer(shape, base, x, K_prev, V_prev, pos):
    """Textbook pre-norm GQA block in float64 from library routines, no adapters.
    K_prev, V_prev [pos, Hkv, D] already-cached (post-RoPE) entries.  Returns y, k_new, v_new."""
    F = torch.nn.functional
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    d, Hq, Hkv, D = shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    x = t(x)
    xn = F.rms_norm(x, (d,), t(base["norm_attn"]), shape.rms_eps)
    q = F.linear(xn, t(base["q"])).view(Hq, D)
    k = F.linear(xn, t(base["k"])).view(Hkv, D)
    v = F.linear(xn, t(base["v"])).view(Hkv, D)
    if shape.qk_norm:
        q = F.rms_norm(q, (D,), t(base["q_norm"]), shape.rms_eps)
        k = F.rms_norm(k, (D,), t(base["k_norm"]), shape.rms_eps)
    w = torch.tensor(shape.rope_theta, dtype=torch.float64) ** (-torch.arange(D // 2, dtype=torch.float64) * 2 / D)
    rot = torch.polar(torch.ones(D // 2, dtype=torch.float64), pos * w)

    def rope(z):
        c = torch.complex(z[:, :D // 2], z[:, D // 2:]) * rot
        return torch.cat([c.real, c.imag], dim=1)
    q, k = rope(q), rope(k)
    kr = t(synth.to_storage(k.numpy().astype(np.float32), shape.bf16)) if shape.bf16 else t(k.numpy().astype(np.float32))
    vr = t(synth.to_storage(v.numpy().astype(np.float32), shape.bf16)) if shape.bf16 else t(v.numpy().astype(np.float32))
    Kall = torch.cat([t(K_prev), kr[None]], 0)       # [n, Hkv, D]
    Vall = torch.cat([t(V_prev), vr[None]], 0)
    g = Hq // Hkv
    Kh = Kall.permute(1, 0, 2).repeat_interleave(g, dim=0)   # [Hq, n, D]
    Vh = Vall.permute(1, 0, 2).repeat_interleave(g, dim=0)
    a = F.scaled_dot_product_attention(q[:, None, :], Kh, Vh)  # [Hq, 1, D]
    z = x + F.linear(a.reshape(Hq * D), t(base["o"]))
    zn = F.rms_norm(z, (d,), t(base["norm_ffn"]), shape.rms_eps)
    h = F.silu(F.linear(zn, t(base["gate"]))) * F.linear(zn, t(base["up"]))
    y = z + F.linear(h, t(base["down"]))
    return y.numpy(), kr.numpy(), vr.numpy()


SHAPES = [
    synth.TINY.replace(d_model=64, n_q_heads=4, n_kv_heads=4, head_dim=16, d_ffn=96),
    synth.LLAMA_SMALL.replace(d_model=128, n_q_heads=8, n_kv_heads=2, head_dim=32, d_ffn=160, lora_rank=4),
    synth.QWEN_SMALL.replace(d_model=96, n_q_heads=6, n_kv_heads=2, head_dim=16, d_ffn=128, lora_rank=4),
]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: s.name)
def test_base_step_equals_library_layer(shape):
    # Sec. 3.1: a decoder-only transformer is the special case with identical encoder and decoder
    # parameters -> with no adapter the step is a plain base-model layer step.
    base = synth.make_base(shape, seed=3, norm_ones=False)
    batch = synth.make_batch(shape, [37], [0], seed=1)
    pool = filled_batch(shape, batch, seed=2)
    cfg = oracle_config(shape, batch.num_blocks)
    orc = oracle.Oracle(cfg, base, None)
    x = synth.make_hidden(shape, 1, seed=4)
    Kp, Vp = read_pool(pool, batch.block_tables[0], 37)
    y, slots = orc.decode_step(pool, batch.block_tables, batch.ctx_lens, batch.row_seq, batch.row_model, x)
    want, k_new, v_new = _torch_layer(shape, base, x[0], Kp, Vp, 37)
    # compare before the output rounding would hide differences: oracle rounds x_out to storage precision
    tol = 2.0 ** -8 if shape.bf16 else 1e-6
    assert np.allclose(y[0], want, rtol=tol, atol=tol * 1e-2 + (0 if shape.bf16 else 1e-7))
    Kn, Vn = read_pool(pool, batch.block_tables[0], 38)
    assert np.array_equal(Kn[37], k_new.astype(np.float32)) and np.array_equal(Vn[37], v_new.astype(np.float32))
    assert slots[0] == int(batch.block_tables[0][37 // 16]) * 16 + 37 % 16


def test_unrounded_output_matches_library_tightly():
    # same as above on an fp32-storage shape, where output rounding is float32: 1e-6 agreement
    shape = SHAPES[0]
    base = synth.make_base(shape, seed=8, norm_ones=False)
    batch = synth.make_batch(shape, [5], [0], seed=1)
    pool = filled_batch(shape, batch, seed=2)
    orc = oracle.Oracle(oracle_config(shape, batch.num_blocks), base, None)
    x = synth.make_hidden(shape, 1, seed=4)
    Kp, Vp = read_pool(pool, batch.block_tables[0], 5)
    y, _ = orc.decode_step(pool, batch.block_tables, batch.ctx_lens, batch.row_seq, batch.row_model, x)
    want, _, _ = _torch_layer(shape, base, x[0], Kp, Vp, 5)
    assert np.max(np.abs(y[0] - want)) / np.max(np.abs(want)) < 5e-7


# --------------------------------------------------------------------------- invariants of the method

def _setup(shape, ctx, n_active, seed=0, zero_b=False, lora_std=0.05):
    base = synth.make_base(shape, seed=seed, norm_ones=False)
    lora = synth.make_lora(shape, seed=seed, zero_b=zero_b, std=lora_std)
    batch = synth.make_batch(shape, ctx, n_active, seed=seed)
    pool = filled_batch(shape, batch, seed=seed)
    orc = oracle.Oracle(oracle_config(shape, batch.num_blocks), base, lora)
    return base, lora, batch, pool, orc


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: s.name)
def test_zero_B_reproduces_base_model(shape):
    # Sec. 3.2: E_base == D_base at initialisation -> B = 0 makes every decoder row equal the encoder row.
    base, lora, batch, pool, orc = _setup(shape.replace(lora_target_mask=synth.ALL_TARGETS), [20, 33], [shape.n_models, 1], zero_b=True)
    x_seq = synth.make_hidden(shape, batch.S, seed=1)
    x = x_seq[batch.row_seq]                       # identical rows within a sequence (layer-1 reality)
    y, _ = orc.decode_step(pool, batch.block_tables, batch.ctx_lens, batch.row_seq, batch.row_model, x)
    for r in range(batch.R):
        enc = int(np.flatnonzero((batch.row_seq == batch.row_seq[r]) & (batch.row_model == -1))[0])
        assert np.array_equal(y[r], y[enc])
    # and equals the adapter-free oracle
    pool2 = filled_batch(shape, batch, seed=0)
    y2, _ = oracle.Oracle(orc.cfg, base, None).decode_step(pool2, batch.block_tables, batch.ctx_lens, batch.row_seq, batch.row_model, x)
    assert np.array_equal(y, y2) and np.array_equal(pool, pool2)


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: s.name)
def test_nonzero_B_changes_decoder_rows_only(shape):
    base, lora, batch, pool, orc = _setup(shape.replace(lora_target_mask=synth.ALL_TARGETS), [20], [2])
    x = synth.make_hidden(shape, 1, seed=1)[batch.row_seq]
    y, _ = orc.decode_step(pool, batch.block_tables, batch.ctx_lens, batch.row_seq, batch.row_model, x)
    assert not np.array_equal(y[1], y[0]) and not np.array_equal(y[2], y[1])
    y0, _ = oracle.Oracle(orc.cfg, base, None).decode_step(filled_batch(shape, batch, 0), batch.block_tables, batch.ctx_lens,
                                                         batch.row_seq[:1], batch.row_model[:1], x[:1])
    assert np.array_equal(y[0], y0[0])             # the encoder row never sees an adapter


def test_cache_is_adapter_independent():
    # Sec. 3.2 / 3.3: the cache for a prompt is identical whatever adapters are loaded or active;
    # adapters on K and V are never read (the decoder produces no KV entries, App. C).
    shape = SHAPES[1]
    base, lora, batch, pool, orc = _setup(shape, [20, 47], [3, 1])
    x_seq = synth.make_hidden(shape, 2, seed=1)
    x = x_seq[batch.row_seq]
    y, slots = orc.decode_step(pool, batch.block_tables, batch.ctx_lens, batch.row_seq, batch.row_model, x)
    # (a) other adapter weights, (b) other active sets, (c) no decoders at all
    lora_b = synth.make_lora(shape, seed=99, std=0.3)
    for lr, n_act in ((lora_b, [3, 1]), (lora, [1, 4]), (None, [0, 0])):
        b2 = synth.make_batch(shape, [20, 47], n_act, seed=0)
        assert np.array_equal(b2.block_tables, batch.block_tables)
        p2 = filled_batch(shape, b2, seed=0)
        o2 = oracle.Oracle(orc.cfg, base, lr)
        _, s2 = o2.decode_step(p2, b2.block_tables, b2.ctx_lens, b2.row_seq, b2.row_model, x_seq[b2.row_seq])
        assert np.array_equal(p2, pool) and np.array_equal(s2, slots)
    # perturbing only the K and V adapters changes neither cache nor outputs
    lora_kv = dict(lora)
    lora_kv["k"] = (lora["k"][0] * 7 + 1, lora["k"][1] * 3 - 2)
    lora_kv["v"] = (lora["v"][0] * 5 - 1, lora["v"][1] * 9 + 2)
    p3 = filled_batch(shape, batch, seed=0)
    y3, _ = oracle.Oracle(orc.cfg, base, lora_kv).decode_step(p3, batch.block_tables, batch.ctx_lens, batch.row_seq, batch.row_model, x)
    assert np.array_equal(p3, pool) and np.array_equal(y3, y)


@pytest.mark.parametrize("shape", [SHAPES[0], SHAPES[2]], ids=lambda s: s.name)
def test_decoder_row_equals_merged_weight_model_on_shared_cache(shape):
    # Eq. 5: D_task = base weights + adapter, reading the cache E_base wrote.  A model whose q, o, gate,
    # up, down weights are W + s B A (K/V weights untouched) and no adapter gives the same row when both
    # see the same input (then the entry E_base appends at the current position is the same too).
    # On the QK-norm shape this also fixes where the per-head norm of q sits: after the adapter's delta, as in
    # the merged model, where it cannot sit anywhere else (a norm taken before the delta would differ by far
    # more than the float32 storage of the merged weights).
    shape = shape.replace(lora_target_mask=synth.ALL_TARGETS)
    base, lora, batch, pool, orc = _setup(shape, [29], [2])
    x = synth.make_hidden(shape, 1, seed=6)
    for j in range(shape.n_models):
        p_l = filled_batch(shape, batch, seed=0)
        yl, _ = orc.decode_step(p_l, batch.block_tables, batch.ctx_lens, [0, 0], [-1, j], np.stack([x[0], x[0]]))
        merged = dict(base)
        for p in ("q", "o", "gate", "up", "down"):
            A, B = lora[p]
            merged[p] = np.float32(base[p].astype(np.float64) + shape.lora_scale * B[j].astype(np.float64) @ A[j].astype(np.float64))
        p_m = filled_batch(shape, batch, seed=0)
        ym, _ = oracle.Oracle(orc.cfg, merged, None).decode_step(p_m, batch.block_tables, batch.ctx_lens, [0], [-1], x)
        assert np.array_equal(p_l, p_m)
        assert np.max(np.abs(yl[1] - ym[0])) / np.max(np.abs(ym[0])) < 2e-6   # float32 storage of merged weights
        assert np.max(np.abs(yl[1] - yl[0])) / np.max(np.abs(yl[0])) > 1e-3   # and the adapter does matter


def test_paged_equals_contiguous():
    # paging is an addressing scheme: any block permutation gives the attention of the contiguous cache
    shape = SHAPES[1]
    cfg = oracle_config(shape, 64)
    orc = oracle.Oracle(cfg, synth.make_base(shape), None)
    n = 53
    K, V = synth.make_kv_tokens(shape, n, seed=5)
    q = synth.make_hidden(shape.replace(d_model=shape.n_q_heads * shape.head_dim), 3, seed=5).reshape(3, shape.n_q_heads, shape.head_dim)
    outs = []
    for perm_seed in (0, 1, None):
        bt = np.arange(4, dtype=np.int32)[None] if perm_seed is None else np.random.default_rng(perm_seed).permutation(64)[:4].astype(np.int32)[None]
        pool = orc.new_pool()
        pool[:] = 123.0                      # garbage in unused slots must not matter
        fill_pool(pool, bt[0], K, V)
        outs.append(orc.attn_shared_kv(q, pool, bt, [n], [0, 0, 0]))
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])
    g = shape.n_q_heads // shape.n_kv_heads
    kv_of = [(u % shape.n_q_heads) // g for u in range(3 * shape.n_q_heads)]
    direct = oracle.attention(q.reshape(-1, shape.head_dim).astype(np.float64), K, V, kv_of)
    assert np.array_equal(outs[0].reshape(-1, shape.head_dim), direct)


def test_head_stacking_is_result_neutral():
    # Sec. 3.3: concatenating the streams' queries on the head axis changes nothing but the cache reads
    shape = SHAPES[1]
    cfg = oracle_config(shape, 16)
    orc = oracle.Oracle(cfg, synth.make_base(shape), None)
    n = 40
    K, V = synth.make_kv_tokens(shape, n, seed=6)
    bt = np.random.default_rng(0).permutation(16)[:3].astype(np.int32)[None]
    pool = orc.new_pool()
    fill_pool(pool, bt[0], K, V)
    q = np.random.default_rng(1).standard_normal((4, shape.n_q_heads, shape.head_dim)).astype(np.float32)
    stacked = orc.attn_shared_kv(q, pool, bt, [n], [0, 0, 0, 0])
    for t in range(4):
        alone = orc.attn_shared_kv(q[t:t + 1], pool, bt, [n], [0])
        assert np.array_equal(stacked[t], alone[0])


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: s.name)
def test_stacked_equals_sequential(shape):
    # Sec. 3.3: running encoder and decoder in one stacked pass is a latency optimisation only
    base, lora, batch, pool, orc = _setup(shape, [17, 31, 16], [2, 0, 1])
    x = synth.make_hidden(shape, batch.R, seed=2)
    pa, pb = pool.copy(), pool.copy()
    ya, sa = orc.decode_step(pa, batch.block_tables, batch.ctx_lens, batch.row_seq, batch.row_model, x, sequential=False)
    yb, sb = orc.decode_step(pb, batch.block_tables, batch.ctx_lens, batch.row_seq, batch.row_model, x, sequential=True)
    assert np.array_equal(ya, yb) and np.array_equal(pa, pb) and np.array_equal(sa, sb)


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: s.name)
def test_prefill_and_decode_write_the_same_cache(shape):
    # App. C: entries produced in prefill and in decode are interchangeable
    base = synth.make_base(shape, seed=1, norm_ones=False)
    lora = synth.make_lora(shape, seed=1)
    n = 21
    batch = synth.make_batch(shape, [0], [1], seed=3, headroom=n + 1)
    cfg = oracle_config(shape, batch.num_blocks)
    orc = oracle.Oracle(cfg, base, lora)
    x = synth.make_hidden(shape, n, seed=3)
    # (a) one prefill call
    pa = orc.new_pool()
    ya, sa = orc.prefill(pa, batch.block_tables, [0], [n], x)
    # (b) two chunks, the second starting mid-block
    pb = orc.new_pool()
    yb1, sb1 = orc.prefill(pb, batch.block_tables, [0], [9], x[:9])
    yb2, sb2 = orc.prefill(pb, batch.block_tables, [9], [n - 9], x[9:])
    assert np.array_equal(pa, pb) and np.array_equal(np.concatenate([yb1, yb2]), ya)
    assert np.array_equal(np.concatenate([sb1, sb2]), sa)
    # (c) token by token through the decode step (encoder row + a decoder row that must not matter)
    pc = orc.new_pool()
    for t in range(n):
        yc, sc = orc.decode_step(pc, batch.block_tables, [t], [0, 0], [-1, t % shape.n_models], np.stack([x[t], x[t]]))
        assert np.array_equal(yc[0], ya[t]) and sc[0] == sa[t]
    assert np.array_equal(pa, pc)
    # slots follow the closed form
    bt = batch.block_tables[0]
    assert [int(v) for v in sa] == [int(bt[t // 16]) * 16 + t % 16 for t in range(n)]


def test_prefill_is_causal_and_select_only_skips_rows():
    shape = SHAPES[1]
    base = synth.make_base(shape, seed=1)
    batch = synth.make_batch(shape, [19, 0], [0, 0], seed=3, headroom=12)
    pool = filled_batch(shape, batch, seed=3)
    orc = oracle.Oracle(oracle_config(shape, batch.num_blocks), base, None)
    x = synth.make_hidden(shape, 20, seed=9)
    p1 = pool.copy()
    y1, _ = orc.prefill(p1, batch.block_tables, [19, 0], [11, 9], x)
    # changing a later token of a sequence leaves earlier rows unchanged (causality)
    x2 = x.copy()
    x2[7] += 1.0
    p2 = pool.copy()
    y2, _ = orc.prefill(p2, batch.block_tables, [19, 0], [11, 9], x2)
    assert np.array_equal(y1[:7], y2[:7]) and not np.array_equal(y1[8], y2[8])
    assert np.array_equal(y1[11:], y2[11:])             # the other sequence is untouched
    # select computes the same values for the chosen rows and writes the same cache
    sel = np.zeros(20, dtype=np.uint8)
    sel[[0, 10, 19]] = 1
    p3 = pool.copy()
    y3, _ = orc.prefill(p3, batch.block_tables, [19, 0], [11, 9], x, select=sel)
    assert np.array_equal(p3, p1)
    assert np.array_equal(y3[[0, 10, 19]], y1[[0, 10, 19]]) and np.isnan(y3[1]).all()


def test_untouched_slots_keep_their_bytes():
    shape = SHAPES[0]
    base, lora, batch, pool, orc = _setup(shape, [16, 15], [1, 2])
    pool[:] = np.where(pool == 0, np.float32(-77.0), pool)   # sentinel in every unfilled slot
    before = pool.copy()
    x = synth.make_hidden(shape, batch.R, seed=2)
    _, slots = orc.decode_step(pool, batch.block_tables, batch.ctx_lens, batch.row_seq, batch.row_model, x)
    changed = np.argwhere((pool != before).any(axis=(1, 2, 4)))
    assert sorted(int(b) * 16 + int(o) for b, o in changed) == sorted(int(s) for s in slots)
    assert slots[0] % 16 == 0 and slots[1] % 16 == 15        # first slot of a fresh block / last of a block
