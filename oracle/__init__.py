"""CPU oracle for the ICaRus shared-KV layer step.  TEST INFRASTRUCTURE ONLY.

Thin ctypes binding over ``icarus_oracle.c`` (plain C, float64 arithmetic).
Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s CPU-baseline
leg may import this package; the product package never does.

Argument marshalling only -- every number is computed in the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "icarus_oracle.c")
_LIB = os.path.join(_HERE, "libicarus_oracle.so")

PROJ = ("q", "k", "v", "o", "gate", "up", "down")
NPROJ = 7


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP over output features / heads)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


class _Cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "block_size", "num_blocks",
        "n_models", "lora_rank", "lora_target_mask", "qk_norm", "bf16")] + [
        ("rope_theta", C.c_double), ("rms_eps", C.c_double), ("lora_scale", C.c_double),
        ("kv_fp8", C.c_int32), ("k_scale", C.c_double), ("v_scale", C.c_double)]


class _Base(C.Structure):
    _fields_ = [("w", C.c_void_p * NPROJ), ("norm_attn", C.c_void_p), ("norm_ffn", C.c_void_p),
                ("q_norm", C.c_void_p), ("k_norm", C.c_void_p)]


class _Lora(C.Structure):
    _fields_ = [("A", C.c_void_p * NPROJ), ("B", C.c_void_p * NPROJ), ("F", C.c_void_p * NPROJ)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_round_bf16.restype = C.c_double
        _lib.orc_round_bf16.argtypes = [C.c_double]
        _lib.orc_round_e4m3.restype = C.c_double
        _lib.orc_round_e4m3.argtypes = [C.c_double]
        _lib.orc_slot.restype = C.c_int64
        _lib.orc_slot.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
        _lib.orc_decode_step.restype = C.c_int
        _lib.orc_prefill.restype = C.c_int
    return _lib


def set_threads(n: int) -> None:
    """Number of OpenMP threads the oracle's loops may use from now on (timing only: no result depends on it,
    the loops split independent output features / heads and no sum is reordered)."""
    lib()   # the OpenMP runtime is loaded with the oracle
    C.CDLL("libgomp.so.1").omp_set_num_threads(int(n))


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a):
    return None if a is None else C.c_void_p(a.ctypes.data)


@dataclass
class LayerConfig:
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    block_size: int = 16
    num_blocks: int = 0
    n_models: int = 0
    lora_rank: int = 0
    lora_target_mask: int = 0
    qk_norm: bool = False
    bf16: bool = True
    rope_theta: float = 1e4
    rms_eps: float = 1e-5
    lora_scale: float = 2.0
    kv_fp8: bool = False        # the cache holds FP8 E4M3 codes: value = code * k_scale (K) or v_scale (V)
    k_scale: float = 1.0
    v_scale: float = 1.0

    def proj_in(self, p: str) -> int:
        return {"q": self.d_model, "k": self.d_model, "v": self.d_model, "gate": self.d_model,
                "up": self.d_model, "o": self.n_q_heads * self.head_dim, "down": self.d_ffn}[p]

    def proj_out(self, p: str) -> int:
        return {"q": self.n_q_heads * self.head_dim, "k": self.n_kv_heads * self.head_dim,
                "v": self.n_kv_heads * self.head_dim, "gate": self.d_ffn, "up": self.d_ffn,
                "o": self.d_model, "down": self.d_model}[p]

    def _c(self) -> _Cfg:
        return _Cfg(self.d_model, self.n_q_heads, self.n_kv_heads, self.head_dim, self.d_ffn,
                    self.block_size, self.num_blocks, self.n_models, self.lora_rank,
                    self.lora_target_mask, int(self.qk_norm), int(self.bf16),
                    float(self.rope_theta), float(self.rms_eps), float(self.lora_scale),
                    int(self.kv_fp8), float(self.k_scale), float(self.v_scale))


class Oracle:
    """Holds float32 views of the weights and calls the C oracle.

    base: dict with "q","k","v","o","gate","up","down" [out,in] and "norm_attn","norm_ffn"
          ([d_model]) and, for qk_norm, "q_norm","k_norm" ([head_dim]).
    lora: dict p -> (A [M,r,in_p], B [M,out_p,r]) for the adapted projections, or None.
    """

    def __init__(self, cfg: LayerConfig, base: dict, lora: dict | None = None, full: dict | None = None):
        """full: dict p -> F [M, out_p, in_p] for p in q, o, gate, up, down: private full weights of every
        decoder (instead of adapters).  K and V always come from the encoder row with the base weights."""
        self.cfg = cfg
        self._keep = []
        self._base = _Base()
        for i, p in enumerate(PROJ):
            w = _f32(base[p])
            assert w.shape == (cfg.proj_out(p), cfg.proj_in(p)), (p, w.shape)
            self._keep.append(w)
            self._base.w[i] = w.ctypes.data
        for name in ("norm_attn", "norm_ffn", "q_norm", "k_norm"):
            if base.get(name) is not None:
                w = _f32(base[name])
                self._keep.append(w)
                setattr(self._base, name, w.ctypes.data)
        self._lora = None
        if lora:
            self._lora = _Lora()
            for i, p in enumerate(PROJ):
                if p in lora and lora[p] is not None:
                    A, B = _f32(lora[p][0]), _f32(lora[p][1])
                    assert A.shape == (cfg.n_models, cfg.lora_rank, cfg.proj_in(p)), (p, A.shape)
                    assert B.shape == (cfg.n_models, cfg.proj_out(p), cfg.lora_rank), (p, B.shape)
                    self._keep += [A, B]
                    self._lora.A[i] = A.ctypes.data
                    self._lora.B[i] = B.ctypes.data
        if full:
            assert not lora, "a decoder has adapters or private weights, not both"
            self._lora = _Lora()
            for i, p in enumerate(PROJ):
                if p in ("k", "v"):
                    continue
                Fw = _f32(full[p])
                assert Fw.shape == (cfg.n_models, cfg.proj_out(p), cfg.proj_in(p)), (p, Fw.shape)
                self._keep.append(Fw)
                self._lora.F[i] = Fw.ctypes.data

    # -- pool helpers -----------------------------------------------------
    def new_pool(self) -> np.ndarray:
        c = self.cfg
        return np.zeros((c.num_blocks, 2, c.n_kv_heads, c.block_size, c.head_dim), dtype=np.float32)

    # -- entry points -----------------------------------------------------
    def decode_step(self, pool, block_tables, ctx_lens, row_seq, row_model, x_in, sequential=False):
        c = self.cfg
        bt = _i32(block_tables)
        S, max_blocks = bt.shape
        ctx, rs, rm = _i32(ctx_lens), _i32(row_seq), _i32(row_model)
        x = _f32(x_in)
        R = x.shape[0]
        assert pool.dtype == np.float32 and pool.flags.c_contiguous
        out = np.zeros((R, c.d_model), dtype=np.float64)
        slots = np.zeros(S, dtype=np.int64)
        cc = c._c()
        rc = lib().orc_decode_step(C.byref(cc), C.byref(self._base),
                                   C.byref(self._lora) if self._lora else None, _p(pool), _p(bt),
                                   C.c_int(max_blocks), C.c_int(S), _p(ctx), C.c_int(R), _p(rs), _p(rm),
                                   _p(x), _p(out), _p(slots), C.c_int(int(sequential)))
        if rc != 0:
            raise ValueError("oracle: malformed row list")
        return out, slots

    def prefill(self, pool, block_tables, ctx_lens, chunk_lens, x_in, select=None, want_out=True):
        c = self.cfg
        bt = _i32(block_tables)
        S, max_blocks = bt.shape
        ctx, ch = _i32(ctx_lens), _i32(chunk_lens)
        x = _f32(x_in)
        n = x.shape[0]
        assert n == int(ch.sum())
        out = np.full((n, c.d_model), np.nan, dtype=np.float64) if want_out else None
        slots = np.zeros(n, dtype=np.int64)
        sel = None if select is None else np.ascontiguousarray(select, dtype=np.uint8)
        cc = c._c()
        lib().orc_prefill(C.byref(cc), C.byref(self._base), _p(pool), _p(bt), C.c_int(max_blocks),
                          C.c_int(S), _p(ctx), _p(ch), _p(x), _p(out), _p(sel), _p(slots))
        return out, slots

    def attn_shared_kv(self, q, pool, block_tables, kv_lens, row_seq):
        c = self.cfg
        bt = _i32(block_tables)
        S, max_blocks = bt.shape
        kl, rs = _i32(kv_lens), _i32(row_seq)
        qf = _f32(q)
        R = qf.shape[0]
        out = np.zeros((R, c.n_q_heads, c.head_dim), dtype=np.float64)
        cc = c._c()
        lib().orc_attn_shared_kv(C.byref(cc), _p(qf), _p(pool), _p(bt), C.c_int(max_blocks), C.c_int(S),
                                 _p(kl), C.c_int(R), _p(rs), _p(out))
        return out


class OracleStack:
    """L layers + token embedding + final norm + LM head (Alg. 3 outer loop; Alg. 1 for the prompt).

    layers: list of Oracle (same shape).  embed, lm_head [vocab, d_model]; final_norm [d_model].
    Every layer has its own pool; all share the block tables.  Only orchestration lives here: the
    embedding lookup is an index operation, every number comes from the C file.
    """

    def __init__(self, layers, embed, final_norm, lm_head):
        self.layers = list(layers)
        self.cfg = self.layers[0].cfg
        self.embed, self.final_norm, self.lm_head = _f32(embed), _f32(final_norm), _f32(lm_head)
        self.vocab = self.lm_head.shape[0]

    def new_pools(self):
        return [l.new_pool() for l in self.layers]

    def _head(self, x):
        x = np.ascontiguousarray(x, dtype=np.float64)
        R, d = x.shape
        logits = np.empty((R, self.vocab), dtype=np.float64)
        tokens = np.empty(R, dtype=np.int32)
        lib().orc_lm_head(_p(x), C.c_int(R), C.c_int(d), _p(self.final_norm), C.c_double(self.cfg.rms_eps),
                          _p(self.lm_head), C.c_int(self.vocab), _p(logits), _p(tokens))
        return logits, tokens

    def decode(self, pools, block_tables, ctx_lens, row_seq, row_model, seq_tokens):
        """One token step.  Every row of sequence s embeds seq_tokens[s] (the streams differ from layer 1
        on).  Returns (logits [R, vocab], tokens [R], slots [S])."""
        x = self.embed[np.asarray(seq_tokens)[np.asarray(row_seq)]]
        slots = None
        for layer, pool in zip(self.layers, pools):
            x, slots = layer.decode_step(pool, block_tables, ctx_lens, row_seq, row_model, x)   # rounded to storage
        logits, tokens = self._head(x)
        return logits, tokens, slots

    def prefill(self, pools, block_tables, ctx_lens, chunk_lens, tokens):
        """The prompt chunk through the frozen encoder of every layer.  Returns (logits [S, vocab],
        first tokens [S]) taken at the last chunk token of each sequence: the first generated token
        comes from the base model (Alg. 1)."""
        x = self.embed[np.asarray(tokens)]
        for layer, pool in zip(self.layers, pools):
            x, _ = layer.prefill(pool, block_tables, ctx_lens, chunk_lens, x)
        last = np.cumsum(np.asarray(chunk_lens)) - 1
        return self._head(x[last])


# -- primitives exposed for the pin tests ------------------------------------

def round_e4m3(x) -> np.ndarray:
    f = np.vectorize(lambda v: lib().orc_round_e4m3(float(v)), otypes=[np.float64])
    return f(np.asarray(x, dtype=np.float64))


def round_bf16(x) -> np.ndarray:
    f = np.vectorize(lambda v: lib().orc_round_bf16(float(v)), otypes=[np.float64])
    return f(np.asarray(x, dtype=np.float64))


def slot(bt_row, pos: int, block_size: int) -> int:
    bt = _i32(bt_row)
    return int(lib().orc_slot(_p(bt), pos, block_size))


def rmsnorm(x, w, eps):
    x = np.ascontiguousarray(x, dtype=np.float64)
    w = _f32(w)
    y = np.empty_like(x)
    lib().orc_rmsnorm(_p(x), _p(w), C.c_double(eps), C.c_int(x.size), _p(y))
    return y


def linear(W, x):
    W = _f32(W)
    x = np.ascontiguousarray(x, dtype=np.float64)
    y = np.empty(W.shape[0], dtype=np.float64)
    lib().orc_linear(_p(W), C.c_int(W.shape[0]), C.c_int(W.shape[1]), _p(x), _p(y))
    return y


def adaptive_linear(A, B, s, x):
    A, B = _f32(A), _f32(B)
    x = np.ascontiguousarray(x, dtype=np.float64)
    y = np.empty(B.shape[0], dtype=np.float64)
    lib().orc_adaptive_linear(_p(A), _p(B), C.c_int(B.shape[0]), C.c_int(A.shape[1]), C.c_int(A.shape[0]),
                              C.c_double(s), _p(x), _p(y))
    return y


def rope(v, pos: int, theta: float):
    v = np.array(v, dtype=np.float64, order="C")
    H, D = v.shape
    lib().orc_rope(_p(v), C.c_int(H), C.c_int(D), C.c_int(pos), C.c_double(theta))
    return v


def attention(q, K, V, kv_of):
    """q [U,D] float64; K,V [n,Hkv,D] float32; kv_of [U] -> o [U,D]."""
    q = np.ascontiguousarray(q, dtype=np.float64)
    K, V = _f32(K), _f32(V)
    kv = _i32(kv_of)
    U, D = q.shape
    n, Hkv, _ = K.shape
    o = np.empty((U, D), dtype=np.float64)
    lib().orc_attention(C.c_int(U), C.c_int(D), C.c_int(Hkv), _p(kv), _p(q), _p(K), _p(V), C.c_int(n), _p(o))
    return o
