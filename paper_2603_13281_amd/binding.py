"""Python binding over libicarus.so: argument marshalling only.

Every step of the layer runs in the library's gfx950 kernels; torch is used for device
memory and streams.  Function names mirror the C ABI (include/icarus.h).  If the library
is missing this module raises at import time: there is no CPU or eager fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libicarus.so")

PROJ = ("q", "k", "v", "o", "gate", "up", "down")
NPROJ = 7
F32, BF16 = 0, 1

STATUS = {0: "OK", 1: "INVALID_ARG", 2: "SHAPE", 3: "ALIGNMENT", 4: "MODEL_ID", 5: "ROW_ORDER",
          6: "CAPACITY", 7: "UNSUPPORTED", 8: "HIP"}

EXPORTS = ("icarus_create", "icarus_destroy", "icarus_last_error", "icarus_workspace_bytes",
           "icarus_validate_decode", "icarus_prefill_kv", "icarus_decode_step", "icarus_attn_shared_kv",
           "icarus_set_kernel_mode", "icarus_timing_enable", "icarus_timing_read", "icarus_bench_copy", "icarus_bench_mfma", "icarus_stack_create", "icarus_stack_destroy",
           "icarus_stack_last_error", "icarus_stack_workspace_bytes", "icarus_stack_prefill", "icarus_stack_decode",
           "icarus_cache_create", "icarus_cache_destroy", "icarus_cache_last_error", "icarus_cache_acquire", "icarus_cache_extend",
           "icarus_cache_commit", "icarus_cache_release", "icarus_cache_get_stats", "icarus_set_full_decoders",
           "icarus_validate_block_tables", "icarus_set_attn_piece_limit", "icarus_attn_shared_kv_static", "icarus_bench_read")

PHASES = ("norm", "lora", "gemm_qkv", "rope_append", "attn", "attn_merge", "gemm_o", "gemm_gateup", "gemm_down",
          "elementwise")


class IcarusError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"icarus status {status} ({STATUS.get(status, '?')}): {message}")
        self.status = status
        self.status_name = STATUS.get(status, "?")


class _Cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "block_size", "num_blocks", "n_models",
        "lora_rank", "lora_target_mask", "dtype", "qk_norm", "max_position", "kv_dtype")] + [
        ("rope_theta", C.c_double), ("rms_eps", C.c_double), ("lora_scale", C.c_double),
        ("k_scale", C.c_double), ("v_scale", C.c_double)]


class _Base(C.Structure):
    _fields_ = [("w", C.c_void_p * NPROJ), ("norm_attn", C.c_void_p), ("norm_ffn", C.c_void_p),
                ("q_norm", C.c_void_p), ("k_norm", C.c_void_p)]


class _Lora(C.Structure):
    _fields_ = [("A", C.c_void_p * NPROJ), ("B", C.c_void_p * NPROJ)]


class _Full(C.Structure):
    _fields_ = [("w", C.c_void_p * NPROJ)]


class _StackCfg(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("vocab", C.c_int32), ("layers", C.POINTER(C.c_void_p)),
                ("embed", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p)]


class _CacheCfg(C.Structure):
    _fields_ = [("num_blocks", C.c_int32), ("block_size", C.c_int32), ("key_by_model", C.c_int32)]


class _CacheStats(C.Structure):
    _fields_ = [("lookups", C.c_int64), ("hit_tokens", C.c_int64), ("miss_tokens", C.c_int64), ("evictions", C.c_int64),
                ("live", C.c_int32), ("cached", C.c_int32), ("free_blocks", C.c_int32), ("peak_live", C.c_int32)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2603_13281_amd.build` "
                          "(there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    lib.icarus_create.restype = C.c_int
    lib.icarus_create.argtypes = [C.POINTER(_Cfg), C.POINTER(_Base), C.POINTER(_Lora), C.POINTER(vp)]
    lib.icarus_destroy.restype = None
    lib.icarus_destroy.argtypes = [vp]
    lib.icarus_last_error.restype = C.c_char_p
    lib.icarus_last_error.argtypes = [vp]
    lib.icarus_workspace_bytes.restype = sz
    lib.icarus_workspace_bytes.argtypes = [vp, i32, i32, i32]
    lib.icarus_validate_decode.restype = C.c_int
    lib.icarus_validate_decode.argtypes = [vp, i32, i32, vp, i32, vp, vp]
    lib.icarus_prefill_kv.restype = C.c_int
    lib.icarus_prefill_kv.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.icarus_decode_step.restype = C.c_int
    lib.icarus_decode_step.argtypes = [vp, vp, vp, i32, i32, vp, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.icarus_attn_shared_kv.restype = C.c_int
    lib.icarus_attn_shared_kv.argtypes = [vp, vp, vp, vp, i32, i32, vp, i32, vp, vp, vp, sz, vp]
    lib.icarus_attn_shared_kv_static.restype = C.c_int
    lib.icarus_attn_shared_kv_static.argtypes = [vp, vp, vp, vp, i32, i32, vp, i32, vp, vp, vp]
    lib.icarus_validate_block_tables.restype = C.c_int
    lib.icarus_validate_block_tables.argtypes = [vp, vp, i32, i32, vp, vp]
    lib.icarus_set_attn_piece_limit.restype = C.c_int
    lib.icarus_set_attn_piece_limit.argtypes = [vp, i32]
    lib.icarus_set_kernel_mode.restype = C.c_int
    lib.icarus_set_kernel_mode.argtypes = [vp, i32]
    lib.icarus_timing_enable.restype = C.c_int
    lib.icarus_timing_enable.argtypes = [vp, i32]
    lib.icarus_timing_read.restype = C.c_int
    lib.icarus_timing_read.argtypes = [vp, vp, vp]
    lib.icarus_bench_copy.restype = C.c_int
    lib.icarus_bench_copy.argtypes = [vp, vp, sz, vp]
    lib.icarus_bench_read.restype = C.c_int
    lib.icarus_bench_read.argtypes = [vp, sz, vp, vp]
    lib.icarus_bench_mfma.restype = C.c_int
    lib.icarus_bench_mfma.argtypes = [vp, C.c_int32, C.c_int32, vp]
    lib.icarus_stack_create.restype = C.c_int
    lib.icarus_stack_create.argtypes = [C.POINTER(_StackCfg), C.POINTER(vp)]
    lib.icarus_stack_destroy.restype = None
    lib.icarus_stack_destroy.argtypes = [vp]
    lib.icarus_stack_last_error.restype = C.c_char_p
    lib.icarus_stack_last_error.argtypes = [vp]
    lib.icarus_stack_workspace_bytes.restype = sz
    lib.icarus_stack_workspace_bytes.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32, C.c_int32]
    lib.icarus_stack_prefill.restype = C.c_int
    lib.icarus_stack_prefill.argtypes = [vp, C.POINTER(vp), vp, C.c_int32, C.c_int32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.icarus_stack_decode.restype = C.c_int
    lib.icarus_stack_decode.argtypes = [vp, C.POINTER(vp), vp, C.c_int32, C.c_int32, vp, C.c_int32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    i32, pi32 = C.c_int32, C.POINTER(C.c_int32)
    lib.icarus_cache_create.restype = C.c_int
    lib.icarus_cache_create.argtypes = [C.POINTER(_CacheCfg), C.POINTER(vp)]
    lib.icarus_cache_destroy.restype = None
    lib.icarus_cache_destroy.argtypes = [vp]
    lib.icarus_cache_last_error.restype = C.c_char_p
    lib.icarus_cache_last_error.argtypes = [vp]
    lib.icarus_cache_acquire.restype = C.c_int
    lib.icarus_cache_acquire.argtypes = [vp, vp, i32, i32, i32, vp, i32, pi32, pi32]
    lib.icarus_cache_extend.restype = C.c_int
    lib.icarus_cache_extend.argtypes = [vp, vp, i32, pi32, i32]
    lib.icarus_cache_commit.restype = C.c_int
    lib.icarus_cache_commit.argtypes = [vp, vp, i32, i32, vp, i32]
    lib.icarus_cache_release.restype = C.c_int
    lib.icarus_cache_release.argtypes = [vp, vp, i32]
    lib.icarus_set_full_decoders.restype = C.c_int
    lib.icarus_set_full_decoders.argtypes = [vp, C.POINTER(_Full)]
    lib.icarus_cache_get_stats.restype = C.c_int
    lib.icarus_cache_get_stats.argtypes = [vp, C.POINTER(_CacheStats)]
    return lib


_lib = _load()


def lib():
    return _lib


@dataclass
class LayerConfig:
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    block_size: int
    num_blocks: int
    n_models: int = 0
    lora_rank: int = 0
    lora_target_mask: int = 0
    bf16: bool = True
    qk_norm: bool = False
    max_position: int = 1 << 17
    rope_theta: float = 5e5
    rms_eps: float = 1e-5
    lora_scale: float = 2.0
    kv_fp8: bool = False      # the KV pool holds FP8 E4M3 codes: value = code * k_scale (K) or v_scale (V)
    k_scale: float = 1.0
    v_scale: float = 1.0

    def _c(self) -> _Cfg:
        return _Cfg(self.d_model, self.n_q_heads, self.n_kv_heads, self.head_dim, self.d_ffn, self.block_size,
                    self.num_blocks, self.n_models, self.lora_rank, self.lora_target_mask,
                    BF16 if self.bf16 else F32, int(self.qk_norm), self.max_position, 1 if self.kv_fp8 else 0,
                    float(self.rope_theta), float(self.rms_eps), float(self.lora_scale), float(self.k_scale), float(self.v_scale))

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.bf16 else torch.float32

    @property
    def pool_dtype(self):
        """Element type of the KV pool tensor (FP8 codes are handed over as raw bytes)."""
        return torch.uint8 if self.kv_fp8 else self.torch_dtype

    def pool_shape(self):
        """[num_blocks, n_kv_heads, 2, block_size*head_dim]: plane 0 = K [Bk, D], plane 1 = V^T [D, Bk]."""
        return (self.num_blocks, self.n_kv_heads, 2, self.block_size * self.head_dim)


def _ptr(t) -> C.c_void_p:
    if t is None:
        return C.c_void_p(0)
    if isinstance(t, torch.Tensor):
        assert t.is_contiguous(), "tensors passed to the library must be contiguous"
        return C.c_void_p(t.data_ptr())
    if isinstance(t, np.ndarray):
        return C.c_void_p(t.ctypes.data)
    if isinstance(t, int):
        return C.c_void_p(t)
    raise TypeError(type(t))


def _host_i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _want(t, what: str, dtype, shape=None, device=None):
    """Marshalling guard: a device tensor handed to the library must have the element type, the shape and the
    device the C signature assumes (a numpy-default int64 block table would be read as pairs of int32)."""
    if not isinstance(t, torch.Tensor):
        raise TypeError(f"{what}: expected a torch tensor, got {type(t).__name__}")
    if t.dtype != dtype:
        raise TypeError(f"{what}: dtype {t.dtype}, the library reads {dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{what}: must be contiguous")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{what}: shape {tuple(t.shape)}, expected {tuple(shape)}")
    if device is not None and t.device != device:
        raise ValueError(f"{what}: on {t.device}, expected {device}")
    if not t.is_cuda:
        raise ValueError(f"{what}: must be a device tensor")


def bench_copy(src: torch.Tensor, dst: torch.Tensor):
    """dst <- src by the library's plain copy kernel (profiler counter calibration)."""
    n = src.numel() * src.element_size()
    rc = _lib.icarus_bench_copy(_ptr(src), _ptr(dst), n, C.c_void_p(torch.cuda.current_stream(src.device).cuda_stream))
    if rc != 0:
        raise IcarusError(rc, "icarus_bench_copy failed")


def bench_read(src: torch.Tensor, reps: int = 5) -> float:
    """Seconds per pass of the library's streaming-read kernel over `src` (whole 8 KB chunks), best of `reps`."""
    n = src.numel() * src.element_size() // 8192 * 8192
    out = torch.zeros(1, dtype=torch.int32, device=src.device)
    stream = C.c_void_p(torch.cuda.current_stream(src.device).cuda_stream)
    best = None
    for _ in range(reps + 1):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        ev[0].record()
        rc = _lib.icarus_bench_read(_ptr(src), n, _ptr(out), stream)
        ev[1].record()
        if rc != 0:
            raise IcarusError(rc, "icarus_bench_read failed")
        torch.cuda.synchronize()
        t = ev[0].elapsed_time(ev[1]) * 1e-3
        best = t if best is None else min(best, t)
    return best


def bench_mfma(waves: int, iters: int, device="cuda:0") -> float:
    """Seconds of the library's register-resident bf16 MFMA loop (flops: 2*32*32*16*8*iters*waves)."""
    out = torch.empty(waves * 64, dtype=torch.float32, device=device)
    stream = C.c_void_p(torch.cuda.current_stream(out.device).cuda_stream)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    if _lib.icarus_bench_mfma(_ptr(out), waves, max(1, iters // 16), stream) != 0:      # warm-up
        raise IcarusError(8, "icarus_bench_mfma failed")
    ev[0].record()
    rc = _lib.icarus_bench_mfma(_ptr(out), waves, iters, stream)
    ev[1].record()
    if rc != 0:
        raise IcarusError(rc, "icarus_bench_mfma failed")
    torch.cuda.synchronize()
    return ev[0].elapsed_time(ev[1]) * 1e-3


class IcarusLayer:
    """One layer context.  base / lora hold torch tensors (device, storage dtype) the caller owns;
    this object keeps references so that they outlive the context.

    base: dict "q","k","v","o","gate","up","down" -> [out,in]; "norm_attn","norm_ffn" -> [d];
          "q_norm","k_norm" -> [D] when qk_norm.
    lora: dict p -> (A [M,r,in_p], B [M,out_p,r]) or None.
    """

    def __init__(self, cfg: LayerConfig, base: dict, lora: dict | None = None):
        self.cfg = cfg
        self._refs = []
        cb = _Base()
        for i, p in enumerate(PROJ):
            cb.w[i] = self._keep(base[p])
        for name in ("norm_attn", "norm_ffn", "q_norm", "k_norm"):
            if base.get(name) is not None:
                setattr(cb, name, self._keep(base[name]))
        cl = _Lora()
        if lora:
            for i, p in enumerate(PROJ):
                if lora.get(p) is not None:
                    cl.A[i] = self._keep(lora[p][0])
                    cl.B[i] = self._keep(lora[p][1])
        cc = cfg._c()
        h = C.c_void_p()
        rc = _lib.icarus_create(C.byref(cc), C.byref(cb), C.byref(cl), C.byref(h))
        if rc != 0:
            raise IcarusError(rc, _lib.icarus_last_error(None).decode())
        self._h = h
        self._ws = None

    def _keep(self, t):
        if isinstance(t, torch.Tensor):
            assert t.is_contiguous()
            self._refs.append(t)
            return t.data_ptr()
        return int(t)  # raw address (host-only validation tests)

    def close(self):
        if getattr(self, "_h", None):
            _lib.icarus_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int):
        if rc != 0:
            raise IcarusError(rc, _lib.icarus_last_error(self._h).decode())

    # -- C ABI mirrors ---------------------------------------------------------------
    def set_full_decoders(self, full: dict | None):
        """full: p -> device tensor [n_models, out_p, in_p] for p in q, o, gate, up, down (private weights of every
        decoder, instead of the adapters); None switches back to the adapters.  The tensors are kept alive here."""
        if full is None:
            self._check(_lib.icarus_set_full_decoders(self._h, None))
            self._full_keep = None
            return
        fw = _Full()
        for i, p in enumerate(PROJ):
            if p in full and full[p] is not None:
                fw.w[i] = full[p].data_ptr()
        self._check(_lib.icarus_set_full_decoders(self._h, C.byref(fw)))
        self._full_keep = dict(full)

    def set_kernel_mode(self, mode: int):
        self._check(_lib.icarus_set_kernel_mode(self._h, mode))

    def timing_enable(self, on: bool):
        self._check(_lib.icarus_timing_enable(self._h, int(on)))

    def timing_read(self) -> dict:
        """{phase: (milliseconds, launches)} accumulated since the last read."""
        ms = np.zeros(len(PHASES), dtype=np.float64)
        n = np.zeros(len(PHASES), dtype=np.int32)
        self._check(_lib.icarus_timing_read(self._h, _ptr(ms), _ptr(n)))
        return {p: (float(ms[i]), int(n[i])) for i, p in enumerate(PHASES)}

    def workspace_bytes(self, max_rows: int, max_seqs: int, max_ctx: int) -> int:
        return int(_lib.icarus_workspace_bytes(self._h, max_rows, max_seqs, max_ctx))

    def set_attn_piece_limit(self, tokens: int):
        """Longest piece of the decode attention's plan, in tokens (0 = automatic); for tests and measurements."""
        self._check(_lib.icarus_set_attn_piece_limit(self._h, int(tokens)))
        self._ws = None

    def validate_block_tables(self, block_tables, ctx_lens, extra=None):
        """Host-side check of a HOST copy of the block tables ([S, max_blocks] int32)."""
        bt = np.ascontiguousarray(block_tables)
        if bt.dtype != np.int32 or bt.ndim != 2:
            raise TypeError(f"block_tables: need a 2-d int32 array, got {bt.dtype} with {bt.ndim} dims")
        ctx_lens = _host_i32(ctx_lens)
        if len(ctx_lens) != bt.shape[0]:
            raise ValueError(f"ctx_lens has {len(ctx_lens)} entries for {bt.shape[0]} table rows")
        ex = None if extra is None else _host_i32(extra)
        if ex is not None and len(ex) != bt.shape[0]:
            raise ValueError(f"extra has {len(ex)} entries for {bt.shape[0]} table rows")
        self._check(_lib.icarus_validate_block_tables(self._h, _ptr(bt), bt.shape[1], bt.shape[0], _ptr(ctx_lens), _ptr(ex)))

    def _check_call(self, kv_pool, block_tables, n_seq_meta, what_meta, x=None, x_cols=None, rows=None, outs=()):
        """Shapes, dtypes and devices of a call's tensors against what the C signature assumes."""
        dev = block_tables.device if isinstance(block_tables, torch.Tensor) else None
        _want(block_tables, "block_tables", torch.int32)
        if block_tables.dim() != 2:
            raise ValueError(f"block_tables: need [S, max_blocks], got {tuple(block_tables.shape)}")
        if block_tables.shape[0] != n_seq_meta:
            raise ValueError(f"{what_meta} has {n_seq_meta} entries for {block_tables.shape[0]} block-table rows")
        _want(kv_pool, "kv_pool", self.cfg.pool_dtype, None, dev)
        want = self.cfg.pool_shape()
        if kv_pool.dim() != 4 or tuple(kv_pool.shape[1:]) != want[1:] or kv_pool.shape[0] < want[0]:
            raise ValueError(f"kv_pool: shape {tuple(kv_pool.shape)}, expected at least {want[0]} blocks of {want[1:]}")
        if x is not None:
            _want(x, "input rows", self.cfg.torch_dtype, (rows, x_cols), dev)
        for name, t, dtype, shape in outs:
            if t is not None:
                _want(t, name, dtype, shape, dev)

    def validate_decode(self, max_blocks, ctx_lens, row_seq, row_model):
        ctx_lens, row_seq, row_model = _host_i32(ctx_lens), _host_i32(row_seq), _host_i32(row_model)
        self._check(_lib.icarus_validate_decode(self._h, max_blocks, len(ctx_lens), _ptr(ctx_lens), len(row_seq),
                                                _ptr(row_seq), _ptr(row_model)))

    def _workspace(self, rows, seqs, max_ctx, device):
        need = self.workspace_bytes(rows, seqs, max_ctx)
        if self._ws is None or self._ws.numel() < need or self._ws.device != device:
            self._ws = torch.empty(need, dtype=torch.uint8, device=device)
        return self._ws

    @staticmethod
    def _stream(device):
        return C.c_void_p(torch.cuda.current_stream(device).cuda_stream)

    def prefill_kv(self, kv_pool, block_tables, ctx_lens, chunk_lens, x_in, x_out=None, slot_out=None,
                   workspace=None, want_out=True):
        ctx_lens, chunk_lens = _host_i32(ctx_lens), _host_i32(chunk_lens)
        if len(ctx_lens) != len(chunk_lens):
            raise ValueError("ctx_lens and chunk_lens differ in length")
        total = int(chunk_lens.sum())
        self._check_call(kv_pool, block_tables, len(ctx_lens), "ctx_lens", x_in, self.cfg.d_model, total,
                         (("x_out", x_out if want_out else None, self.cfg.torch_dtype, (total, self.cfg.d_model)),
                          ("slot_out", slot_out, torch.int64, (total,))))
        S, max_blocks = block_tables.shape
        if want_out and x_out is None:
            x_out = torch.empty_like(x_in)
        if not want_out:
            x_out = None
        max_ctx = int((ctx_lens + chunk_lens).max()) if S else 0
        ws = workspace if workspace is not None else self._workspace(total, S, max_ctx, x_in.device)
        self._check(_lib.icarus_prefill_kv(self._h, _ptr(kv_pool), _ptr(block_tables), max_blocks, S, _ptr(ctx_lens),
                                           _ptr(chunk_lens), _ptr(x_in), _ptr(x_out), _ptr(slot_out), _ptr(ws),
                                           ws.numel(), self._stream(x_in.device)))
        return x_out

    def decode_step(self, kv_pool, block_tables, ctx_lens, row_seq, row_model, x_in, x_out=None, slot_out=None,
                    workspace=None):
        ctx_lens, row_seq, row_model = _host_i32(ctx_lens), _host_i32(row_seq), _host_i32(row_model)
        R = len(row_seq)
        if len(row_model) != R:
            raise ValueError("row_seq and row_model differ in length")
        self._check_call(kv_pool, block_tables, len(ctx_lens), "ctx_lens", x_in, self.cfg.d_model, R,
                         (("x_out", x_out, self.cfg.torch_dtype, (R, self.cfg.d_model)), ("slot_out", slot_out, torch.int64, (len(ctx_lens),))))
        S, max_blocks = block_tables.shape
        if x_out is None:
            x_out = torch.empty_like(x_in)
        max_ctx = int(ctx_lens.max()) + 1 if S else 0
        ws = workspace if workspace is not None else self._workspace(R, S, max_ctx, x_in.device)
        self._check(_lib.icarus_decode_step(self._h, _ptr(kv_pool), _ptr(block_tables), max_blocks, S, _ptr(ctx_lens),
                                            R, _ptr(row_seq), _ptr(row_model), _ptr(x_in), _ptr(x_out), _ptr(slot_out),
                                            _ptr(ws), ws.numel(), self._stream(x_in.device)))
        return x_out

    def _check_attn(self, q, kv_pool, block_tables, kv_lens, row_seq, out):
        R = len(row_seq)
        self._check_call(kv_pool, block_tables, len(kv_lens), "kv_lens")
        _want(q, "q", self.cfg.torch_dtype, None, block_tables.device)
        if q.numel() != R * self.cfg.n_q_heads * self.cfg.head_dim:
            raise ValueError(f"q has {q.numel()} elements for {R} rows of {self.cfg.n_q_heads} x {self.cfg.head_dim}")
        if out is not None:
            _want(out, "out", self.cfg.torch_dtype, tuple(q.shape), block_tables.device)

    def attn_shared_kv_static(self, q, kv_pool, block_tables, kv_lens, row_seq, out):
        """icarus_attn_shared_kv_static: no workspace, nothing allocated (the caller passes `out`)."""
        kv_lens, row_seq = _host_i32(kv_lens), _host_i32(row_seq)
        self._check_attn(q, kv_pool, block_tables, kv_lens, row_seq, out)
        S, max_blocks = block_tables.shape
        self._check(_lib.icarus_attn_shared_kv_static(self._h, _ptr(q), _ptr(kv_pool), _ptr(block_tables), max_blocks, S,
                                                      _ptr(kv_lens), len(row_seq), _ptr(row_seq), _ptr(out), self._stream(q.device)))
        return out

    def attn_shared_kv(self, q, kv_pool, block_tables, kv_lens, row_seq, out=None, workspace=None):
        kv_lens, row_seq = _host_i32(kv_lens), _host_i32(row_seq)
        self._check_attn(q, kv_pool, block_tables, kv_lens, row_seq, out)
        S, max_blocks = block_tables.shape
        R = len(row_seq)
        if out is None:
            out = torch.empty_like(q)
        max_ctx = int(kv_lens.max()) if S else 0
        ws = workspace if workspace is not None else self._workspace(R, S, max_ctx, q.device)
        self._check(_lib.icarus_attn_shared_kv(self._h, _ptr(q), _ptr(kv_pool), _ptr(block_tables), max_blocks, S,
                                               _ptr(kv_lens), R, _ptr(row_seq), _ptr(out), _ptr(ws), ws.numel(),
                                               self._stream(q.device)))
        return out


class IcarusStack:
    """A stack of IcarusLayer contexts with token embedding, final norm and LM head (marshalling only).
    layers: list of IcarusLayer (kept alive); embed, final_norm, lm_head: device tensors, storage dtype."""

    def __init__(self, layers, embed, final_norm, lm_head):
        self.layers = list(layers)
        self._t = [embed.contiguous(), final_norm.contiguous(), lm_head.contiguous()]
        self.vocab = int(lm_head.shape[0])
        arr = (C.c_void_p * len(self.layers))(*[l._h for l in self.layers])
        self._arr = arr
        cfg = _StackCfg(len(self.layers), self.vocab, C.cast(arr, C.POINTER(C.c_void_p)), self._t[0].data_ptr(),
                        self._t[1].data_ptr(), self._t[2].data_ptr())
        h = C.c_void_p()
        rc = _lib.icarus_stack_create(C.byref(cfg), C.byref(h))
        if rc != 0:
            raise IcarusError(rc, _lib.icarus_stack_last_error(None).decode())
        self._h = h
        self._ws = None

    def close(self):
        if getattr(self, "_h", None):
            _lib.icarus_stack_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc):
        if rc != 0:
            raise IcarusError(rc, _lib.icarus_stack_last_error(self._h).decode())

    def workspace_bytes(self, max_rows, max_seqs, max_ctx, max_logit_rows) -> int:
        return int(_lib.icarus_stack_workspace_bytes(self._h, max_rows, max_seqs, max_ctx, max_logit_rows))

    def _workspace(self, rows, seqs, max_ctx, logit_rows, device):
        need = self.workspace_bytes(rows, seqs, max_ctx, logit_rows)
        if self._ws is None or self._ws.numel() < need or self._ws.device != device:
            self._ws = torch.empty(need, dtype=torch.uint8, device=device)
        return self._ws

    @staticmethod
    def _pools(kv_pools):
        return (C.c_void_p * len(kv_pools))(*[p.data_ptr() for p in kv_pools])

    def prefill(self, kv_pools, block_tables, ctx_lens, chunk_lens, tokens, want_logits=False):
        """Returns (next_token [S] int32 device, logits [S, vocab] float32 device or None)."""
        ctx_lens, chunk_lens, tokens = _host_i32(ctx_lens), _host_i32(chunk_lens), _host_i32(tokens)
        S, max_blocks = block_tables.shape
        dev = block_tables.device
        R = int(chunk_lens.sum())
        nxt = torch.empty(S, dtype=torch.int32, device=dev)
        logits = torch.empty((S, self.vocab), dtype=torch.float32, device=dev) if want_logits else None
        ws = self._workspace(R, S, int((ctx_lens + chunk_lens).max()) if S else 0, S, dev)
        stream = C.c_void_p(torch.cuda.current_stream(dev).cuda_stream)
        self._check(_lib.icarus_stack_prefill(self._h, self._pools(kv_pools), _ptr(block_tables), max_blocks, S, _ptr(ctx_lens),
                                              _ptr(chunk_lens), _ptr(tokens), _ptr(nxt), _ptr(logits), _ptr(ws), ws.numel(), stream))
        return nxt, logits

    def decode(self, kv_pools, block_tables, ctx_lens, row_seq, row_model, seq_token, seq_next=None, want_logits=False):
        """seq_token: device int32 [S].  Returns (row_next [R] int32 device, logits [R, vocab] or None);
        seq_next (device int32 [S], may be seq_token itself) receives each sequence's last row's token."""
        ctx_lens, row_seq, row_model = _host_i32(ctx_lens), _host_i32(row_seq), _host_i32(row_model)
        S, max_blocks = block_tables.shape
        dev = block_tables.device
        R = len(row_seq)
        row_next = torch.empty(R, dtype=torch.int32, device=dev)
        logits = torch.empty((R, self.vocab), dtype=torch.float32, device=dev) if want_logits else None
        ws = self._workspace(R, S, int(ctx_lens.max()) + 1 if S else 0, R, dev)
        stream = C.c_void_p(torch.cuda.current_stream(dev).cuda_stream)
        self._check(_lib.icarus_stack_decode(self._h, self._pools(kv_pools), _ptr(block_tables), max_blocks, S, _ptr(ctx_lens), R,
                                             _ptr(row_seq), _ptr(row_model), _ptr(seq_token), _ptr(row_next), _ptr(seq_next),
                                             _ptr(logits), _ptr(ws), ws.numel(), stream))
        return row_next, logits


class PrefixCache:
    """icarus_cache_*: the cross-model prefix-cache manager (host side).  Marshalling only."""

    def __init__(self, num_blocks: int, block_size: int, key_by_model: bool):
        self.num_blocks, self.block_size, self.key_by_model = int(num_blocks), int(block_size), bool(key_by_model)
        self._h = C.c_void_p()
        cfg = _CacheCfg(self.num_blocks, self.block_size, int(self.key_by_model))
        rc = _lib.icarus_cache_create(C.byref(cfg), C.byref(self._h))
        if rc != 0:
            raise IcarusError(rc, (_lib.icarus_cache_last_error(None) or b"").decode())

    def close(self):
        if getattr(self, "_h", None):
            _lib.icarus_cache_destroy(self._h)
            self._h = None

    __del__ = close

    def _check(self, rc):
        if rc != 0:
            raise IcarusError(rc, (_lib.icarus_cache_last_error(self._h) or b"").decode())

    @staticmethod
    def _i32(a):
        return np.ascontiguousarray(a, dtype=np.int32)

    def acquire(self, tokens, model: int, reserve: int = 0):
        """-> (block ids of the sequence, number of leading tokens whose K/V is already cached)"""
        t = self._i32(tokens)
        cap = (len(t) + reserve + self.block_size - 1) // self.block_size
        out = np.empty(max(cap, 1), dtype=np.int32)
        nb, nc = C.c_int32(0), C.c_int32(0)
        self._check(_lib.icarus_cache_acquire(self._h, t.ctypes.data, len(t), int(model), int(reserve), out.ctypes.data, cap,
                                              C.byref(nb), C.byref(nc)))
        return out[: nb.value].tolist(), nc.value

    def extend(self, blocks, n_tokens_total: int):
        cap = max(len(blocks), (int(n_tokens_total) + self.block_size - 1) // self.block_size, 1)
        buf = np.empty(cap, dtype=np.int32)
        buf[: len(blocks)] = blocks
        nb = C.c_int32(len(blocks))
        self._check(_lib.icarus_cache_extend(self._h, buf.ctypes.data, cap, C.byref(nb), int(n_tokens_total)))
        return buf[: nb.value].tolist()

    def commit(self, tokens, model: int, blocks):
        t, b = self._i32(tokens), self._i32(blocks)
        self._check(_lib.icarus_cache_commit(self._h, t.ctypes.data, len(t), int(model), b.ctypes.data, len(b)))

    def release(self, blocks):
        b = self._i32(blocks)
        self._check(_lib.icarus_cache_release(self._h, b.ctypes.data, len(b)))

    def counts(self) -> dict:
        st = _CacheStats()
        self._check(_lib.icarus_cache_get_stats(self._h, C.byref(st)))
        return dict(lookups=st.lookups, hit_tokens=st.hit_tokens, miss_tokens=st.miss_tokens, evictions=st.evictions,
                    peak_live=st.peak_live, live=st.live, cached=st.cached, free=st.free_blocks)
