"""GPU-side test glue: upload seeded inputs, move pools between the oracle's layout and the library's."""
import numpy as np
import torch

from paper_2603_13281_amd import binding, synth


def dev(a: np.ndarray, bf16: bool, device="cuda:0") -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.to(device=device, dtype=torch.bfloat16 if bf16 else torch.float32).contiguous()


def host(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu", torch.float32).numpy()


def pool_to_device_layout(pool: np.ndarray) -> np.ndarray:
    """oracle [nb, 2, Hkv, Bk, D] -> library [nb, Hkv, 2, Bk*D] (K token-major, V transposed)."""
    nb, _, Hkv, Bk, D = pool.shape
    K = pool[:, 0].reshape(nb, Hkv, Bk * D)
    Vt = pool[:, 1].transpose(0, 1, 3, 2).reshape(nb, Hkv, D * Bk)
    return np.ascontiguousarray(np.stack([K, Vt], axis=2))


def pool_from_device_layout(dpool: np.ndarray, Bk: int, D: int) -> np.ndarray:
    nb, Hkv = dpool.shape[:2]
    K = dpool[:, :, 0].reshape(nb, Hkv, Bk, D)
    V = dpool[:, :, 1].reshape(nb, Hkv, D, Bk).transpose(0, 1, 3, 2)
    return np.ascontiguousarray(np.stack([K, V], axis=1))


def layer_config(shape: synth.LayerShape, num_blocks: int, max_position: int = 1 << 17) -> binding.LayerConfig:
    return binding.LayerConfig(
        d_model=shape.d_model, n_q_heads=shape.n_q_heads, n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim,
        d_ffn=shape.d_ffn, block_size=shape.block_size, num_blocks=num_blocks, n_models=shape.n_models,
        lora_rank=shape.lora_rank, lora_target_mask=shape.lora_target_mask, bf16=shape.bf16, qk_norm=shape.qk_norm,
        max_position=max_position, rope_theta=shape.rope_theta, rms_eps=shape.rms_eps, lora_scale=shape.lora_scale)


def make_layer(shape, base, lora, num_blocks, device="cuda:0", max_position=1 << 17, **cfg_overrides) -> binding.IcarusLayer:
    dbase = {k: dev(v, shape.bf16, device) for k, v in base.items()}
    dlora = None
    if lora is not None:
        dlora = {p: (dev(A, shape.bf16, device), dev(B, shape.bf16, device)) for p, (A, B) in lora.items()}
    cfg = layer_config(shape, num_blocks, max_position)
    if lora is None:
        cfg.n_models, cfg.lora_rank, cfg.lora_target_mask = 0, 0, 0
    for k, v in cfg_overrides.items():
        setattr(cfg, k, v)
    return binding.IcarusLayer(cfg, dbase, dlora)


def fp8_pool_to_float(dpool: torch.Tensor, k_scale: float, v_scale: float) -> np.ndarray:
    """Device pool of FP8 E4M3 codes [nb, Hkv, 2, Bk*D] (uint8) -> float32 values, library layout."""
    vals = dpool.cpu().view(torch.float8_e4m3fn).to(torch.float32).numpy()
    vals[:, :, 0] *= np.float32(k_scale)
    vals[:, :, 1] *= np.float32(v_scale)
    return vals


def e4m3_step(x: np.ndarray, scale: float) -> np.ndarray:
    """Spacing of the FP8 E4M3 grid (times scale) at |x|."""
    a = np.maximum(np.abs(x.astype(np.float64)) / scale, 2.0 ** -6)
    return 2.0 ** (np.floor(np.log2(a)) - 3) * scale


def bf16_ulp(x: np.ndarray) -> np.ndarray:
    """Spacing of bfloat16 at |x| (8 significant bits)."""
    ax = np.maximum(np.abs(x.astype(np.float64)), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(ax)) - 7)
