"""Host-side checks of the C ABI that need no GPU: the library loads, exports every declared
symbol, and rejects malformed configurations and batches before touching a device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2603_13281_amd import binding
from paper_2603_13281_amd.binding import IcarusError, IcarusLayer, LayerConfig

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000  # a 16-byte aligned non-null address; never dereferenced on the host


def _cfg(**kw):
    base = dict(d_model=256, n_q_heads=8, n_kv_heads=2, head_dim=64, d_ffn=512, block_size=16, num_blocks=64,
                n_models=4, lora_rank=8, lora_target_mask=0x7F, bf16=True, max_position=4096)
    base.update(kw)
    return LayerConfig(**base)


def _weights(addr=FAKE):
    base = {p: addr for p in binding.PROJ}
    base.update(norm_attn=addr, norm_ffn=addr, q_norm=addr, k_norm=addr)
    lora = {p: (addr, addr) for p in binding.PROJ}
    return base, lora


def test_library_exports_every_declared_symbol():
    import glob
    hdr = "".join(open(h).read() for h in sorted(glob.glob(os.path.join(ROOT, "include", "*.h"))))
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(icarus_[a-z_0-9]+)\s*\(", hdr))
    assert declared == set(binding.EXPORTS), declared ^ set(binding.EXPORTS)
    lib = C.CDLL(binding.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def test_create_and_workspace_are_host_only():
    base, lora = _weights()
    layer = IcarusLayer(_cfg(), base, lora)
    small = layer.workspace_bytes(9, 1, 4097)
    big = layer.workspace_bytes(576, 64, 16484)
    assert 0 < small < big
    assert layer.workspace_bytes(-1, 1, 1) == 0
    layer.close()


@pytest.mark.parametrize("kw,status", [
    (dict(n_q_heads=6, n_kv_heads=4), "SHAPE"),
    (dict(head_dim=63), "SHAPE"),
    (dict(head_dim=512), "SHAPE"),
    (dict(d_model=0), "SHAPE"),
    (dict(num_blocks=0), "SHAPE"),
    (dict(max_position=0), "SHAPE"),
    (dict(rope_theta=0.5), "INVALID_ARG"),
])
def test_create_rejects_bad_config(kw, status):
    base, lora = _weights()
    with pytest.raises(IcarusError) as e:
        IcarusLayer(_cfg(**kw), base, lora)
    assert e.value.status_name == status


def test_create_rejects_bad_pointers():
    base, lora = _weights()
    b2 = dict(base, q=0)
    with pytest.raises(IcarusError) as e:
        IcarusLayer(_cfg(), b2, lora)
    assert e.value.status_name == "INVALID_ARG"
    b3 = dict(base, down=FAKE + 8)
    with pytest.raises(IcarusError) as e:
        IcarusLayer(_cfg(), b3, lora)
    assert e.value.status_name == "ALIGNMENT"
    l2 = dict(lora, o=None)
    with pytest.raises(IcarusError) as e:
        IcarusLayer(_cfg(), base, l2)
    assert e.value.status_name == "INVALID_ARG"
    # adapters for K and V are never read: they may be absent
    l3 = dict(lora, k=None, v=None)
    IcarusLayer(_cfg(), base, l3).close()
    # and no adapters at all is a plain base model
    IcarusLayer(_cfg(n_models=0, lora_rank=0), base, None).close()


def test_validate_decode_row_rules():
    base, lora = _weights()
    layer = IcarusLayer(_cfg(), base, lora)
    ok = lambda ctx, rs, rm, mb=8: layer.validate_decode(mb, ctx, rs, rm)
    ok([5, 100], [0, 0, 0, 1], [-1, 2, 0, -1])          # m = 2 and m = 0
    ok([0], [0], [-1])

    def bad(status, *a, **k):
        with pytest.raises(IcarusError) as e:
            ok(*a, **k)
        assert e.value.status_name == status, str(e.value)
    bad("ROW_ORDER", [5, 7], [0, 1, 0], [-1, -1, 1])     # rows of sequence 0 not contiguous
    bad("ROW_ORDER", [5], [0, 0], [1, -1])               # encoder row not first
    bad("ROW_ORDER", [5], [0, 0], [-1, -1])              # two encoder rows
    bad("ROW_ORDER", [5, 7], [0, 0], [-1, 1])            # sequence 1 has no rows
    bad("MODEL_ID", [5], [0, 0], [-1, 4])                # id out of range
    bad("MODEL_ID", [5], [0, 0], [-1, -2])
    bad("MODEL_ID", [5], [0, 0, 0], [-1, 3, 3])          # repeated
    bad("CAPACITY", [128], [0], [-1], mb=8)              # position 128 needs 9 blocks
    bad("CAPACITY", [4096], [0], [-1], mb=1000)          # beyond max_position
    bad("INVALID_ARG", [-1], [0], [-1])
    ok([127], [0], [-1], mb=8)
    layer.close()


def test_validate_block_tables_on_a_host_copy():
    """Ids outside the pool, rows too short for the call and two sequences appending into one block are refused
    on the host; shared read-only prefix blocks are fine.  No table, good or bad, is given to a kernel here."""
    base, lora = _weights()
    layer = IcarusLayer(_cfg(num_blocks=32), base, lora)
    bt = np.int32([[3, 4, 5, 0], [3, 4, 9, 0]])                  # blocks 3, 4: a common cached prefix, read only
    layer.validate_block_tables(bt, [40, 35])                     # decode: one new token each, into blocks 5 and 9
    layer.validate_block_tables(bt, [32, 33], extra=[15, 15])     # chunks that stay inside blocks 5 and 9
    layer.validate_block_tables(bt, [47, 0], extra=[1, 0])        # last slot of block 5; sequence 1 touches nothing
    layer.validate_block_tables(bt[:, :3], [47, 40])

    def bad(status, table, ctx, extra=None):
        with pytest.raises(IcarusError) as e:
            layer.validate_block_tables(table, ctx, extra)
        assert e.value.status_name == status, str(e.value)
    bad("CAPACITY", np.int32([[3, 32, 5, 0]]), [40])              # id == num_blocks inside the range read
    bad("CAPACITY", np.int32([[3, -1, 5, 0]]), [40])
    bad("CAPACITY", np.int32([[3, 4, 5, 77]]), [47], [2])         # the chunk spills into entry 3
    layer.validate_block_tables(np.int32([[3, 4, 5, 77]]), [40])  # ... which a call that stops before it never reads
    bad("CAPACITY", bt, [63, 10], [2, 1])                         # 65 tokens need 5 blocks, the row has 4
    bad("INVALID_ARG", np.int32([[3, 4, 5, 0], [6, 7, 5, 0]]), [40, 39])      # both append into block 5
    bad("INVALID_ARG", np.int32([[3, 4, 5, 0], [3, 4, 9, 0]]), [20, 20])      # both append into the "shared" block 4
    bad("INVALID_ARG", bt, [-1, 3])
    with pytest.raises(TypeError):
        layer.validate_block_tables(np.int64([[1, 2]]), [3])      # a numpy-default table would be read as int32 pairs
    with pytest.raises(ValueError):
        layer.validate_block_tables(bt, [3])
    layer.close()


def test_binding_refuses_tensors_the_c_signature_would_misread():
    """The marshalling layer checks element type, shape and placement before a pointer crosses the boundary."""
    import torch
    base, lora = _weights()
    layer = IcarusLayer(_cfg(num_blocks=4), base, lora)
    pool = torch.zeros(layer.cfg.pool_shape(), dtype=torch.bfloat16)
    x = torch.zeros(2, 256, dtype=torch.bfloat16)
    with pytest.raises(TypeError):       # int64 table
        layer.decode_step(pool, torch.zeros(1, 4, dtype=torch.int64), [3], [0, 0], [-1, 0], x)
    with pytest.raises(ValueError):      # ctx_lens shorter than the table
        layer.decode_step(pool, torch.zeros(2, 4, dtype=torch.int32), [3], [0, 0], [-1, 0], x)
    with pytest.raises(ValueError):      # host tensors are not device memory
        layer.decode_step(pool, torch.zeros(1, 4, dtype=torch.int32), [3], [0, 0], [-1, 0], x)
    layer.close()
