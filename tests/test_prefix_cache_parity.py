"""The library's prefix-cache manager (host code, through the C ABI) against the oracle: block ids, hit
lengths and counters must be identical, operation by operation.  No GPU is needed: this is host logic."""
import numpy as np
import pytest

from oracle.prefix_cache import CacheFull, OraclePrefixCache
from paper_2603_13281_amd import binding, cache_sim, synth


def both(num_blocks, block_size, per_model):
    return binding.PrefixCache(num_blocks, block_size, per_model), OraclePrefixCache(num_blocks, block_size, per_model)


@pytest.mark.parametrize("pattern", ["round_robin", "skewed"])
@pytest.mark.parametrize("per_model", [False, True])
@pytest.mark.parametrize("num_blocks", [260, 100000])
def test_agent_schedule_matches_oracle(pattern, per_model, num_blocks):
    sched = synth.make_agent_schedule(12, 4, 5, seed=2, pattern=pattern, prompt_len=(300, 700), concurrency=3)
    lib, orc = both(num_blocks, 16, per_model)
    rl, ro = [], []
    out_l = cache_sim.run_schedule(lib, sched, record=rl)
    out_o = cache_sim.run_schedule(orc, sched, record=ro)
    assert rl == ro
    assert out_l == out_o
    if num_blocks == 260:
        assert out_l["evictions"] > 0


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
@pytest.mark.parametrize("per_model", [False, True])
def test_random_operations_with_live_sequences_match_oracle(seed, per_model):
    """Several sequences live at once (duplicates of one prefix, evictions under them, repeated commits,
    failed acquires): every observable result equal, including after a full pool refused a request."""
    rng = np.random.default_rng(seed)
    B, N = 4, 48
    lib, orc = both(N, B, per_model)
    stems = [rng.integers(0, 6, size=rng.integers(5, 40)).astype(np.int32) for _ in range(5)]   # few symbols: shared prefixes
    live = []      # (tokens, model, blocks_lib, blocks_orc)
    n_fail = 0
    for step in range(1500):
        op = rng.random()
        if op < 0.40 or not live:
            stem = stems[rng.integers(len(stems))]
            cut = int(rng.integers(1, len(stem) + 1))
            extra = rng.integers(0, 6, size=rng.integers(0, 9)).astype(np.int32)
            toks = np.concatenate([stem[:cut], extra])
            model, reserve = int(rng.integers(0, 3)), int(rng.integers(0, 6))
            try:
                bo, ho = orc.acquire(toks, model, reserve)
            except CacheFull:
                with pytest.raises(binding.IcarusError) as e:
                    lib.acquire(toks, model, reserve)
                assert e.value.status_name == "CAPACITY"
                n_fail += 1
                assert lib.counts() == orc.counts()
                continue
            bl, hl = lib.acquire(toks, model, reserve)
            assert (bl, hl) == (bo, ho)
            live.append([toks, model, bl, bo])
        elif op < 0.55:
            s = live[rng.integers(len(live))]
            grow = rng.integers(0, 6, size=rng.integers(1, 10)).astype(np.int32)
            toks = np.concatenate([s[0], grow])
            try:
                bo = orc.extend(s[3], len(toks))
            except CacheFull:
                with pytest.raises(binding.IcarusError):
                    lib.extend(s[2], len(toks))
                n_fail += 1
                continue
            bl = lib.extend(s[2], len(toks))
            assert bl == bo
            s[0], s[2], s[3] = toks, bl, bo
        elif op < 0.75:
            s = live[rng.integers(len(live))]
            n = int(rng.integers(0, len(s[0]) + 1))      # commit a prefix of what the sequence holds
            lib.commit(s[0][:n], s[1], s[2])
            orc.commit(s[0][:n], s[1], s[3])
        else:
            s = live.pop(rng.integers(len(live)))
            lib.release(s[2])
            orc.release(s[3])
        if step % 50 == 0:
            assert lib.counts() == orc.counts()
    for s in live:
        lib.release(s[2]); orc.release(s[3])
    assert lib.counts() == orc.counts()
    assert lib.counts()["live"] == 0
    assert n_fail > 0 and lib.counts()["evictions"] > 0


def test_argument_errors():
    lib = binding.PrefixCache(8, 4, True)
    with pytest.raises(binding.IcarusError) as e:
        lib.acquire(np.arange(5, dtype=np.int32), -1)
    assert e.value.status_name == "MODEL_ID"
    with pytest.raises(binding.IcarusError) as e:
        lib.acquire(np.arange(40, dtype=np.int32), 0)              # 10 blocks from a pool of 8
    assert e.value.status_name == "CAPACITY"
    blocks, hit = lib.acquire(np.arange(6, dtype=np.int32), 0)
    with pytest.raises(binding.IcarusError) as e:
        lib.release(blocks + blocks)                                  # released more often than referenced
    assert e.value.status_name == "INVALID_ARG"
    assert lib.counts()["live"] == 2                                  # the failed call changed nothing
    with pytest.raises(binding.IcarusError):
        lib.commit(np.arange(6, dtype=np.int32), 0, [7])              # a block that is not live
    lib.release(blocks)
    with pytest.raises(binding.IcarusError):
        binding.PrefixCache(0, 4, False)
