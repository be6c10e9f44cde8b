"""Host-side logic of the library (no GPU): replica lists, coverage check and
tiling plan, checked against the oracle, brute force and their defining
properties."""
import itertools

import numpy as np
import pytest

from paper_2605_10670_amd import binding, synth


def test_replica_lists_match_oracle_and_definition(oracle):
    rng = np.random.default_rng(4)
    for trial in range(200):
        R, S = int(rng.integers(1, 9)), int(rng.integers(1, 6))
        S_prim = int(rng.integers(0, S + 1))
        E = int(rng.integers(1, 12))
        p2l = rng.integers(-1, E, size=R * S).astype(np.int32)
        off, lst = binding.host_replica_lists(p2l, E, S, S_prim)
        o_off, o_lst = oracle.tables(p2l, E, S, S_prim)
        assert np.array_equal(off, o_off) and np.array_equal(lst, o_lst)
        for e in range(E):
            want = sorted((p for p in range(R * S) if p2l[p] == e),
                          key=lambda p: ((p % S) >= S_prim, p))
            assert lst[off[e]:off[e + 1]].tolist() == want


def test_replica_lists_reject_bad_entries():
    with pytest.raises(binding.EepError):
        binding.host_replica_lists(np.array([0, 5], np.int32), 4, 2, 1)
    with pytest.raises(binding.EepError):
        binding.host_replica_lists(np.array([0, 1, 2], np.int32), 4, 2, 1)   # P % S != 0


def test_uncovered_experts_all_masks(oracle):
    R, S, E = 4, 2, 5
    rng = np.random.default_rng(2)
    for trial in range(50):
        p2l = rng.integers(-1, E, size=R * S).astype(np.int32)
        for mask in itertools.product([0, 1], repeat=R):
            want = sum(1 for e in range(E)
                       if not any(p2l[p] == e and mask[p // S] for p in range(R * S)))
            assert binding.host_uncovered_experts(p2l, mask, E, S) == want
            assert oracle.uncovered_experts(p2l, np.array(mask, np.int32), E, S) == want


def test_workload_placements_are_covered():
    for wl in (synth.tiny("a"), synth.tiny("c"), synth.decode(T=32, H=8),
               synth.decode_failed_zipf(T=32, H=8), synth.prefill_fp8(T=32, H=128)):
        assert binding.host_uncovered_experts(wl.p2l, wl.active, wl.E, wl.S) == 0
    wl = synth.tiny("b")
    assert binding.host_uncovered_experts(wl.p2l, wl.active, wl.E, wl.S) == 1


@pytest.mark.parametrize("R", [1, 3, 16, 32, 64])
def test_tiling_partitions_every_source_rank(R):
    for per_rank in [0, 1, 2, 63, 64, 127, 128, 129, 131, 255, 256, 257, 512, 643, 1000]:
        T = R * per_rank
        g = binding.host_tiling(T, R)
        if T == 0:
            assert g["num_tiles"] == 0
            continue
        assert g["tokens_per_rank"] == per_rank and g["num_tiles"] == R * g["tiles_per_rank"]
        assert 1 <= g["tile_tokens"] <= 128
        # tiles of one rank cover its tokens exactly once and never cross into the next rank
        covered = []
        for sub in range(g["tiles_per_rank"]):
            lo = sub * g["tile_tokens"]
            hi = min(lo + g["tile_tokens"], per_rank)
            assert lo < hi, "empty tile"
            covered += list(range(lo, hi))
        assert covered == list(range(per_rank))
        # the fewest tiles that respect the 128-token limit
        assert g["tiles_per_rank"] == -(-per_rank // 128)
    with pytest.raises(binding.EepError):
        binding.host_tiling(R + 1 if R > 1 else -1, R)
