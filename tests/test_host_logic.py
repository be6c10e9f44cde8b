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


def test_every_argument_check_of_the_host_entry_points():
    """One invalid argument at a time (each size, each pointer, the first id on either side of
    the valid range) must be refused with EEP_ERR_INVALID_ARG; the unchanged call succeeds."""
    import ctypes
    lib = binding.load()
    BAD = binding.ERR_INVALID_ARG
    R, S, S_prim, E = 3, 2, 1, 4
    P = R * S
    I = lambda *v: np.array(v, np.int32)
    cur, tgt = I(0, 1, 2, 3, -1, 0), I(1, 0, 2, 3, 3, -1)
    act, wr = I(1, 0, 1), I(1, 1, 1)
    new, kind, src = (np.zeros(P, np.int32) for _ in range(3))
    summ = np.zeros(4, np.int32)
    load = np.ones(E, np.float32)
    p = lambda a: None if a is None else a.ctypes.data

    def repair(R=R, S=S, S_prim=S_prim, E=E, cur=cur, act=act, load=load, new=new, kind=kind,
               src=src, summ=summ):
        return lib.eep_plan_repair(R, S, S_prim, E, p(cur), p(act), p(load), p(new), p(kind), p(src),
                                   p(summ))

    def transition(R=R, S=S, S_prim=S_prim, E=E, cur=cur, tgt=tgt, act=act, wr=wr, new=new,
                   kind=kind, src=src, summ=summ):
        return lib.eep_plan_transition(R, S, S_prim, E, p(cur), p(tgt), p(act), p(wr), p(new),
                                       p(kind), p(src), p(summ))

    off, lst = np.zeros(E + 1, np.int32), np.zeros(P, np.int32)

    def lists(P=P, E=E, S=S, S_prim=S_prim, p2l=cur, off=off, lst=lst):
        return lib.eep_host_replica_lists(P, E, S, S_prim, p(p2l), p(off), p(lst))

    def uncovered(P=P, E=E, S=S, p2l=cur, act=act):
        return lib.eep_host_uncovered_experts(P, E, S, p(p2l), p(act))

    out4 = np.zeros(4, np.int32)

    def tiling(T=12, R=R, out=out4):
        return lib.eep_host_tiling(T, R, p(out))

    assert repair() == binding.OK and repair(load=None) == binding.OK
    assert transition() == binding.OK and lists() == binding.OK and tiling() == binding.OK
    assert uncovered() == 2 and tiling(T=0) == binding.OK       # experts 2 and 3 live on the dead rank only
    hi, lo = cur.copy(), cur.copy()
    hi[2], lo[3] = E, -2
    sizes = [dict(R=0), dict(S=0), dict(S_prim=-1), dict(S_prim=S + 1), dict(E=0)]
    for kw in sizes + [dict(cur=None), dict(act=None), dict(new=None), dict(kind=None),
                       dict(src=None), dict(summ=None), dict(cur=hi), dict(cur=lo),
                       dict(load=np.array([1, -1, 1, 1], np.float32)),
                       dict(load=np.array([1, np.nan, 1, 1], np.float32))]:
        assert repair(**kw) == BAD, kw
    for kw in sizes + [dict(cur=None), dict(tgt=None), dict(act=None), dict(wr=None),
                       dict(new=None), dict(kind=None), dict(src=None), dict(summ=None),
                       dict(cur=hi), dict(cur=lo), dict(tgt=hi), dict(tgt=lo)]:
        assert transition(**kw) == BAD, kw
    for kw in [dict(P=0), dict(E=0), dict(S=0), dict(S_prim=-1), dict(S_prim=S + 1), dict(P=P - 1),
               dict(p2l=None), dict(off=None), dict(lst=None), dict(p2l=hi), dict(p2l=lo)]:
        assert lists(**kw) == BAD, kw
    for kw in [dict(P=0), dict(E=0), dict(S=0), dict(P=P - 1), dict(p2l=None), dict(act=None),
               dict(p2l=hi), dict(p2l=lo)]:
        assert uncovered(**kw) == BAD, kw
    for kw in [dict(T=-3), dict(R=0), dict(T=13), dict(out=None)]:
        assert tiling(**kw) == BAD, kw
    # sizes that are wrong although every entry would pass: no experts with all slots empty,
    # no slots per rank with no primary slots
    empty = np.full(P, -1, np.int32)
    assert lists(E=0, p2l=empty) == BAD and uncovered(E=0, p2l=empty) == BAD
    assert repair(E=0, cur=empty, load=None) == BAD and transition(E=0, cur=empty, tgt=empty) == BAD
    assert lists(S=0, S_prim=0) == BAD and repair(S=0, S_prim=0) == BAD
    # the ids on the valid side of each boundary are accepted
    edge = cur.copy()
    edge[2], edge[3] = E - 1, -1
    assert repair(cur=edge) in (binding.OK, binding.ERR_COVERAGE) and transition(cur=edge, tgt=edge) == binding.OK
    assert lists(p2l=edge) == binding.OK and uncovered(p2l=edge) >= 0
