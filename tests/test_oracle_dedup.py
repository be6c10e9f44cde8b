"""Pins for the oracle's de-duplicated dispatch (one row per (token, destination
rank), expanded on the destination): its two stages together must give exactly
what the plain pack gives, and its counts are library set operations."""
import numpy as np
import pytest

import oracle
from paper_2605_10670_amd import synth


def _case(seed, T=96, R=8, sp=2, sr=1, k=6, failed=()):
    rng = np.random.default_rng(seed)
    E = R * sp
    idx, w = synth.router_topk(rng.standard_normal((T, E)).astype(np.float32), k)
    idx = idx.copy()
    idx[rng.random(idx.shape) < 0.05] = -1                       # some masked pairs
    pref = synth.preferred_placement(R, sp, sr)
    p2l = synth.repaired_placement(pref, failed, R, sp, sr) if failed else pref
    lay = oracle.step_layout(idx, p2l, synth.active_mask(R, failed), E, R, sp + sr, sp, oracle.SPREAD)
    x = rng.integers(0, 2 ** 16, size=(T, 24), dtype=np.uint16)
    return lay, x, R, sp + sr, k


@pytest.mark.parametrize("seed", range(6))
def test_two_stages_equal_the_plain_pack(seed):
    lay, x, R, S, k = _case(seed, failed=(3,) if seed % 2 else ())
    d = oracle.dedup_layout(lay["slot_of"], lay["row_of"], R, S)
    recv_d = oracle.pack_dedup(x, d["dedup_row"], d["lead"], fill=0xAAAA)
    recv = oracle.expand(recv_d, d["expand_of"], lay["N"], fill=0xBBBB)
    plain = oracle.pack(x, lay["row_of"], fill=0xBBBB)
    assert np.array_equal(recv, plain)
    assert (recv_d[d["N_d"]:] == 0xAAAA).all()                   # nothing written past N_d


@pytest.mark.parametrize("seed", range(6))
def test_counts_rows_and_leads_are_what_sets_say(seed):
    lay, x, R, S, k = _case(100 + seed, T=64, k=8, R=4)          # 4 ranks, 8 experts: much sharing
    slot = lay["slot_of"]
    d = oracle.dedup_layout(slot, lay["row_of"], R, S)
    T = slot.shape[0]
    ranks = [set((slot[t][slot[t] >= 0] // S).tolist()) for t in range(T)]
    count = np.array([sum(r in s for s in ranks) for r in range(R)])
    assert np.array_equal(d["dedup_count"], count)
    assert np.array_equal(d["dedup_offset"], np.concatenate([[0], np.cumsum(count)]))
    assert d["N_d"] == sum(len(s) for s in ranks) <= lay["N"]
    assert d["N_d"] < lay["N"]                                   # sharing does occur here
    for r in range(R):                                           # token-ascending inside a rank
        toks = [t for t in range(T) if r in ranks[t]]
        for n, t in enumerate(toks):
            js = [j for j in range(k) if slot[t, j] >= 0 and slot[t, j] // S == r]
            assert all(d["dedup_row"][t, j] == d["dedup_offset"][r] + n for j in js)
            assert d["lead"][t, js].tolist() == [1] + [0] * (len(js) - 1)
    routed = slot >= 0
    assert (d["dedup_row"][~routed] == -1).all() and (d["lead"][~routed] == 0).all()
    assert d["lead"].sum() == d["N_d"]
    # every de-duplicated row is used by at least one expert-major row, and no other
    used = d["expand_of"][:lay["N"]]
    assert set(used.tolist()) == set(range(d["N_d"]))
    assert (d["expand_of"][lay["N"]:] == -1).all()


def test_no_sharing_means_no_saving_and_full_sharing_one_row_per_token():
    R, S, k, T = 4, 2, 2, 8
    slot = np.array([[0, 2]] * T, np.int32)                      # two experts on two ranks
    lay = oracle.layout(slot, R, S)
    d = oracle.dedup_layout(slot, lay["row_of"], R, S)
    assert d["N_d"] == T * k and d["lead"].all()
    slot = np.array([[4, 5]] * T, np.int32)                      # both experts on rank 2
    lay = oracle.layout(slot, R, S)
    d = oracle.dedup_layout(slot, lay["row_of"], R, S)
    assert d["N_d"] == T and d["dedup_count"].tolist() == [0, 0, T, 0]
    assert d["dedup_row"][:, 0].tolist() == d["dedup_row"][:, 1].tolist() == list(range(T))
