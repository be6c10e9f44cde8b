"""Pins of the oracle's failure-detection round (paper Sec. 3.4; Sec. 4.1, the
paragraph on per-rank signal counters; the time-out remark in Fig. 7): an active
peer whose signal does not arrive is dropped by the waiting side, which goes on
without it; the report reaches the host after the step."""
import numpy as np
import pytest

from paper_2605_10670_amd import synth


def _step_out(oracle, idx, w, x, scale, p2l, active, arrived, R, S, S_prim, E, policy=0):
    lay = oracle.step_layout(idx, p2l, active, E, R, S, S_prim, policy)
    recv = oracle.pack(x, lay["row_of"])
    y = oracle.stub_scale(recv, oracle.F32, lay["N"], lay["offset"], p2l, scale)
    det = oracle.detect_round(lay["slot_of"], lay["row_of"], active, arrived, S)
    out = oracle.combine(y, oracle.F32, w, det["row_of"])
    return lay, det, out


@pytest.mark.parametrize("silent", [(), (1,), (0, 3), (0, 1, 2, 3)])
def test_closed_form_without_replicas(oracle, silent):
    """Slot p holds expert p, so expert e lives on rank e // S and nowhere else.  With the
    scalar stand-in y = s[e] * x the combined row is
        out[t] = (sum over j whose rank stayed reachable of w[t,j] * s[e_j]) * x[t],
    whatever the layout did in between."""
    rng = np.random.default_rng(11)
    R, S, k, T, H = 4, 3, 4, 64, 8
    E = R * S
    x = rng.standard_normal((T, H)).astype(np.float32)
    idx, w = synth.router_topk(rng.standard_normal((T, E)).astype(np.float32), k)
    scale = (1.0 + np.arange(E) / 8.0).astype(np.float32)
    arrived = np.ones(R, np.int32)
    arrived[list(silent)] = 0
    lay, det, out = _step_out(oracle, idx, w, x, scale, np.arange(E, dtype=np.int32),
                              np.ones(R, np.int32), arrived, R, S, S, E)
    reachable = ~np.isin(idx // S, silent)
    coeff = (w.astype(np.float64) * scale[idx] * reachable).sum(axis=1)
    np.testing.assert_allclose(out, coeff[:, None] * x.astype(np.float64), rtol=1e-6, atol=1e-7)
    assert det["report"].tolist() == [int(r in silent) for r in range(R)]
    assert det["active"].tolist() == [int(r not in silent) for r in range(R)]
    assert det["withdrawn"] == int((~reachable).sum())


def test_only_active_peers_are_awaited_and_a_full_round_changes_nothing(oracle):
    wl = synth.tiny("c")                       # rank 2 already failed, experts remapped
    lay = oracle.step_layout(wl.topk_idx, wl.p2l, wl.active, wl.E, wl.R, wl.S, wl.S_prim, 0)
    everyone_but_the_dead = wl.active.copy()   # rank 2 sends nothing, and nobody waits for it
    det = oracle.detect_round(lay["slot_of"], lay["row_of"], wl.active, everyone_but_the_dead, wl.S)
    assert det["report"].sum() == 0 and det["withdrawn"] == 0
    assert np.array_equal(det["active"], wl.active)
    assert np.array_equal(det["row_of"], lay["row_of"])
    nobody = np.zeros(wl.R, np.int32)
    det = oracle.detect_round(lay["slot_of"], lay["row_of"], wl.active, nobody, wl.S)
    assert det["report"].tolist() == wl.active.tolist()       # every awaited peer, not rank 2
    assert det["active"].sum() == 0 and (det["row_of"] == -1).all()
    assert det["withdrawn"] == lay["N"]


def test_a_rank_from_which_nothing_is_expected_is_not_awaited(oracle):
    """Sec. 3.4: a side waits for the EXPECTED arrivals from the active peer set.  Here no
    token routes to rank 3 in this step, so its silence goes unnoticed (and is noticed in the
    first round in which it holds rows)."""
    R, S, k, T, H = 4, 2, 2, 8, 4
    E = R * S
    idx = np.tile(np.array([[0, 3]], np.int32), (T, 1))          # experts of ranks 0 and 1 only
    silent = np.array([1, 1, 1, 0], np.int32)
    lay = oracle.step_layout(idx, np.arange(E, dtype=np.int32), np.ones(R, np.int32), E, R, S, S, 0)
    assert lay["rank_count"].tolist() == [T, T, 0, 0]
    det = oracle.detect_round(lay["slot_of"], lay["row_of"], np.ones(R, np.int32), silent, S)
    assert det["report"].sum() == 0 and det["active"].tolist() == [1, 1, 1, 1]
    idx2 = np.tile(np.array([[0, 6]], np.int32), (T, 1))         # now rank 3 holds rows
    lay = oracle.step_layout(idx2, np.arange(E, dtype=np.int32), np.ones(R, np.int32), E, R, S, S, 0)
    det = oracle.detect_round(lay["slot_of"], lay["row_of"], np.ones(R, np.int32), silent, S)
    assert det["report"].tolist() == [0, 0, 0, 1] and det["withdrawn"] == T


@pytest.mark.parametrize("policy", [0, 1])
def test_replicated_placement_invariants(oracle, policy):
    """Decode-like tables with replicas: the rows withdrawn are exactly the dropped ranks'
    receive partitions, the next step routes nothing to them, and the outputs follow the
    closed form with the reachable pairs read off slot_of."""
    rng = np.random.default_rng(5)
    R, S_prim, S_red, k, T, H = 8, 4, 2, 4, 128, 4
    S, E = S_prim + S_red, R * S_prim
    p2l = synth.preferred_placement(R, S_prim, S_red)
    active = synth.active_mask(R, (6,))
    p2l = synth.repaired_placement(p2l, (6,), R, S_prim, S_red)
    x = rng.standard_normal((T, H)).astype(np.float32)
    idx, w = synth.router_topk(rng.standard_normal((T, E)).astype(np.float32), k)
    scale = (0.5 + np.arange(E) / E).astype(np.float32)
    arrived = np.ones(R, np.int32)
    arrived[[2, 6]] = 0                        # 2 goes silent now; 6 was dropped earlier
    lay, det, out = _step_out(oracle, idx, w, x, scale, p2l, active, arrived, R, S, S_prim, E,
                              policy)
    assert det["report"].tolist() == [0, 0, 1, 0, 0, 0, 0, 0]
    assert det["withdrawn"] == lay["rank_count"][2] > 0
    lost = det["row_of"] != lay["row_of"]
    rows_of_rank2 = np.arange(lay["rank_offset"][2], lay["rank_offset"][3])
    assert sorted(lay["row_of"][lost].tolist()) == rows_of_rank2.tolist()
    reachable = lay["slot_of"] // S != 2
    coeff = (w.astype(np.float64) * scale[idx] * reachable).sum(axis=1)
    np.testing.assert_allclose(out, coeff[:, None] * x.astype(np.float64), rtol=1e-6, atol=1e-7)
    nxt = oracle.step_layout(idx, p2l, det["active"], E, R, S, S_prim, policy)
    assert nxt["rank_count"][2] == 0 and nxt["rank_count"][6] == 0
    assert nxt["N"] + nxt["n_uncovered"] == T * k
