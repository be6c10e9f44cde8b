"""Pins for the oracle's weight movement (paper Sec. 3.5, Sec. 5.1; Fig. 5 middle
panel): what a repaired instance must hold, and where each copy came from.

Weights are tagged so the source of every byte is visible: the backup of expert e
is (0, e, e, ...); the copy living in slot q is (q + 1, e, e, ...).  A slot that
was filled from a peer therefore shows the peer's tag, one filled from DRAM shows
tag 0, and an untouched slot keeps its own.
"""
import numpy as np
import pytest

from oracle import planner as ref
from test_oracle_tables_map import parse_fig5
from test_planner import _panel_placement

W = 8


def tagged_store(p2l, E):
    backup = [bytes([0] + [e] * (W - 1)) for e in range(E)]
    weights = [bytes([q + 1] + [max(int(e), 0) if e >= 0 else 255] * (W - 1))
               for q, e in enumerate(p2l)]
    return weights, backup


def test_fig5_sources_as_the_footnote_states():
    meta, panels = parse_fig5()
    S, S_prim, E, R = meta["slots_per_rank"], meta["primary_slots"], meta["experts"], 4
    before = _panel_placement(panels[0], R, S)
    active = panels[1]["active"]
    plan = ref.plan_repair(before, active, R, S, S_prim, E)
    weights, backup = tagged_store(before, E)
    after, outcome = ref.carry_out_repair(weights, backup, plan["p2l"], plan["kind"],
                                          plan["src_slot"], active, S)
    e6_slot, e2_slot = 0 * S + 2, 1 * S + 2                       # R0's and R1's third slot
    assert after[e6_slot] == backup[6] and outcome[e6_slot] == ref.FROM_DRAM
    r3_copy = 3 * S + 2                                           # E2' on R3
    assert after[e2_slot] == weights[r3_copy] and after[e2_slot][0] == r3_copy + 1
    assert outcome[e2_slot] == ref.FROM_PEER
    moved = {e6_slot, e2_slot}
    for p in range(R * S):
        if p not in moved:
            assert after[p] == weights[p] and outcome[p] == ref.UNTOUCHED
    # the failed rank's memory is never written
    assert after[2 * S:3 * S] == weights[2 * S:3 * S]


@pytest.mark.parametrize("seed", range(5))
def test_every_live_slot_ends_up_holding_what_the_placement_names(seed):
    rng = np.random.default_rng(100 + seed)
    for trial in range(60):
        R, S = int(rng.integers(2, 9)), int(rng.integers(1, 5))
        S_prim = int(rng.integers(0, S + 1))
        E = int(rng.integers(1, min(R * S + 3, 250)))
        cur = rng.integers(-1, E, size=R * S).astype(np.int32)
        active = (rng.random(R) < 0.7).astype(np.int32)
        if not active.any():
            active[0] = 1
        plan = ref.plan_repair(cur, active, R, S, S_prim, E)
        weights, backup = tagged_store(cur, E)
        # between planning and moving, one more rank may drop out
        later = active.copy()
        if trial % 2 and active.sum() > 1:
            later[rng.choice(np.nonzero(active)[0])] = 0
        after, outcome = ref.carry_out_repair(weights, backup, plan["p2l"], plan["kind"],
                                              plan["src_slot"], later, S)
        for p in range(R * S):
            e, kind = plan["p2l"][p], plan["kind"][p]
            if kind in (ref.NONE, ref.LOCAL):
                assert after[p] == weights[p] and outcome[p] == ref.UNTOUCHED
                continue
            assert after[p][1:] == backup[e][1:]                  # the right expert's weights
            if kind == ref.DRAM:
                assert after[p][0] == 0 and outcome[p] == ref.FROM_DRAM
            elif later[plan["src_slot"][p] // S]:
                assert after[p][0] == plan["src_slot"][p] + 1     # the planned peer's copy
                assert outcome[p] == ref.FROM_PEER
            else:
                assert after[p][0] == 0                           # planned source died: DRAM
                assert outcome[p] == ref.FROM_DRAM_FALLBACK
        # a planned source is never overwritten by the same batch
        dests = {p for p in range(R * S) if plan["kind"][p] in (ref.PEER, ref.DRAM)}
        assert not dests & {plan["src_slot"][p] for p in dests if plan["kind"][p] == ref.PEER}


def _rejoin_plan(impl_transition):
    meta, panels = parse_fig5()
    S, S_prim, E, R = meta["slots_per_rank"], meta["primary_slots"], meta["experts"], 4
    normal = _panel_placement(panels[0], R, S)
    shrunk_mask = np.asarray(panels[1]["active"], np.int32)
    shrunk = _panel_placement(panels[1], R, S, stale=normal)
    shrunk[2 * S:3 * S] = -1                                      # the relaunched rank holds nothing yet
    target = _panel_placement(panels[2], R, S)
    assert np.array_equal(target, normal)                         # Fig. 5: the preferred placement returns
    plan = impl_transition(shrunk, target, shrunk_mask, np.ones(R, np.int32), R, S, S_prim)
    return S, E, shrunk, target, shrunk_mask, plan


def test_fig5_rejoin_restores_the_preferred_placement():
    S, E, shrunk, target, mask, plan = _rejoin_plan(ref.plan_transition)
    assert plan["p2l"] == target.tolist()
    kind, src = plan["kind"], plan["src_slot"]
    # R2 gets E2 and E6 back from the copies the repair made on R1 and R0
    assert kind[2 * S] == ref.PEER and src[2 * S] == 1 * S + 2
    assert kind[2 * S + 1] == ref.PEER and src[2 * S + 1] == 0 * S + 2
    # the repair's extra copies are given up (slots empty again), everything else stays
    assert kind[0 * S + 2] == ref.NONE and kind[1 * S + 2] == ref.NONE
    assert plan["local"] == 7 and plan["peer"] == 2 and plan["dram"] == 0
    weights, backup = tagged_store(shrunk, E)
    after, outcome = ref.carry_out_repair(weights, backup, plan["p2l"], kind, src, mask, S)
    for p, e in enumerate(target):                                # loaded while R2 is still inactive
        if e >= 0:
            assert after[p][1:] == backup[e][1:]
    assert after[2 * S][0] == (1 * S + 2) + 1 and after[2 * S + 1][0] == (0 * S + 2) + 1


@pytest.mark.parametrize("seed", range(4))
def test_transition_plans_reach_any_target(seed):
    rng = np.random.default_rng(500 + seed)
    for trial in range(60):
        R, S = int(rng.integers(2, 9)), int(rng.integers(1, 5))
        S_prim = int(rng.integers(0, S + 1))
        E = int(rng.integers(1, min(R * S + 3, 250)))
        cur = rng.integers(-1, E, size=R * S).astype(np.int32)
        target = rng.integers(-1, E, size=R * S).astype(np.int32)
        active = (rng.random(R) < 0.7).astype(np.int32)
        writable = np.maximum(active, (rng.random(R) < 0.3).astype(np.int32))
        plan = ref.plan_transition(cur, target, active, writable, R, S, S_prim)
        weights, backup = tagged_store(cur, E)
        after, outcome = ref.carry_out_repair(weights, backup, plan["p2l"], plan["kind"],
                                              plan["src_slot"], active, S)
        for p in range(R * S):
            if not writable[p // S]:
                assert plan["p2l"][p] == cur[p] and after[p] == weights[p]
                continue
            e = plan["p2l"][p]
            assert e == target[p]
            if e < 0:
                assert after[p] == weights[p]
            elif e == cur[p]:
                assert after[p] == weights[p] and plan["kind"][p] == ref.LOCAL
            else:
                assert after[p][1:] == backup[e][1:]
                live_copy = any(active[q // S] and cur[q] == e and
                                not (writable[q // S] and target[q] >= 0 and target[q] != cur[q])
                                for q in range(R * S))
                assert (plan["kind"][p] == ref.PEER) == live_copy  # DRAM only when no copy survives
                if live_copy:
                    assert after[p][0] == plan["src_slot"][p] + 1
