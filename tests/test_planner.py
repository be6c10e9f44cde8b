"""Placement-repair planner (paper Sec. 3.5, Sec. 5.1): the library's C++ version
and the plain Python statement in oracle/planner.py against the paper's worked
example (Fig. 5, middle panel), the coverage requirement, the definitions of the
three weight sources, and each other."""
import numpy as np
import pytest

from oracle import planner as ref
from paper_2605_10670_amd import binding, synth
from test_oracle_tables_map import parse_fig5

IMPLS = {"library": lambda *a, **k: binding.plan_repair(*a, **k),
         "oracle": lambda *a, **k: ref.plan_repair(*a, **k)}


def _panel_placement(panel, R, S, stale=None):
    p2l = np.full(R * S, -1, np.int32)
    for r, slots in panel["ranks"].items():
        if slots is None:
            p2l[r * S:(r + 1) * S] = stale[r * S:(r + 1) * S]
        else:
            p2l[r * S:r * S + S] = slots
    return p2l


@pytest.mark.parametrize("impl", sorted(IMPLS))
def test_fig5_repair_reproduces_middle_panel(impl):
    meta, panels = parse_fig5()
    S, S_prim, E, R = meta["slots_per_rank"], meta["primary_slots"], meta["experts"], 4
    normal, shrunk = panels[0], panels[1]
    before = _panel_placement(normal, R, S)
    want = _panel_placement(shrunk, R, S, stale=before)
    out = IMPLS[impl](before, shrunk["active"], R, S, S_prim, E)
    assert np.array_equal(np.asarray(out["p2l"]), want)
    assert out["unplaced"] == 0
    kind, src = np.asarray(out["kind"]), np.asarray(out["src_slot"])
    for e_tok, r_tok, how, *rest in shrunk["sources"]:
        e, r = int(e_tok[1:]), int(r_tok[1:])
        slot = r * S + (S - 1)
        assert want[slot] == e
        if how == "dram":
            assert kind[slot] == ref.DRAM
        else:
            assert kind[slot] == ref.PEER and src[slot] // S == int(rest[0][1:])
    assert (kind[2 * S:3 * S] == ref.NONE).all()            # failed rank untouched
    assert out["local"] == 7 and out["peer"] == 1 and out["dram"] == 1


def _check_plan(out, cur, active, R, S, S_prim, E):
    P = R * S
    new, kind, src = (np.asarray(out[k]) for k in ("p2l", "kind", "src_slot"))
    live = np.asarray(active)[np.arange(P) // S] != 0
    assert np.array_equal(new[~live], cur[~live])                      # failed ranks untouched
    assert (kind[~live] == ref.NONE).all()
    covered = set(new[live].tolist()) - {-1}
    assert len(covered) == E - out["unplaced"]
    for p in np.nonzero(live)[0]:
        if new[p] < 0:
            assert kind[p] == ref.NONE
        elif kind[p] == ref.LOCAL:
            assert new[p] == cur[p]                                    # weights already there
        elif kind[p] == ref.PEER:
            q = src[p]
            assert live[q] and cur[q] == new[p] and q // S != p // S   # a surviving copy elsewhere
        else:
            assert kind[p] == ref.DRAM
            assert not ((cur == new[p]) & live).any()                  # no GPU-resident copy left
    # What Sec. 3.5 fixes without naming an algorithm.  (1) Nothing that is already in
    # place is moved: a live slot that keeps its expert is local reuse, never a copy.
    keeps = live & (new == cur) & (cur >= 0)
    assert (kind[keeps] == ref.LOCAL).all()
    # (2) The backup tier is used exactly for the experts that lost every GPU copy, once
    # each: that is the least movement that restores coverage.
    lost = [e for e in range(E) if not ((cur == e) & live).any()]
    from_dram = sorted(new[kind == ref.DRAM].tolist())
    assert len(from_dram) == len(set(from_dram)) == len(lost) - out["unplaced"]
    assert set(from_dram) <= set(lost)
    # (3) An expert that had a live copy still has one (coverage never regresses).
    had_live = set(cur[live].tolist()) - {-1}
    assert had_live <= covered
    return covered


def _brute_force_best(cur, active, R, S, E):
    """All ways to fill the live slots: the best reachable coverage and the fewest slots
    that must be rewritten to reach it."""
    import itertools
    P = R * S
    live = [p for p in range(P) if active[p // S]]
    best = (-1, 0)
    for choice in itertools.product(range(-1, E), repeat=len(live)):
        covered = len(set(choice) - {-1})
        rewrites = sum(1 for p, e in zip(live, choice) if e != cur[p])
        best = max(best, (covered, -rewrites))
    return best[0], -best[1]


@pytest.mark.parametrize("impl", sorted(IMPLS))
def test_coverage_is_maximal_and_backup_movement_minimal_by_brute_force(impl):
    rng = np.random.default_rng(2024)
    for trial in range(120):
        R, S = int(rng.integers(1, 4)), int(rng.integers(1, 3))
        E = int(rng.integers(1, 5))
        cur = rng.integers(-1, E, size=R * S).astype(np.int32)
        active = (rng.random(R) < 0.7).astype(np.int32)
        out = IMPLS[impl](cur, active, R, S, int(rng.integers(0, S + 1)), E)
        best_cov, min_rewrites = _brute_force_best(cur.tolist(), active.tolist(), R, S, E)
        assert E - out["unplaced"] == best_cov, (trial, cur, active)
        assert out["dram"] == min_rewrites, (trial, cur, active)


@pytest.mark.parametrize("seed", range(6))
def test_library_matches_plain_statement_and_invariants(seed):
    rng = np.random.default_rng(seed)
    for trial in range(40):
        R, S = int(rng.integers(2, 9)), int(rng.integers(1, 5))
        S_prim = int(rng.integers(0, S + 1))
        E = int(rng.integers(1, R * S + 3))
        cur = rng.integers(-1, E, size=R * S).astype(np.int32)
        active = (rng.random(R) < 0.7).astype(np.int32)
        load = rng.integers(0, 5, size=E).astype(np.float32) if trial % 2 else None
        a = binding.plan_repair(cur, active, R, S, S_prim, E, load)
        b = ref.plan_repair(cur, active, R, S, S_prim, E, load)
        for key in ("p2l", "kind", "src_slot"):
            assert np.array_equal(np.asarray(a[key]), np.asarray(b[key])), key
        assert (a["local"], a["peer"], a["dram"], a["unplaced"]) == \
               (b["local"], b["peer"], b["dram"], b["unplaced"])
        _check_plan(a, cur, active, R, S, S_prim, E)
        _check_plan(b, cur, active, R, S, S_prim, E)
        # pigeonhole: coverage is reached exactly when the live slots can hold E experts
        live_slots = int(active.sum()) * S
        assert a["unplaced"] == max(0, E - live_slots)
        assert binding.host_uncovered_experts(a["p2l"], active, E, S) == a["unplaced"]
        # the library's return code says the same: coverage error exactly when experts are left over
        assert a["status"] == (binding.ERR_COVERAGE if a["unplaced"] else binding.OK)


def test_failure_scales_shift_from_peer_to_dram():
    """Sec. 6.3 (repair-source mix): with few failed ranks most repaired experts
    still have a surviving GPU copy; as more ranks fail, a growing share must come
    from the DRAM backup.  DSV3-like instance with spare capacity: 32 ranks x
    (8 primary + 8 redundant slots), experts 0-3 of every rank replicated once,
    four redundant slots per rank empty."""
    R, S_prim, S_red, E = 32, 8, 8, 256
    S = S_prim + S_red
    pref = synth.preferred_placement(R, S_prim, S_red).reshape(R, S)
    pref[:, 12:] = -1
    pref = pref.ravel()
    order = np.random.default_rng(0).permutation(R)
    dram_share = []
    for n_failed in (1, 2, 4, 8, 16):
        active = synth.active_mask(R, order[:n_failed])
        out = binding.plan_repair(pref, active, R, S, S_prim, E)
        _check_plan(out, pref, active, R, S, S_prim, E)
        assert out["unplaced"] == 0
        dram_share.append(out["dram"] / (out["dram"] + out["peer"]))
    assert all(b >= a for a, b in zip(dram_share, dram_share[1:]))
    assert dram_share[0] < 0.5 < dram_share[-1]


def test_dsv3_8_plus_1_slots_tolerate_three_failed_ranks():
    """32 x (8+1) slots hold 288 experts' worth of weights: up to 3 failed ranks
    can be covered (261 live slots >= 256), 4 cannot (252 < 256)."""
    R, S_prim, S_red, E = 32, 8, 1, 256
    pref = synth.preferred_placement(R, S_prim, S_red)
    for n_failed, want_unplaced in ((1, 0), (3, 0), (4, 4)):
        active = synth.active_mask(R, range(5, 5 + n_failed))
        out = binding.plan_repair(pref, active, R, S_prim + S_red, S_prim, E)
        assert out["unplaced"] == want_unplaced
        _check_plan(out, pref, active, R, S_prim + S_red, S_prim, E)


def test_tiny_infeasible_case_reports_one_uncovered_expert():
    wl = synth.tiny("b")
    out = binding.plan_repair(wl.p2l_preferred, wl.active, wl.R, wl.S, wl.S_prim, wl.E)
    assert out["unplaced"] == 1                       # 15 live slots < 16 experts
    assert out["status"] == binding.ERR_COVERAGE


def test_bad_arguments():
    with pytest.raises(binding.EepError):
        binding.plan_repair(np.array([0, 9], np.int32), [1, 1], 2, 1, 1, 2)
    with pytest.raises(binding.EepError):
        binding.plan_repair(np.array([0, 1], np.int32), [1, 1], 2, 1, 1, 2, load=[-1.0, 1.0])


def test_transition_library_matches_plain_statement():
    rng = np.random.default_rng(77)
    for trial in range(300):
        R, S = int(rng.integers(1, 9)), int(rng.integers(1, 5))
        S_prim = int(rng.integers(0, S + 1))
        E = int(rng.integers(1, R * S + 3))
        cur = rng.integers(-1, E, size=R * S).astype(np.int32)
        target = rng.integers(-1, E, size=R * S).astype(np.int32)
        if trial % 3 == 0:                                         # mostly-unchanged targets too
            keep = rng.random(R * S) < 0.8
            target[keep] = cur[keep]
        active = (rng.random(R) < 0.7).astype(np.int32)
        writable = np.maximum(active, (rng.random(R) < 0.3).astype(np.int32))
        got = binding.plan_transition(cur, target, active, writable, R, S, S_prim, E)
        want = ref.plan_transition(cur, target, active, writable, R, S, S_prim)
        for key in ("p2l", "kind", "src_slot"):
            assert np.asarray(got[key]).tolist() == list(want[key]), (trial, key)
        assert (got["local"], got["peer"], got["dram"]) == (want["local"], want["peer"], want["dram"])
        assert got["unplaced"] == want["unplaced"] == 0           # a transition places what it is told


def test_codes_are_the_ones_the_header_declares():
    """The plain statement's source kinds and outcome codes are compared with the library's by
    value in the GPU tests, so they must be the header's values (and distinct)."""
    import os
    import re
    text = open(os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))),
                             "include", "eep.h")).read()
    enum = {m.group(1): int(m.group(2)) for m in re.finditer(r"\b(EEP_[A-Z_]+)\s*=\s*(-?\d+)", text)}
    assert (ref.NONE, ref.LOCAL, ref.PEER, ref.DRAM) == (
        enum["EEP_SRC_NONE"], enum["EEP_SRC_LOCAL"], enum["EEP_SRC_PEER"], enum["EEP_SRC_DRAM"])
    assert (ref.UNTOUCHED, ref.FROM_PEER, ref.FROM_DRAM, ref.FROM_DRAM_FALLBACK) == (
        enum["EEP_REPAIR_UNTOUCHED"], enum["EEP_REPAIR_FROM_PEER"], enum["EEP_REPAIR_FROM_DRAM"],
        enum["EEP_REPAIR_FROM_DRAM_FALLBACK"])
    assert len({ref.NONE, ref.LOCAL, ref.PEER, ref.DRAM}) == 4
    assert len({ref.UNTOUCHED, ref.FROM_PEER, ref.FROM_DRAM, ref.FROM_DRAM_FALLBACK}) == 4


def test_transition_argument_errors():
    ok = np.zeros(4, np.int32)
    one = np.ones(2, np.int32)
    with pytest.raises(binding.EepError):
        binding.plan_transition(ok, np.array([0, 0, 0, 9], np.int32), one, one, 2, 2, 1, 4)
    with pytest.raises(binding.EepError):
        binding.plan_transition(ok - 2, ok, one, one, 2, 2, 1, 4)
    with pytest.raises(ValueError):
        binding.plan_transition(ok, ok, one, np.ones(3, np.int32), 2, 2, 1, 4)
