"""Pins for the oracle's table building (O1) and pair mapping (O2).

What fixes the expected values here is the paper, not the oracle: the three
panels of Fig. 5 (golden text file), the validity contract of Sec. 3.2, the
skip-inactive rule of Fig. 7, and brute force over every mask on tiny cases
written directly with Python list comprehensions.
"""
import itertools
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "fig5_overview.txt")


def parse_fig5():
    meta, panels, cur = {}, [], None
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if not line:
            continue
        tok = line.split()
        if tok[0] in ("slots_per_rank", "primary_slots", "experts"):
            meta[tok[0]] = int(tok[1])
        elif tok[0] == "panel":
            cur = dict(name=tok[1], ranks={}, routes={})
            panels.append(cur)
        elif tok[0] == "active":
            cur["active"] = [int(v) for v in tok[1:]]
        elif tok[0] == "source":
            cur.setdefault("sources", []).append(tok[1:])
        elif tok[0] == "route":
            cur["routes"][int(tok[1][1:])] = int(tok[2][1:])
        elif tok[0][0] == "R":
            r = int(tok[0][1:])
            if tok[1] == "failed":
                cur["ranks"][r] = None
            else:
                cur["ranks"][r] = [-1 if v == "-" else int(v[1:]) for v in tok[1:]]
    return meta, panels


@pytest.mark.parametrize("dead_slots", ["empty", "stale"])
def test_fig5_three_panels_first_live(oracle, dead_slots):
    meta, panels = parse_fig5()
    S, S_prim, E = meta["slots_per_rank"], meta["primary_slots"], meta["experts"]
    R = 4
    assert [p["name"] for p in panels] == ["normal", "shrunk", "rejoined"]
    stale = None
    for panel in panels:
        p2l = np.full(R * S, -1, np.int32)
        for r, slots in panel["ranks"].items():
            if slots is None:
                # the panel prints only "failed"; what the dead rank's slots still
                # say must not matter because its active bit is 0
                if dead_slots == "stale":
                    p2l[r * S:(r + 1) * S] = stale[r * S:(r + 1) * S]
                continue
            p2l[r * S:r * S + S] = slots
        stale = p2l.copy()
        active = np.array(panel["active"], np.int32)
        assert oracle.uncovered_experts(p2l, active, E, S) == 0
        off, lst = oracle.tables(p2l, E, S, S_prim)
        # one token per logical expert, top-1
        idx = np.arange(E, dtype=np.int32).reshape(E, 1)
        slot_of, n_unc, n_msk = oracle.map_pairs(idx, off, lst, active, E, S, oracle.FIRST_LIVE)
        assert (n_unc, n_msk) == (0, 0)
        for e, rank in panel["routes"].items():
            assert slot_of[e, 0] // S == rank, (panel["name"], e)
        # every expert lands on a live rank that hosts it
        for e in range(E):
            p = slot_of[e, 0]
            assert active[p // S] == 1 and p2l[p] == e
        # a failed rank receives nothing (validity condition 1)
        lay = oracle.layout(slot_of, R, S)
        for r in range(R):
            if active[r] == 0:
                assert lay["rank_count"][r] == 0


def test_canonical_order_primary_before_redundant(oracle):
    # expert 0 has replicas in slot 5 (redundant of rank 1), slot 3 (primary of
    # rank 1) and slot 2 (redundant of rank 0): order must be 3, 2, 5
    S, S_prim, E = 3, 2, 2
    p2l = np.array([1, -1, 0, 0, -1, 0], np.int32)
    off, lst = oracle.tables(p2l, E, S, S_prim)
    assert off.tolist() == [0, 3, 4]
    assert lst.tolist()[:4] == [3, 2, 5, 0]
    assert lst.tolist()[4:] == [-1, -1]


def test_tables_reject_out_of_range(oracle):
    with pytest.raises(ValueError):
        oracle.tables(np.array([0, 7], np.int32), 4, 2, 1)
    with pytest.raises(ValueError):
        oracle.tables(np.array([0, -2], np.int32), 4, 2, 1)
    with pytest.raises(ValueError):
        oracle.tables(np.array([0, 4], np.int32), 4, 2, 1)      # E itself is the first invalid id
    oracle.tables(np.array([3, -1], np.int32), 4, 2, 1)         # E - 1 and "empty" are the last valid


def _brute_slot(e, t, p2l, active, S, S_prim, E, policy, earlier):
    """Independent statement of O2 for one pair, with Python builtins only."""
    if not (0 <= e < E) or e in earlier:
        return -1, "masked"
    reps = sorted((p for p in range(len(p2l)) if p2l[p] == e),
                  key=lambda p: ((p % S) >= S_prim, p))
    live = [p for p in reps if active[p // S]]
    if not live:
        return -1, "uncovered"
    return (live[0] if policy == 1 else live[t % len(live)]), "ok"


@pytest.mark.parametrize("policy", [0, 1])
def test_brute_force_all_masks_and_many_placements(oracle, policy):
    """R=4, S=2 (1 primary + 1 redundant), E=4: every one of the 2^4 masks, a few
    hundred random placements (empty slots, multi-replica experts, out-of-range
    and repeated indices included)."""
    R, S, S_prim, E, k, T = 4, 2, 1, 4, 3, 8
    rng = np.random.default_rng(7 + policy)
    for trial in range(150):
        p2l = rng.integers(-1, E, size=R * S).astype(np.int32)
        idx = rng.integers(-1, E + 1, size=(T, k)).astype(np.int32)
        off, lst = oracle.tables(p2l, E, S, S_prim)
        for mask in itertools.product([0, 1], repeat=R):
            active = np.array(mask, np.int32)
            slot_of, n_unc, n_msk = oracle.map_pairs(idx, off, lst, active, E, S, policy)
            exp_unc = exp_msk = 0
            for t in range(T):
                for j in range(k):
                    want, why = _brute_slot(int(idx[t, j]), t, p2l.tolist(), mask, S, S_prim, E,
                                            policy, [int(v) for v in idx[t, :j]])
                    assert slot_of[t, j] == want, (trial, mask, t, j)
                    exp_unc += why == "uncovered"
                    exp_msk += why == "masked"
            assert (n_unc, n_msk) == (exp_unc, exp_msk)
            live_missing = sum(1 for e in range(E)
                               if not any(p2l[p] == e and mask[p // S] for p in range(R * S)))
            assert oracle.uncovered_experts(p2l, active, E, S) == live_missing


@pytest.mark.parametrize("policy", [0, 1])
def test_validity_invariants_random(oracle, policy):
    """Validity contract (Sec. 3.2) on a mid-size random case with 3 failed ranks."""
    from paper_2605_10670_amd import synth
    R, S_prim, S_red, E, k, T = 8, 4, 2, 32, 4, 256
    S = S_prim + S_red
    rng = np.random.default_rng(99)
    failed = (1, 6)
    p2l = synth.repaired_placement(synth.preferred_placement(R, S_prim, S_red), failed, R, S_prim,
                                   S_red)
    active = synth.active_mask(R, failed)
    idx, _ = synth.router_topk(rng.standard_normal((T, E)).astype(np.float32), k)
    res = oracle.step_layout(idx, p2l, active, E, R, S, S_prim, policy)
    slot_of = res["slot_of"]
    assert res["n_uncovered"] == 0 and res["n_masked"] == 0
    assert (slot_of >= 0).all()                                   # exactly one slot per pair
    assert (active[slot_of // S] == 1).all()                      # ... on a live rank
    assert (p2l[slot_of] == idx).all()                            # ... that hosts the expert
    assert res["rank_count"][list(failed)].sum() == 0             # failed ranks get nothing
    assert res["count"].sum() == T * k == res["N"]                # counts sum to T*k
    if policy == 0:
        # SPREAD really uses more than one replica of a replicated expert
        multi = [e for e in range(E) if ((p2l == e) & (active[np.arange(R * S) // S] == 1)).sum() > 1]
        assert multi
        for e in multi[:4]:
            assert len(set(slot_of[idx == e].tolist())) > 1


def test_uncovered_and_masked_are_counted(oracle):
    from paper_2605_10670_amd import synth
    w = synth.tiny("b")
    res = oracle.step_layout(w.topk_idx, w.p2l, w.active, w.E, w.R, w.S, w.S_prim, oracle.SPREAD)
    assert oracle.uncovered_experts(w.p2l, w.active, w.E, w.S) == 1
    lost = 11
    assert res["n_uncovered"] == int((w.topk_idx == lost).sum()) > 0
    assert res["N"] + res["n_uncovered"] + res["n_masked"] == w.T * w.k
    assert (res["slot_of"][w.topk_idx == lost] == -1).all()


def test_spread_balances_and_depends_only_on_token_and_live_set(oracle):
    """The paper names no replica-selection rule, so the expected slots of SPREAD cannot come
    from it.  What any sensible spreading rule must satisfy is pinned instead, without
    restating the oracle's formula: consecutive tokens that want one expert are dealt over
    its live replicas evenly (every window of n tokens touches all n live replicas, so the
    per-replica counts differ by at most one), the choice does not depend on the pair's
    position j, on the token's other experts, or on replicas that are not live."""
    R, S, S_prim, E, T = 6, 3, 2, 8, 60
    # expert 6: primary on rank 2 (its second primary slot), redundant copies on ranks 0, 3 and 4
    p2l = np.full(R * S, -1, np.int32)
    for r in range(R):
        p2l[r * S + 0] = r                     # experts 0..5 primary on their rank
    p2l[2 * S + 1] = 6
    for r in (0, 3, 4):
        p2l[r * S + 2] = 6                     # three redundant copies of expert 6
    p2l[5 * S + 1] = 7
    off, lst = oracle.tables(p2l, E, S, S_prim)
    rng = np.random.default_rng(11)
    for mask in ([1] * R, [1, 1, 0, 1, 1, 1], [0, 1, 1, 1, 0, 1], [0, 1, 0, 1, 0, 1]):
        active = np.array(mask, np.int32)
        live = [p for p in range(R * S) if p2l[p] == 6 and mask[p // S]]
        n = len(live)
        # every token wants expert 6, at a random position j among two other experts
        k = 3
        idx = np.empty((T, k), np.int32)
        pos = rng.integers(0, k, size=T)
        for t in range(T):
            others = rng.choice([0, 1, 3, 5, 7], size=k - 1, replace=False)
            idx[t] = np.insert(others, pos[t], 6)
        slot_of, _, _ = oracle.map_pairs(idx, off, lst, active, E, S, 0)
        chosen = np.array([slot_of[t, pos[t]] for t in range(T)])
        assert set(chosen.tolist()) <= set(live)
        for t0 in range(T - n + 1):                                  # every window is a full deal
            assert set(chosen[t0:t0 + n].tolist()) == set(live), (mask, t0)
        counts = np.bincount(chosen, minlength=R * S)[live]
        assert counts.max() - counts.min() <= 1
        # the same tokens with expert 6 alone in the token, at j = 0: same choices
        alone, _, _ = oracle.map_pairs(np.full((T, 1), 6, np.int32), off, lst, active, E, S, 0)
        assert np.array_equal(alone[:, 0], chosen)
        # emptying the slots of dead ranks changes nothing
        pruned = p2l.copy()
        pruned[[p for p in range(R * S) if not mask[p // S]]] = -1
        off2, lst2 = oracle.tables(pruned, E, S, S_prim)
        again, _, _ = oracle.map_pairs(idx, off2, lst2, active, E, S, 0)
        assert np.array_equal(np.array([again[t, pos[t]] for t in range(T)]), chosen)
