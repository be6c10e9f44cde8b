"""Pins of the oracle's statement of double-buffered staging (paper Sec. 4.1):
which issue orders are free of hazards, and that a valid overlapped pass yields
every step's stand-alone result under the tables of its dispatch."""
import numpy as np
import pytest

from oracle import pipeline as pl
from paper_2605_10670_amd import synth


def test_two_batch_overlap_is_valid_and_drained():
    for n in range(0, 7):
        ev = pl.two_batch_overlap(n)
        pl.validate(ev)
        assert [a for w, a in ev if w == pl.D] == list(range(n))
        assert [a for w, a in ev if w == pl.C] == list(range(n))
        # D(i+1) is issued before C(i): that is the overlap
        for i in range(n - 1):
            assert ev.index((pl.D, i + 1)) < ev.index((pl.C, i))


@pytest.mark.parametrize("events", [
    [(pl.D, 0), (pl.D, 1), (pl.D, 2)],                                   # set 0 refilled too early
    [(pl.D, 0), (pl.C, 1)],                                              # nothing to combine there
    [(pl.D, 0), (pl.UPDATE_PLACEMENT, None), (pl.C, 0)],                 # slots change under a step
    [(pl.D, 0), (pl.D, 1), (pl.C, 0), (pl.UPDATE_PLACEMENT, None), (pl.C, 1)],
    [(pl.D, 0)],                                                         # never combined
])
def test_hazards_are_refused(events):
    with pytest.raises(pl.ScheduleError):
        pl.validate(events)


def test_placement_updates_only_when_no_step_is_in_flight():
    """Sec. 3.1: repair happens between forward passes.  With the pipeline drained a placement
    update is accepted and binds to the steps dispatched after it; with one or both staging
    sets holding a dispatched step it is refused."""
    seen = []
    drained = [(pl.D, 0), (pl.D, 1), (pl.C, 0), (pl.C, 1), (pl.UPDATE_PLACEMENT, "B"),
               (pl.D, 2), (pl.C, 2)]
    pl.validate(drained)
    pl.validate([(pl.UPDATE_PLACEMENT, "B")])                          # an idle pipeline too
    got = pl.run(drained, lambda i, p2l, act: seen.append((i, p2l, act)) or (i, p2l), "A", "m")
    assert seen == [(0, "A", "m"), (1, "A", "m"), (2, "B", "m")]
    assert got == {0: (0, "A"), 1: (1, "A"), 2: (2, "B")}
    for busy in ([(pl.D, 0), (pl.UPDATE_PLACEMENT, "B"), (pl.C, 0)],                    # one set
                 [(pl.D, 0), (pl.D, 1), (pl.UPDATE_PLACEMENT, "B"), (pl.C, 0), (pl.C, 1)],  # both
                 [(pl.D, 0), (pl.D, 1), (pl.C, 0), (pl.UPDATE_PLACEMENT, "B"), (pl.C, 1)]):
        with pytest.raises(pl.ScheduleError):
            pl.validate(busy)
    with pytest.raises(pl.ScheduleError):
        pl.validate([("rewind", 0)])                                    # unknown events too


def test_membership_updates_are_allowed_mid_flight_and_bind_at_dispatch(oracle):
    """The scalar stand-in gives out[t] = (sum over covered j of w_j s[e_j]) x[t]; which pairs
    are covered depends only on the mask in force at the step's dispatch.  Placement without
    replicas (slot p holds expert p), so the covered pairs can be read off the router indices."""
    rng = np.random.default_rng(3)
    R, S, k, T, H, n = 4, 2, 2, 32, 4, 4
    E = R * S
    p2l = np.arange(E, dtype=np.int32)
    scale = (1.0 + np.arange(E) / 4.0).astype(np.float32)
    steps = []
    for i in range(n):
        x = rng.standard_normal((T, H)).astype(np.float32)
        idx, w = synth.router_topk(rng.standard_normal((T, E)).astype(np.float32), k)
        steps.append((x, idx, w))

    def step_alone(i, p2l_now, active):
        x, idx, w = steps[i]
        lay = oracle.step_layout(idx, p2l_now, active, E, R, S, S, 0)
        y = oracle.stub_scale(oracle.pack(x, lay["row_of"]), oracle.F32, lay["N"], lay["offset"],
                              p2l_now, scale)
        return oracle.combine(y, oracle.F32, w, lay["row_of"])

    all_live, one_dead = np.ones(R, np.int32), synth.active_mask(R, (1,))
    events = [(pl.D, 0), (pl.D, 1), (pl.C, 0),
              (pl.SET_MEMBERSHIP, one_dead),          # while step 1 waits for its combine
              (pl.D, 2), (pl.C, 1), (pl.D, 3), (pl.C, 2),
              (pl.SET_MEMBERSHIP, all_live), (pl.C, 3)]
    got = pl.run(events, step_alone, p2l, all_live)
    mask_at_dispatch = [all_live, all_live, one_dead, one_dead]
    for i, (x, idx, w) in enumerate(steps):
        covered = mask_at_dispatch[i][idx // S] != 0
        coeff = (w.astype(np.float64) * scale[idx] * covered).sum(axis=1)
        np.testing.assert_allclose(got[i], coeff[:, None] * x.astype(np.float64), rtol=1e-6,
                                   atol=1e-7)
