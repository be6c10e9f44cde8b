"""One EP instance, several MoE layers (paper Sec. 4.1: one GPU-resident peer
table; Sec. 5.1: expert-location metadata per layer): contexts created with
eep_create_attached share the membership mask and keep their own placement."""
import numpy as np
import pytest
import torch

from paper_2605_10670_amd import binding, synth

import gpu_util as gu

pytestmark = pytest.mark.gpu


def _layer_workload(seed, H):
    wl = synth.decode(T=512, H=H, seed_offset=seed)
    return wl


def _check(oracle, ctx, dev, wl, p2l, active, version):
    dev.step()
    dev.sync()
    lay = oracle.step_layout(wl.topk_idx, p2l, active, wl.E, wl.R, wl.S, wl.S_prim, oracle.SPREAD)
    got = ctx.read_layout(wl.T)
    gu.assert_layout_equal(got, lay, wl.T, wl.k)
    assert got["version"] == version
    recv = oracle.pack(wl.x, lay["row_of"])
    chain = oracle.f32_to_bf16(oracle.combine_chain32(recv, oracle.BF16, wl.topk_w, lay["row_of"]))
    assert np.array_equal(gu.to_host(dev.out, np.uint16), chain)
    return got


def test_two_layers_share_one_membership(oracle):
    wl_a, wl_b = _layer_workload(21, 256), _layer_workload(22, 512)
    R, S, S_prim, S_red, E = wl_a.R, wl_a.S, wl_a.S_prim, wl_a.S_red, wl_a.E
    # layer B places its experts differently: every rank holds the experts of rank r+3
    p2l_b = np.roll(wl_a.p2l.reshape(R, S), 3, axis=0).ravel().copy()
    failed = (9,)
    dead, live = synth.active_mask(R, failed), synth.active_mask(R)
    rep_a = synth.repaired_placement(wl_a.p2l, failed, R, S_prim, S_red)
    rep_b = binding.plan_repair(p2l_b, dead, R, S, S_prim, E)["p2l"]
    a = gu.make_context(wl_a)
    b = binding.Context(num_ranks=R, slots_per_rank=S, primary_slots=S_prim, num_logical=E,
                        max_tokens=wl_b.T, topk=wl_b.k, hidden=wl_b.H, parent=a)
    try:
        assert a.view_pointers()["active"] == b.view_pointers()["active"]      # one table
        assert a.view_pointers()["phys_to_logical"] != b.view_pointers()["phys_to_logical"]
        a.update_placement(wl_a.p2l)
        b.update_placement(p2l_b)
        dev_a, dev_b = gu.DeviceStep(a, wl_a), gu.DeviceStep(b, wl_b)
        _check(oracle, a, dev_a, wl_a, wl_a.p2l, live, 1)
        _check(oracle, b, dev_b, wl_b, p2l_b, live, 1)

        # rank 9 fails.  The mask is shared, so it cannot be cleared while ANY layer
        # would lose an expert: repairing only layer A is not enough.
        a.update_placement(rep_a)
        with pytest.raises(binding.EepError) as ei:
            a.set_membership(dead)
        assert ei.value.code == binding.ERR_COVERAGE
        assert a.read("active", R).tolist() == live.tolist()
        b.update_placement(rep_b)
        b.set_membership(dead)                      # through either context: one mask
        got_a = _check(oracle, a, dev_a, wl_a, rep_a, dead, 3)
        got_b = _check(oracle, b, dev_b, wl_b, rep_b, dead, 3)
        assert got_a["rank_count"][9] == 0 and got_b["rank_count"][9] == 0

        # rejoin through the other context
        a.set_membership(live)
        a.update_placement(wl_a.p2l)
        b.update_placement(p2l_b)
        _check(oracle, a, dev_a, wl_a, wl_a.p2l, live, 5)
        _check(oracle, b, dev_b, wl_b, p2l_b, live, 5)

        # the first context of an instance goes last
        with pytest.raises(binding.EepError) as ei:
            a.destroy()
        assert ei.value.code == binding.ERR_STATE
    finally:
        b.destroy()
        a.destroy()


def test_failure_detected_in_one_layer_drops_the_rank_for_all(oracle):
    sets = synth.churn_inputs(2, T=256, H=256)
    wl_a, wl_b = sets
    R = wl_a.R
    a = gu.make_context(wl_a, strict=False)
    b = binding.Context(num_ranks=R, slots_per_rank=wl_b.S, primary_slots=wl_b.S_prim,
                        num_logical=wl_b.E, max_tokens=wl_b.T, topk=wl_b.k, hidden=wl_b.H,
                        strict_coverage=False, parent=a)
    try:
        a.update_placement(wl_a.p2l)
        b.update_placement(wl_b.p2l)
        a.set_detection(200_000)
        dev_a, dev_b = gu.DeviceStep(a, wl_a), gu.DeviceStep(b, wl_b)
        w = np.zeros(R, np.int32)
        w[3] = 1
        a.debug_withhold_signal(w)
        dev_a.step()                                  # layer A times out on rank 3
        dev_a.sync()
        dead = synth.active_mask(R, (3,))
        assert b.read("active", R).tolist() == dead.tolist()
        dev_b.step()                                  # layer B already routes around it
        dev_b.sync()
        lay = oracle.step_layout(wl_b.topk_idx, wl_b.p2l, dead, wl_b.E, R, wl_b.S, wl_b.S_prim, 0)
        got = b.read_layout(wl_b.T)
        gu.assert_layout_equal(got, lay, wl_b.T, wl_b.k)
        assert got["rank_count"][3] == 0 and got["n_uncovered"] > 0
        assert a.read_failures().tolist() == w.tolist()
    finally:
        b.destroy()
        a.destroy()


def test_two_contexts_in_flight_on_two_streams(oracle):
    """Two micro-batches of one layer kept in flight at once: two contexts of one
    instance (own layout arrays each), each on its own stream, 20 overlapping steps,
    a table patch half-way.  Both must match the oracle every time."""
    wl_a, wl_b = synth.decode(T=1024, H=1024, seed_offset=51), synth.decode(T=1024, H=1024,
                                                                            seed_offset=52)
    R = wl_a.R
    failed = (4,)
    dead, live = synth.active_mask(R, failed), synth.active_mask(R)
    repaired = synth.repaired_placement(wl_a.p2l, failed, R, wl_a.S_prim, wl_a.S_red)
    a = gu.make_context(wl_a)
    b = binding.Context(num_ranks=R, slots_per_rank=wl_b.S, primary_slots=wl_b.S_prim,
                        num_logical=wl_b.E, max_tokens=wl_b.T, topk=wl_b.k, hidden=wl_b.H,
                        parent=a)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    try:
        a.update_placement(wl_a.p2l)
        b.update_placement(wl_a.p2l)
        torch.cuda.synchronize()
        dev_a, dev_b = gu.DeviceStep(a, wl_a, sa), gu.DeviceStep(b, wl_b, sb)
        torch.cuda.synchronize()

        def expected(wl, p2l, active):
            lay = oracle.step_layout(wl.topk_idx, p2l, active, wl.E, R, wl.S, wl.S_prim, 0)
            recv = oracle.pack(wl.x, lay["row_of"])
            return lay, oracle.f32_to_bf16(oracle.combine_chain32(recv, oracle.BF16, wl.topk_w,
                                                                  lay["row_of"]))

        want = {(n, f): expected(wl, repaired if f else wl_a.p2l, dead if f else live)
                for n, wl in (("a", wl_a), ("b", wl_b)) for f in (False, True)}
        for step in range(20):
            down = step >= 10
            if step == 10:                                  # both layers repaired, then the mask
                torch.cuda.synchronize()
                a.update_placement(repaired)
                b.update_placement(repaired)
                a.set_membership(dead)
                torch.cuda.synchronize()
            dev_a.out.zero_()
            dev_b.out.zero_()
            torch.cuda.synchronize()
            dev_a.step()                                    # queued on sa ...
            dev_b.step()                                    # ... and on sb, no wait in between
            torch.cuda.synchronize()
            for name, ctx, dev, wl in (("a", a, dev_a, wl_a), ("b", b, dev_b, wl_b)):
                lay, chain = want[(name, down)]
                gu.assert_layout_equal(ctx.read_layout(wl.T), lay, wl.T, wl.k)
                assert np.array_equal(gu.to_host(dev.out, np.uint16), chain), (step, name)
    finally:
        b.destroy()
        a.destroy()
