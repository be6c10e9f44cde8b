"""Membership churn under a captured hipGraph (paper Sec. 2.3, Fig. 4, Fig. 8,
Sec. 4.2): one graph of dispatch_layout -> dispatch -> expert stub -> combine is
captured once and replayed 1000 times while rank 5 is toggled failed / rejoined
every 100 steps by table writes only.  Every step is compared with the oracle."""
import numpy as np
import pytest
import torch

from paper_2605_10670_amd import binding, synth

import gpu_util as gu

pytestmark = pytest.mark.gpu

STEPS, PERIOD, RANK = 1000, 100, 5


def test_churn_1000_replays_one_instantiation(oracle):
    sets = synth.churn_inputs(8)
    wl0 = sets[0]
    T, k, H, R = wl0.T, wl0.k, wl0.H, wl0.R
    pref = wl0.p2l_preferred
    repaired = synth.repaired_placement(pref, (RANK,), R, wl0.S_prim, wl0.S_red)
    live, dead = synth.active_mask(R), synth.active_mask(R, (RANK,))

    # oracle results for the 16 (input set, membership) combinations
    expect = {}
    for si, wl in enumerate(sets):
        for failed in (False, True):
            p2l, act = (repaired, dead) if failed else (pref, live)
            lay = oracle.step_layout(wl.topk_idx, p2l, act, wl.E, R, wl.S, wl.S_prim, oracle.SPREAD)
            recv = oracle.pack(wl.x, lay["row_of"])
            y = oracle.stub_scale(recv, oracle.BF16, lay["N"], lay["offset"], p2l, wl.expert_scale)
            out64 = oracle.combine(y, oracle.BF16, wl.topk_w, lay["row_of"])
            chain = oracle.f32_to_bf16(oracle.combine_chain32(y, oracle.BF16, wl.topk_w,
                                                              lay["row_of"]))
            # closed form: out = (sum_j w_j s[e_j]) * x, whatever the membership
            closed = ((wl.topk_w.astype(np.float64) * wl.expert_scale[wl.topk_idx]).sum(1)[:, None]
                      * gu.bf16_to_f64(wl.x))
            assert np.abs(out64 - closed).max() <= 2.0 ** -7 * np.abs(closed).max()
            gu.check_combine(chain, "bf16", out64)
            assert lay["N"] == T * k and (lay["rank_count"][RANK] == 0) == failed
            expect[(si, failed)] = dict(lay=lay, chain=chain)

    ctx = gu.make_context(wl0)
    stream = torch.cuda.Stream()
    try:
        gu.apply_tables(ctx, pref, live, stream)
        dev_sets = [(gu.to_dev(w.topk_idx), gu.to_dev(w.topk_w), gu.to_dev(w.x)) for w in sets]
        idx = torch.empty_like(dev_sets[0][0])
        wts = torch.empty_like(dev_sets[0][1])
        x = torch.empty_like(dev_sets[0][2])
        scale = gu.to_dev(wl0.expert_scale)
        recv = torch.zeros((T * k, H), dtype=torch.int16, device="cuda")
        y = torch.zeros_like(recv)
        out = torch.zeros((T, H), dtype=torch.int16, device="cuda")
        torch.cuda.synchronize()

        def step_calls():
            ctx.dispatch_layout(idx, T, stream)
            ctx.dispatch(x, recv, T, stream=stream)
            ctx.expert_stub("scale", recv, y, T, expert_scale=scale, stream=stream)
            ctx.combine(y, wts, out, T, stream=stream)

        with torch.cuda.stream(stream):
            for dst, src in zip((idx, wts, x), dev_sets[0]):
                dst.copy_(src, non_blocking=True)
        step_calls()                      # warm-up outside the graph
        stream.synchronize()
        ctx.graph_begin(stream)
        step_calls()
        graph = ctx.graph_end(stream)

        version = 2
        was_failed = False
        for s in range(STEPS):
            failed = (s // PERIOD) % 2 == 1
            if failed != was_failed:      # exactly two table calls per toggle, nothing else
                if failed:
                    ctx.update_placement(repaired, stream)
                    ctx.set_membership(dead, stream)
                else:
                    ctx.set_membership(live, stream)
                    ctx.update_placement(pref, stream)
                version += 2
                was_failed = failed
            si = s % len(sets)
            with torch.cuda.stream(stream):
                for dst, src in zip((idx, wts, x), dev_sets[si]):
                    dst.copy_(src, non_blocking=True)
            graph.launch(stream)
            stream.synchronize()
            want = expect[(si, failed)]
            got = ctx.read_layout(T, stream)
            gu.assert_layout_equal(got, want["lay"], T, k)
            assert got["version"] == version
            assert np.array_equal(gu.to_host(out, np.uint16), want["chain"]), f"step {s}"
        c = graph.counters()
        assert c == dict(instantiations=1, exec_updates=0, launches=STEPS)
        graph.destroy()
    finally:
        ctx.destroy()


@pytest.mark.parametrize("router", ["uniform", "zipf"])
def test_decode_full_size_as_the_benchmark_launches_it(oracle, router):
    """The launch configuration the benchmark times: DeepSeek-V3 decode shape at full
    size, identity expert (y aliases the receive buffer), EIGHT steps captured in one
    hipGraph on a side stream, replayed with table patches and eager work in between.
    Every output row of every step of every replay is compared with the oracle.
    "zipf": the router of the failed-rank configuration, whose hottest experts are the ones
    that move to redundant slots when rank 13 fails (the hottest slot takes ~4000 rows)."""
    wl = synth.decode() if router == "uniform" else synth.decode_failed_zipf()
    wl.p2l = wl.p2l_preferred                     # start healthy; the failure comes mid-test
    T, k, H, R = wl.T, wl.k, wl.H, wl.R
    failed = (13,)
    dead, live = synth.active_mask(R, failed), synth.active_mask(R)
    repaired = synth.repaired_placement(wl.p2l, failed, R, wl.S_prim, wl.S_red)

    def expected(p2l, active):
        lay = oracle.step_layout(wl.topk_idx, p2l, active, wl.E, R, wl.S, wl.S_prim, oracle.SPREAD)
        recv = oracle.pack(wl.x, lay["row_of"])
        chain = oracle.f32_to_bf16(oracle.combine_chain32(recv, oracle.BF16, wl.topk_w, lay["row_of"]))
        gu.check_combine(chain, "bf16", oracle.combine(recv, oracle.BF16, wl.topk_w, lay["row_of"]))
        return lay, recv, chain

    want_live, want_dead = expected(wl.p2l, live), expected(repaired, dead)
    assert want_dead[0]["rank_count"][13] == 0 and want_dead[0]["N"] == T * k

    ctx = gu.make_context(wl)
    stream = torch.cuda.Stream()
    steps_per_graph = 8
    try:
        gu.apply_tables(ctx, wl.p2l, live, stream)
        idx, w, x = gu.to_dev(wl.topk_idx), gu.to_dev(wl.topk_w), gu.to_dev(wl.x)
        recv = torch.zeros((T * k, H), dtype=torch.int16, device="cuda")
        outs = [torch.zeros((T, H), dtype=torch.int16, device="cuda") for _ in range(steps_per_graph)]
        torch.cuda.synchronize()

        def step(out):
            ctx.dispatch_layout(idx, T, stream)
            ctx.dispatch(x, recv, T, stream=stream)
            ctx.combine(recv, w, out, T, stream=stream)

        step(outs[0])
        stream.synchronize()
        ctx.graph_begin(stream)
        for out in outs:
            step(out)
        graph = ctx.graph_end(stream)

        def replay_and_check(want, version):
            for out in outs:
                out.zero_()
            torch.cuda.synchronize()
            graph.launch(stream)
            stream.synchronize()
            lay, rows, chain = want
            got = ctx.read_layout(T, stream)
            gu.assert_layout_equal(got, lay, T, k)
            assert got["version"] == version
            assert np.array_equal(gu.to_host(recv, np.uint16)[:lay["N"]], rows[:lay["N"]])
            for i, out in enumerate(outs):
                assert np.array_equal(gu.to_host(out, np.uint16), chain), f"step {i} of the graph"

        replay_and_check(want_live, 2)
        ctx.update_placement(repaired, stream)          # rank 13 fails: two table patches
        ctx.set_membership(dead, stream)
        replay_and_check(want_dead, 4)
        step(outs[0])                                   # eager work between replays
        stream.synchronize()
        replay_and_check(want_dead, 4)
        ctx.set_membership(live, stream)                # and rejoins
        ctx.update_placement(wl.p2l, stream)
        replay_and_check(want_live, 6)
        assert graph.counters() == dict(instantiations=1, exec_updates=0, launches=4)
        graph.destroy()
    finally:
        ctx.destroy()
