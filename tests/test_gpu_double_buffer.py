"""Double-buffered staging (paper Sec. 4.1) through the C ABI: a context and its
staging context hold two staging sets; the dispatch side of step i+1 runs on a
side stream beside the expert + combine side of step i (event fork / join).
Every step must still be bit-equal to the oracle's stand-alone step under the
tables in force at its dispatch -- eagerly with a membership change in mid
flight, and as one captured hipGraph per pass with changes between passes."""
import numpy as np
import pytest
import torch

from oracle import pipeline as pl
from paper_2605_10670_amd import binding, synth

import gpu_util as gu

pytestmark = pytest.mark.gpu


def _oracle_step(oracle, wl, p2l, active):
    lay = oracle.step_layout(wl.topk_idx, p2l, active, wl.E, wl.R, wl.S, wl.S_prim, oracle.SPREAD)
    recv = oracle.pack(wl.x, lay["row_of"])
    y = oracle.stub_scale(recv, oracle.BF16, lay["N"], lay["offset"], p2l, wl.expert_scale)
    chain = oracle.f32_to_bf16(oracle.combine_chain32(y, oracle.BF16, wl.topk_w, lay["row_of"]))
    return dict(lay=lay, out=chain)


class _Pipe:
    """Two staging sets with device buffers of their own, and per-step input/output buffers."""

    def __init__(self, sets, strict):
        self.wls = sets
        wl = sets[0]
        self.T, self.k = wl.T, wl.k
        self.main, self.side = torch.cuda.Stream(), torch.cuda.Stream()
        self.ctx = [gu.make_context(wl, strict=strict)]
        self.ctx.append(self.ctx[0].staging())
        self.recv = [gu.dev_empty(wl.T * wl.k, wl.H, "bf16", fill=0) for _ in range(2)]
        self.y = [gu.dev_empty(wl.T * wl.k, wl.H, "bf16", fill=0) for _ in range(2)]
        self.scale = gu.to_dev(wl.expert_scale)
        self.idx = [gu.to_dev(w.topk_idx) for w in sets]
        self.x = [gu.to_dev(w.x) for w in sets]
        self.w = [gu.to_dev(w.topk_w) for w in sets]
        self.out = [gu.dev_empty(wl.T, wl.H, "bf16", fill=0) for _ in sets]

    def dispatch_side(self, i, stream):          # not overlapped (prologue, or after a drain)
        s = i % 2
        self.ctx[s].dispatch_layout(self.idx[i], self.T, stream)
        self.ctx[s].dispatch(self.x[i], self.recv[s], self.T, stream=stream)

    def fork_dispatch(self, i):
        s = i % 2
        self.ctx[s].staging_fork(self.idx[i], self.x[i], self.recv[s], self.T, self.main, self.side)

    def join(self, i):
        self.ctx[i % 2].staging_join(self.main, self.side)

    def combine_side(self, i):
        s = i % 2
        self.ctx[s].expert_stub("scale", self.recv[s], self.y[s], self.T, expert_scale=self.scale,
                                stream=self.main)
        self.ctx[s].combine(self.y[s], self.w[i], self.out[i], self.T, self.main)

    def overlapped_pass(self, steps):
        """D(first); then D(i+1) beside C(i) for every step; drained at the end."""
        self.dispatch_side(steps[0], self.main)
        for a, b in zip(steps, steps[1:] + [None]):
            if b is not None:
                self.fork_dispatch(b)
            self.combine_side(a)
            if b is not None:
                self.join(b)

    def destroy(self):
        self.ctx[1].destroy()
        self.ctx[0].destroy()


def test_eager_overlap_with_a_membership_change_in_mid_flight(oracle):
    sets = synth.churn_inputs(6, T=512, H=512)
    wl = sets[0]
    R = wl.R
    pipe = _Pipe(sets, strict=False)
    try:
        ctx = pipe.ctx[0]
        gu.apply_tables(ctx, wl.p2l, wl.active, pipe.main)
        dead = synth.active_mask(R, (5,))
        repaired = synth.repaired_placement(wl.p2l, (5,), R, wl.S_prim, wl.S_red)
        events, got_lay = [], {}

        def D(i, overlapped):
            events.append((pl.D, i))
            pipe.fork_dispatch(i) if overlapped else pipe.dispatch_side(i, pipe.main)

        def C(i, joined_step=None):
            events.append((pl.C, i))
            pipe.combine_side(i)
            if joined_step is not None:
                pipe.join(joined_step)
            # the set is read back before the schedule refills it (this wait is the test's, not
            # the schedule's: by now both sides of the overlap have been queued)
            pipe.main.synchronize()
            got_lay[i] = pipe.ctx[i % 2].read_layout(pipe.T, pipe.main)

        D(0, False)
        D(1, True); C(0, 1)
        # rank 5 drops out between steps, mask only (no drain needed): step 1 was routed
        # before, step 2 is routed after; the experts that lived only there go uncovered
        events.append((pl.SET_MEMBERSHIP, dead))
        pipe.ctx[1].set_membership(dead, pipe.main)          # through the staging context
        D(2, True); C(1, 2)
        D(3, True); C(2, 3)
        C(3)                                                # drain: nothing dispatched is pending
        # now the repair: placement (needs the drained pipeline), mask unchanged
        events.append((pl.UPDATE_PLACEMENT, repaired))
        pipe.ctx[1].update_placement(repaired, pipe.main)    # acts on the shared tables
        D(4, False)
        D(5, True); C(4, 5)
        C(5)
        torch.cuda.synchronize()

        want = pl.run(events, lambda i, p2l, act: _oracle_step(oracle, sets[i], p2l, act),
                      wl.p2l, wl.active)
        for i in range(6):
            gu.assert_layout_equal(got_lay[i], want[i]["lay"], pipe.T, pipe.k)
            assert np.array_equal(gu.to_host(pipe.out[i], np.uint16), want[i]["out"]), f"step {i}"
        assert got_lay[1]["rank_count"][5] > 0 and got_lay[2]["rank_count"][5] == 0
        assert got_lay[2]["n_uncovered"] > 0 and got_lay[4]["n_uncovered"] == 0
        # both contexts see one set of tables
        assert np.array_equal(pipe.ctx[0].read("phys_to_logical", ctx.P), repaired)
        assert pipe.ctx[0].view_pointers()["phys_to_logical"] == \
            pipe.ctx[1].view_pointers()["phys_to_logical"]
        assert pipe.ctx[0].view_pointers()["row_of"] != pipe.ctx[1].view_pointers()["row_of"]
    finally:
        pipe.destroy()


def test_overlapped_pass_as_one_graph_replayed_across_failure_and_rejoin(oracle):
    """A pass of 6 steps (think: 3 MoE layers x 2 micro-batches) captured ONCE with the
    overlap inside; the pipeline is drained at the ends of the graph, so table updates
    between replays are updates between forward passes."""
    sets = synth.churn_inputs(6, T=1024, H=1024)
    wl = sets[0]
    R = wl.R
    pipe = _Pipe(sets, strict=True)
    try:
        ctx = pipe.ctx[0]
        gu.apply_tables(ctx, wl.p2l, wl.active, pipe.main)
        steps = list(range(6))
        pipe.overlapped_pass(steps)                  # warm-up, eager
        torch.cuda.synchronize()
        ctx.graph_begin(pipe.main)
        pipe.overlapped_pass(steps)
        graph = ctx.graph_end(pipe.main)

        dead = synth.active_mask(R, (5,))
        repaired = synth.repaired_placement(wl.p2l, (5,), R, wl.S_prim, wl.S_red)
        for phase, (p2l, active) in enumerate([(wl.p2l, wl.active), (repaired, dead),
                                               (wl.p2l, wl.active)]):
            if phase == 1:      # failure: placement, then mask
                ctx.update_placement(p2l, pipe.main)
                ctx.set_membership(active, pipe.main)
            elif phase == 2:    # rejoin: mask, then placement
                ctx.set_membership(active, pipe.main)
                ctx.update_placement(p2l, pipe.main)
            for o in pipe.out:
                o.fill_(0)
            torch.cuda.synchronize()
            for _ in range(2):  # replays of one executable graph, eager work between them
                graph.launch(pipe.main)
                pipe.main.synchronize()
                for i in steps:
                    want = _oracle_step(oracle, sets[i], p2l, active)
                    assert np.array_equal(gu.to_host(pipe.out[i], np.uint16), want["out"]), \
                        f"phase {phase} step {i}"
                    if i >= 4:   # the two sets still hold the layouts of the last two steps
                        gu.assert_layout_equal(pipe.ctx[i % 2].read_layout(pipe.T, pipe.main),
                                               want["lay"], pipe.T, pipe.k)
        assert graph.counters() == dict(instantiations=1, exec_updates=0, launches=6)
        graph.destroy()
    finally:
        pipe.destroy()


def test_staging_argument_checks_and_lifetime():
    wl = synth.churn_inputs(1, T=64, H=256)[0]
    a = gu.make_context(wl)
    b = a.staging()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    try:
        with pytest.raises(binding.EepError) as ei:          # staging sets go first
            a.destroy()
        assert ei.value.code == binding.ERR_STATE
        with pytest.raises(binding.EepError) as ei:
            b.staging_join(s1, s2)                            # no fork before
        assert ei.value.code == binding.ERR_STATE
        with pytest.raises(binding.EepError) as ei:
            b.staging_fork(None, None, None, wl.T, s1, s1)    # one stream twice
        assert ei.value.code == binding.ERR_INVALID_ARG
    finally:
        b.destroy()
        a.destroy()
