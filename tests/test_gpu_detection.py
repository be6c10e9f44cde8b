"""GPU-side failure detection (paper Sec. 3.4, Sec. 4.1, Fig. 7): a rank that
never signals is dropped by the waiting kernel itself -- active bit cleared on
the device, failure reported after the kernel exits, its pairs skipped in that
step -- and a captured graph keeps replaying on the reduced membership.  The
silence is injected from the host (the withhold knob); every wait in the kernel
is bounded by the timeout, so all kernels exit normally."""
import numpy as np
import pytest
import torch

from paper_2605_10670_amd import binding, synth

import gpu_util as gu

pytestmark = pytest.mark.gpu
TIMEOUT_NS = 200_000   # 200 us instead of the paper's 1 s
SILENT = 6


def _oracle_out(oracle, wl, p2l, active, silent=()):
    """One step of the oracle under the mask `active`, with the ranks in `silent`
    sending no signal: layout, the rows the combine uses, the combined output, and what
    the detection round leaves behind (mask for later steps, report for the host)."""
    lay = oracle.step_layout(wl.topk_idx, p2l, active, wl.E, wl.R, wl.S, wl.S_prim, oracle.SPREAD)
    recv = oracle.pack(wl.x, lay["row_of"])
    y = oracle.stub_scale(recv, oracle.BF16, lay["N"], lay["offset"], p2l, wl.expert_scale)
    arrived = np.ones(wl.R, np.int32)
    arrived[list(silent)] = 0
    det = oracle.detect_round(lay["slot_of"], lay["row_of"], active, arrived, wl.S)
    chain = oracle.f32_to_bf16(oracle.combine_chain32(y, oracle.BF16, wl.topk_w, det["row_of"]))
    return lay, det, chain


@pytest.mark.parametrize("T_batch", [512, 64])   # tiled layout / single-workgroup layout
@pytest.mark.parametrize("use_graph", [False, True])
def test_silent_rank_is_dropped_by_the_kernel(oracle, use_graph, T_batch):
    wl = synth.churn_inputs(1, T=T_batch, H=512)[0]
    T, k, R = wl.T, wl.k, wl.R
    ctx = gu.make_context(wl)
    stream = torch.cuda.Stream()
    try:
        gu.apply_tables(ctx, wl.p2l, wl.active, stream)
        ctx.set_detection(TIMEOUT_NS)
        dev = gu.DeviceStep(ctx, wl, stream)
        dev.step()                          # warm-up (also outside the graph)
        stream.synchronize()
        if use_graph:
            ctx.graph_begin(stream)
            dev.step()
            graph = ctx.graph_end(stream)
            run = lambda: graph.launch(stream)
        else:
            run = dev.step

        def run_and_read():
            run()
            stream.synchronize()
            return ctx.read_layout(T, stream), gu.to_host(dev.out, np.uint16)

        live = wl.active
        dead = synth.active_mask(R, (SILENT,))
        # 1. healthy step: every rank signals, nothing is dropped
        lay, det, chain = _oracle_out(oracle, wl, wl.p2l, live)
        got, out = run_and_read()
        gu.assert_layout_equal(got, lay, T, k)
        assert np.array_equal(out, chain)
        assert ctx.read_failures(stream).sum() == 0
        assert ctx.read("active", R, stream).tolist() == [1] * R
        version = got["version"]

        # 2. rank SILENT stops signalling: the combine-side wait times out
        w = np.zeros(R, np.int32)
        w[SILENT] = 1
        ctx.debug_withhold_signal(w, stream)
        lay, det, chain = _oracle_out(oracle, wl, wl.p2l, live, silent=(SILENT,))
        got, out = run_and_read()
        assert np.array_equal(got["slot_of"], lay["slot_of"])      # routed before the failure
        assert np.array_equal(got["row_of"], det["row_of"])        # its pairs lost their row
        assert np.array_equal(out, chain)
        assert det["withdrawn"] == lay["rank_count"][SILENT] > 0
        assert ctx.check_layout(T, stream).tolist() == [0, 0, 0, det["withdrawn"]]
        assert det["active"].tolist() == dead.tolist()
        assert ctx.read("active", R, stream).tolist() == dead.tolist()   # cleared by the kernel
        assert got["version"] == version       # this step's layout ran before the drop

        # 3. next step, no host action on the tables yet: routing already avoids the rank;
        #    experts that lived only there are uncovered and counted
        lay, det, chain = _oracle_out(oracle, wl, wl.p2l, dead, silent=(SILENT,))
        assert det["report"].sum() == 0            # a rank that is no longer active is not awaited
        got, out = run_and_read()
        gu.assert_layout_equal(got, lay, T, k)
        assert got["rank_count"][SILENT] == 0 and got["n_uncovered"] > 0
        assert np.array_equal(out, chain)
        assert got["version"] == version + 1       # the drop shows in the table version

        # until the host has read the report its copy of the mask is out of date: a membership
        # update (here: another rank toggled) is refused rather than bringing the rank back
        other = synth.active_mask(R, (SILENT + 1,))
        with pytest.raises(binding.EepError) as ei:
            ctx.set_membership(other, stream)
        assert ei.value.code == binding.ERR_STATE
        with pytest.raises(binding.EepError) as ei:     # strict context: coverage needs the mask
            ctx.update_placement(wl.p2l, stream)
        assert ei.value.code == binding.ERR_STATE
        assert ctx.read("active", R, stream).tolist() == dead.tolist()

        # 4. the host learns of it, repairs the placement, service is complete again
        failed = ctx.read_failures(stream)
        assert failed.tolist() == w.tolist()
        assert ctx.read_failures(stream).sum() == 0                # report was cleared
        # the placement that was fine a moment ago is now refused for what it is: uncovered
        with pytest.raises(binding.EepError) as ei:
            ctx.update_placement(wl.p2l, stream)
        assert ei.value.code == binding.ERR_COVERAGE
        plan = binding.plan_repair(wl.p2l, dead, R, wl.S, wl.S_prim, wl.E)
        assert plan["unplaced"] == 0
        ctx.update_placement(plan["p2l"], stream)                  # passes the coverage check
        lay, det, chain = _oracle_out(oracle, wl, plan["p2l"], dead, silent=(SILENT,))
        got, out = run_and_read()
        gu.assert_layout_equal(got, lay, T, k)
        assert got["n_uncovered"] == 0 and got["N"] == T * k
        assert np.array_equal(out, chain)

        # 5. rejoin: the rank signals again, mask then preferred placement
        ctx.debug_withhold_signal(np.zeros(R, np.int32), stream)
        assert ctx.read_failures(stream).sum() == 0                # the host is up to date
        ctx.set_membership(live, stream)
        ctx.update_placement(wl.p2l, stream)
        lay, det, chain = _oracle_out(oracle, wl, wl.p2l, live)
        got, out = run_and_read()
        gu.assert_layout_equal(got, lay, T, k)
        assert np.array_equal(out, chain)
        assert ctx.read_failures(stream).sum() == 0
        if use_graph:
            assert graph.counters() == dict(instantiations=1, exec_updates=0, launches=5)
            graph.destroy()
    finally:
        ctx.destroy()


def test_detection_argument_checks():
    wl = synth.decode(T=64, H=256)
    ctx = gu.make_context(wl)
    try:
        with pytest.raises(binding.EepError):
            ctx.set_detection(-1)
        with pytest.raises(binding.EepError):
            ctx.set_detection(3_000_000_000)
        ctx.set_detection(0)
    finally:
        ctx.destroy()
