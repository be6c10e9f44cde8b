"""De-duplicated dispatch on the GPU (one row per (token, destination rank), expansion on
the destination) against the oracle, and against the plain dispatch: the expanded buffer
must be byte-equal to what eep_dispatch writes."""
import numpy as np
import pytest
import torch

from paper_2605_10670_amd import binding, synth

import gpu_util as gu

pytestmark = pytest.mark.gpu


def _workload(R, T, k, sp, sr, H, failed=(), seed=0, dtype="bf16", masked=False):
    rng = np.random.default_rng(4000 + seed + R + T + k)
    E = R * sp
    idx, w = synth.router_topk(rng.standard_normal((T, E)).astype(np.float32), min(k, E))
    if masked:
        idx = idx.copy()
        idx[rng.random(idx.shape) < 0.1] = -1
    x32 = rng.standard_normal((T, H), dtype=np.float32)
    x = x32 if dtype == "f32" else synth.f32_to_bf16_bits(x32)
    pref = synth.preferred_placement(R, sp, sr)
    p2l = synth.repaired_placement(pref, failed, R, sp, sr) if failed else pref
    return synth.Workload("dedup", T, H, E, idx.shape[1], R, sp, sr, dtype, dtype, dtype, "identity",
                          failed, idx, w, x, p2l, synth.active_mask(R, failed))


CASES = [
    dict(R=32, T=4096, k=8, sp=8, sr=1, H=256, failed=(13,)),            # decode shape, one failed rank
    dict(R=4, T=512, k=8, sp=4, sr=1, H=512, masked=True),               # 4 ranks, top-8: heavy sharing
    dict(R=8, T=64, k=6, sp=2, sr=2, H=64, failed=(2, 5)),               # single-workgroup layout path
    dict(R=32, T=16384, k=8, sp=8, sr=1, H=64, failed=(7, 20)),          # 128 tiles
    dict(R=2, T=600, k=2, sp=1, sr=3, H=8, dtype="f32"),                 # more replicas than experts
    dict(R=1, T=77, k=4, sp=8, sr=0, H=1024),                            # one rank: one row per token
    dict(R=16, T=32, k=32, sp=4, sr=1, H=128),                           # k = 32
    dict(R=4, T=0, k=2, sp=4, sr=1, H=128),                              # empty batch
]


@pytest.mark.parametrize("case", CASES)
def test_dedup_dispatch_matches_oracle_and_plain_dispatch(oracle, case):
    wl = _workload(**case)
    T, k, H, R, S = wl.T, wl.k, wl.H, wl.R, wl.S
    ctx = gu.make_context(wl, strict=False)
    try:
        gu.apply_tables(ctx, wl.p2l, wl.active)
        dev = gu.DeviceStep(ctx, wl)
        fill = 0x5A5A if wl.x_dtype == "bf16" else 7.0
        recv_d = gu.dev_empty(T * k, H, wl.x_dtype, fill=0x5A5A if wl.x_dtype == "bf16" else 7.0)
        expanded = gu.dev_empty(T * k, H, wl.x_dtype, fill=0)
        dev.layout()
        ctx.dedup_layout(T)
        dev.dispatch()                                   # the plain dispatch, for comparison
        ctx.dispatch_dedup(dev.x, recv_d, T)
        ctx.expand(recv_d, expanded, T)
        torch.cuda.synchronize()

        lay = oracle.step_layout(wl.topk_idx, wl.p2l, wl.active, wl.E, R, S, wl.S_prim, oracle.SPREAD)
        gu.assert_layout_equal(ctx.read_layout(T), lay, T, k)
        want = oracle.dedup_layout(lay["slot_of"], lay["row_of"], R, S)
        got = ctx.read_dedup(T)
        assert got["N_d"] == want["N_d"]
        assert np.array_equal(got["dedup_count"], want["dedup_count"])
        assert np.array_equal(got["dedup_offset"], want["dedup_offset"])
        assert np.array_equal(got["dedup_row"], want["dedup_row"])
        assert np.array_equal(got["dedup_dst"], np.where(want["lead"] == 1, want["dedup_row"], -1))
        assert np.array_equal(got["expand_of"], want["expand_of"])
        if T == 0:
            return
        N, N_d = lay["N"], want["N_d"]
        npdt = gu.NP_OF[wl.x_dtype]
        want_d = oracle.pack_dedup(wl.x, want["dedup_row"], want["lead"])
        got_d = gu.to_host(recv_d, npdt)
        assert np.array_equal(got_d[:N_d].view(np.uint8), want_d[:N_d].view(np.uint8))
        untouched = got_d[N_d:].view(np.uint16 if wl.x_dtype == "bf16" else np.float32)
        assert (untouched == fill).all(), "rows past N_d were written"
        plain = gu.to_host(dev.recv, npdt)
        exp = gu.to_host(expanded, npdt)
        assert np.array_equal(exp[:N].view(np.uint8), plain[:N].view(np.uint8))
        assert np.array_equal(exp[:N].view(np.uint8),
                              oracle.pack(wl.x, lay["row_of"])[:N].view(np.uint8))
        assert (exp[N:].view(np.uint8) == 0).all(), "rows past N were written"
        if case["R"] <= 4 and k >= 8:
            assert N_d < 0.6 * N                           # sharing really happens here
    finally:
        ctx.destroy()


def test_dedup_call_order_and_refusals():
    wl = _workload(R=4, T=64, k=4, sp=4, sr=1, H=128)
    ctx = gu.make_context(wl)
    try:
        gu.apply_tables(ctx, wl.p2l, wl.active)
        dev = gu.DeviceStep(ctx, wl)
        other = torch.zeros_like(dev.recv)
        with pytest.raises(binding.EepError) as ei:
            ctx.dedup_layout(wl.T)                         # no layout yet
        assert ei.value.code == binding.ERR_STATE
        dev.layout()
        with pytest.raises(binding.EepError) as ei:
            ctx.dispatch_dedup(dev.x, other, wl.T)         # no de-duplicated layout yet
        assert ei.value.code == binding.ERR_STATE
        ctx.dedup_layout(wl.T)
        with pytest.raises(binding.EepError) as ei:
            ctx.expand(other, other, wl.T)                 # in place is not possible
        assert ei.value.code == binding.ERR_INVALID_ARG
        with pytest.raises(binding.EepError) as ei:
            ctx.dispatch_dedup(dev.x, other, wl.T - 4)
        assert ei.value.code == binding.ERR_STATE
        ctx.dispatch_dedup(dev.x, other, wl.T)
        ctx.expand(other, dev.recv, wl.T)
        # a new layout of the same T invalidates the de-duplicated tables of the old one
        dev.layout()
        with pytest.raises(binding.EepError) as ei:
            ctx.dispatch_dedup(dev.x, other, wl.T)
        assert ei.value.code == binding.ERR_STATE
        with pytest.raises(binding.EepError) as ei:
            ctx.expand(other, dev.recv, wl.T)
        assert ei.value.code == binding.ERR_STATE
        ctx.dedup_layout(wl.T)
        ctx.dispatch_dedup(dev.x, other, wl.T)
        torch.cuda.synchronize()
    finally:
        ctx.destroy()
    fp8 = synth.prefill_fp8(T=64, H=1024)
    ctx = gu.make_context(fp8)
    try:
        gu.apply_tables(ctx, fp8.p2l, fp8.active)
        dev = gu.DeviceStep(ctx, fp8)
        dev.layout()
        ctx.dedup_layout(fp8.T)                            # the layout itself is payload-agnostic
        with pytest.raises(binding.EepError) as ei:
            ctx.dispatch_dedup(dev.x, dev.recv, fp8.T)
        assert ei.value.code == binding.ERR_INVALID_ARG
    finally:
        ctx.destroy()
