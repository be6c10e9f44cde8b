"""eep_dispatch_layout_noalloc (the entry point for callers that cannot allocate
device memory) against eep_dispatch_layout and against the oracle: every output
array bit-equal, on calls in a row that share the static scratch array, later
calls with smaller inputs than earlier ones."""
import numpy as np
import pytest
import torch

from paper_2605_10670_amd import binding, synth

import gpu_util as gu

pytestmark = pytest.mark.gpu


def _device_outputs(T_max, k, R, P, fill):
    shapes = dict(slot_of=T_max * k, row_of=T_max * k, src_of=T_max * k, count=P, offset=P + 1,
                  rank_count=R, rank_offset=R + 1, cnt_src=R * P, status=4)
    return {n: torch.full((m,), fill, dtype=torch.int32, device="cuda") for n, m in shapes.items()}


def _host(out, T, k, R, P):
    h = {n: t.cpu().numpy() for n, t in out.items()}
    st = h.pop("status")
    res = dict(slot_of=h["slot_of"][:T * k].reshape(T, k), row_of=h["row_of"][:T * k].reshape(T, k),
               src_of=h["src_of"][:T * k], count=h["count"], offset=h["offset"],
               rank_count=h["rank_count"], rank_offset=h["rank_offset"],
               cnt_src=h["cnt_src"].reshape(R, P), N=int(st[0]), n_uncovered=int(st[1]),
               n_masked=int(st[2]), version=int(st[3]))
    tail = {n: h[n][T * k:] for n in ("slot_of", "row_of", "src_of")}
    return res, tail


def _workload(T, failed, seed_offset):
    wl = synth.decode(T=T, H=64, seed_offset=seed_offset)
    if failed:
        wl.p2l = synth.repaired_placement(wl.p2l_preferred, failed, wl.R, wl.S_prim, wl.S_red)
        wl.active = synth.active_mask(wl.R, failed)
    return wl


# T = 16384: 128 tiles, the three-launch path (tile prefixes in the scratch);
# T = 4096: 32 tiles, the fused two-launch path; T = 1024: 32 tiles of 32 tokens;
# T = 64: the single-workgroup path (no scratch besides the step counter).
@pytest.mark.parametrize("sizes", [(16384, 4096, 64), (4096, 1024), (8192, 16384, 2048)])
@pytest.mark.parametrize("policy", [binding.SPREAD, binding.FIRST_LIVE])
def test_noalloc_layout_equals_the_context_entry_point(oracle, sizes, policy):
    T_max = max(sizes)
    base = _workload(T_max, (), 40)
    R, S, P, E, k = base.R, base.S, base.P, base.E, base.k
    ctx = gu.make_context(base, policy=policy, T_max=T_max)
    try:
        out = _device_outputs(T_max, k, R, P, fill=-7)
        ptr = ctx.view_pointers()
        version = torch.tensor([1234], dtype=torch.int32, device="cuda")
        for step, T in enumerate(sizes):
            failed = () if step == 0 else (3 + step, 20)
            wl = _workload(T, failed, 41 + step)
            if step > 0:
                ctx.set_membership(np.ones(R, np.int32))  # rejoin first, then the next failure
            gu.apply_tables(ctx, wl.p2l, wl.active)
            idx = gu.to_dev(wl.topk_idx)
            ctx.dispatch_layout(idx, T)
            torch.cuda.synchronize()
            want = ctx.read_layout(T)
            free_before = torch.cuda.mem_get_info()[0]
            binding.dispatch_layout_noalloc(
                R=R, S=S, E=E, k=k, policy=policy, topk_idx=idx, active=ptr["active"],
                l2p_off=ptr["l2p_off"], l2p_list=ptr["l2p_list"], out=out, T=T,
                table_version=version if step % 2 == 0 else None)
            torch.cuda.synchronize()
            if step > 0:     # (the first call may still load code; later ones must take nothing)
                assert torch.cuda.mem_get_info()[0] == free_before, "device memory was allocated"
            got, tail = _host(out, T, k, R, P)
            gu.assert_layout_equal(got, want, T, k)
            assert got["version"] == (1234 if step % 2 == 0 else 0)
            ref = oracle.step_layout(wl.topk_idx, wl.p2l, wl.active, E, R, S, wl.S_prim, policy)
            gu.assert_layout_equal(got, ref, T, k)
            if step == 0:    # entries past T*k are not the call's to write
                assert all((a == -7).all() for a in tail.values())
    finally:
        ctx.destroy()


def test_noalloc_layout_tiny_other_topk(oracle):
    """k != 8 (the run-time-k kernels), R = 4, one failed rank."""
    wl = synth.tiny("c", T=512)
    R, S, P, E, k = wl.R, wl.S, wl.P, wl.E, wl.k
    off, lst = binding.host_replica_lists(wl.p2l, E, S, wl.S_prim)
    out = _device_outputs(wl.T, k, R, P, fill=-7)
    binding.dispatch_layout_noalloc(R=R, S=S, E=E, k=k, policy=binding.SPREAD,
                                    topk_idx=gu.to_dev(wl.topk_idx), active=gu.to_dev(wl.active),
                                    l2p_off=gu.to_dev(off), l2p_list=gu.to_dev(lst), out=out,
                                    T=wl.T)
    torch.cuda.synchronize()
    got, _ = _host(out, wl.T, k, R, P)
    ref = oracle.step_layout(wl.topk_idx, wl.p2l, wl.active, E, R, S, wl.S_prim, oracle.SPREAD)
    gu.assert_layout_equal(got, ref, wl.T, k)
    assert got["rank_count"][2] == 0


def test_noalloc_layout_of_an_empty_batch():
    R, S, E, k = 4, 3, 8, 2
    out = _device_outputs(8, k, R, R * S, fill=-7)
    binding.dispatch_layout_noalloc(R=R, S=S, E=E, k=k, policy=0, topk_idx=None, out=out, T=0,
                                    active=torch.ones(R, dtype=torch.int32, device="cuda"),
                                    l2p_off=torch.zeros(E + 1, dtype=torch.int32, device="cuda"),
                                    l2p_list=torch.zeros(R * S, dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    got, tail = _host(out, 0, k, R, R * S)
    assert got["N"] == 0 and got["n_uncovered"] == 0 and got["n_masked"] == 0
    assert not got["count"].any() and not got["offset"].any() and not got["cnt_src"].any()
    assert not got["rank_count"].any() and not got["rank_offset"].any()
    assert all((a == -7).all() for a in tail.values())        # no pair, nothing per pair written


def test_noalloc_layout_inside_a_captured_graph(oracle):
    """What the entry point is for: a caller under stream capture.  Captured once, replayed
    with new router outputs and a new mask in the same device buffers, with eager work in
    between; every replay is compared with the oracle."""
    T = 2048
    wls = [_workload(T, (), 60), _workload(T, (11,), 61), _workload(T, (11, 30), 62)]
    wl = wls[0]
    R, S, P, E, k = wl.R, wl.S, wl.P, wl.E, wl.k
    out = _device_outputs(T, k, R, P, fill=-7)
    idx = gu.to_dev(wl.topk_idx)
    off, lst = binding.host_replica_lists(wl.p2l, E, S, wl.S_prim)
    active, l2p_off, l2p_list = gu.to_dev(wl.active), gu.to_dev(off), gu.to_dev(lst)
    stream = torch.cuda.Stream()
    call = lambda: binding.dispatch_layout_noalloc(
        R=R, S=S, E=E, k=k, policy=binding.SPREAD, topk_idx=idx, active=active, l2p_off=l2p_off,
        l2p_list=l2p_list, out=out, T=T, stream=stream)
    call()                               # eager once: the scratch address is resolved here
    stream.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        call()
    for step in range(5):
        w = wls[step % 3]
        off, lst = binding.host_replica_lists(w.p2l, E, S, w.S_prim)
        idx.copy_(gu.to_dev(w.topk_idx))                 # eager work between the replays
        active.copy_(gu.to_dev(w.active))
        l2p_off.copy_(gu.to_dev(off))
        l2p_list.copy_(gu.to_dev(lst))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got, _ = _host(out, T, k, R, P)
        ref = oracle.step_layout(w.topk_idx, w.p2l, w.active, E, R, S, w.S_prim, oracle.SPREAD)
        gu.assert_layout_equal(got, ref, T, k)
        assert not got["rank_count"][w.active == 0].any()


def test_noalloc_layout_refuses_what_does_not_fit():
    R, S, E, k = 32, 9, 256, 8
    out = _device_outputs(64, k, R, R * S, fill=0)
    small = torch.zeros(64 * k, dtype=torch.int32, device="cuda")
    tables = dict(active=torch.ones(R, dtype=torch.int32, device="cuda"),
                  l2p_off=torch.zeros(E + 1, dtype=torch.int32, device="cuda"),
                  l2p_list=torch.zeros(R * S, dtype=torch.int32, device="cuda"))
    T_big = 32 * 128 * 2048          # 65536 tiles x 288 slots: far beyond the 4 MiB array
    assert binding.noalloc_scratch_needed(R, S, T_big) > binding.NOALLOC_SCRATCH_BYTES
    with pytest.raises(binding.EepError) as ei:    # refused on the host: nothing is launched
        binding.dispatch_layout_noalloc(R=R, S=S, E=E, k=k, policy=0, topk_idx=small, out=out,
                                        T=T_big, **tables)
    assert ei.value.code == binding.ERR_SCRATCH
    with pytest.raises(binding.EepError) as ei:
        binding.dispatch_layout_noalloc(R=R, S=S, E=E, k=k, policy=0, topk_idx=small, out=out,
                                        T=33, **tables)
    assert ei.value.code == binding.ERR_INVALID_ARG
    with pytest.raises(binding.EepError) as ei:
        binding.dispatch_layout_noalloc(R=R, S=S, E=E, k=k, policy=0, topk_idx=small,
                                        out=dict(out, status=None), T=64, **tables)
    assert ei.value.code == binding.ERR_INVALID_ARG
    torch.cuda.synchronize()
