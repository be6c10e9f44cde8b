"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the
same seeded inputs.  Integer results and moved bytes must be bit-exact; combine
outputs must meet the 1e-3 gate against the fp64 oracle and be bit-equal to the
oracle's fp32 ascending fused-multiply-add chain."""
import numpy as np
import pytest
import torch

from paper_2605_10670_amd import binding, synth

import gpu_util as gu

pytestmark = pytest.mark.gpu
ODT = {"f32": 0, "bf16": 1}


def oracle_step(oracle, wl, policy=0, p2l=None, active=None):
    p2l = wl.p2l if p2l is None else p2l
    active = wl.active if active is None else active
    lay = oracle.step_layout(wl.topk_idx, p2l, active, wl.E, wl.R, wl.S, wl.S_prim, policy)
    recv = oracle.pack(wl.x, lay["row_of"])
    recv_scale = oracle.pack(wl.x_scale, lay["row_of"]) if wl.x_scale is not None else None
    N = lay["N"]
    if wl.stub == "identity":
        y = recv
    elif wl.stub == "scale":
        y = oracle.stub_scale(recv, ODT[wl.x_dtype], N, lay["offset"], p2l, wl.expert_scale)
    else:
        y = oracle.stub_dequant(recv, recv_scale, N, 128)
    out64 = oracle.combine(y, ODT[wl.y_dtype], wl.topk_w, lay["row_of"])
    chain = oracle.combine_chain32(y, ODT[wl.y_dtype], wl.topk_w, lay["row_of"])
    chain_bits = chain.view(np.uint32) if wl.out_dtype == "f32" else oracle.f32_to_bf16(chain)
    return dict(lay=lay, recv=recv, recv_scale=recv_scale, y=y, out64=out64, chain_bits=chain_bits)


def run_and_compare(oracle, wl, policy=binding.SPREAD, strict=True):
    ctx = gu.make_context(wl, policy=policy, strict=strict)
    try:
        gu.apply_tables(ctx, wl.p2l, wl.active)
        dev = gu.DeviceStep(ctx, wl)
        dev.step()
        dev.sync()
        ref = oracle_step(oracle, wl, policy)
        got = ctx.read_layout(wl.T)
        gu.assert_layout_equal(got, ref["lay"], wl.T, wl.k)
        assert ctx.check_layout(wl.T).tolist() == [0, 0, 0, 0]      # the device-side bounds check
        N = got["N"]
        recv = gu.to_host(dev.recv, gu.NP_OF[wl.x_dtype])
        assert np.array_equal(recv[:N].view(np.uint8), ref["recv"][:N].view(np.uint8)), "packed rows"
        if wl.stub != "identity":
            assert (recv[N:].view(np.uint8) == 0).all(), "rows past N were written"
        if wl.x_scale is not None:
            rs = dev.recv_scale.cpu().numpy()
            assert np.array_equal(rs[:N].view(np.uint32), ref["recv_scale"][:N].view(np.uint32))
        if wl.stub != "identity":
            y = gu.to_host(dev.y, gu.NP_OF[wl.y_dtype])
            assert np.array_equal(y[:N].view(np.uint8), ref["y"][:N].view(np.uint8)), "stub rows"
        out = gu.to_host(dev.out, gu.NP_OF[wl.out_dtype])
        bits = out.view(np.uint32) if wl.out_dtype == "f32" else out
        gu.check_combine(out, wl.out_dtype, ref["out64"], None)
        assert np.array_equal(bits, ref["chain_bits"]), "combine != fp32 ascending fma chain"
        return got, ref
    finally:
        ctx.destroy()


@pytest.mark.parametrize("variant", ["a", "c"])
@pytest.mark.parametrize("policy", [binding.SPREAD, binding.FIRST_LIVE])
def test_tiny_step(oracle, variant, policy):
    wl = synth.tiny(variant)
    got, ref = run_and_compare(oracle, wl, policy)
    assert got["N"] == wl.T * wl.k
    if variant == "c":
        assert got["rank_count"][2] == 0          # the failed rank receives nothing
        # closed form: y = s[e]*x  =>  out = (sum_j w_j s[e_j]) x, mask-independent
        want = ((wl.topk_w.astype(np.float64) * wl.expert_scale[wl.topk_idx]).sum(1)[:, None]
                * wl.x.astype(np.float64))
        np.testing.assert_allclose(ref["out64"], want, rtol=1e-6, atol=1e-6)


def test_tiny_infeasible_coverage(oracle):
    """4+1 slots, rank 2 failed: 15 live slots < 16 experts (pigeonhole)."""
    wl = synth.tiny("b")
    ctx = gu.make_context(wl, strict=True)
    try:
        ctx.update_placement(wl.p2l)
        with pytest.raises(binding.EepError) as ei:
            ctx.set_membership(wl.active)
        assert ei.value.code == binding.ERR_COVERAGE
        # refused update left the tables alone: all ranks still live
        assert ctx.read("active", wl.R).tolist() == [1] * wl.R
    finally:
        ctx.destroy()
    got, ref = run_and_compare(oracle, wl, strict=False)
    assert got["n_uncovered"] == int((wl.topk_idx == 11).sum()) > 0
    assert got["N"] + got["n_uncovered"] + got["n_masked"] == wl.T * wl.k


@pytest.mark.parametrize("T", [0, 32, 96, 4128, 4192])
def test_decode_shape_ragged_sizes(oracle, T):
    """T/R = 0, 1, 3, 129 and 131 tokens per rank: empty input, tiles smaller
    than a wavefront, and ranks split into two ragged tiles (65+64, 66+65)."""
    wl = synth.decode(T=T, H=512)
    got, _ = run_and_compare(oracle, wl)
    assert got["N"] == T * wl.k


@pytest.mark.parametrize("R,T", [(32, 16384), (32, 20576), (3, 600), (1, 77), (64, 64 * 130)])
def test_many_tiles_and_odd_rank_counts(oracle, R, T):
    """More than 64 tiles (several tiles per scan lane), ragged tiles inside a
    source rank, rank counts that are not powers of two, a single rank."""
    rng = np.random.default_rng(R + T)
    H, k, sp, sr = 128, 8, 4, 1
    E = R * sp
    k = min(k, E)
    x = synth.f32_to_bf16_bits(rng.standard_normal((T, H), dtype=np.float32))
    idx, w = synth.router_topk(rng.standard_normal((T, E)).astype(np.float32), k)
    failed = (R // 2,) if R >= 8 else ()
    pref = synth.preferred_placement(R, sp, sr)
    p2l = synth.repaired_placement(pref, failed, R, sp, sr) if failed else pref
    wl = synth.Workload("tiles", T, H, E, k, R, sp, sr, "bf16", "bf16", "bf16", "identity", failed,
                        idx, w, x, p2l, synth.active_mask(R, failed))
    got, _ = run_and_compare(oracle, wl)
    assert got["N"] == T * k


@pytest.mark.parametrize("T", [96, 256])   # single-workgroup layout / tiled layout
def test_masked_repeated_and_out_of_range_indices(oracle, T):
    wl = synth.decode(T=T, H=256)
    rng = np.random.default_rng(5)
    idx = wl.topk_idx.copy()
    idx[rng.random(idx.shape) < 0.05] = -1
    idx[rng.random(idx.shape) < 0.02] = wl.E + 3
    rep = rng.random(idx.shape[0]) < 0.2
    idx[rep, 5] = idx[rep, 1]                       # a repeated expert inside a token
    idx[7, :] = -1                                  # a token with nothing routed
    wl.topk_idx = idx
    got, ref = run_and_compare(oracle, wl)
    assert got["n_masked"] > 0 and got["N"] + got["n_masked"] == wl.T * wl.k
    assert (ref["out64"][7] == 0).all()


@pytest.mark.parametrize("dtypes", [("f32", "f32", "f32", "scale"), ("bf16", "bf16", "f32", "scale"),
                                    ("f32", "f32", "bf16", "identity"),
                                    ("bf16", "bf16", "bf16", "scale")])
@pytest.mark.parametrize("k", [1, 2, 6, 8])
def test_dtype_and_topk_matrix(oracle, dtypes, k):
    xd, yd, od, stub = dtypes
    rng = np.random.default_rng(17 + k)
    T, H, E, R, sp, sr = 192, 384, 24, 6, 4, 2
    x32 = rng.standard_normal((T, H), dtype=np.float32)
    x = x32 if xd == "f32" else synth.f32_to_bf16_bits(x32)
    idx, w = synth.router_topk(rng.standard_normal((T, E)).astype(np.float32), k)
    failed = (4,)
    pref = synth.preferred_placement(R, sp, sr)
    p2l = synth.repaired_placement(pref, failed, R, sp, sr)
    wl = synth.Workload("matrix", T, H, E, k, R, sp, sr, xd, yd, od, stub, failed, idx, w, x, p2l,
                        synth.active_mask(R, failed),
                        expert_scale=(0.25 + rng.random(E)).astype(np.float32))
    got, _ = run_and_compare(oracle, wl)
    assert got["rank_count"][4] == 0


@pytest.mark.parametrize("shape", [
    dict(R=128, sp=2, sr=1, k=4, T=128 * 16, H=256, xd="bf16"),    # P=384 slots, many ranks
    dict(R=8, sp=8, sr=2, k=32, T=8 * 128, H=128, xd="bf16"),      # k=32: tile pairs > fused limit
    dict(R=4, sp=4, sr=1, k=3, T=4 * 50, H=8192, xd="bf16"),       # 16 KiB rows, small batch: split in 2 KiB pieces
    dict(R=4, sp=4, sr=1, k=3, T=4 * 300, H=8192, xd="bf16"),      # 16 KiB rows, large batch: two passes per wavefront
    dict(R=4, sp=4, sr=1, k=3, T=4 * 300, H=6656, xd="bf16"),      # 13 vectors per lane, one pass
    dict(R=4, sp=4, sr=1, k=3, T=4 * 40, H=6656, xd="bf16"),       # 13 is prime: small batch split into single passes of 13
    dict(R=4, sp=4, sr=1, k=5, T=4 * 7, H=5000, xd="f32"),         # 20000-byte fp32 rows, ragged parts
    dict(R=2, sp=1, sr=3, k=2, T=2 * 300, H=8, xd="bf16"),         # 16-byte rows, more replicas than experts
    dict(R=4, sp=2, sr=1, k=4, T=4 * 33, H=4608, xd="bf16"),       # 9 vectors per lane (pass width 9)
    dict(R=4, sp=2, sr=1, k=4, T=4 * 20, H=11264, xd="bf16"),      # 22 per lane: two passes of 11
])
def test_wide_and_odd_shapes(oracle, shape):
    R, sp, sr, k, T, H, xd = (shape[n] for n in ("R", "sp", "sr", "k", "T", "H", "xd"))
    rng = np.random.default_rng(T + H)
    E = R * sp
    x32 = rng.standard_normal((T, H), dtype=np.float32)
    x = x32 if xd == "f32" else synth.f32_to_bf16_bits(x32)
    idx, w = synth.router_topk(rng.standard_normal((T, E)).astype(np.float32), min(k, E))
    k = idx.shape[1]
    p2l = synth.preferred_placement(R, sp, sr)
    wl = synth.Workload("wide", T, H, E, k, R, sp, sr, xd, xd, xd, "scale", (), idx, w, x, p2l,
                        synth.active_mask(R), expert_scale=(0.5 + rng.random(E)).astype(np.float32))
    got, _ = run_and_compare(oracle, wl)
    assert got["N"] == T * k


@pytest.mark.parametrize("R,T,H,k", [
    (32, 8192, 512, 4),      # 1 vector per lane: 4 tokens per wavefront (2048 wavefronts)
    (32, 8192, 2560, 3),     # 5 per lane: 4 tokens per wavefront
    (32, 8192, 6656, 2),     # 13 per lane: 4 x 13 = 52 vectors per lane, the widest multi-token form
    (32, 12288, 3584, 2),    # 7 per lane, T = 3 * 4096: 4 tokens per wavefront (8 would leave 1536 wavefronts)
    (32, 16384, 1536, 2),    # 3 per lane: 8 tokens per wavefront
    (6, 8190, 1024, 4),      # T is even but not a multiple of 4: 2 tokens per wavefront
])
def test_pack_with_several_tokens_per_wavefront(oracle, R, T, H, k):
    """Batches of 8192 tokens and more take the pack form in which a wavefront moves 2, 4 or 8
    tokens; every combination of pass width and token count used here goes through the
    whole step and is compared with the oracle."""
    rng = np.random.default_rng(T + H + k)
    sp, sr = 2, 1
    E = R * sp
    x = synth.f32_to_bf16_bits(rng.standard_normal((T, H), dtype=np.float32))
    idx, w = synth.router_topk(rng.standard_normal((T, E)).astype(np.float32), k)
    pref = synth.preferred_placement(R, sp, sr)
    failed = (R // 3,)
    p2l = synth.repaired_placement(pref, failed, R, sp, sr)
    wl = synth.Workload("multi", T, H, E, k, R, sp, sr, "bf16", "bf16", "bf16", "identity", failed,
                        idx, w, x, p2l, synth.active_mask(R, failed))
    got, _ = run_and_compare(oracle, wl)
    assert got["N"] == T * k and got["rank_count"][failed[0]] == 0


@pytest.mark.parametrize("seed", range(24))
def test_random_configurations(oracle, seed):
    """Seeded random instances: rank/slot/expert counts, top-k, token counts that
    leave ragged tiles, dtypes, replica policies, random placements with empty
    slots and multi-replica experts, random masks (coverage not guaranteed, so
    strict checking is off and uncovered pairs are counted), stray indices."""
    rng = np.random.default_rng(1000 + seed)
    R = int(rng.choice([1, 2, 3, 4, 6, 8, 16, 32]))
    S = int(rng.integers(1, 7))
    S_prim = int(rng.integers(0, S + 1))
    E = int(rng.integers(1, R * S + 4))
    k = int(rng.integers(1, min(E, 12) + 1))
    T = R * int(rng.choice([1, 2, 5, 31, 64, 100, 129, 200]))
    xd, yd, od, stub = [("f32", "f32", "f32", "scale"), ("bf16", "bf16", "bf16", "scale"),
                        ("bf16", "bf16", "f32", "identity"), ("f32", "f32", "bf16", "identity")][seed % 4]
    H = int(rng.choice([8, 40, 256, 520])) * (1 if xd == "f32" else 2)
    x32 = rng.standard_normal((T, H), dtype=np.float32)
    x = x32 if xd == "f32" else synth.f32_to_bf16_bits(x32)
    idx, w = synth.router_topk(rng.standard_normal((T, E)).astype(np.float32), k)
    idx = idx.copy()
    idx[rng.random(idx.shape) < 0.03] = -1
    idx[rng.random(idx.shape) < 0.03] = E + 1
    p2l = rng.integers(-1, E, size=R * S).astype(np.int32)
    active = (rng.random(R) < 0.75).astype(np.int32)
    wl = synth.Workload(f"random-{seed}", T, H, E, k, R, S_prim, S - S_prim, xd, yd, od, stub, (),
                        idx, w, x, p2l, active,
                        expert_scale=(0.5 + rng.random(E)).astype(np.float32))
    got, ref = run_and_compare(oracle, wl, policy=seed % 2, strict=False)
    assert got["N"] + got["n_uncovered"] + got["n_masked"] == T * k
    dead = np.nonzero(active == 0)[0]
    assert got["rank_count"][dead].sum() == 0


def test_large_tables_near_the_lds_limit(oracle):
    """1024 slots and 1024 logical experts: the map kernel's LDS tables take ~41 KB
    and the scan walks 1024 slots per workgroup; a shape whose tables cannot fit
    is refused at create time."""
    rng = np.random.default_rng(77)
    R, sp, sr, k, T, H = 64, 14, 2, 8, 64 * 64, 64
    E = R * sp + 128                      # more experts than primary slots: some live only in
    S = sp + sr                           # redundant slots, some are uncovered
    p2l = np.full(R * S, -1, np.int32)
    p2l[:] = rng.permutation(np.concatenate([np.arange(E), rng.integers(0, E, R * S - E)]))[:R * S] \
        if R * S >= E else rng.integers(0, E, R * S)
    active = synth.active_mask(R, (5, 40))
    x = synth.f32_to_bf16_bits(rng.standard_normal((T, H), dtype=np.float32))
    idx, w = synth.router_topk(rng.standard_normal((T, E)).astype(np.float32), k)
    wl = synth.Workload("large-tables", T, H, E, k, R, sp, sr, "bf16", "bf16", "bf16", "identity",
                        (5, 40), idx, w, x, p2l, active)
    got, _ = run_and_compare(oracle, wl, strict=False)
    assert got["rank_count"][[5, 40]].sum() == 0
    assert got["N"] + got["n_uncovered"] == T * k
    with pytest.raises(binding.EepError) as ei:
        binding.Context(num_ranks=512, slots_per_rank=32, primary_slots=16, num_logical=4096,
                        max_tokens=512, topk=8, hidden=64)
    assert ei.value.code == binding.ERR_INVALID_ARG


def test_prefill_fp8_reduced(oracle):
    wl = synth.prefill_fp8(T=1024, H=1024)
    got, _ = run_and_compare(oracle, wl)
    assert got["rank_count"][7] == 0 and got["rank_count"][20] == 0


def test_prefill_fp8_full_size_every_token(oracle):
    """Prefill shape at full size (T=16384, fp8 payload + scales, two failed
    ranks).  Layout compared in full.  Then every token goes through the oracle
    in chunks of 1024: the oracle packs the chunk's tokens into a compact receive
    buffer (row c of it is the chunk's c-th routed pair), dequantises and
    combines; the GPU's rows at row_of[chunk] must equal the compact rows byte
    for byte (payload, scales, dequantised rows) and the combined rows must be
    bit-equal to the fp32 chain.  Together the chunks cover all 131072 rows."""
    wl = synth.prefill_fp8()
    T, k, H = wl.T, wl.k, wl.H
    ctx = gu.make_context(wl)
    try:
        gu.apply_tables(ctx, wl.p2l, wl.active)
        dev = gu.DeviceStep(ctx, wl)
        dev.recv.fill_(0x55)                    # nothing may survive from the buffers' fill
        dev.y.fill_(0x5555)
        dev.step()
        dev.sync()
        lay = oracle.step_layout(wl.topk_idx, wl.p2l, wl.active, wl.E, wl.R, wl.S, wl.S_prim, 0)
        got = ctx.read_layout(T)
        gu.assert_layout_equal(got, lay, T, k)
        N = got["N"]
        assert N == T * k and got["rank_count"][7] == 0 and got["rank_count"][20] == 0
        seen = np.zeros(N, bool)
        chunk = 1024
        for t0 in range(0, T, chunk):
            toks = np.arange(t0, t0 + chunk)
            rows = lay["row_of"][toks]                                # [chunk, k], all routed
            assert (rows >= 0).all()
            seen[rows.ravel()] = True
            compact = np.arange(rows.size, dtype=np.int32).reshape(rows.shape)
            recv_c = oracle.pack(wl.x[toks], compact)
            scale_c = oracle.pack(wl.x_scale[toks], compact)
            y_c = oracle.stub_dequant(recv_c, scale_c, rows.size, 128)
            rows_dev = torch.from_numpy(rows.ravel()).cuda().long()
            assert np.array_equal(dev.recv.index_select(0, rows_dev).cpu().numpy(), recv_c), \
                f"packed fp8 rows, tokens from {t0}"
            assert np.array_equal(dev.recv_scale.index_select(0, rows_dev).cpu().numpy()
                                  .view(np.uint32), scale_c.view(np.uint32)), \
                f"scale rows, tokens from {t0}"
            y_got = gu.to_host(dev.y.index_select(0, rows_dev), np.uint16)
            assert np.array_equal(y_got, y_c), f"dequantised rows, tokens from {t0}"
            out64 = oracle.combine(y_c, oracle.BF16, wl.topk_w[toks], compact)
            chain = oracle.f32_to_bf16(oracle.combine_chain32(y_c, oracle.BF16, wl.topk_w[toks],
                                                              compact))
            out_got = gu.to_host(dev.out[t0:t0 + chunk], np.uint16)
            gu.check_combine(out_got, "bf16", out64)
            assert np.array_equal(out_got, chain), f"combined rows, tokens from {t0}"
            print(f"prefill parity: tokens {t0}..{t0 + chunk - 1} ok", flush=True)
        assert seen.all()                       # the chunks' rows are all N rows of the buffer

        # the same step in the launch configuration the benchmark times: eight steps captured
        # into one hipGraph and replayed; every buffer must come out as in the eager step that
        # was just compared with the oracle
        want = [t.clone() for t in (dev.recv, dev.recv_scale, dev.y, dev.out)]
        lay_eager = got
        stream = torch.cuda.Stream()
        dev.stream = stream
        ctx.graph_begin(stream)
        for _ in range(8):
            dev.step()
        graph = ctx.graph_end(stream)
        for replay in range(2):
            for t in (dev.recv, dev.recv_scale, dev.y, dev.out):
                t.fill_(0)
            torch.cuda.synchronize()
            graph.launch(stream)
            stream.synchronize()
            gu.assert_layout_equal(ctx.read_layout(T, stream), lay_eager, T, k)
            for name, a, b in zip(("payload", "scales", "dequantised", "combined"),
                                  (dev.recv, dev.recv_scale, dev.y, dev.out), want):
                assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), \
                    f"{name} rows differ in graph replay {replay}"
        assert graph.counters() == dict(instantiations=1, exec_updates=0, launches=2)
        graph.destroy()
    finally:
        ctx.destroy()


def test_buffers_beyond_4_gib_sampled(oracle):
    """32x the decode batch (T=131072, 1024 tiles, one failed rank, Zipf-skewed load): the
    receive buffer is 15 GB, so row addresses need 64-bit arithmetic and the tile prefix
    takes several rounds.  Token rows are built on the GPU (row t = row t mod 4096 of a
    random block, with t stamped into its first two elements) so that the host never holds
    them all.  Layout compared in full with the oracle; moved rows in full against a torch
    gather; pack and combine against the oracle on 512 sampled tokens, the ones with the
    highest and lowest rows included."""
    T, H, B = 131072, 7168, 4096
    small = synth.decode_failed_zipf(T=T, H=16)                    # router, placement, mask
    k, R = small.k, small.R
    block = synth.decode(T=B, H=H, seed_offset=41).x               # [B, H] bf16 bits

    def host_rows(toks):
        rows = block[toks % B].copy()
        rows[:, 0] = toks & 0x3FFF                                 # small finite bf16 patterns
        rows[:, 1] = toks >> 14
        return rows

    ctx = binding.Context(num_ranks=R, slots_per_rank=small.S, primary_slots=small.S_prim,
                          num_logical=small.E, max_tokens=T, topk=k, hidden=H)
    try:
        gu.apply_tables(ctx, small.p2l, small.active)
        x = gu.to_dev(block).repeat(T // B, 1)
        t_dev = torch.arange(T, device="cuda")
        x[:, 0] = (t_dev & 0x3FFF).to(torch.int16)
        x[:, 1] = (t_dev >> 14).to(torch.int16)
        idx, w = gu.to_dev(small.topk_idx), gu.to_dev(small.topk_w)
        recv = torch.empty((T * k, H), dtype=torch.int16, device="cuda")
        out = torch.empty((T, H), dtype=torch.int16, device="cuda")
        ctx.dispatch_layout(idx, T)
        ctx.dispatch(x, recv, T)
        ctx.combine(recv, w, out, T)
        torch.cuda.synchronize()
        lay = oracle.step_layout(small.topk_idx, small.p2l, small.active, small.E, R, small.S,
                                 small.S_prim, 0)
        got = ctx.read_layout(T)
        gu.assert_layout_equal(got, lay, T, k)
        N = got["N"]
        assert N == T * k and N * H * 2 > 3 * 2 ** 32 and got["rank_count"][13] == 0
        src_tok = torch.from_numpy(lay["src_of"][:N] // k).cuda().long()
        assert torch.equal(recv[:N], x.index_select(0, src_tok)), "packed rows"
        del src_tok
        rng = np.random.default_rng(12)
        by_row = np.argsort(lay["row_of"].max(axis=1))
        toks = np.unique(np.concatenate([rng.choice(T, 448, replace=False), by_row[-32:],
                                         by_row[:32]]))
        rows = lay["row_of"][toks]
        assert rows.max() == N - 1
        compact = np.arange(rows.size, dtype=np.int32).reshape(rows.shape)
        y_c = oracle.pack(host_rows(toks), compact)
        rows_dev = torch.from_numpy(rows.ravel()).cuda().long()
        assert np.array_equal(gu.to_host(recv.index_select(0, rows_dev), np.uint16), y_c)
        w_c = small.topk_w[toks]
        out64 = oracle.combine(y_c, oracle.BF16, w_c, compact)
        chain = oracle.f32_to_bf16(oracle.combine_chain32(y_c, oracle.BF16, w_c, compact))
        out_got = gu.to_host(out.index_select(0, torch.from_numpy(toks).cuda().long()), np.uint16)
        gu.check_combine(out_got, "bf16", out64)
        assert np.array_equal(out_got, chain)
    finally:
        ctx.destroy()


@pytest.mark.parametrize("T,H,group", [(256, 1024, 128), (4096, 7168, 128), (64, 1024, 64),
                                       (96, 256, 16)])
def test_dispatch_with_fused_quantisation(oracle, T, H, group):
    """bf16 tokens in, e4m3 codes + fp32 scales out (quantise-on-dispatch
    variant): codes and scales of every routed row bit-equal to the oracle's
    quantiser followed by its pack; then dequantising stand-in and combine."""
    wl = synth.decode(T=T, H=H)
    rng = np.random.default_rng(T)
    xf = synth.bf16_bits_to_f32(wl.x) * np.exp(rng.standard_normal((T, 1))).astype(np.float32)
    xf[3, :group] = 0.0                                  # an all-zero group
    xf[5, 7] = 3.0e4                                     # an outlier that sets its group's scale
    xb = synth.f32_to_bf16_bits(xf)
    failed = (9,)
    p2l = synth.repaired_placement(wl.p2l, failed, wl.R, wl.S_prim, wl.S_red)
    active = synth.active_mask(wl.R, failed)
    ctx = binding.Context(num_ranks=wl.R, slots_per_rank=wl.S, primary_slots=wl.S_prim,
                          num_logical=wl.E, max_tokens=T, topk=wl.k, hidden=H, x_dtype="fp8",
                          y_dtype="bf16", out_dtype="bf16", scale_group=group)
    try:
        gu.apply_tables(ctx, p2l, active)
        idx, w, x = gu.to_dev(wl.topk_idx), gu.to_dev(wl.topk_w), gu.to_dev(xb)
        recv = torch.zeros((T * wl.k, H), dtype=torch.uint8, device="cuda")
        recv_scale = torch.zeros((T * wl.k, H // group), dtype=torch.float32, device="cuda")
        y = torch.zeros((T * wl.k, H), dtype=torch.int16, device="cuda")
        out = torch.zeros((T, H), dtype=torch.int16, device="cuda")
        ctx.dispatch_layout(idx, T)
        ctx.dispatch_quant(x, recv, recv_scale, T)
        ctx.expert_stub("dequant", recv, y, T, recv_scale=recv_scale)
        ctx.combine(y, w, out, T)
        torch.cuda.synchronize()
        lay = oracle.step_layout(wl.topk_idx, p2l, active, wl.E, wl.R, wl.S, wl.S_prim, 0)
        got = ctx.read_layout(T)
        gu.assert_layout_equal(got, lay, T, wl.k)
        N = lay["N"]
        q, sc = oracle.quantize_e4m3(xb, group)
        want_q, want_sc = oracle.pack(q, lay["row_of"]), oracle.pack(sc, lay["row_of"])
        assert np.array_equal(recv.cpu().numpy()[:N], want_q[:N]), "fp8 codes"
        assert np.array_equal(recv_scale.cpu().numpy()[:N].view(np.uint32),
                              want_sc[:N].view(np.uint32)), "scales"
        want_y = oracle.stub_dequant(want_q, want_sc, N, group)
        assert np.array_equal(gu.to_host(y, np.uint16)[:N], want_y[:N])
        chain = oracle.f32_to_bf16(oracle.combine_chain32(want_y, oracle.BF16, wl.topk_w,
                                                          lay["row_of"]))
        out_h = gu.to_host(out, np.uint16)
        assert np.array_equal(out_h, chain)
        gu.check_combine(out_h, "bf16", oracle.combine(want_y, oracle.BF16, wl.topk_w,
                                                       lay["row_of"]))
        # end to end the quantisation error stays at the fp8 level: out ~= x
        ref = synth.bf16_bits_to_f32(xb).astype(np.float64)
        err = np.abs(gu.bf16_to_f64(out_h) - ref)
        amax = np.abs(ref.reshape(T, H // group, group)).max(2, keepdims=True)
        # half an e4m3 step at the top binade (16/448 of the group maximum) plus two bf16 roundings
        ok = err.reshape(T, H // group, group) <= amax / 448 * 20 + 1e-30
        assert ok.all(), f"{(~ok).sum()} elements off by more than the fp8 step"
    finally:
        ctx.destroy()


def test_decode_full_size(oracle):
    """DeepSeek-V3 decode shape at full size, every output compared."""
    wl = synth.decode()
    got, ref = run_and_compare(oracle, wl)
    assert got["N"] == 4096 * 8
    # identity expert and softmax weights: out ~= x
    x = gu.bf16_to_f64(wl.x)
    assert np.abs(ref["out64"] - x).max() <= 1e-5 * np.abs(x).max()


def test_decode_failed_rank_zipf_full_size(oracle):
    wl = synth.decode_failed_zipf()
    got, _ = run_and_compare(oracle, wl)
    assert got["rank_count"][13] == 0 and got["N"] == 4096 * 8
    S = wl.S
    hot = got["count"].argsort()[::-1][:8]
    assert all(p % S == S - 1 for p in hot)        # hottest slots are redundant replicas


def test_failure_then_planned_repair_then_rejoin(oracle):
    """The paper's sequence (Fig. 5, Fig. 6) on the decode shape: healthy step;
    ranks 3 and 17 fail; the planner repairs the placement from the observed
    per-expert load; tables are patched (placement, then mask); degraded step;
    ranks rejoin (mask, then preferred placement); healthy step again.  Every
    step must match the oracle under the tables in force."""
    wl = synth.decode(T=1024, H=512)
    failed = (3, 17)
    ctx = gu.make_context(wl)
    try:
        gu.apply_tables(ctx, wl.p2l, wl.active)
        dev = gu.DeviceStep(ctx, wl)

        def step_and_check(p2l, active):
            dev.step()
            dev.sync()
            ref = oracle_step(oracle, wl, 0, p2l, active)
            got = ctx.read_layout(wl.T)
            gu.assert_layout_equal(got, ref["lay"], wl.T, wl.k)
            out = gu.to_host(dev.out, np.uint16)
            assert np.array_equal(out, ref["chain_bits"])
            return got

        got = step_and_check(wl.p2l, wl.active)
        load = np.bincount(wl.topk_idx.ravel(), minlength=wl.E).astype(np.float32)
        dead = synth.active_mask(wl.R, failed)
        plan = binding.plan_repair(wl.p2l, dead, wl.R, wl.S, wl.S_prim, wl.E, load)
        assert plan["unplaced"] == 0 and plan["dram"] + plan["peer"] > 0
        ctx.update_placement(plan["p2l"])
        ctx.set_membership(dead)
        got = step_and_check(plan["p2l"], dead)
        assert got["rank_count"][list(failed)].sum() == 0 and got["N"] == wl.T * wl.k
        ctx.set_membership(wl.active)
        ctx.update_placement(wl.p2l)
        step_and_check(wl.p2l, wl.active)
    finally:
        ctx.destroy()


@pytest.mark.parametrize("dtypes", [("f32", "f32"), ("bf16", "bf16"), ("bf16", "f32")])
def test_special_values_follow_ieee(oracle, dtypes):
    """Denormals, infinities, signed zeros and huge values in rows and weights:
    the fp32 chain must keep denormals (no flush) and round like the oracle, so
    outputs stay bit-equal; NaNs must appear in exactly the same places."""
    yd, od = dtypes
    rng = np.random.default_rng(3)
    wl = synth.decode(T=64, H=256)
    specials = np.array([0.0, -0.0, 1e-40, -1e-40, 1.2e-38, 3e38, -3e38, np.inf, -np.inf, 1.0,
                         2.0 ** -126, 2.0 ** -133, 65504.0, -1.5], np.float32)
    x32 = rng.choice(specials, size=(wl.T, wl.H)).astype(np.float32)
    mix = rng.random(x32.shape) < 0.4
    x32[mix] = rng.standard_normal(int(mix.sum())).astype(np.float32)
    w = wl.topk_w.copy()
    w[::3, 0] = 0.0
    w[1::5, 1] = 1e-39          # denormal weight
    w[2::7, 2] = -2.5
    w[3::11, 3] = 3e38          # overflow to infinity in the chain
    nan_rows = np.zeros_like(x32, bool)
    nan_rows[5, 10] = nan_rows[17, 0] = True
    x32[nan_rows] = np.nan
    wl.topk_w = w
    wl.x = x32 if yd == "f32" else synth.f32_to_bf16_bits(x32)
    wl.x_dtype = wl.y_dtype = yd
    wl.out_dtype = od
    ctx = gu.make_context(wl)
    try:
        gu.apply_tables(ctx, wl.p2l, wl.active)
        dev = gu.DeviceStep(ctx, wl)
        dev.step()
        dev.sync()
        lay = oracle.step_layout(wl.topk_idx, wl.p2l, wl.active, wl.E, wl.R, wl.S, wl.S_prim, 0)
        recv = oracle.pack(wl.x, lay["row_of"])
        assert np.array_equal(gu.to_host(dev.recv, gu.NP_OF[yd]).view(np.uint8), recv.view(np.uint8))
        chain = oracle.combine_chain32(recv, ODT[yd], wl.topk_w, lay["row_of"])
        out = gu.to_host(dev.out, gu.NP_OF[od])
        got32 = out if od == "f32" else synth.bf16_bits_to_f32(out)
        want_nan = np.isnan(chain)
        assert want_nan.any() and np.array_equal(np.isnan(got32), want_nan)
        want_bits = chain.view(np.uint32) if od == "f32" else oracle.f32_to_bf16(chain)
        got_bits = out.view(np.uint32) if od == "f32" else out
        assert np.array_equal(got_bits[~want_nan], want_bits[~want_nan])
        assert np.isinf(chain).any() and (np.abs(chain[np.isfinite(chain)]) < 1e-37).any()
    finally:
        ctx.destroy()


def test_device_side_layout_check_sees_planted_errors():
    """eep_debug_check_layout on a sound layout and on layouts whose arrays were overwritten
    from the host (the check itself never indexes with an unchecked value)."""
    import ctypes
    hip = ctypes.CDLL("libamdhip64.so")
    wl = synth.decode(T=512, H=256)
    ctx = gu.make_context(wl)
    try:
        gu.apply_tables(ctx, wl.p2l, wl.active)
        idx = gu.to_dev(wl.topk_idx)
        ctx.dispatch_layout(idx, wl.T)
        assert ctx.check_layout(wl.T).tolist() == [0, 0, 0, 0]
        lay = ctx.read_layout(wl.T)
        ptr = ctx.view_pointers()

        def poke(field, host):
            host = np.ascontiguousarray(host, np.int32)
            assert hip.hipMemcpy(ctypes.c_void_p(ptr[field]), host.ctypes.data_as(ctypes.c_void_p),
                                 ctypes.c_size_t(host.nbytes), 1) == 0

        rows = lay["row_of"].ravel().copy()
        bad = rows.copy()
        bad[5] = wl.T * wl.k + 17                  # beyond the buffer
        bad[9] = -5                                # negative, not the marker
        a, b = 100, 101                            # two pairs swap rows: each row is in range
        bad[a], bad[b] = rows[b], rows[a]          # of the other's slot at best, and src_of
        poke("row_of", bad)                        # no longer points back
        got = ctx.check_layout(wl.T)
        assert got[0] + got[1] >= 4 and got[3] == 0
        poke("row_of", rows)
        assert ctx.check_layout(wl.T).tolist() == [0, 0, 0, 0]
        src = lay["src_of"].copy()
        src[3] = wl.T * wl.k                       # out of range
        src[7] = src[8]                            # a pair that holds another row
        poke("src_of", src)
        got = ctx.check_layout(wl.T)
        assert got[2] == 2 and got[1] == 2 and got[0] == 0
        poke("src_of", lay["src_of"])
        withdrawn = rows.copy()
        withdrawn[40:48] = -1                      # what a dropped rank leaves behind
        poke("row_of", withdrawn)
        assert ctx.check_layout(wl.T).tolist() == [0, 0, 0, 8]
        with pytest.raises(binding.EepError) as ei:
            ctx.check_layout(wl.T - 32)
        assert ei.value.code == binding.ERR_STATE
    finally:
        ctx.destroy()


def test_call_order_and_argument_errors():
    wl = synth.decode(T=64, H=256)
    ctx = gu.make_context(wl)
    try:
        gu.apply_tables(ctx, wl.p2l, wl.active)
        dev = gu.DeviceStep(ctx, wl)
        with pytest.raises(binding.EepError) as ei:
            dev.dispatch()                          # no layout yet
        assert ei.value.code == binding.ERR_STATE
        with pytest.raises(binding.EepError) as ei:
            ctx.dispatch_layout(dev.idx, 65)        # not a multiple of R
        assert ei.value.code == binding.ERR_INVALID_ARG
        with pytest.raises(binding.EepError) as ei:
            ctx.dispatch_layout(dev.idx, 128)       # > T_max
        assert ei.value.code == binding.ERR_INVALID_ARG
        dev.layout()
        with pytest.raises(binding.EepError) as ei:
            ctx.dispatch(dev.x.data_ptr() + 2, dev.recv, wl.T)
        assert ei.value.code == binding.ERR_ALIGN
        bad = wl.p2l.copy()
        bad[0] = wl.E
        with pytest.raises(binding.EepError) as ei:
            ctx.update_placement(bad)
        assert ei.value.code == binding.ERR_INVALID_ARG
        dev.step()
        dev.sync()
    finally:
        ctx.destroy()
    with pytest.raises(binding.EepError) as ei:     # 2-byte rows cannot be moved 16 B at a time
        binding.Context(num_ranks=2, slots_per_rank=2, primary_slots=1, num_logical=2,
                        max_tokens=4, topk=1, hidden=3)
    assert ei.value.code == binding.ERR_ALIGN


def test_context_in_caller_owned_workspace(oracle):
    """eep_create_with_workspace: the tables and layout arrays live inside a torch tensor."""
    wl = synth.tiny("a")
    shape = dict(num_ranks=wl.R, slots_per_rank=wl.S, primary_slots=wl.S_prim, num_logical=wl.E,
                 max_tokens=wl.T, topk=wl.k, hidden=wl.H, x_dtype=wl.x_dtype, y_dtype=wl.y_dtype,
                 out_dtype=wl.out_dtype)
    need = binding.workspace_bytes(**shape)
    torch.cuda.empty_cache()
    ws = torch.full((need + 4096,), 0x7F, dtype=torch.uint8, device="cuda")
    guard = ws[need:].clone()
    for bad in (ws[:need - 256], ws[1:need + 1],
                torch.empty(need, dtype=torch.uint8, pin_memory=True)):
        with pytest.raises(binding.EepError) as ei:
            binding.Context(workspace=bad, **shape)
        assert ei.value.code == binding.ERR_INVALID_ARG
    ctx = binding.Context(workspace=ws[:need], **shape)
    try:
        lo, hi = ws.data_ptr(), ws.data_ptr() + need
        assert all(lo <= p < hi for p in ctx.view_pointers().values())
        gu.apply_tables(ctx, wl.p2l, wl.active)
        dev = gu.DeviceStep(ctx, wl)
        dev.step()
        dev.sync()
        ref = oracle_step(oracle, wl)
        gu.assert_layout_equal(ctx.read_layout(wl.T), ref["lay"], wl.T, wl.k)
        assert np.array_equal(gu.to_host(dev.out, gu.NP_OF[wl.out_dtype]).view(np.uint32),
                              ref["chain_bits"].view(np.uint32))
    finally:
        ctx.destroy()
    assert torch.equal(ws[need:], guard)                 # nothing written past the stated size
    ws.fill_(1)                                          # still the caller's memory after destroy
    torch.cuda.synchronize()


def test_one_context_many_batch_sizes_in_a_row(oracle):
    """The same context and buffers serve batches of different sizes back to back, crossing
    between the few-tile and the many-tile layout paths, with a membership change in the
    middle: nothing left over from a larger earlier batch may leak into a later one."""
    R, sp, sr, k, H = 32, 8, 1, 8, 256
    E, T_max = R * sp, 12288                                      # 96 tiles at full size
    rng = np.random.default_rng(77)
    pref = synth.preferred_placement(R, sp, sr)
    failed = (11,)
    repaired = synth.repaired_placement(pref, failed, R, sp, sr)
    ctx = binding.Context(num_ranks=R, slots_per_rank=sp + sr, primary_slots=sp, num_logical=E,
                          max_tokens=T_max, topk=k, hidden=H)
    try:
        ctx.update_placement(pref)
        recv = torch.zeros((T_max * k, H), dtype=torch.int16, device="cuda")
        out = torch.zeros((T_max, H), dtype=torch.int16, device="cuda")
        p2l, active = pref, synth.active_mask(R)
        for step, T in enumerate([12288, 4096, 96, 0, 8192, 32, 12288, 4128]):
            if step == 4:
                ctx.update_placement(repaired)
                ctx.set_membership(synth.active_mask(R, failed))
                p2l, active = repaired, synth.active_mask(R, failed)
            x = synth.f32_to_bf16_bits(rng.standard_normal((T, H), dtype=np.float32))
            idx, w = synth.router_topk(rng.standard_normal((T, E)).astype(np.float32), k)
            if T:
                x_d, idx_d, w_d = gu.to_dev(x), gu.to_dev(idx), gu.to_dev(w)
            else:
                x_d = idx_d = w_d = None
            ctx.dispatch_layout(idx_d, T)
            ctx.dispatch(x_d, recv, T)
            ctx.combine(recv, w_d, out, T)
            torch.cuda.synchronize()
            lay = oracle.step_layout(idx, p2l, active, E, R, sp + sr, sp, oracle.SPREAD)
            gu.assert_layout_equal(ctx.read_layout(T), lay, T, k)
            if T == 0:
                continue
            rows = oracle.pack(x, lay["row_of"])
            N = lay["N"]
            assert np.array_equal(gu.to_host(recv[:N], np.uint16), rows[:N]), (step, T)
            chain = oracle.f32_to_bf16(oracle.combine_chain32(rows, oracle.BF16, w, lay["row_of"]))
            assert np.array_equal(gu.to_host(out[:T], np.uint16), chain), (step, T)
    finally:
        ctx.destroy()


@pytest.mark.parametrize("policy", [binding.SPREAD, binding.FIRST_LIVE])
@pytest.mark.parametrize("R,T,k,failed", [(32, 128, 8, (13,)), (32, 160, 8, (13,)), (32, 192, 8, (31,)),
                                          (32, 224, 8, (0,)), (4, 192, 2, (1,)), (4, 196, 2, ()),
                                          (4, 128, 2, ()),
                                          (8, 40, 20, (2, 5)), (2, 128, 8, ()), (64, 128, 8, (0, 63)),
                                          (16, 32, 32, (7,)), (1, 128, 8, ())])
def test_small_batches_around_the_single_workgroup_limit(oracle, policy, R, T, k, failed):
    """Batches of at most 192 tokens and 1536 pairs are laid out by one workgroup in one
    launch; just above either limit the tiled path runs.  Both must give the oracle's
    layout: rank boundaries inside a bitmap word, k up to 32, failed first and last
    ranks, one rank only."""
    rng = np.random.default_rng(1000 + R * 7 + T + k)
    sr, H = 2, 128
    sp = -(-max(R * 4, k) // R)
    E = R * sp
    x = synth.f32_to_bf16_bits(rng.standard_normal((T, H), dtype=np.float32))
    idx, w = synth.router_topk(rng.standard_normal((T, E)).astype(np.float32), k)
    pref = synth.preferred_placement(R, sp, sr)
    p2l = synth.repaired_placement(pref, failed, R, sp, sr) if failed else pref
    wl = synth.Workload("small", T, H, E, k, R, sp, sr, "bf16", "bf16", "bf16", "identity", failed,
                        idx, w, x, p2l, synth.active_mask(R, failed))
    got, _ = run_and_compare(oracle, wl, policy=policy, strict=False)
    for r in failed:
        assert got["rank_count"][r] == 0


def test_smoke_in_a_fresh_process_that_loads_the_library_before_torch():
    """build() ends with binding.load(); a process that goes on to smoke() has then loaded the
    library before it imports torch.  The binding brings torch (and its HIP runtime) in first
    by itself, so the order in the caller's code does not matter."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = ("import sys; sys.path.insert(0, %r)\n"
            "from paper_2605_10670_amd import binding\n"
            "assert 'torch' not in sys.modules\n"
            "binding.load()\n"
            "import __graft_entry__ as g\n"
            "g.smoke()\n" % root)
    done = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300,
                          cwd=root)
    assert done.returncode == 0, done.stdout[-2000:] + done.stderr[-2000:]
    assert "smoke ok" in done.stdout
