"""Pins for the oracle's counting/offset/position steps (O3-O5), pack (O6),
stubs (O7) and combine (O8).

Expected values come from library routines that define the same thing
(numpy.bincount, cumsum, stable argsort, fancy indexing, float64 einsum,
torch dtype casts) and from closed forms, never from the oracle itself.
"""
import numpy as np
import pytest
import torch

from paper_2605_10670_amd import synth


def _random_slots(rng, T, k, P, frac_invalid=0.1):
    """slot_of with distinct slots inside a token and some -1 entries."""
    slot_of = np.stack([rng.permutation(P)[:k] for _ in range(T)]).astype(np.int32)
    slot_of[rng.random((T, k)) < frac_invalid] = -1
    return slot_of


@pytest.mark.parametrize("T,k,R,S", [(64, 4, 4, 3), (96, 8, 8, 5), (8, 1, 8, 1), (0, 2, 2, 2)])
def test_layout_is_stable_counting_sort(oracle, T, k, R, S):
    rng = np.random.default_rng(T + k)
    P = R * S
    slot_of = _random_slots(rng, T, k, P) if T else np.zeros((0, k), np.int32)
    lay = oracle.layout(slot_of, R, S)
    flat = slot_of.ravel()
    valid = np.nonzero(flat >= 0)[0]
    N = valid.size
    assert np.array_equal(lay["count"], np.bincount(flat[valid], minlength=P))
    assert np.array_equal(lay["offset"], np.concatenate([[0], np.cumsum(lay["count"])]))
    assert np.array_equal(lay["rank_count"], lay["count"].reshape(R, S).sum(1))
    assert np.array_equal(lay["rank_offset"][:-1], lay["offset"][:-1:S])
    assert lay["rank_offset"][-1] == N
    # stable sort of the valid pairs by slot == the receive-buffer order
    order = valid[np.argsort(flat[valid], kind="stable")]
    assert np.array_equal(lay["src_of"][:N], order)
    assert (lay["src_of"][N:] == -1).all()
    row_flat = lay["row_of"].ravel()
    assert (row_flat[flat < 0] == -1).all()
    assert np.array_equal(row_flat[order], np.arange(N))          # src_of o row_of = id
    if T:
        per = T // R
        src_rank = (np.arange(T * k) // k) // per
        want = np.zeros((R, P), np.int64)
        np.add.at(want, (src_rank[valid], flat[valid]), 1)
        assert np.array_equal(lay["cnt_src"], want)
        # inside a slot the source tokens strictly increase
        for p in range(P):
            rows = lay["src_of"][lay["offset"][p]:lay["offset"][p + 1]] // k
            assert (np.diff(rows) > 0).all()


def test_layout_requires_T_multiple_of_R(oracle):
    with pytest.raises(ValueError):
        oracle.layout(np.zeros((5, 2), np.int32), 2, 2)


@pytest.mark.parametrize("dtype", [np.float32, np.uint16, np.uint8])
def test_pack_is_a_row_gather(oracle, dtype):
    rng = np.random.default_rng(3)
    T, k, R, S, H = 48, 4, 4, 4, 40
    slot_of = _random_slots(rng, T, k, R * S)
    lay = oracle.layout(slot_of, R, S)
    x = rng.integers(0, 250, size=(T, H)).astype(dtype)
    recv = oracle.pack(x, lay["row_of"], fill=7)
    N = int(lay["offset"][-1])
    assert np.array_equal(recv[:N], x[lay["src_of"][:N] // k])
    assert (recv[N:] == 7).all()


def test_bf16_and_e4m3_formats_match_torch(oracle):
    all16 = np.arange(65536, dtype=np.uint16)
    want = torch.from_numpy(all16.view(np.int16)).view(torch.bfloat16).float().numpy()
    got = oracle.bf16_to_f32(all16)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.standard_normal(200000).astype(np.float32) * 10,
                        # exact ties and neighbours, denormals, big values
                        (np.arange(0x3F800000, 0x3F800000 + 0x40000, 0x2000, dtype=np.uint32)
                         .view(np.float32)),
                        np.array([0.0, -0.0, 1e-40, -1e-40, 3.38e38, -3.38e38, np.inf, -np.inf],
                                 np.float32)])
    want16 = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oracle.f32_to_bf16(x), want16)
    assert np.array_equal(synth.f32_to_bf16_bits(x), want16)
    # NaN stays NaN with its sign (IEEE 754 conversion; which payload bits survive is not fixed,
    # only that the result is a quiet NaN), whatever the payload: also one that lives only in
    # the 16 bits that the narrower format drops
    nan_bits = np.array([0x7FC00000, 0xFFC00000, 0x7F800001, 0xFF800001, 0x7F80FFFF, 0x7FFFFFFF,
                         0xFFFFFFFF, 0x7FA00000], np.uint32)
    got_nan = oracle.f32_to_bf16(nan_bits.view(np.float32)).astype(np.uint32)
    assert ((got_nan & 0x7F80) == 0x7F80).all() and ((got_nan & 0x007F) != 0).all()
    assert ((got_nan & 0x0040) != 0).all()                                   # quiet
    assert np.array_equal(got_nan >> 15, nan_bits >> 31)                     # sign kept
    codes = np.arange(256, dtype=np.uint8)
    want8 = torch.from_numpy(codes).view(torch.float8_e4m3fn).float().numpy()
    got8 = oracle.e4m3_to_f32(codes)
    assert np.array_equal(np.isnan(got8), np.isnan(want8))
    assert np.array_equal(got8[~np.isnan(got8)], want8[~np.isnan(want8)])
    assert got8[0x7E] == 448.0 and np.isnan(got8[0x7F]) and got8[0x01] == 2.0 ** -9


def test_combine_matches_float64_einsum(oracle):
    rng = np.random.default_rng(11)
    T, k, R, S, H = 32, 4, 4, 3, 24
    slot_of = _random_slots(rng, T, k, R * S, frac_invalid=0.2)
    lay = oracle.layout(slot_of, R, S)
    y = rng.standard_normal((T * k, H)).astype(np.float32)
    w = rng.random((T, k)).astype(np.float32)
    rows = lay["row_of"]
    gathered = np.where((rows >= 0)[:, :, None], y[np.maximum(rows, 0)].astype(np.float64), 0.0)
    want = np.einsum("tk,tkh->th", w.astype(np.float64), gathered)
    got = oracle.combine(y, oracle.F32, w, rows)
    np.testing.assert_allclose(got, want, rtol=1e-14, atol=1e-14)
    got32 = oracle.combine_chain32(y, oracle.F32, w, rows)
    # fp32 chain of <= k fused multiply-adds: error <= k * 2^-24 * sum|w*y|
    bound = k * 2.0 ** -24 * np.einsum("tk,tkh->th", w.astype(np.float64), np.abs(gathered))
    assert (np.abs(got32.astype(np.float64) - want) <= bound + 1e-30).all()
    # bf16 rows go through the same sum after widening
    yb = synth.f32_to_bf16_bits(y)
    got_b = oracle.combine(yb, oracle.BF16, w, rows)
    gathered_b = np.where((rows >= 0)[:, :, None],
                          synth.bf16_bits_to_f32(yb)[np.maximum(rows, 0)].astype(np.float64), 0.0)
    np.testing.assert_allclose(got_b, np.einsum("tk,tkh->th", w.astype(np.float64), gathered_b),
                               rtol=1e-14, atol=1e-14)


def test_chain32_order_and_fma_are_what_they_claim(oracle):
    """One token, values chosen so that (a) a separate multiply-then-add and
    (b) the reverse order give different fp32 results than the fused ascending
    chain; the expected number is computed exactly with Python fractions."""
    from fractions import Fraction
    w = np.array([[1.0, 1.0 + 2.0 ** -12, 2.0 ** -30]], np.float32)
    y = np.array([[-1.0], [1.0 + 2.0 ** -12], [1.0]], np.float32)
    rows = np.array([[0, 1, 2]], np.int32)

    def rnd(fr):  # exact rational -> nearest float32 (ties to even) via float64 is safe here
        return np.float32(float(fr))

    acc = Fraction(0)
    for j in range(3):
        acc = Fraction(float(rnd(Fraction(float(w[0, j])) * Fraction(float(y[j, 0])) + acc)))
    got = oracle.combine_chain32(y, oracle.F32, w, rows)
    assert got[0, 0] == np.float32(float(acc))
    unfused = np.float32(0)
    for j in range(3):
        unfused = np.float32(np.float32(w[0, j] * y[j, 0]) + unfused)
    assert unfused != got[0, 0]
    assert got[0, 0] == np.float32(2.0 ** -11 + 2.0 ** -24 + 2.0 ** -30)
    rev = oracle.combine_chain32(y[::-1].copy(), oracle.F32, w[:, ::-1].copy(), rows)
    assert rev[0, 0] != got[0, 0]


def _run_pipeline(oracle, wl, p2l, active, policy=0):
    lay = oracle.step_layout(wl.topk_idx, p2l, active, wl.E, wl.R, wl.S, wl.S_prim, policy)
    recv = oracle.pack(wl.x, lay["row_of"])
    return lay, recv


def test_closed_form_scalar_stub_is_mask_and_placement_invariant(oracle):
    """With y = s[e] * x the result is (sum_j w_j s[e_j]) * x[t], whatever the
    mask, placement and policy -- as long as every expert is covered."""
    wl = synth.tiny("c")
    want = ((wl.topk_w.astype(np.float64) * wl.expert_scale[wl.topk_idx].astype(np.float64))
            .sum(1)[:, None] * wl.x.astype(np.float64))
    cases = [(wl.p2l, wl.active, 0), (wl.p2l, wl.active, 1),
             (wl.p2l_preferred, synth.active_mask(wl.R), 0),
             (wl.p2l, synth.active_mask(wl.R), 0)]
    outs = []
    for p2l, active, policy in cases:
        lay, recv = _run_pipeline(oracle, wl, p2l, active, policy)
        assert lay["N"] == wl.T * wl.k
        y = oracle.stub_scale(recv, oracle.F32, lay["N"], lay["offset"], p2l, wl.expert_scale)
        out = oracle.combine(y, oracle.F32, wl.topk_w, lay["row_of"])
        np.testing.assert_allclose(out, want, rtol=1e-6, atol=1e-6)
        outs.append(out)
    # the failed-rank layout really differs from the all-live one
    a = oracle.step_layout(wl.topk_idx, wl.p2l, wl.active, wl.E, wl.R, wl.S, wl.S_prim, 0)
    b = oracle.step_layout(wl.topk_idx, wl.p2l_preferred, synth.active_mask(wl.R), wl.E, wl.R,
                           wl.S, wl.S_prim, 0)
    assert not np.array_equal(a["row_of"], b["row_of"])
    assert a["rank_count"][2] == 0 and b["rank_count"][2] > 0


def test_identity_stub_returns_weighted_sum_of_x(oracle):
    """Identity expert: out[t] = (sum_j w[t,j]) * x[t] = x[t] up to the rounding
    of the weights (they are a softmax, so they sum to 1)."""
    wl = synth.decode(T=64, H=256)
    lay, recv = _run_pipeline(oracle, wl, wl.p2l, wl.active)
    out = oracle.combine(recv, oracle.BF16, wl.topk_w, lay["row_of"])
    x = synth.bf16_bits_to_f32(wl.x).astype(np.float64)
    np.testing.assert_allclose(out, wl.topk_w.astype(np.float64).sum(1)[:, None] * x, rtol=1e-12,
                               atol=1e-12)
    np.testing.assert_allclose(out, x, rtol=1e-6, atol=1e-6)


def test_uncovered_pairs_contribute_nothing(oracle):
    wl = synth.tiny("b")
    lay, recv = _run_pipeline(oracle, wl, wl.p2l, wl.active)
    y = oracle.stub_scale(recv, oracle.F32, lay["N"], lay["offset"], wl.p2l, wl.expert_scale)
    out = oracle.combine(y, oracle.F32, wl.topk_w, lay["row_of"])
    keep = (lay["slot_of"] >= 0)
    want = ((wl.topk_w.astype(np.float64) * wl.expert_scale[wl.topk_idx] * keep).sum(1)[:, None]
            * wl.x.astype(np.float64))
    np.testing.assert_allclose(out, want, rtol=1e-6, atol=1e-6)
    assert (~keep).any()


def test_stub_scale_bf16_and_dequant_match_torch(oracle):
    rng = np.random.default_rng(21)
    R, S, E, H, N = 2, 2, 3, 32, 9
    p2l = np.array([2, 0, 1, 0], np.int32)
    count = np.array([3, 1, 4, 1], np.int32)
    offset = np.concatenate([[0], np.cumsum(count)]).astype(np.int32)
    s = np.array([0.3, 1.7, -2.2], np.float32)
    x = rng.standard_normal((12, H)).astype(np.float32)
    xb = synth.f32_to_bf16_bits(x)
    row_e = np.repeat(p2l, count)
    y = oracle.stub_scale(xb, oracle.BF16, N, offset, p2l, s)
    want = (torch.from_numpy(synth.bf16_bits_to_f32(xb[:N])) * torch.from_numpy(s[row_e])[:, None])
    want = want.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(y[:N], want)
    assert (y[N:] == 0).all()
    yf = oracle.stub_scale(x, oracle.F32, N, offset, p2l, s)
    assert np.array_equal(yf[:N], x[:N] * s[row_e][:, None])
    # fp8 dequant
    big = rng.standard_normal((6, 256)).astype(np.float32) * 3
    q, sc = synth.quantize_e4m3(big, 128)
    yd = oracle.stub_dequant(q, sc, 5, 128)
    deq = torch.from_numpy(q).view(torch.float8_e4m3fn).float() * torch.from_numpy(
        np.repeat(sc, 128, axis=1))
    want_d = deq.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(yd[:5], want_d[:5]) and (yd[5:] == 0).all()
    # and the quantiser is sane: dequantised values are close to the originals
    assert np.abs(deq.numpy() - big).max() <= np.abs(big).max() / 448 * 16 + 1e-6


def test_e4m3_encoder_matches_torch_and_the_format(oracle):
    """Pins for the quantise-on-dispatch definition: torch's float8_e4m3fn cast
    (round to nearest even) on every in-range value class, exact ties, the
    saturation rule, and the independent searchsorted quantiser of synth."""
    rng = np.random.default_rng(13)
    codes = np.arange(256, dtype=np.uint8)
    vals = oracle.e4m3_to_f32(codes)
    finite = ~np.isnan(vals)
    assert np.array_equal(oracle.f32_to_e4m3(vals[finite]), codes[finite])   # round trip
    pos = np.sort(vals[finite & (codes < 0x80)])
    mids = ((pos[:-1].astype(np.float64) + pos[1:]) / 2).astype(np.float32)  # exact in binary32
    x = np.concatenate([rng.standard_normal(100000).astype(np.float32) * 100,
                        rng.standard_normal(100000).astype(np.float32) * 0.01,
                        mids, -mids, np.nextafter(mids, np.float32(0)),
                        np.nextafter(mids, np.float32(1000)),
                        np.array([0.0, -0.0, 447.9, 448.0, -448.0, 2.0 ** -9, 2.0 ** -10,
                                  1.5 * 2.0 ** -10, 2.5 * 2.0 ** -9], np.float32)])
    x = x[np.abs(x) <= 448]
    want = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = oracle.f32_to_e4m3(x)
    assert np.array_equal(got, want)
    # ties go to the even code
    tie_codes = oracle.f32_to_e4m3(mids)
    assert (tie_codes % 2 == 0).all()
    # saturation and NaN
    big = np.array([449.0, 463.9, 464.0, 1e6, np.inf, -500.0, np.nan], np.float32)
    assert oracle.f32_to_e4m3(big).tolist()[:6] == [0x7E, 0x7E, 0x7E, 0x7E, 0x7E, 0xFE]
    assert oracle.f32_to_e4m3(big)[6] & 0x7F == 0x7F
    # whole-tensor definition against the generator's quantiser (a third method)
    xb = synth.f32_to_bf16_bits(rng.standard_normal((64, 512), dtype=np.float32) * 3)
    xb[5, 128:256] = 0                                          # an all-zero group
    q, sc = oracle.quantize_e4m3(xb, 128)
    q2, sc2 = synth.quantize_e4m3(synth.bf16_bits_to_f32(xb), 128)
    assert np.array_equal(sc, sc2) and np.array_equal(q, q2)
    assert sc[5, 1] == 1.0 and (q[5, 128:256] == 0).all()
    assert np.abs(oracle.e4m3_to_f32(q)).max() == 448.0
