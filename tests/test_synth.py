"""The seeded input generators produce what the workloads' recipe promises."""
import numpy as np
import torch

from paper_2605_10670_amd import synth


def test_router_topk_is_distinct_descending_and_normalised():
    rng = np.random.default_rng(1)
    logits = rng.standard_normal((64, 32)).astype(np.float32)
    logits[3, 5] = logits[3, 9] = logits[3].max() + 1  # a tie at the top
    idx, w = synth.router_topk(logits, 8)
    want = torch.topk(torch.from_numpy(logits).double(), 8, dim=1)
    assert all(len(set(r)) == 8 for r in idx.tolist())
    assert np.array_equal(np.sort(idx, 1)[np.arange(64) != 3],
                          np.sort(want.indices.numpy(), 1)[np.arange(64) != 3])
    assert idx[3, 0] == 5 and idx[3, 1] == 9          # ties -> lower index first
    assert (np.diff(np.take_along_axis(logits, idx, 1), axis=1) <= 0).all()
    np.testing.assert_allclose(w.sum(1), 1.0, atol=1e-6)
    np.testing.assert_allclose(w, torch.softmax(want.values, 1).numpy(), atol=1e-6)


def test_placements_cover_every_expert_on_live_ranks():
    for R, sp, sr, failed in [(32, 8, 1, ()), (32, 8, 1, (13,)), (32, 8, 1, (7, 20)),
                              (16, 8, 1, (5,)), (4, 4, 2, (2,))]:
        S = sp + sr
        pref = synth.preferred_placement(R, sp, sr)
        assert np.array_equal(pref.reshape(R, S)[:, :sp].ravel(), np.arange(R * sp))
        p2l = synth.repaired_placement(pref, failed, R, sp, sr) if failed else pref
        active = synth.active_mask(R, failed)
        live = active[np.arange(R * S) // S] == 1
        assert set(p2l[live].tolist()) >= set(range(R * sp))
        for f in failed:  # lost experts now sit only in redundant slots of live ranks
            for e in range(f * sp, (f + 1) * sp):
                where = np.nonzero((p2l == e) & live)[0]
                assert len(where) >= 1 and (where % S >= sp).all()


def test_workload_shapes():
    w = synth.decode(T=256, H=512)
    assert w.topk_idx.shape == (256, 8) and w.x.dtype == np.uint16 and w.P == 288
    z = synth.decode_failed_zipf(T=1024, H=64)
    hot = np.bincount(z.topk_idx.ravel(), minlength=256).argsort()[::-1][:8]
    assert set(hot.tolist()) == set(range(13 * 8, 14 * 8))
    p = synth.prefill_fp8(T=64, H=256)
    assert p.x.dtype == np.uint8 and p.x_scale.shape == (64, 2)
    back = torch.from_numpy(p.x).view(torch.float8_e4m3fn).float().numpy()
    assert np.isfinite(back).all() and np.abs(back).max() == 448.0
