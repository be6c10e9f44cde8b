"""Seeded synthetic inputs for the dispatch/combine step.

This module only PRODUCES inputs (router choices, activations, placements,
masks).  It contains none of the dispatch/combine method and is the one piece
that both the GPU tests and the CPU oracle's tests draw from.  The tensors
stand in for DeepSeek-V3 serving traffic (paper Sec. 6.1: 256 routed experts,
32-rank decode EP instance): same shapes and routing statistics, random
values, no model weights.

All randomness comes from numpy.random.default_rng(BASE_SEED + offset).
"""
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

BASE_SEED = 260510670


# ----------------------------------------------------------------------------
# number formats (input preparation only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round-to-nearest-even."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32).astype(np.uint64)
    rounded = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, np.uint16).astype(np.uint32) << 16).view(np.float32)


def _e4m3_positive_values() -> np.ndarray:
    """The 127 finite non-negative e4m3fn values in code order 0x00..0x7E."""
    codes = np.arange(0x7F)
    ex, man = codes >> 3, codes & 7
    return np.where(ex == 0, man / 8.0 * 2.0 ** -6, (1 + man / 8.0) * 2.0 ** (ex - 7.0))


def quantize_e4m3(x: np.ndarray, group: int = 128):
    """Per-token, per-`group`-channel fp8 quantisation of float32 rows.

    scale = max|x| / 448 over the group (1 if the group is all zero), in fp32;
    q = e4m3fn(x / scale), round-to-nearest-even, saturating at +-448.
    Returns (q uint8 [T, H], scale float32 [T, H/group]).
    """
    x = np.ascontiguousarray(x, np.float32)
    T, H = x.shape
    assert H % group == 0
    vals = _e4m3_positive_values()
    mids = (vals[:-1] + vals[1:]) / 2
    q = np.empty((T, H), np.uint8)
    scale = np.empty((T, H // group), np.float32)
    for t0 in range(0, T, 512):  # row blocks keep the float64 temporaries small
        xg = x[t0:t0 + 512].reshape(-1, H // group, group)
        amax = np.abs(xg).max(axis=2)
        sc = (amax / np.float32(448.0)).astype(np.float32)
        sc[sc == 0] = 1.0
        a = (xg / sc[:, :, None]).astype(np.float32).reshape(-1, H)
        mag = np.minimum(np.abs(a).astype(np.float64), 448.0)
        lo = np.searchsorted(mids, mag, side="left")
        hi = np.searchsorted(mids, mag, side="right")
        code = np.where(lo == hi, lo, np.where(lo % 2 == 0, lo, hi))  # tie -> even code
        q[t0:t0 + 512] = (code | np.where(np.signbit(a), 0x80, 0)).astype(np.uint8)
        scale[t0:t0 + 512] = sc
    return q, scale


# ----------------------------------------------------------------------------
# router
# ----------------------------------------------------------------------------
def router_topk(logits: np.ndarray, k: int):
    """Top-k by descending logit (ties -> lower expert index), indices kept in
    that order; weights = softmax over the k selected logits, computed in
    float64 and stored as float32."""
    order = np.argsort(-logits.astype(np.float64), axis=1, kind="stable")[:, :k]
    sel = np.take_along_axis(logits.astype(np.float64), order, axis=1)
    ex = np.exp(sel - sel.max(axis=1, keepdims=True))
    w = ex / ex.sum(axis=1, keepdims=True)
    return order.astype(np.int32), w.astype(np.float32)


# ----------------------------------------------------------------------------
# placements
# ----------------------------------------------------------------------------
def preferred_placement(R: int, S_prim: int, S_red: int) -> np.ndarray:
    """All-live placement: primary slot (r, s) holds expert r*S_prim + s; the
    i-th redundant slot of rank r replicates expert ((r+1+i) mod R)*S_prim + i
    (with one redundant slot: the first expert of the next rank, like E2' on
    R3 in the paper's Fig. 5)."""
    S = S_prim + S_red
    p2l = np.full(R * S, -1, np.int32)
    for r in range(R):
        for s in range(S_prim):
            p2l[r * S + s] = r * S_prim + s
        for i in range(S_red):
            p2l[r * S + S_prim + i] = ((r + 1 + i) % R) * S_prim + (i % max(S_prim, 1))
    return p2l


def repaired_placement(p2l: np.ndarray, failed, R: int, S_prim: int, S_red: int) -> np.ndarray:
    """Placement after the ranks in `failed` are lost: each lost rank's primary
    experts are written into redundant slots of the following live ranks,
    round-robin, replacing whatever replica was there.  Failed ranks are handled
    in ascending order; a redundant slot is reused only after every live rank's
    redundant slots have been taken once."""
    S = S_prim + S_red
    out = np.array(p2l, np.int32, copy=True)
    failed = sorted(int(f) for f in failed)
    live = [r for r in range(R) if r not in failed]
    taken = set()
    for f in failed:
        cursor = f
        for i in range(S_prim):
            e = f * S_prim + i
            placed = False
            for _ in range(R * max(S_red, 1) + 1):
                cursor = (cursor + 1) % R
                if cursor not in live:
                    continue
                for s in range(S_prim, S):
                    if (cursor, s) not in taken:
                        out[cursor * S + s] = e
                        taken.add((cursor, s))
                        placed = True
                        break
                if placed:
                    break
            if not placed:
                raise ValueError("not enough redundant slots on live ranks")
    return out


def active_mask(R: int, failed=()) -> np.ndarray:
    a = np.ones(R, np.int32)
    for f in failed:
        a[f] = 0
    return a


# ----------------------------------------------------------------------------
# workloads
# ----------------------------------------------------------------------------
@dataclass
class Workload:
    name: str
    T: int
    H: int
    E: int
    k: int
    R: int
    S_prim: int
    S_red: int
    x_dtype: str            # "f32" | "bf16" | "fp8"
    y_dtype: str            # "f32" | "bf16"
    out_dtype: str          # "f32" | "bf16"
    stub: str               # "identity" | "scale" | "dequant"
    failed: tuple
    topk_idx: np.ndarray    # int32 [T, k]
    topk_w: np.ndarray      # float32 [T, k]
    x: np.ndarray           # float32 [T,H] | uint16 bf16 bits | uint8 fp8 codes
    p2l: np.ndarray         # int32 [P], placement in force for the step
    active: np.ndarray      # int32 [R]
    x_scale: Optional[np.ndarray] = None      # float32 [T, H/128] for fp8
    expert_scale: Optional[np.ndarray] = None  # float32 [E] for the scale stub
    p2l_preferred: Optional[np.ndarray] = None
    extra: dict = field(default_factory=dict)

    @property
    def S(self):
        return self.S_prim + self.S_red

    @property
    def P(self):
        return self.R * self.S


def _x_bf16(rng, T, H):
    return f32_to_bf16_bits(rng.standard_normal((T, H), dtype=np.float32))


def tiny(variant: str = "c", T: int = 128, seed_offset: int = 1) -> Workload:
    """Tiny CPU-checkable step: H=1024 fp32, E=16, top-2, R=4, scalar stub.

    variant "a": 4 primary + 1 redundant slot per rank, all ranks live;
    variant "b": same slots, rank 2 failed.  3 live ranks x 5 slots = 15 < 16
                 experts, so one expert is necessarily uncovered;
    variant "c": 4 primary + 2 redundant slots, rank 2 failed, fully covered.
    """
    rng = np.random.default_rng(BASE_SEED + seed_offset)
    H, E, k, R, S_prim = 1024, 16, 2, 4, 4
    S_red = 2 if variant == "c" else 1
    failed = () if variant == "a" else (2,)
    x = rng.standard_normal((T, H), dtype=np.float32)
    logits = rng.standard_normal((T, E), dtype=np.float32)
    idx, w = router_topk(logits, k)
    pref = preferred_placement(R, S_prim, S_red)
    if variant == "b":
        # only 3 redundant slots exist on live ranks: experts 8, 9, 10 move, 11 is lost
        p2l = pref.copy()
        S = S_prim + S_red
        for i, r in enumerate((3, 0, 1)):
            p2l[r * S + S_prim] = 2 * S_prim + i
    else:
        p2l = repaired_placement(pref, failed, R, S_prim, S_red) if failed else pref
    scale = (1.0 + np.arange(E) / 16.0).astype(np.float32)
    return Workload(f"tiny-{variant}", T, H, E, k, R, S_prim, S_red, "f32", "f32", "f32", "scale",
                    failed, idx, w, x, p2l, active_mask(R, failed), expert_scale=scale,
                    p2l_preferred=pref)


def decode(T: int = 4096, H: int = 7168, seed_offset: int = 2) -> Workload:
    """DeepSeek-V3-shaped decode step: R=32 ranks x T/32 tokens, bf16, E=256,
    top-8, 8 primary + 1 redundant slot per rank, all live, identity stub."""
    rng = np.random.default_rng(BASE_SEED + seed_offset)
    E, k, R, S_prim, S_red = 256, 8, 32, 8, 1
    x = _x_bf16(rng, T, H)
    logits = rng.standard_normal((T, E), dtype=np.float32)
    idx, w = router_topk(logits, k)
    pref = preferred_placement(R, S_prim, S_red)
    return Workload("dsv3-decode", T, H, E, k, R, S_prim, S_red, "bf16", "bf16", "bf16",
                    "identity", (), idx, w, x, pref, active_mask(R), p2l_preferred=pref)


def decode_failed_zipf(T: int = 4096, H: int = 7168, failed_rank: int = 13,
                       seed_offset: int = 3) -> Workload:
    """Decode shape with one failed rank whose 8 experts live only in redundant
    slots of other ranks; logits carry a Zipf(1.2) per-expert bias whose eight
    hottest experts are the remapped ones."""
    rng = np.random.default_rng(BASE_SEED + seed_offset)
    E, k, R, S_prim, S_red = 256, 8, 32, 8, 1
    x = _x_bf16(rng, T, H)
    logits = rng.standard_normal((T, E), dtype=np.float32)
    lost = np.arange(failed_rank * S_prim, (failed_rank + 1) * S_prim)
    others = np.setdiff1d(np.arange(E), lost)
    zrank = np.empty(E, np.int64)
    zrank[lost] = np.arange(1, S_prim + 1)
    zrank[rng.permutation(others)] = np.arange(S_prim + 1, E + 1)
    logits = logits + (-1.2 * np.log(zrank)).astype(np.float32)[None, :]
    idx, w = router_topk(logits, k)
    pref = preferred_placement(R, S_prim, S_red)
    p2l = repaired_placement(pref, (failed_rank,), R, S_prim, S_red)
    return Workload("dsv3-decode-failed-zipf", T, H, E, k, R, S_prim, S_red, "bf16", "bf16",
                    "bf16", "identity", (failed_rank,), idx, w, x, p2l,
                    active_mask(R, (failed_rank,)), p2l_preferred=pref)


def prefill_fp8(T: int = 16384, H: int = 7168, failed=(7, 20), seed_offset: int = 4) -> Workload:
    """Prefill-shaped step: fp8 e4m3 payload + fp32 scale per 128 channels,
    dequantising stub, bf16 combine, two failed ranks, uniform logits."""
    rng = np.random.default_rng(BASE_SEED + seed_offset)
    E, k, R, S_prim, S_red = 256, 8, 32, 8, 1
    x32 = rng.standard_normal((T, H), dtype=np.float32)
    q, scale = quantize_e4m3(x32, 128)
    del x32
    logits = rng.random((T, E), dtype=np.float32)
    idx, w = router_topk(logits, k)
    pref = preferred_placement(R, S_prim, S_red)
    p2l = repaired_placement(pref, failed, R, S_prim, S_red)
    return Workload("dsv3-prefill-fp8", T, H, E, k, R, S_prim, S_red, "fp8", "bf16", "bf16",
                    "dequant", tuple(failed), idx, w, q, p2l, active_mask(R, failed),
                    x_scale=scale, p2l_preferred=pref)


def churn_inputs(n_sets: int = 8, T: int = 2048, H: int = 4096, seed_offset: int = 5):
    """Qwen3-MoE-like churn workload: E=128, top-8, R=16, 8+1 slots, bf16,
    per-expert scalar stub.  Returns a list of `n_sets` Workloads (all-live
    placement/mask filled in; the test toggles rank 5)."""
    E, k, R, S_prim, S_red = 128, 8, 16, 8, 1
    pref = preferred_placement(R, S_prim, S_red)
    scale = (0.5 + np.arange(E) / E).astype(np.float32)
    sets = []
    for s in range(n_sets):
        rng = np.random.default_rng(BASE_SEED + seed_offset + 1000 + s)
        x = _x_bf16(rng, T, H)
        logits = rng.standard_normal((T, E), dtype=np.float32)
        idx, w = router_topk(logits, k)
        sets.append(Workload(f"churn-{s}", T, H, E, k, R, S_prim, S_red, "bf16", "bf16", "bf16",
                             "scale", (), idx, w, x, pref, active_mask(R), expert_scale=scale,
                             p2l_preferred=pref))
    return sets
