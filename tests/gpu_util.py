"""Helpers shared by the GPU parity tests: move a synth.Workload to the GPU, run
the step through the C-ABI binding, bring results back as numpy arrays."""
import numpy as np
import torch

from paper_2605_10670_amd import binding

NP_OF = {"f32": np.float32, "bf16": np.uint16, "fp8": np.uint8}
LAYOUT_KEYS = ["slot_of", "row_of", "src_of", "count", "offset", "rank_count", "rank_offset",
               "cnt_src"]


def to_dev(a):
    """numpy -> cuda tensor of the same bytes (uint16 travels as int16)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(a).cuda()


def to_host(t, np_dtype):
    a = t.cpu().numpy()
    return a.view(np_dtype) if a.dtype != np_dtype else a


def dev_empty(rows, H, kind, fill=None):
    tdt = {"f32": torch.float32, "bf16": torch.int16, "fp8": torch.uint8}[kind]
    t = torch.empty((rows, H), dtype=tdt, device="cuda")
    if fill is not None:
        t.fill_(fill)
    return t


def make_context(wl, policy=binding.SPREAD, strict=True, T_max=None):
    return binding.Context(num_ranks=wl.R, slots_per_rank=wl.S, primary_slots=wl.S_prim,
                           num_logical=wl.E, max_tokens=T_max or wl.T, topk=wl.k, hidden=wl.H,
                           x_dtype=wl.x_dtype, y_dtype=wl.y_dtype, out_dtype=wl.out_dtype,
                           policy=policy, strict_coverage=strict)


def apply_tables(ctx, p2l, active, stream=None):
    """Placement first, then membership: the order the paper uses on a failure."""
    ctx.update_placement(p2l, stream)
    ctx.set_membership(active, stream)


class DeviceStep:
    """Device buffers of one workload plus the per-step calls on them."""

    def __init__(self, ctx, wl, stream=None):
        self.ctx, self.wl, self.stream = ctx, wl, stream
        T, k, H = wl.T, wl.k, wl.H
        self.idx = to_dev(wl.topk_idx)
        self.w = to_dev(wl.topk_w)
        self.x = to_dev(wl.x)
        self.x_scale = to_dev(wl.x_scale) if wl.x_scale is not None else None
        self.recv = dev_empty(T * k, H, wl.x_dtype, fill=0)
        self.recv_scale = (torch.zeros((T * k, H // 128), dtype=torch.float32, device="cuda")
                           if wl.x_scale is not None else None)
        self.expert_scale = to_dev(wl.expert_scale) if wl.expert_scale is not None else None
        if wl.stub == "identity":
            self.y = self.recv          # alias, as a real caller would
        else:
            self.y = dev_empty(T * k, H, wl.y_dtype, fill=0)
        self.out = dev_empty(T, H, wl.out_dtype, fill=0)

    def layout(self):
        self.ctx.dispatch_layout(self.idx, self.wl.T, self.stream)

    def dispatch(self):
        self.ctx.dispatch(self.x, self.recv, self.wl.T, self.x_scale, self.recv_scale, self.stream)

    def stub(self):
        if self.wl.stub != "identity":
            self.ctx.expert_stub(self.wl.stub, self.recv, self.y, self.wl.T,
                                 recv_scale=self.recv_scale, expert_scale=self.expert_scale,
                                 stream=self.stream)

    def combine(self):
        self.ctx.combine(self.y, self.w, self.out, self.wl.T, self.stream)

    def step(self):
        self.layout()
        self.dispatch()
        self.stub()
        self.combine()

    def sync(self):
        torch.cuda.synchronize()


def assert_layout_equal(got, want, T, k):
    for key in LAYOUT_KEYS:
        assert np.array_equal(got[key], want[key]), f"layout field {key} differs"
    for key in ("N", "n_uncovered", "n_masked"):
        assert got[key] == want[key], f"{key}: {got[key]} != {want[key]}"


def bf16_to_f64(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def check_combine(got, out_dtype, want64, chain32_bits=None):
    """The benchmark spec gate: 1e-3 relative on the fp32-accumulated sum (row-rms floor);
    bf16 outputs within one bf16 ulp of the exact sum.  If the fp32-chain result
    is given, also demand bit equality with it (same order, same rounding)."""
    rms = np.sqrt((want64 ** 2).mean(axis=1, keepdims=True))
    if out_dtype == "f32":
        g = got.astype(np.float64)
        tol = 1e-3 * np.abs(want64) + 1e-3 * rms
    else:
        g = bf16_to_f64(got)
        tol = 2.0 ** -7 * np.abs(want64) + 1e-3 * rms
    bad = np.abs(g - want64) > tol
    assert not bad.any(), f"{bad.sum()} combine outputs outside tolerance"
    if chain32_bits is not None:
        assert np.array_equal(got.view(chain32_bits.dtype), chain32_bits), \
            "combine is not bit-equal to the fp32 ascending fused-multiply-add chain"
