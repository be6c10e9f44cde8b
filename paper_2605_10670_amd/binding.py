"""ctypes binding of libeep.so (include/eep.h).  Argument marshalling only:
every step of the path runs in the library's HIP kernels.  Device buffers are
torch tensors (or raw integer addresses); streams are raw hipStream_t handles
(`torch.cuda.Stream.cuda_stream`).
"""
import ctypes
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libeep.so")

OK, ERR_INVALID_ARG, ERR_ALIGN, ERR_COVERAGE, ERR_HIP, ERR_STATE, ERR_SCRATCH = 0, -1, -2, -3, -4, -5, -6
NOALLOC_SCRATCH_BYTES = 4 * 1024 * 1024
F32, BF16, FP8_E4M3 = 0, 1, 2
SPREAD, FIRST_LIVE = 0, 1
STUB_IDENTITY, STUB_SCALE, STUB_DEQUANT = 0, 1, 2
DTYPES = {"f32": F32, "bf16": BF16, "fp8": FP8_E4M3}
STUBS = {"identity": STUB_IDENTITY, "scale": STUB_SCALE, "dequant": STUB_DEQUANT}

VIEW_FIELDS = ["active", "phys_to_logical", "l2p_off", "l2p_list", "slot_of", "row_of", "src_of",
               "count", "offset", "rank_count", "rank_offset", "cnt_src", "status"]


class EepError(RuntimeError):
    def __init__(self, code, what):
        self.code = code
        super().__init__(f"{what}: {_strerror(code)} ({code})")


class _Config(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "num_ranks", "slots_per_rank", "primary_slots", "num_logical", "max_tokens", "topk",
        "hidden", "x_dtype", "y_dtype", "out_dtype", "scale_group", "policy", "strict_coverage")]


class _View(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in VIEW_FIELDS]


class _LayoutShape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("num_ranks", "slots_per_rank", "num_logical", "topk",
                                              "policy")]


LAYOUT_OUT_FIELDS = ["slot_of", "row_of", "src_of", "count", "offset", "rank_count", "rank_offset",
                     "cnt_src", "status"]


class _LayoutOut(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in LAYOUT_OUT_FIELDS]


_lib = None


def load():
    """Load libeep.so, building it first if it does not exist; raises if that fails
    (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        # nothing built yet: compile the HIP sources once (hipcc cross-compiles without a GPU)
        try:
            from . import build as _build
            _build.build()
        except Exception as exc:
            raise RuntimeError(f"{LIB_PATH} is missing and could not be built with hipcc ({exc}); "
                               "there is no fallback path") from exc
    # torch brings a HIP runtime of its own.  It has to be in the process before this library
    # binds its hip* symbols, so that both use the same one: two runtimes in one process do
    # not share a device context, and tensors of one are not valid arguments for the other.
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    sig = {
        "eep_create": [ctypes.POINTER(_Config), ctypes.POINTER(vp)],
        "eep_workspace_bytes": [ctypes.POINTER(_Config), ctypes.POINTER(i64)],
        "eep_create_with_workspace": [ctypes.POINTER(_Config), vp, i64, ctypes.POINTER(vp)],
        "eep_create_attached": [ctypes.POINTER(_Config), vp, ctypes.POINTER(vp)],
        "eep_create_staging": [vp, ctypes.POINTER(vp)],
        "eep_staging_fork": [vp, vp, vp, vp, vp, vp, i32, vp, vp],
        "eep_staging_join": [vp, vp, vp],
        "eep_destroy": [vp],
        "eep_set_membership": [vp, vp, vp],
        "eep_update_placement": [vp, vp, vp],
        "eep_dispatch_layout": [vp, vp, i32, vp],
        "eep_dispatch_layout_noalloc": [ctypes.POINTER(_LayoutShape), vp, vp, vp, vp, vp,
                                        ctypes.POINTER(_LayoutOut), i32, vp],
        "eep_dispatch": [vp, vp, vp, vp, vp, i32, vp],
        "eep_dispatch_quant": [vp, vp, vp, vp, i32, vp],
        "eep_combine": [vp, vp, vp, vp, i32, vp],
        "eep_expert_stub": [vp, i32, vp, vp, vp, vp, i32, vp],
        "eep_debug_check_layout": [vp, i32, vp, vp],
        "eep_get_view": [vp, ctypes.POINTER(_View)],
        "eep_read_view": [vp, i32, vp, i64, vp],
        "eep_last_hip_error": [vp],
        "eep_calibration_copy": [vp, vp, i64, vp],
        "eep_calibration_stream": [vp, vp, i64, i64, i32, i32, vp],
        "eep_host_replica_lists": [i32, i32, i32, i32, vp, vp, vp],
        "eep_host_uncovered_experts": [i32, i32, i32, vp, vp],
        "eep_host_tiling": [i32, i32, vp],
        "eep_plan_repair": [i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp],
        "eep_plan_transition": [i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp],
        "eep_apply_repair": [vp, vp, vp, i64, vp, vp, vp, vp],
        "eep_read_repair_outcome": [vp, vp],
        "eep_dedup_layout": [vp, i32, vp],
        "eep_dispatch_dedup": [vp, vp, vp, i32, vp],
        "eep_expand": [vp, vp, vp, i32, vp],
        "eep_get_dedup_view": [vp, vp],
        "eep_read_dedup": [vp, i32, vp, i64, vp],
        "eep_set_detection": [vp, i64],
        "eep_signal_experts_done": [vp, vp],
        "eep_debug_withhold_signal": [vp, vp, vp],
        "eep_read_failures": [vp, vp, vp],
        "eep_graph_begin": [vp, vp],
        "eep_graph_end": [vp, vp, ctypes.POINTER(vp)],
        "eep_graph_launch": [vp, vp],
        "eep_graph_destroy": [vp],
        "eep_graph_counters": [vp, ctypes.POINTER(i64 * 3)],
    }
    for name, argtypes in sig.items():
        fn = getattr(lib, name)
        fn.argtypes = argtypes
        fn.restype = ctypes.c_int
    lib.eep_noalloc_scratch_needed.argtypes = [i32, i32, i32]
    lib.eep_noalloc_scratch_needed.restype = i64
    lib.eep_strerror.argtypes = [ctypes.c_int]
    lib.eep_strerror.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _library():
    """`load` under a name that arguments called `load` cannot shadow."""
    return load()


def _strerror(code):
    return load().eep_strerror(code).decode()


def _ptr(t):
    """Device address of a torch tensor (must be contiguous), an int, or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return t.data_ptr()


def _stream(s):
    if s is None:
        return None
    return s if isinstance(s, int) else s.cuda_stream


def _check(code, what, ctx=None):
    if code != OK:
        err = EepError(code, what)
        if code == ERR_HIP and ctx is not None:
            err.args = (err.args[0] + f" [hipError {load().eep_last_hip_error(ctx)}]",)
        raise err


def calibration_copy(dst, src, nbytes, stream=None):
    """Plain copy kernel of known size (yardstick for HBM counters)."""
    _check(load().eep_calibration_copy(_ptr(dst), _ptr(src), nbytes, _stream(stream)),
           "eep_calibration_copy")


def calibration_stream(dst, src, plane_bytes, plane_stride_bytes, reads, writes, stream=None):
    """Sequential streaming kernel with a given read:write mix (yardstick for the data kernels)."""
    _check(load().eep_calibration_stream(_ptr(dst), _ptr(src), plane_bytes, plane_stride_bytes,
                                         reads, writes, _stream(stream)),
           "eep_calibration_stream")


def host_replica_lists(p2l, E, S, S_prim):
    """CSR of every logical expert's replicas (host only) -> (l2p_off, l2p_list)."""
    p2l = np.ascontiguousarray(p2l, np.int32)
    off, lst = np.empty(E + 1, np.int32), np.empty(p2l.size, np.int32)
    _check(load().eep_host_replica_lists(p2l.size, E, S, S_prim, p2l.ctypes.data, off.ctypes.data,
                                         lst.ctypes.data), "eep_host_replica_lists")
    return off, lst


def host_uncovered_experts(p2l, active, E, S):
    p2l = np.ascontiguousarray(p2l, np.int32)
    active = np.ascontiguousarray(active, np.int32)
    n = load().eep_host_uncovered_experts(p2l.size, E, S, p2l.ctypes.data, active.ctypes.data)
    if n < 0:
        _check(n, "eep_host_uncovered_experts")
    return n


def host_tiling(T, R):
    out = np.empty(4, np.int32)
    _check(load().eep_host_tiling(T, R, out.ctypes.data), "eep_host_tiling")
    return dict(tokens_per_rank=int(out[0]), tiles_per_rank=int(out[1]), tile_tokens=int(out[2]),
                num_tiles=int(out[3]))


def noalloc_scratch_needed(R, S, T):
    """Bytes of the static scratch array a batch of T tokens needs (host only)."""
    n = load().eep_noalloc_scratch_needed(R, S, T)
    if n < 0:
        _check(int(n), "eep_noalloc_scratch_needed")
    return int(n)


def dispatch_layout_noalloc(*, R, S, E, k, policy, topk_idx, active, l2p_off, l2p_list, out, T,
                            table_version=None, stream=None):
    """eep_dispatch_layout_noalloc: tables and outputs are device tensors (or raw
    addresses) the caller owns; `out` maps the names in LAYOUT_OUT_FIELDS to them."""
    shape = _LayoutShape(R, S, E, k, policy)
    o = _LayoutOut(*[_ptr(out[n]) for n in LAYOUT_OUT_FIELDS])
    _check(load().eep_dispatch_layout_noalloc(ctypes.byref(shape), _ptr(topk_idx), _ptr(active),
                                              _ptr(l2p_off), _ptr(l2p_list), _ptr(table_version),
                                              ctypes.byref(o), T, _stream(stream)),
           "eep_dispatch_layout_noalloc")


SRC_NONE, SRC_LOCAL, SRC_PEER, SRC_DRAM = -1, 0, 1, 2


def plan_repair(cur_p2l, active, R, S, S_prim, E, load=None):
    """Repaired placement + source of every slot's weights (host only).
    Returns dict(p2l, kind, src_slot, local, peer, dram, unplaced, status); status is the
    library's return code: OK, or ERR_COVERAGE when experts stayed unplaced."""
    cur = np.ascontiguousarray(cur_p2l, np.int32)
    act = np.ascontiguousarray(active, np.int32)
    if cur.size != R * S or act.size != R:
        raise ValueError("cur_p2l must have R*S entries and active R")
    ld = None if load is None else np.ascontiguousarray(load, np.float32)
    new, kind, src = (np.empty(R * S, np.int32) for _ in range(3))
    summary = np.zeros(4, np.int32)
    rc = _library().eep_plan_repair(R, S, S_prim, E, cur.ctypes.data, act.ctypes.data,
                                None if ld is None else ld.ctypes.data, new.ctypes.data,
                                kind.ctypes.data, src.ctypes.data, summary.ctypes.data)
    if rc not in (OK, ERR_COVERAGE):
        _check(rc, "eep_plan_repair")
    return dict(p2l=new, kind=kind, src_slot=src, local=int(summary[0]), peer=int(summary[1]),
                dram=int(summary[2]), unplaced=int(summary[3]), status=rc)


def workspace_bytes(*, num_ranks, slots_per_rank, primary_slots, num_logical, max_tokens, topk, hidden,
                    x_dtype="bf16", y_dtype="bf16", out_dtype="bf16", scale_group=None,
                    policy=SPREAD, strict_coverage=True):
    """Bytes of device memory a context of this shape needs (host only)."""
    xd = DTYPES[x_dtype] if isinstance(x_dtype, str) else x_dtype
    if scale_group is None:
        scale_group = 128 if xd == FP8_E4M3 else 0
    cfg = _Config(num_ranks, slots_per_rank, primary_slots, num_logical, max_tokens, topk, hidden,
                  xd, DTYPES[y_dtype] if isinstance(y_dtype, str) else y_dtype,
                  DTYPES[out_dtype] if isinstance(out_dtype, str) else out_dtype, scale_group,
                  policy, 1 if strict_coverage else 0)
    n = ctypes.c_int64()
    _check(_library().eep_workspace_bytes(ctypes.byref(cfg), ctypes.byref(n)), "eep_workspace_bytes")
    return n.value


def plan_transition(cur_p2l, target_p2l, active, writable, R, S, S_prim, E):
    """Sources for moving to a given target placement (host only); same dict as plan_repair."""
    cur, tgt = (np.ascontiguousarray(a, np.int32) for a in (cur_p2l, target_p2l))
    act, wr = (np.ascontiguousarray(a, np.int32) for a in (active, writable))
    if cur.size != R * S or tgt.size != R * S or act.size != R or wr.size != R:
        raise ValueError("placements must have R*S entries and masks R")
    new, kind, src = (np.empty(R * S, np.int32) for _ in range(3))
    summary = np.zeros(4, np.int32)
    _check(_library().eep_plan_transition(R, S, S_prim, E, cur.ctypes.data, tgt.ctypes.data,
                                          act.ctypes.data, wr.ctypes.data, new.ctypes.data,
                                          kind.ctypes.data, src.ctypes.data, summary.ctypes.data),
           "eep_plan_transition")
    return dict(p2l=new, kind=kind, src_slot=src, local=int(summary[0]), peer=int(summary[1]),
                dram=int(summary[2]), unplaced=0)


class Graph:
    def __init__(self, handle):
        self._h = handle

    def launch(self, stream):
        _check(load().eep_graph_launch(self._h, _stream(stream)), "eep_graph_launch")

    def counters(self):
        c = (ctypes.c_int64 * 3)()
        _check(load().eep_graph_counters(self._h, ctypes.byref(c)), "eep_graph_counters")
        return dict(instantiations=c[0], exec_updates=c[1], launches=c[2])

    def destroy(self):
        if self._h:
            load().eep_graph_destroy(self._h)
            self._h = None


class Context:
    """One EP instance on the current GPU."""

    def __init__(self, *, num_ranks, slots_per_rank, primary_slots, num_logical, max_tokens, topk,
                 hidden, x_dtype="bf16", y_dtype="bf16", out_dtype="bf16", scale_group=None,
                 policy=SPREAD, strict_coverage=True, parent=None, workspace=None,
                 _staging_of=None):
        xd = DTYPES[x_dtype] if isinstance(x_dtype, str) else x_dtype
        if scale_group is None:
            scale_group = 128 if xd == FP8_E4M3 else 0
        self.cfg = _Config(num_ranks, slots_per_rank, primary_slots, num_logical, max_tokens, topk,
                           hidden, xd, DTYPES[y_dtype] if isinstance(y_dtype, str) else y_dtype,
                           DTYPES[out_dtype] if isinstance(out_dtype, str) else out_dtype,
                           scale_group, policy, 1 if strict_coverage else 0)
        self._h = ctypes.c_void_p()
        self._parent = parent      # keeps the instance's first context alive
        self._workspace = workspace    # caller-owned slab (a uint8 device tensor), kept alive
        if _staging_of is not None:
            self._parent = _staging_of
            _check(load().eep_create_staging(_staging_of._h, ctypes.byref(self._h)),
                   "eep_create_staging")
        elif workspace is not None:
            if parent is not None:
                raise ValueError("workspace and parent cannot be combined")
            _check(load().eep_create_with_workspace(ctypes.byref(self.cfg), _ptr(workspace),
                                                    workspace.numel() * workspace.element_size(),
                                                    ctypes.byref(self._h)),
                   "eep_create_with_workspace")
        elif parent is None:
            _check(load().eep_create(ctypes.byref(self.cfg), ctypes.byref(self._h)), "eep_create")
        else:   # same EP instance: shared membership, own placement and layout
            _check(load().eep_create_attached(ctypes.byref(self.cfg), parent._h,
                                              ctypes.byref(self._h)), "eep_create_attached")
        self.R, self.S, self.E, self.k = num_ranks, slots_per_rank, num_logical, topk
        self.P = num_ranks * slots_per_rank
        self.T_max = max_tokens

    def staging(self):
        """A second staging set of this layer (shared membership and placement tables,
        own layout arrays): eep_create_staging."""
        c = self.cfg
        return Context(num_ranks=c.num_ranks, slots_per_rank=c.slots_per_rank,
                       primary_slots=c.primary_slots, num_logical=c.num_logical,
                       max_tokens=c.max_tokens, topk=c.topk, hidden=c.hidden, x_dtype=c.x_dtype,
                       y_dtype=c.y_dtype, out_dtype=c.out_dtype, scale_group=c.scale_group,
                       policy=c.policy, strict_coverage=bool(c.strict_coverage),
                       _staging_of=self)

    def staging_fork(self, topk_idx, x, recv_x, T, stream, side_stream, x_scale=None,
                     recv_scale=None):
        _check(load().eep_staging_fork(self._h, _ptr(topk_idx), _ptr(x), _ptr(x_scale),
                                       _ptr(recv_x), _ptr(recv_scale), T, _stream(stream),
                                       _stream(side_stream)), "eep_staging_fork", self._h)

    def staging_join(self, stream, side_stream):
        _check(load().eep_staging_join(self._h, _stream(stream), _stream(side_stream)),
               "eep_staging_join", self._h)

    # -- table updates -------------------------------------------------------
    def set_membership(self, active, stream=None):
        a = np.ascontiguousarray(active, np.int32)
        if a.size != self.R:
            raise ValueError("active must have R entries")
        _check(load().eep_set_membership(self._h, a.ctypes.data, _stream(stream)),
               "eep_set_membership", self._h)

    def update_placement(self, phys_to_logical, stream=None):
        p = np.ascontiguousarray(phys_to_logical, np.int32)
        if p.size != self.P:
            raise ValueError("phys_to_logical must have P entries")
        _check(load().eep_update_placement(self._h, p.ctypes.data, _stream(stream)),
               "eep_update_placement", self._h)

    def apply_repair(self, weights, backup, slot_bytes, plan, stream=None):
        """weights: device tensor [P, slot_bytes]; backup: device or pinned-host tensor
        [E, slot_bytes] (or None); plan: the dict plan_repair returns."""
        arrays = [np.ascontiguousarray(plan[key], np.int32) for key in ("p2l", "kind", "src_slot")]
        if any(a.size != self.P for a in arrays):
            raise ValueError("plan arrays must have P entries")
        _check(load().eep_apply_repair(self._h, _ptr(weights), _ptr(backup), slot_bytes,
                                       arrays[0].ctypes.data, arrays[1].ctypes.data,
                                       arrays[2].ctypes.data, _stream(stream)),
               "eep_apply_repair", self._h)

    def read_repair_outcome(self):
        out = np.zeros(self.P, np.int32)
        _check(load().eep_read_repair_outcome(self._h, out.ctypes.data),
               "eep_read_repair_outcome", self._h)
        return out

    # -- per-step calls ------------------------------------------------------
    def dispatch_layout(self, topk_idx, T, stream=None):
        _check(load().eep_dispatch_layout(self._h, _ptr(topk_idx), T, _stream(stream)),
               "eep_dispatch_layout", self._h)

    def dispatch(self, x, recv_x, T, x_scale=None, recv_scale=None, stream=None):
        _check(load().eep_dispatch(self._h, _ptr(x), _ptr(x_scale), _ptr(recv_x),
                                   _ptr(recv_scale), T, _stream(stream)), "eep_dispatch", self._h)

    def dispatch_quant(self, x_bf16, recv_x, recv_scale, T, stream=None):
        _check(load().eep_dispatch_quant(self._h, _ptr(x_bf16), _ptr(recv_x), _ptr(recv_scale), T,
                                         _stream(stream)), "eep_dispatch_quant", self._h)

    def combine(self, y, topk_w, out, T, stream=None):
        _check(load().eep_combine(self._h, _ptr(y), _ptr(topk_w), _ptr(out), T, _stream(stream)),
               "eep_combine", self._h)

    def expert_stub(self, kind, recv_x, y, T, recv_scale=None, expert_scale=None, stream=None):
        kind = STUBS[kind] if isinstance(kind, str) else kind
        _check(load().eep_expert_stub(self._h, kind, _ptr(recv_x), _ptr(recv_scale),
                                      _ptr(expert_scale), _ptr(y), T, _stream(stream)),
               "eep_expert_stub", self._h)

    # -- GPU-side failure detection -------------------------------------------
    def set_detection(self, timeout_ns):
        _check(load().eep_set_detection(self._h, int(timeout_ns)), "eep_set_detection", self._h)

    def signal_experts_done(self, stream=None):
        _check(load().eep_signal_experts_done(self._h, _stream(stream)),
               "eep_signal_experts_done", self._h)

    def debug_withhold_signal(self, withhold, stream=None):
        w = np.ascontiguousarray(withhold, np.int32)
        if w.size != self.R:
            raise ValueError("withhold must have R entries")
        _check(load().eep_debug_withhold_signal(self._h, w.ctypes.data, _stream(stream)),
               "eep_debug_withhold_signal", self._h)

    def read_failures(self, stream=None):
        out = np.zeros(self.R, np.int32)
        _check(load().eep_read_failures(self._h, out.ctypes.data, _stream(stream)),
               "eep_read_failures", self._h)
        return out

    # -- introspection -------------------------------------------------------
    def view_pointers(self):
        v = _View()
        _check(load().eep_get_view(self._h, ctypes.byref(v)), "eep_get_view")
        return {n: getattr(v, n) for n in VIEW_FIELDS}

    def read(self, field, n, stream=None):
        """Host copy (numpy int32[n]) of one view array, after waiting for `stream`."""
        out = np.empty(n, np.int32)
        _check(load().eep_read_view(self._h, VIEW_FIELDS.index(field), out.ctypes.data, n,
                                    _stream(stream)), "eep_read_view", self._h)
        return out

    def check_layout(self, T, stream=None):
        """eep_debug_check_layout -> int32[4] violation counts (see eep.h)."""
        out = np.zeros(4, np.int32)
        _check(load().eep_debug_check_layout(self._h, T, out.ctypes.data, _stream(stream)),
               "eep_debug_check_layout", self._h)
        return out

    def read_layout(self, T, stream=None):
        k, R, P = self.k, self.R, self.P
        st = self.read("status", 4, stream)
        return dict(
            slot_of=self.read("slot_of", T * k).reshape(T, k),
            row_of=self.read("row_of", T * k).reshape(T, k),
            src_of=self.read("src_of", T * k), count=self.read("count", P),
            offset=self.read("offset", P + 1), rank_count=self.read("rank_count", R),
            rank_offset=self.read("rank_offset", R + 1),
            cnt_src=self.read("cnt_src", R * P).reshape(R, P),
            N=int(st[0]), n_uncovered=int(st[1]), n_masked=int(st[2]), version=int(st[3]))

    # -- de-duplicated dispatch ------------------------------------------------
    def dedup_layout(self, T, stream=None):
        _check(load().eep_dedup_layout(self._h, T, _stream(stream)), "eep_dedup_layout", self._h)

    def dispatch_dedup(self, x, recv_dedup, T, stream=None):
        _check(load().eep_dispatch_dedup(self._h, _ptr(x), _ptr(recv_dedup), T, _stream(stream)),
               "eep_dispatch_dedup", self._h)

    def expand(self, recv_dedup, recv_x, T, stream=None):
        _check(load().eep_expand(self._h, _ptr(recv_dedup), _ptr(recv_x), T, _stream(stream)),
               "eep_expand", self._h)

    def read_dedup(self, T, stream=None):
        fields = ["dedup_count", "dedup_offset", "dedup_row", "dedup_dst", "expand_of", "status"]
        sizes = [self.R, self.R + 1, T * self.k, T * self.k, T * self.k, 1]
        out = {}
        for i, (name, n) in enumerate(zip(fields, sizes)):
            a = np.zeros(n, np.int32)
            _check(load().eep_read_dedup(self._h, i, a.ctypes.data, n, _stream(stream)),
                   "eep_read_dedup", self._h)
            out[name] = a
        out["dedup_row"] = out["dedup_row"].reshape(T, self.k)
        out["dedup_dst"] = out["dedup_dst"].reshape(T, self.k)
        out["N_d"] = int(out.pop("status")[0])
        return out

    # -- graphs --------------------------------------------------------------
    def graph_begin(self, stream):
        _check(load().eep_graph_begin(self._h, _stream(stream)), "eep_graph_begin", self._h)

    def graph_end(self, stream):
        g = ctypes.c_void_p()
        _check(load().eep_graph_end(self._h, _stream(stream), ctypes.byref(g)), "eep_graph_end",
               self._h)
        return Graph(g)

    def destroy(self):
        if self._h:
            _check(load().eep_destroy(self._h), "eep_destroy")
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass
