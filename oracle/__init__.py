"""Python face of the C oracle (oracle/eep_oracle.c).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the CPU-baseline leg of
the benchmark may import this; the product package never does.  This file only
marshals numpy arrays into the C functions; all arithmetic lives in the C file.
"""
import ctypes
import os

import numpy as np

from . import build as _build

SPREAD, FIRST_LIVE = 0, 1
F32, BF16 = 0, 1

_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(_build.build(force=False))
        _lib.eeo_tables.restype = ctypes.c_int
        _lib.eeo_uncovered_experts.restype = ctypes.c_int
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def tables(p2l, E, S, S_prim):
    """O1 -> (l2p_off[E+1], l2p_list[P])."""
    p2l = _i32(p2l)
    P = p2l.size
    off = np.empty(E + 1, np.int32)
    lst = np.empty(P, np.int32)
    rc = lib().eeo_tables(P, E, S, S_prim, _p(p2l), _p(off), _p(lst))
    if rc != 0:
        raise ValueError("phys_to_logical entry outside [-1, E)")
    return off, lst


def uncovered_experts(p2l, active, E, S):
    p2l, active = _i32(p2l), _i32(active)
    return lib().eeo_uncovered_experts(p2l.size, E, S, _p(p2l), _p(active))


def map_pairs(topk_idx, l2p_off, l2p_list, active, E, S, policy):
    """O2 -> (slot_of[T,k], n_uncovered, n_masked)."""
    topk_idx = _i32(topk_idx)
    T, k = topk_idx.shape
    slot_of = np.empty((T, k), np.int32)
    counters = np.zeros(2, np.int64)
    lib().eeo_map(T, k, E, S, policy, _p(topk_idx), _p(_i32(l2p_off)), _p(_i32(l2p_list)),
                  _p(_i32(active)), _p(slot_of), _p(counters))
    return slot_of, int(counters[0]), int(counters[1])


def layout(slot_of, R, S):
    """O3-O5 -> dict(count, rank_count, cnt_src, offset, rank_offset, row_of, src_of)."""
    slot_of = _i32(slot_of)
    T, k = slot_of.shape
    if T % R != 0:
        raise ValueError("T must be a multiple of R")
    P = R * S
    out = dict(count=np.empty(P, np.int32), rank_count=np.empty(R, np.int32),
               cnt_src=np.empty((R, P), np.int32), offset=np.empty(P + 1, np.int32),
               rank_offset=np.empty(R + 1, np.int32), row_of=np.empty((T, k), np.int32),
               src_of=np.empty(T * k, np.int32))
    cursor = np.empty(P, np.int32)
    lib().eeo_layout(T, k, R, S, _p(slot_of), _p(out["count"]), _p(out["rank_count"]),
                     _p(out["cnt_src"]), _p(out["offset"]), _p(out["rank_offset"]),
                     _p(out["row_of"]), _p(out["src_of"]), _p(cursor))
    return out


def pack(x, row_of, fill=0):
    """O6.  x: [T, ...] any dtype, contiguous -> recv [T*k, ...]; untouched rows = fill."""
    x = np.ascontiguousarray(x)
    row_of = _i32(row_of)
    T, k = row_of.shape
    recv = np.full((T * k,) + x.shape[1:], fill, dtype=x.dtype)
    row_bytes = x[0].nbytes if T else 0
    lib().eeo_pack(T, k, ctypes.c_int64(row_bytes), _p(x), _p(row_of), _p(recv))
    return recv


def pack_into(x, row_of, recv):
    """O6 into an existing receive buffer: recv[row_of[t, j]] = x[t] for the tokens given
    (x and row_of may be a token range of a larger step; recv is the whole buffer)."""
    x = np.ascontiguousarray(x)
    row_of = _i32(row_of)
    T, k = row_of.shape
    assert recv.flags.c_contiguous and recv.dtype == x.dtype and recv.shape[1:] == x.shape[1:]
    assert T == 0 or int(row_of.max()) < recv.shape[0]
    row_bytes = x[0].nbytes if T else 0
    lib().eeo_pack(T, k, ctypes.c_int64(row_bytes), _p(x), _p(row_of), _p(recv))
    return recv


def dedup_layout(slot_of, row_of, R, S):
    """De-duplicated dispatch layout -> dict(dedup_count, dedup_offset, dedup_row, lead, expand_of, N_d)."""
    slot_of, row_of = _i32(slot_of), _i32(row_of)
    T, k = slot_of.shape
    out = dict(dedup_count=np.empty(R, np.int32), dedup_offset=np.empty(R + 1, np.int32),
               dedup_row=np.empty((T, k), np.int32), lead=np.empty((T, k), np.int32),
               expand_of=np.empty(T * k, np.int32))
    seen = np.empty(R, np.int32)
    lib().eeo_dedup_layout(T, k, R, S, _p(slot_of), _p(row_of), _p(out["dedup_count"]),
                           _p(out["dedup_offset"]), _p(out["dedup_row"]), _p(out["lead"]),
                           _p(out["expand_of"]), _p(seen))
    out["N_d"] = int(out["dedup_offset"][-1])
    return out


def pack_dedup(x, dedup_row, lead, fill=0):
    """Stage 1: x [T, ...] -> recv_d [T*k, ...] (only the first N_d rows are written)."""
    x = np.ascontiguousarray(x)
    dedup_row, lead = _i32(dedup_row), _i32(lead)
    T, k = dedup_row.shape
    recv_d = np.full((T * k,) + x.shape[1:], fill, dtype=x.dtype)
    row_bytes = x[0].nbytes if T else 0
    lib().eeo_pack_dedup(T, k, ctypes.c_int64(row_bytes), _p(x), _p(dedup_row), _p(lead), _p(recv_d))
    return recv_d


def expand(recv_d, expand_of, N, fill=0):
    """Stage 2: recv[row] = recv_d[expand_of[row]] for row < N."""
    recv_d = np.ascontiguousarray(recv_d)
    expand_of = _i32(expand_of)
    recv = np.full_like(recv_d, fill)
    row_bytes = recv_d[0].nbytes if recv_d.shape[0] else 0
    lib().eeo_expand(int(N), ctypes.c_int64(row_bytes), _p(recv_d), _p(expand_of), _p(recv))
    return recv


def stub_scale(recv, dtype, N, offset, p2l, expert_scale):
    """O7 scalar stub.  recv: [rows, H] float32 (dtype F32) or uint16 bf16 bits (BF16)."""
    recv = np.ascontiguousarray(recv)
    y = np.zeros_like(recv)
    H = recv.shape[1]
    p2l = _i32(p2l)
    lib().eeo_stub_scale(int(N), H, p2l.size, dtype, _p(recv), _p(_i32(offset)), _p(p2l),
                         _p(np.ascontiguousarray(expert_scale, np.float32)), _p(y))
    return y


def stub_dequant(q, scale, N, group):
    """O7 fp8 stub -> bf16 bits [rows, H]."""
    q = np.ascontiguousarray(q, np.uint8)
    scale = np.ascontiguousarray(scale, np.float32)
    y = np.zeros(q.shape, np.uint16)
    lib().eeo_stub_dequant(int(N), q.shape[1], group, _p(q), _p(scale), _p(y))
    return y


def combine(y, y_dtype, w, row_of):
    """O8 in double -> float64 [T, H]."""
    y = np.ascontiguousarray(y)
    w = np.ascontiguousarray(w, np.float32)
    row_of = _i32(row_of)
    T, k = row_of.shape
    H = y.shape[1]
    out = np.empty((T, H), np.float64)
    lib().eeo_combine(T, k, H, y_dtype, _p(y), _p(w), _p(row_of), _p(out))
    return out


def combine_chain32(y, y_dtype, w, row_of):
    """O8, fp32 fused-multiply-add chain in ascending j -> float32 [T, H]."""
    y = np.ascontiguousarray(y)
    w = np.ascontiguousarray(w, np.float32)
    row_of = _i32(row_of)
    T, k = row_of.shape
    H = y.shape[1]
    out = np.empty((T, H), np.float32)
    lib().eeo_combine_chain32(T, k, H, y_dtype, _p(y), _p(w), _p(row_of), _p(out))
    return out


def detect_round(slot_of, row_of, active, arrived, S):
    """One combine-side wait for the signals of the active ranks (Sec. 3.4, Sec. 4.1).
    -> dict(active, report, row_of, withdrawn): the mask later steps see, the failure
    report the host reads after the step, the rows the combine of THIS step uses."""
    slot_of, rows = _i32(slot_of), _i32(row_of).copy()
    act, arr = _i32(active).copy(), _i32(arrived)
    T, k = slot_of.shape
    report = np.zeros(act.size, np.int32)
    fn = lib().eeo_detect_round
    fn.restype = ctypes.c_int64
    n = fn(T, k, act.size, S, _p(slot_of), _p(arr), _p(act), _p(report), _p(rows))
    return dict(active=act, report=report, row_of=rows, withdrawn=int(n))


def bf16_to_f32(bits):
    bits = np.ascontiguousarray(bits, np.uint16)
    out = np.empty(bits.shape, np.float32)
    lib().eeo_bf16_to_f32_array(ctypes.c_int64(bits.size), _p(bits), _p(out))
    return out


def f32_to_bf16(x):
    x = np.ascontiguousarray(x, np.float32)
    out = np.empty(x.shape, np.uint16)
    lib().eeo_f32_to_bf16_array(ctypes.c_int64(x.size), _p(x), _p(out))
    return out


def e4m3_to_f32(q):
    q = np.ascontiguousarray(q, np.uint8)
    out = np.empty(q.shape, np.float32)
    lib().eeo_e4m3_to_f32_array(ctypes.c_int64(q.size), _p(q), _p(out))
    return out


def f32_to_e4m3(x):
    x = np.ascontiguousarray(x, np.float32)
    out = np.empty(x.shape, np.uint8)
    lib().eeo_f32_to_e4m3_array(ctypes.c_int64(x.size), _p(x), _p(out))
    return out


def quantize_e4m3(x_bf16_bits, group=128):
    """Quantise-on-dispatch definition: bf16 bits [T,H] -> (codes uint8 [T,H], scale f32 [T,H/group])."""
    x = np.ascontiguousarray(x_bf16_bits, np.uint16)
    T, H = x.shape
    q = np.empty((T, H), np.uint8)
    scale = np.empty((T, H // group), np.float32)
    lib().eeo_quantize_e4m3(T, H, group, _p(x), _p(q), _p(scale))
    return q, scale


def step_layout(topk_idx, p2l, active, E, R, S, S_prim, policy):
    """O1-O5 in one call -> dict with slot_of, counters and every layout array."""
    off, lst = tables(p2l, E, S, S_prim)
    slot_of, n_unc, n_msk = map_pairs(topk_idx, off, lst, active, E, S, policy)
    lay = layout(slot_of, R, S)
    lay.update(slot_of=slot_of, n_uncovered=n_unc, n_masked=n_msk, l2p_off=off, l2p_list=lst,
               N=int(lay["offset"][-1]))
    return lay
