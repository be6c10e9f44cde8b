#!/usr/bin/env python3
"""Benchmark of the dispatch/combine hot path on ONE MI355X.

A step = eep_dispatch_layout + eep_dispatch + eep_combine over one synthetic
DeepSeek-V3-shaped decode batch (T=4096 tokens of 32 virtual ranks, hidden 7168
bf16, 256 experts, top-8, 8+1 slots per rank, all ranks live, identity expert:
y aliases the receive buffer).  Inputs are resident in HBM before timing starts.

Prints ONE JSON line.  `value` is achieved GB/s = algorithmic bytes per step /
time per step; `ms_per_step` carries the latency.  `roofline` describes the
dominant kernel against the 8 TB/s HBM peak, `cpu_baseline` is the CPU oracle
timed on this machine's host cores on the same workload.
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs, each scaled by the
# same counter's reading for the 512 MiB k_calibration_copy.  The file is written by
# `bench.py --traffic-from FETCH.csv WRITE.csv --workload W` when the counters are
# refreshed and records a hash of the kernel sources it was measured with; figures taken
# with other sources are not reported.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")
CALIB_BYTES = 512 << 20
STAGE_KERNELS = {"dispatch": ("k_pack", "k_pack_multi", "k_pack_quant", "k_scale_rows"),
                 "combine": ("k_combine",)}


def source_hash():
    """Hash of the HIP sources that hold every kernel of the step (layout.hip, data.hip); the
    built .so travels with them."""
    import hashlib
    h = hashlib.sha256()
    for name in ("data.hip", "layout.hip"):
        h.update(name.encode())
        h.update(open(os.path.join(ROOT, "paper_2605_10670_amd", "csrc", name), "rb").read())
    return h.hexdigest()[:16]


def load_traffic(workload):
    """{stage: HBM bytes per launch} measured with the current sources, or {}."""
    try:
        entry = json.load(open(TRAFFIC_FILE))["workloads"][workload]
    except (OSError, KeyError, ValueError):
        return {}
    if entry.get("source_hash") != source_hash():
        return {}
    return {st: v["fetch_bytes"] + v["write_bytes"] for st, v in entry["stages"].items()}


def write_traffic(workload, fetch_csv, write_csv):
    """Turn two rocprofv3 --pmc counter_collection.csv files (FETCH_SIZE, WRITE_SIZE; runs of
    `bench.py --calib --mode eager`) into the workload's entry of profiles/hbm_traffic.json."""
    import csv
    import re

    def per_kernel(path, counter):
        acc = {}
        for row in csv.DictReader(open(path)):
            if row["Counter_Name"] != counter:
                continue
            m = re.search(r"eep::(k_\w+)", row["Kernel_Name"])
            if m:
                a = acc.setdefault(m.group(1), [0, 0.0])
                a[0] += 1
                a[1] += float(row["Counter_Value"])
        return acc

    fetch, write = per_kernel(fetch_csv, "FETCH_SIZE"), per_kernel(write_csv, "WRITE_SIZE")
    scale = {}
    for name, acc in (("FETCH_SIZE", fetch), ("WRITE_SIZE", write)):
        n, total = acc["k_calibration_copy"]
        scale[name] = (CALIB_BYTES / 1024) / (total / n)      # true KiB per counted KiB
    stages = {}
    for stage, kernels in STAGE_KERNELS.items():
        steps = max(fetch.get("k_combine", [1])[0], 1)          # one combine launch per step
        kib = lambda acc: sum(acc[k][1] for k in kernels if k in acc) / steps
        stages[stage] = {"fetch_bytes": round(kib(fetch) * scale["FETCH_SIZE"] * 1024),
                         "write_bytes": round(kib(write) * scale["WRITE_SIZE"] * 1024),
                         "kernels": sorted(k for k in kernels if k in fetch)}
    try:
        doc = json.load(open(TRAFFIC_FILE))
    except (OSError, ValueError):
        doc = {"workloads": {}}
    doc["workloads"][workload] = {"source_hash": source_hash(), "counter_scale": scale,
                                  "stages": stages}
    json.dump(doc, open(TRAFFIC_FILE, "w"), indent=1, sort_keys=True)
    print(json.dumps(doc["workloads"][workload]))


def algorithmic_bytes(T, k, H, x_bytes, y_bytes, out_bytes, scale_row_bytes=0):
    """Bytes the method must move per step: read each token row once and write
    one row per routed pair (dispatch); read each expert-output row once and
    write each token row once (combine); plus the per-pair metadata."""
    pairs = T * k
    dispatch = T * (H * x_bytes + scale_row_bytes) + pairs * (H * x_bytes + scale_row_bytes)
    combine = pairs * H * y_bytes + T * H * out_bytes
    # layout: read topk_idx, write slot_of/row_of/src_of; dispatch+combine: read row_of, topk_w
    meta = pairs * 4 * 4 + pairs * 4 * 3
    return dict(dispatch=dispatch + pairs * 4, combine=combine + pairs * 8, layout=pairs * 16,
                total=dispatch + combine + meta)


def time_events(stream, fn, reps):
    import torch
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(reps):
        fn()
    e1.record(stream)
    e1.synchronize()
    return e0.elapsed_time(e1) / reps  # ms


def streaming_yardsticks(stream, plane_d, plane_c):
    """What the memory system gives the step's two read:write mixes when nothing is scattered:
    perfectly sequential kernels (eep_calibration_stream: same loads and stores as pack and
    combine) that read one plane of plane_d bytes and write eight (dispatch's mix), read eight
    planes of plane_c bytes and write one (combine's mix), each looped alone and the two
    alternating as in a step (x -> receive rows -> out), plus a copy of 512 MiB."""
    import torch
    from paper_2605_10670_amd import binding
    pad = 4368 * 16                      # keeps the planes from being a power of two apart
    stride = max(plane_d, plane_c) + pad
    size = max(8 * stride, 512 << 20)
    a = torch.ones(size, dtype=torch.uint8, device="cuda")
    b = torch.zeros(size, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    d_mix = lambda: binding.calibration_stream(b, a, plane_d, stride, 1, 8, stream)
    c_mix = lambda: binding.calibration_stream(a, b, plane_c, stride, 8, 1, stream)
    copy = lambda: binding.calibration_stream(b, a, 512 << 20, 512 << 20, 1, 1, stream)

    def pair():
        d_mix()
        c_mix()

    out = {}
    for name, fn, nbytes in (("copy_512MiB", copy, 2 * (512 << 20)), ("read1_write8", d_mix, 9 * plane_d),
                             ("read8_write1", c_mix, 9 * plane_c),
                             ("read1_write8_then_read8_write1", pair, 9 * (plane_d + plane_c))):
        for _ in range(3):
            fn()
        us = time_events(stream, fn, 16) * 1e3
        out[name] = {"us": us, "bytes": nbytes, "gbs": nbytes / us / 1e3,
                     "frac_of_hbm_peak": nbytes / us / 1e3 / HBM_PEAK_GBS}
    del a, b
    return out


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(wl, bytes_total, quant=False, budget_s=12.0):
    """The oracle as it stands on the same workload: the same three calls as the GPU step
    (layout, pack, combine; y comes from outside).  Two legs: one thread, and the row copies
    and the combine split over the host cores by token range (threads around the same C
    functions, which release the interpreter lock; the layout stays serial)."""
    import concurrent.futures as cf
    import numpy as np
    import oracle
    ydt = oracle.BF16 if wl.y_dtype == "bf16" else oracle.F32
    T = wl.T
    y_ext = None
    if wl.stub != "identity":   # expert stand-in output, prepared outside the timed region like on the GPU
        y_ext = np.zeros((T * wl.k, wl.H), np.uint16 if wl.y_dtype == "bf16" else np.float32)
    cores = max(1, min(16, len(os.sched_getaffinity(0))))

    def one_step(pool, workers):
        lay = oracle.step_layout(wl.topk_idx, wl.p2l, wl.active, wl.E, wl.R, wl.S, wl.S_prim,
                                 oracle.SPREAD)
        rows = lay["row_of"]
        bounds = [T * i // workers for i in range(workers + 1)]
        ranges = [(a, b) for a, b in zip(bounds, bounds[1:]) if b > a]
        x, xs = wl.x, wl.x_scale
        if quant:
            q_sc = list(pool.map(lambda r: oracle.quantize_e4m3(wl.x[r[0]:r[1]], 128), ranges))
            x = np.concatenate([q for q, _ in q_sc])
            xs = np.concatenate([sc for _, sc in q_sc])
        recv = np.empty((T * wl.k,) + x.shape[1:], x.dtype)
        list(pool.map(lambda r: oracle.pack_into(x[r[0]:r[1]], rows[r[0]:r[1]], recv), ranges))
        if xs is not None:
            rs = np.empty((T * wl.k,) + xs.shape[1:], xs.dtype)
            list(pool.map(lambda r: oracle.pack_into(xs[r[0]:r[1]], rows[r[0]:r[1]], rs), ranges))
        y = recv if y_ext is None else y_ext
        list(pool.map(lambda r: oracle.combine(y, ydt, wl.topk_w[r[0]:r[1]], rows[r[0]:r[1]]),
                      ranges))

    def leg(workers):
        with cf.ThreadPoolExecutor(workers) as pool:
            one_step(pool, workers)                 # warm-up (page faults of the big buffers)
            times, t_all = [], time.perf_counter()
            while len(times) < 3 or (time.perf_counter() - t_all < budget_s and len(times) < 10):
                t0 = time.perf_counter()
                one_step(pool, workers)
                times.append(time.perf_counter() - t0)
        med = statistics.median(times)
        return {"value": bytes_total / med / 1e9, "unit": "GB/s", "cores": workers,
                "ms_per_step": med * 1e3,
                "sample": f"{len(times)} full {wl.name} steps (T={T}), median"}

    single = leg(1)
    out = leg(cores) if cores > 1 else dict(single)
    out.update({"kind": "oracle", "cpu_model": cpu_model(), "host_cpus": os.cpu_count(),
                "single_thread": single,
                "note": "layout serial; row copies and combine split over `cores` threads by "
                        "token range"})
    return out


WORKLOADS = {
    "tiny": ("tiny CPU-checkable step: T=128, H=1024 fp32, E=16, top-2, R=4 x (4+2) slots, rank 2 failed "
             "and remapped, per-expert scalar stand-in (launch-latency-bound)"),
    "decode": ("dsv3-decode: T=4096 (32 ranks x 128), H=7168 bf16, E=256, top-8, 8+1 slots/rank, "
               "all live, identity expert"),
    "decode_failed_zipf": ("dsv3-decode, rank 13 failed and remapped to redundant slots, "
                           "Zipf(1.2)-skewed logits: T=4096, H=7168 bf16, E=256, top-8"),
    "prefill_fp8": ("dsv3-prefill: T=16384, H=7168 fp8 e4m3 + fp32 scale/128 dispatch, bf16 combine, "
                    "E=256, top-8, ranks 7 and 20 failed"),
    "decode_quant": ("dsv3-decode with quantise-on-dispatch: T=4096, H=7168, bf16 tokens -> fp8 e4m3 "
                     "+ fp32 scale/128 receive rows (eep_dispatch_quant), bf16 combine, all live"),
    "decode_dedup": ("dsv3-decode with de-duplicated dispatch: T=4096, H=7168 bf16, one row per (token, "
                     "destination rank) (eep_dedup_layout + eep_dispatch_dedup); the expert stage is "
                     "taken to gather through expand_of, y prepared once by eep_expand, untimed"),
    "decode_double_buffer": ("dsv3-decode with double-buffered staging: two micro-batches of T=4096 "
                             "(H=7168 bf16, E=256, top-8, all live) alternate through two staging sets "
                             "(eep_create_staging); the dispatch side of one runs on a side stream beside "
                             "the combine of the other (eep_staging_fork / eep_staging_join); a pass of 8 "
                             "steps is one hipGraph, drained at both ends"),
    "churn": "qwen3-moe-like: T=2048, H=4096 bf16, E=128, top-8, R=16, 8+1 slots/rank, all live",
    "repair": ("weight movement after a rank failure (eep_apply_repair; not the hot path): 32 ranks "
               "x (8+2) slots, one redundant slot empty, E=256, 44 MB per expert (three 7168x2048 "
               "fp8 matrices), rank 13 fails; backup in pinned host memory"),
    "repair_scales": ("weight movement vs failure scale (the one-GPU analogue of the paper's recovery "
                      "breakdown, Sec. 6.3): 32 ranks x (8+8) slots, experts 0-3 of every rank "
                      "replicated once, four redundant slots per rank empty, E=256, 44 MB per expert; "
                      "1, 2, 4, 8, 16 failed ranks; backup in pinned host memory"),
}
BYTES_OF = {"f32": 4, "bf16": 2, "fp8": 1}


def bench_repair(args, stream, copy_gbs):
    """Times eep_apply_repair per source tier: the peer copies (HBM to HBM here; xGMI
    in a real deployment), the reloads from the pinned-host backup (PCIe), and the
    whole planned batch in one launch."""
    import numpy as np
    import torch
    from paper_2605_10670_amd import binding, synth

    R, S_prim, S, E = 32, 8, 10, 256
    slot_bytes = 3 * 7168 * 2048
    p2l = np.full((R, S), -1, np.int32)
    p2l[:, :S_prim + 1] = synth.preferred_placement(R, S_prim, 1).reshape(R, -1)
    p2l = p2l.ravel().copy()
    dead = synth.active_mask(R, (13,))
    plan = binding.plan_repair(p2l, dead, R, S, S_prim, E)
    assert plan["unplaced"] == 0
    weights = torch.empty((R * S, slot_bytes), dtype=torch.uint8, device="cuda")
    backup = torch.empty((E, slot_bytes), dtype=torch.uint8, pin_memory=True)
    ctx = binding.Context(num_ranks=R, slots_per_rank=S, primary_slots=S_prim, num_logical=E,
                          max_tokens=R, topk=8, hidden=64, strict_coverage=False)

    def subset(keep):
        sub = {key: np.array(plan[key], copy=True) for key in ("p2l", "kind", "src_slot")}
        drop = np.isin(plan["kind"], (binding.SRC_PEER, binding.SRC_DRAM)) & (plan["kind"] != keep)
        sub["kind"][drop], sub["src_slot"][drop], sub["p2l"][drop] = binding.SRC_NONE, -1, p2l[drop]
        return sub

    def timed(pl, reps):
        times = []
        for _ in range(reps + 1):
            ctx.update_placement(p2l, stream)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            ctx.apply_repair(weights, backup, slot_bytes, pl, stream)
            e1.record(stream)
            e1.synchronize()
            times.append(e0.elapsed_time(e1))
        return statistics.median(times[1:])

    n_peer, n_dram = plan["peer"], plan["dram"]
    reps = max(1, min(args.steps, 20))
    ms_peer = timed(subset(binding.SRC_PEER), reps)
    ms_dram = timed(subset(binding.SRC_DRAM), reps)
    ms_all = timed(plan, reps)
    moved = (n_peer + n_dram) * slot_bytes
    print(json.dumps({
        "metric": "repair_weight_move_gbs", "value": round(moved / (ms_all * 1e-3) / 1e9, 2),
        "unit": "GB/s", "n_gpus": 1, "steps": reps, "warmup": 1, "ms_per_step": round(ms_all, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u8",
        "data": "synthetic", "config": {"workload": WORKLOADS["repair"]},
        "plan": {"local": plan["local"], "peer": n_peer, "dram": n_dram,
                 "mb_per_expert": round(slot_bytes / 1e6, 2)},
        "peer_tier": {"ms": round(ms_peer, 4), "moved_gbs": round(n_peer * slot_bytes / ms_peer / 1e6, 1),
                      "hbm_read_plus_write_gbs": round(2 * n_peer * slot_bytes / ms_peer / 1e6, 1),
                      "copy_ceiling_gbs": round(copy_gbs, 1)},
        "dram_tier": {"ms": round(ms_dram, 4), "moved_gbs": round(n_dram * slot_bytes / ms_dram / 1e6, 1),
                      "note": "kernel reads pinned host memory over the host link"},
    }))
    ctx.destroy()


def bench_double_buffer(args, stream, copy_gbs):
    """Two staging sets, dispatch of one micro-batch beside the combine of the other, against
    the same 8 steps queued one after the other on one stream."""
    import numpy as np
    import torch
    from paper_2605_10670_amd import binding, synth

    wls = [synth.decode(seed_offset=2), synth.decode(seed_offset=12)]
    wl = wls[0]
    T, k, H = wl.T, wl.k, wl.H
    side = torch.cuda.Stream()
    ctx = [binding.Context(num_ranks=wl.R, slots_per_rank=wl.S, primary_slots=wl.S_prim,
                           num_logical=wl.E, max_tokens=T, topk=k, hidden=H)]
    ctx.append(ctx[0].staging())
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a).view(np.int16)
                                     if a.dtype == np.uint16 else np.ascontiguousarray(a)).cuda()
    idx, w, x = ([dev(getattr(v, n)) for v in wls] for n in ("topk_idx", "topk_w", "x"))
    recv = [torch.empty((T * k, H), dtype=torch.int16, device="cuda") for _ in range(2)]
    out = [torch.empty((T, H), dtype=torch.int16, device="cuda") for _ in range(2)]
    ctx[0].update_placement(wl.p2l, stream)
    ctx[0].set_membership(wl.active, stream)
    steps_per_pass = 8

    def d_side(s, st):
        ctx[s].dispatch_layout(idx[s], T, st)
        ctx[s].dispatch(x[s], recv[s], T, stream=st)

    def c_side(s):
        ctx[s].combine(recv[s], w[s], out[s], T, stream)

    def overlapped():
        d_side(0, stream)
        for i in range(steps_per_pass):
            s, nxt = i % 2, (i + 1) % 2
            last = i + 1 == steps_per_pass
            if not last:
                ctx[nxt].staging_fork(idx[nxt], x[nxt], recv[nxt], T, stream, side)
            c_side(s)
            if not last:
                ctx[nxt].staging_join(stream, side)

    def sequential():
        for i in range(steps_per_pass):
            d_side(i % 2, stream)
            c_side(i % 2)

    result = {}
    for name, fn in (("sequential", sequential), ("overlapped", overlapped)):
        fn()
        stream.synchronize()
        ctx[0].graph_begin(stream)
        fn()
        g = ctx[0].graph_end(stream)
        for _ in range(max(1, args.warmup // steps_per_pass)):
            g.launch(stream)
        stream.synchronize()
        n_rep = max(25, args.steps // steps_per_pass)
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(n_rep)]
        for e in ev:
            e[0].record(stream)
            g.launch(stream)
            e[1].record(stream)
        stream.synchronize()
        per = sorted(e[0].elapsed_time(e[1]) * 1e3 / steps_per_pass for e in ev)
        result[name] = {"p10": per[n_rep // 10], "p50": per[n_rep // 2], "p90": per[(n_rep * 9) // 10],
                        "replays": n_rep}
        g.destroy()
    nbytes = algorithmic_bytes(T, k, H, 2, 2, 2)["total"]
    us = result["overlapped"]["p50"]
    print(json.dumps({
        "metric": "dispatch+combine achieved HBM GB/s (algorithmic bytes / step time), "
                  "decode_double_buffer", "value": nbytes / us / 1e3, "unit": "GB/s", "n_gpus": 1,
        "steps": result["overlapped"]["replays"] * steps_per_pass, "warmup": args.warmup,
        "ms_per_step": us / 1e3, "us_per_step": us, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": WORKLOADS["decode_double_buffer"], "mode": "graph",
                   "steps_per_graph": steps_per_pass, "algorithmic_bytes_per_step": nbytes},
        "frac_of_hbm_peak": nbytes / us / 1e3 / HBM_PEAK_GBS, "copy_ceiling_gbs": copy_gbs,
        "overlapped_us_per_step": result["overlapped"],
        "sequential_us_per_step": result["sequential"]}))
    ctx[1].destroy()
    ctx[0].destroy()


def bench_repair_scales(args, stream):
    """Plan + carry out the repair for 1..16 failed ranks of 32: which tier the weights come
    from and how long planning (host) and moving (GPU) take."""
    import numpy as np
    import torch
    from paper_2605_10670_amd import binding, synth

    R, S_prim, S_red, E = 32, 8, 8, 256
    S = S_prim + S_red
    slot_bytes = 3 * 7168 * 2048
    pref = synth.preferred_placement(R, S_prim, S_red).reshape(R, S)
    pref[:, 12:] = -1
    pref = pref.ravel().copy()
    order = np.random.default_rng(0).permutation(R)
    weights = torch.empty((R * S, slot_bytes), dtype=torch.uint8, device="cuda")
    backup = torch.empty((E, slot_bytes), dtype=torch.uint8, pin_memory=True)
    ctx = binding.Context(num_ranks=R, slots_per_rank=S, primary_slots=S_prim, num_logical=E,
                          max_tokens=R, topk=8, hidden=64)
    rows = []
    for n_failed in (1, 2, 4, 8, 16):
        dead = synth.active_mask(R, order[:n_failed])
        ctx.update_placement(pref, stream)
        ctx.set_membership(np.ones(R, np.int32), stream)
        stream.synchronize()
        t0 = time.perf_counter()
        plan = binding.plan_repair(pref, dead, R, S, S_prim, E)
        plan_ms = (time.perf_counter() - t0) * 1e3
        assert plan["unplaced"] == 0
        times = []
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            ctx.apply_repair(weights, backup, slot_bytes, plan, stream)
            ctx.set_membership(dead, stream)            # placement first, then the mask
            e1.record(stream)
            e1.synchronize()
            times.append(e0.elapsed_time(e1))
            ctx.set_membership(np.ones(R, np.int32), stream)     # rejoin: mask, then placement
            ctx.update_placement(pref, stream)
        move_ms = statistics.median(times)
        moved = (plan["peer"] + plan["dram"]) * slot_bytes
        rows.append({"failed_ranks": n_failed, "local": plan["local"], "peer": plan["peer"],
                     "dram": plan["dram"],
                     "dram_share": round(plan["dram"] / max(1, plan["dram"] + plan["peer"]), 3),
                     "plan_ms_host": round(plan_ms, 3), "move_and_publish_ms": round(move_ms, 3),
                     "moved_mb": round(moved / 1e6, 1),
                     "moved_gbs": round(moved / (move_ms * 1e-3) / 1e9, 1)})
    print(json.dumps({
        "metric": "repair_move_ms_by_failure_scale", "value": rows[0]["move_and_publish_ms"],
        "unit": "ms", "n_gpus": 1, "steps": 3, "warmup": 0,
        "ms_per_step": rows[0]["move_and_publish_ms"], "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": WORKLOADS["repair_scales"]}, "scales": rows}))
    ctx.destroy()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--mode", choices=["graph", "eager"], default="graph",
                    help="replay a captured hipGraph of the step (default) or launch eagerly")
    ap.add_argument("--steps-per-graph", type=int, default=8,
                    help="steps captured into one hipGraph (a decode forward pass holds one such "
                         "step per MoE layer in a single graph); reduced to a divisor of --steps")
    ap.add_argument("--workload", choices=sorted(WORKLOADS), default="decode",
                    help="decode (default) is the configuration the headline metric is quoted on")
    ap.add_argument("--tokens", type=int, default=0,
                    help="decode workloads only: batch size T (a multiple of 32) instead of 4096, "
                         "e.g. 32..256 for the low-concurrency decode regime")
    ap.add_argument("--detect", action="store_true",
                    help="switch GPU-side failure detection on (1 s timeout as in the paper): adds "
                         "the signal kernel after dispatch and the bounded wait before combine")
    ap.add_argument("--isolated", action="store_true",
                    help="also time dispatch alone and combine alone in loops of their own (out of "
                         "sequence: inside a step part of what dispatch writes is still draining "
                         "to HBM while combine runs, so the split between the two differs)")
    ap.add_argument("--stage-only", choices=["dispatch", "combine"],
                    help="for counter runs: after one whole step, launch only this stage --steps "
                         "times (out of sequence) and print its mean time; nothing else is measured")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline")
    ap.add_argument("--no-yardsticks", action="store_true",
                    help="skip the sequential streaming kernels with the step's read:write mixes")
    ap.add_argument("--calib", action="store_true",
                    help="first launch 5 plain copy kernels of 512 MiB (k_calibration_copy), the "
                         "yardstick for rocprofv3 FETCH_SIZE / WRITE_SIZE counters")
    ap.add_argument("--traffic-from", nargs=2, metavar=("FETCH_CSV", "WRITE_CSV"),
                    help="no GPU work: read two rocprofv3 --pmc counter_collection.csv files "
                         "(FETCH_SIZE run, WRITE_SIZE run, both of `--calib --mode eager` for "
                         "--workload) and record the HBM bytes per launch in profiles/hbm_traffic.json")
    args = ap.parse_args()
    if args.traffic_from:
        return write_traffic(args.workload, *args.traffic_from)
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (virtual EP ranks share one HBM); "
                 "use --gpus 1")

    import numpy as np
    import torch
    from paper_2605_10670_amd import binding, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    stream = torch.cuda.Stream()

    # plain-copy ceiling of this GPU (and, with --calib, the counters' yardstick)
    a = torch.ones(512 << 20, dtype=torch.uint8, device="cuda")
    b = torch.empty_like(a)
    torch.cuda.synchronize()
    copy = lambda: binding.calibration_copy(b, a, a.numel(), stream)
    for _ in range(5 if args.calib else 2):
        copy()
    stream.synchronize()
    copy_gbs = 2 * a.numel() / (time_events(stream, copy, 10) * 1e-3) / 1e9
    del a, b

    if args.workload == "repair":
        return bench_repair(args, stream, copy_gbs)
    if args.workload == "repair_scales":
        return bench_repair_scales(args, stream)
    if args.workload == "decode_double_buffer":
        return bench_double_buffer(args, stream, copy_gbs)

    quant = args.workload == "decode_quant"
    dedup = args.workload == "decode_dedup"
    if args.workload in ("decode", "decode_quant", "decode_dedup"):
        wl = synth.decode(T=args.tokens) if args.tokens else synth.decode()
        if quant:   # receive rows are fp8 + scales; the stand-in dequantises them once, untimed
            wl.x_dtype, wl.stub = "fp8", "dequant"
    elif args.workload == "decode_failed_zipf":
        wl = synth.decode_failed_zipf()
    elif args.workload == "prefill_fp8":
        wl = synth.prefill_fp8()
    elif args.workload == "tiny":
        wl = synth.tiny("c")
    else:
        wl = synth.churn_inputs(1)[0]
        wl.stub = "identity"
    T, k, H = wl.T, wl.k, wl.H
    scale_row = (H // 128) * 4 if (wl.x_scale is not None or quant) else 0
    nbytes = algorithmic_bytes(T, k, H, BYTES_OF[wl.x_dtype], BYTES_OF[wl.y_dtype],
                               BYTES_OF[wl.out_dtype], scale_row)
    if quant:   # the token rows are read as bf16 (2 B) and carry no scales on the way in
        delta = T * H * (2 - 1) - T * scale_row
        nbytes["dispatch"] += delta
        nbytes["total"] += delta

    ctx = binding.Context(num_ranks=wl.R, slots_per_rank=wl.S, primary_slots=wl.S_prim,
                          num_logical=wl.E, max_tokens=T, topk=k, hidden=H, x_dtype=wl.x_dtype,
                          y_dtype=wl.y_dtype, out_dtype=wl.out_dtype)

    def dev(arr):
        arr = np.ascontiguousarray(arr)
        return torch.from_numpy(arr.view(np.int16) if arr.dtype == np.uint16 else arr).cuda()

    tdt = {"f32": torch.float32, "bf16": torch.int16, "fp8": torch.uint8}
    idx, w, x = dev(wl.topk_idx), dev(wl.topk_w), dev(wl.x)
    x_scale = dev(wl.x_scale) if wl.x_scale is not None else None
    recv = torch.empty((T * k, H), dtype=tdt[wl.x_dtype], device="cuda")
    recv_scale = (torch.empty((T * k, H // 128), dtype=torch.float32, device="cuda")
                  if (x_scale is not None or quant) else None)
    # identity expert: y aliases the receive buffer; otherwise the stand-in fills y once, untimed
    y = (recv if wl.stub == "identity" and not dedup else
         torch.empty((T * k, H), dtype=tdt[wl.y_dtype], device="cuda"))
    out = torch.empty((T, H), dtype=tdt[wl.out_dtype], device="cuda")
    torch.cuda.synchronize()
    ctx.update_placement(wl.p2l, stream)
    ctx.set_membership(wl.active, stream)

    def layout():
        ctx.dispatch_layout(idx, T, stream)
        if dedup:
            ctx.dedup_layout(T, stream)

    def dispatch():
        if dedup:       # recv holds the rank-major, de-duplicated rows
            ctx.dispatch_dedup(x, recv, T, stream)
        elif quant:
            ctx.dispatch_quant(x, recv, recv_scale, T, stream)
        else:
            ctx.dispatch(x, recv, T, x_scale, recv_scale, stream)

    def combine():
        ctx.combine(y, w, out, T, stream=stream)

    if args.detect:
        ctx.set_detection(1_000_000_000)

    def step():
        layout()
        dispatch()
        if args.detect:   # the expert stage (here: nothing) announces its outputs
            ctx.signal_experts_done(stream)
        combine()

    layout()
    dispatch()
    if dedup:           # expansion on the destination, once, untimed: y = expert-major rows
        ctx.expand(recv, y, T, stream)
    elif wl.stub != "identity":
        ctx.expert_stub(wl.stub, recv, y, T, recv_scale=recv_scale,
                        expert_scale=dev(wl.expert_scale) if wl.expert_scale is not None else None,
                        stream=stream)
    elif args.detect:
        ctx.signal_experts_done(stream)
    combine()
    stream.synchronize()
    if args.stage_only:
        fn = dispatch if args.stage_only == "dispatch" else combine
        for _ in range(args.warmup):
            fn()
        us = time_events(stream, fn, args.steps) * 1e3
        print(json.dumps({"workload": args.workload, "stage_only": args.stage_only,
                          "steps": args.steps, "us_per_launch": us}))
        ctx.destroy()
        return
    dedup_info = None
    if dedup:           # one row per (token, rank): N_d rows are written instead of N
        n_d = ctx.read_dedup(T, stream)["N_d"]
        delta = (n_d - T * k) * H * BYTES_OF[wl.x_dtype]
        nbytes["dispatch"] += delta
        nbytes["total"] += delta
        dedup_info = {"rows_expert_major": T * k, "rows_dedup": n_d,
                      "expand_us": time_events(stream, lambda: ctx.expand(recv, y, T, stream), 20) * 1e3}
    graph = None
    spg = 1
    if args.mode == "graph":
        import math
        spg = math.gcd(max(1, args.steps_per_graph), args.steps) if args.steps > 0 else 1
        ctx.graph_begin(stream)
        for _ in range(spg):
            step()
        graph = ctx.graph_end(stream)
        run = lambda: graph.launch(stream)
    else:
        run = step

    for _ in range(-(-args.warmup // spg)):
        run()
    stream.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ms = time_events(stream, run, args.steps // spg) / spg     # exactly args.steps steps
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps

    # distribution over individually timed replays (an event pair around each)
    replay_pct = None
    if graph is not None:
        n_rep = max(200, args.steps // spg)
        rev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(n_rep)]
        for e in rev:
            e[0].record(stream)
            run()
            e[1].record(stream)
        stream.synchronize()
        per = sorted(e[0].elapsed_time(e[1]) * 1e3 / spg for e in rev)
        replay_pct = {"replays": n_rep, "p10": per[n_rep // 10], "p50": per[n_rep // 2],
                      "p90": per[(n_rep * 9) // 10]}

    # Per-call durations inside whole steps (eager launches, HIP events recorded on
    # the launch stream between the calls), so that every launch of a kernel in
    # this process happens in the same context: after the previous stage of a step.
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    for e in ev:
        e[0].record(stream)
        layout()
        e[1].record(stream)
        dispatch()
        if args.detect:
            ctx.signal_experts_done(stream)
        e[2].record(stream)
        combine()
        e[3].record(stream)
    stream.synchronize()
    stage_ms = {name: sum(e[i].elapsed_time(e[i + 1]) for e in ev) / len(ev)
                for i, name in enumerate(("layout", "dispatch", "combine"))}
    # what two consecutive event records measure with no kernel between them (reported for
    # information; between two kernels a record costs less than this)
    gap_ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
    for e in gap_ev:
        step()          # a whole step, so that no kernel is ever launched out of sequence
        e[0].record(stream)
        e[1].record(stream)
    stream.synchronize()
    event_gap_ms = sum(e[0].elapsed_time(e[1]) for e in gap_ev) / len(gap_ev)
    per_step = sorted(e[0].elapsed_time(e[3]) * 1e3 for e in ev)
    pct = lambda q: per_step[min(len(per_step) - 1, int(q * len(per_step)))]
    other_ms = time_events(stream, step, args.steps)   # eager steps, no inner events
    isolated = None
    if args.isolated:
        isolated = {"dispatch": time_events(stream, dispatch, args.steps) * 1e3,
                    "combine": time_events(stream, combine, args.steps) * 1e3}
    if graph is not None:
        graph.destroy()

    # A handful of replays is a noisy clock: with fewer than 50 timed replays the headline is
    # the median of the individually timed replays above (>= 200 of them); the mean over
    # exactly --steps steps is reported beside it.
    timed_ms = ms
    timed_replays = args.steps // spg if graph is not None else args.steps
    if replay_pct is not None and timed_replays < 50:
        ms = replay_pct["p50"] / 1e3
    traffic = load_traffic(args.workload) if not args.tokens else {}
    kernel_of = {"dispatch": "k_pack_quant" if quant else "k_pack", "combine": "k_combine"}
    # (with de-duplication the layout stage holds four launches and the dispatch stage k_pack)
    event_cost_ms = max(0.0, (sum(stage_ms.values()) - other_ms) / 3)
    kernels = {}
    for stage, kname in kernel_of.items():
        # launch duration = event-to-event time of the stage minus the cost of the event record
        # that sits between two calls, estimated in the same run as (sum of the three stage
        # times - time of an eager step without inner events) / 3; agrees with rocprofv3's
        # kernel durations to within 0.5 % (profiles/).  With an fp8 payload the dispatch
        # stage is the payload kernel plus the small k_scale_rows launch.
        launch_ms = stage_ms[stage] - event_cost_ms
        gbs = nbytes[stage] / (launch_ms * 1e-3) / 1e9
        kernels[kname] = {"avg_launch_us": launch_ms * 1e3,
                          "algorithmic_bytes_per_launch": nbytes[stage], "achieved": gbs,
                          "frac": gbs / HBM_PEAK_GBS,
                          "traffic": traffic.get(stage)}
    dom = max(kernels, key=lambda n: kernels[n]["avg_launch_us"])
    result = {
        "metric": "dispatch+combine achieved HBM GB/s (algorithmic bytes / step time), "
                  + ("DSV3 decode shape" if args.workload == "decode" else args.workload),
        "value": nbytes["total"] / (ms * 1e-3) / 1e9,
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "us_per_step": ms * 1e3,
        "ms_per_step_is": ("median of %d individually timed graph replays" % replay_pct["replays"]
                           if ms != timed_ms else "mean over exactly --steps steps"),
        "timed_ms_per_step": timed_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"f32": "f32", "bf16": "bf16", "fp8": "u8"}[wl.x_dtype], "data": "synthetic",
        "config": {"workload": WORKLOADS[args.workload] if not args.tokens else
                   WORKLOADS[args.workload].replace("T=4096 (32 ranks x 128)", f"T={args.tokens}")
                   .replace("T=4096", f"T={args.tokens}"), "mode": args.mode,
                   "steps_per_graph": spg if args.mode == "graph" else None,
                   "failure_detection": bool(args.detect), "step": "dispatch_layout + dispatch + combine",
                   "algorithmic_bytes_per_step": nbytes["total"]},
        "frac_of_hbm_peak": nbytes["total"] / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "wall_ms_per_step": wall_ms,
        "copy_ceiling_gbs": copy_gbs,
        "frac_of_copy_ceiling": nbytes["total"] / (ms * 1e-3) / 1e9 / copy_gbs,
        "stages_us": {n: v * 1e3 for n, v in stage_ms.items()},
        "event_gap_us": event_gap_ms * 1e3, "event_cost_in_sequence_us": event_cost_ms * 1e3,
        "graph_replay_us_per_step": replay_pct,
        "eager_us_per_step": other_ms * 1e3,
        "eager_step_with_events_us": {"p10": pct(0.10), "p50": pct(0.50), "p90": pct(0.90)},
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": kernels[dom]["achieved"],
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": kernels[dom]["frac"],
                     "traffic": kernels[dom]["traffic"],
                     "traffic_source": ("profiles/hbm_traffic.json, sources " + source_hash()
                                        if kernels[dom]["traffic"] else None),
                     "algorithmic_bytes_per_launch": kernels[dom]["algorithmic_bytes_per_launch"],
                     "avg_launch_us": kernels[dom]["avg_launch_us"]},
        "kernels": kernels,
    }
    if isolated is not None:
        result["isolated_us"] = isolated
    if k == 8 and not args.no_yardsticks:
        # same byte counts as the two data stages, perfectly sequential (no permutation)
        result["streaming_yardsticks"] = streaming_yardsticks(
            stream, nbytes["dispatch"] // 9 // 16 * 16, nbytes["combine"] // 9 // 16 * 16)
    if dedup_info is not None:
        result["dedup"] = dedup_info
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(wl, nbytes["total"], quant)
    ctx.destroy()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
