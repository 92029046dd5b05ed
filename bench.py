#!/usr/bin/env python3
"""Benchmark of the RaggedShard / DBuffer hot path on one MI355X.

A step is one pass of the whole path over the Llama-3-8B-shaped workload (W = 64, 128x128
FP8 blocks): for each of 32 decoder units back to back
    ragged_pack (per-parameter grads -> DBuffer), shard_reduce over rank 0's shard (64 partials),
    dequant_unpack of the gathered FP8 unit,
then block_quant of rank 0's shard of all 32 units in one batched launch.
All inputs are synthetic and resident in HBM before the timed region.  One JSON line is printed:
whole-step algorithmic GB/s as `value`, per-kernel figures, the roofline of the dominant
kernel (HIP events inside the timed region around the launches of every 4th unit: bracketing
every launch costs ~6 % of the step) and the CPU oracle timed on a bounded sample of the
same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 1..5] [--event-every N] [--no-cpu]
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X HBM3E, published

# HBM bytes per launch on the default workload, from two rocprofv3 --pmc runs (FETCH_SIZE, then
# WRITE_SIZE), each scaled by what the counter reads for the plain copy launch of known size
# (fetch x 1.99991, write x 0.99987).  Offline measurements: they cannot be taken inside this
# process, so they are recorded here next to the algorithmic bytes they are compared with.
PMC_TRAFFIC_CONFIG2 = {"ragged_pack": 920.2e6, "shard_reduce": 418.9e6, "block_quant": 319.5e6,
                       "dequant_unpack": 668.5e6}


def algorithmic_bytes(E, W, S, payload_r, nb_r, nb):
    """Bytes each op must move per unit (bf16 = 2, fp32 = 4, fp8 = 1)."""
    return {
        "ragged_pack": 2 * E + 2 * W * S,                    # read every tensor, write the whole DBuffer
        "shard_reduce": 2 * W * payload_r + 4 * S,           # W partials of the payload, fp32 shard out
        "block_quant": 2 * payload_r + S + 4 * nb_r,         # bf16 shard in, codes (padding zeroed) + scales out
        "dequant_unpack": E + 4 * nb + 2 * E,                # codes + scales in, bf16 tensors out
    }


def cpu_baseline(wl, seed=1):
    """The oracle as it stands, on a bounded sample of the workload: one of the 32 units (unit 0,
    all nine tensors) for pack / quant / dequant, and rank 0's whole shard with all W partials for
    reduce (about 10 s of numpy on the GPU machine's host, 30 s on a slow one)."""
    import numpy as np
    from oracle import dbuffer as OD
    from oracle import fp8 as OF
    from oracle import plan as OP
    from workloads import gen_param, gen_partial

    specs = [OP.TensorSpec(t.rows, t.cols, t.mode) for t in wl.tensors]
    plan = OP.make_plan(specs, wl.world, wl.align_bytes, wl.min_itemsize)
    k = len(specs)
    params = [gen_param(wl, seed, t) for t in range(k)]
    total_s = plan.offsets[k - 1] + specs[k - 1].e
    E_s = sum(s.e for s in specs[:k])
    n_red = plan.S
    parts = np.stack([gen_partial(wl, seed, w, n_red) for w in range(wl.world)])
    segs = [(t, so, do, min(n, n_red - do)) for t, so, do, n in plan.rank_segments(wl.rank) if do < n_red]
    payload_red = sum(s[3] for s in segs)

    t0 = time.perf_counter()
    db = OD.ragged_pack(params, plan.offsets[:k], total_s)
    t1 = time.perf_counter()
    OD.shard_reduce(parts, segs)
    t2 = time.perf_counter()
    qs = [OF.quantise_tensor(db[l:l + s.e], s) for s, l in zip(specs[:k], plan.offsets[:k])]
    t3 = time.perf_counter()
    for (c, sc), s in zip(qs, specs[:k]):
        OF.dequantise_tensor(c, sc, s)
    t4 = time.perf_counter()
    nb_s = sum(s.num_blocks for s in specs[:k])
    moved = {
        "ragged_pack": 2 * E_s + 2 * total_s,
        "shard_reduce": 2 * wl.world * payload_red + 4 * n_red,
        "block_quant": 3 * E_s + 4 * nb_s,
        "dequant_unpack": 3 * E_s + 4 * nb_s,
    }
    secs = {"ragged_pack": t1 - t0, "shard_reduce": t2 - t1, "block_quant": t3 - t2, "dequant_unpack": t4 - t3}
    total_bytes, total_s_ = sum(moved.values()), sum(secs.values())
    return {
        "value": round(total_bytes / total_s_ / 1e9, 4),
        "unit": "GB/s",
        "cores": 1,
        "kind": "oracle",
        "sample": (f"unit 0, first {k} tensors ({E_s} of {plan.payload} elements) for pack/quant/dequant; "
                   f"reduce over {wl.world} partials of the first {n_red} elements of rank {wl.rank}'s shard; "
                   f"{total_s_:.1f} s of numpy (single thread)"),
        "per_op_GBps": {k_: round(moved[k_] / secs[k_] / 1e9, 4) for k_ in moved},
    }


def cpu_baseline_all_cores(wl, seed=1):
    """The same sample through the C / OpenMP statement of the oracle on every host core the
    process may use: context for the single-thread numpy figure, not a target."""
    import numpy as np
    from oracle import c_oracle as OC
    from oracle import plan as OP
    from workloads import gen_param, gen_partial

    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    OC.set_num_threads(cores)
    specs = [OP.TensorSpec(t.rows, t.cols, t.mode) for t in wl.tensors]
    plan = OP.make_plan(specs, wl.world, wl.align_bytes, wl.min_itemsize)
    params = [gen_param(wl, seed, t) for t in range(len(specs))]
    parts = np.stack([gen_partial(wl, seed, w, plan.S) for w in range(wl.world)])
    segs = plan.rank_segments(wl.rank)
    payload_red = sum(s[3] for s in segs)
    E = plan.payload

    def shape(s):
        return ((1, s.rows, 1, 128) if s.cols == 0 else
                (s.rows, s.cols, 128, 128) if s.mode == OP.BLOCK_128x128 else (s.rows, s.cols, 1, 128))
    t0 = time.perf_counter()
    db = OC.ragged_pack(params, plan.offsets, plan.total)
    t1 = time.perf_counter()
    OC.shard_reduce(parts, segs)
    t2 = time.perf_counter()
    q = []
    for s, l in zip(specs, plan.offsets):
        R, C, bh, bw = shape(s)
        q.append(OC.quantise_matrix(db[l:l + s.e].reshape(R, C), bh, bw) + (bh, bw))
    t3 = time.perf_counter()
    for c, sc, bh, bw in q:
        OC.dequantise_matrix(c, sc, bh, bw)
    t4 = time.perf_counter()
    nb = sum(s.num_blocks for s in specs)
    moved = {"ragged_pack": 2 * E + 2 * plan.total, "shard_reduce": 2 * wl.world * payload_red + 4 * plan.S,
             "block_quant": 3 * E + 4 * nb, "dequant_unpack": 3 * E + 4 * nb}
    secs = {"ragged_pack": t1 - t0, "shard_reduce": t2 - t1, "block_quant": t3 - t2, "dequant_unpack": t4 - t3}
    return {"value": round(sum(moved.values()) / sum(secs.values()) / 1e9, 3), "unit": "GB/s", "cores": cores,
            "kind": "oracle (plain C with OpenMP, the numpy oracle's cross-check)",
            "sample": f"the same sample as cpu_baseline; {sum(secs.values()):.2f} s",
            "per_op_GBps": {k: round(moved[k] / secs[k] / 1e9, 3) for k in moved}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--units", type=int, default=0, help="units per step (default: the workload's 32)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle leg")
    ap.add_argument("--event-every", type=int, default=4,
                    help="bracket the launches of every N-th unit with HIP events (1 = all); events cost "
                         "about 1.5 us per launch, so bracketing every launch slows the step by ~6 %%")
    ap.add_argument("--graph", action="store_true",
                    help="also replay the step from a HIP graph (captured once) and report its time as "
                         "graph_ms_per_step; the timed steps themselves stay eager because their per-kernel "
                         "events cannot be recorded inside a graph")
    ap.add_argument("--workload", type=int, default=2,
                    help="configuration 1-5 (default 2, the one the metric is quoted on)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU's share of the path; this build has no multi-GPU code "
              "(--gpus must be 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2602_22437_amd import binding as B   # raises if the HIP library is missing
    from workloads import WORKLOADS

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    wl = WORKLOADS[args.workload]
    units = args.units or wl.units
    quant = wl.quantised
    desc = [(t.rows, t.cols, t.mode) for t in wl.tensors]
    plan = B.rs_plan_create(desc, wl.world, wl.align_bytes, wl.min_itemsize)
    B.rs_plan_upload(plan, 0)
    S, total, E = B.rs_plan_shard_elems(plan), B.rs_plan_total_elems(plan), B.rs_plan_payload_elems(plan)
    W, rank = wl.world, wl.rank
    nb = B.rs_plan_num_scales(plan)
    lo, hi = B.rs_plan_scale_range(plan, rank)
    payload_r = sum(s[3] for s in B.rs_plan_rank_segments(plan, rank))
    per_unit = algorithmic_bytes(E, W, S, payload_r, hi - lo, nb)
    if not quant:   # bf16-only path: pack, reduce, plain unpack
        per_unit = {"ragged_pack": per_unit["ragged_pack"], "shard_reduce": per_unit["shard_reduce"],
                    "unpack_bf16": 2 * E + 2 * E}

    # ---- synthetic inputs, resident in HBM ----
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1234)
    U = []
    for u in range(units):
        src = [torch.empty(t.numel, dtype=torch.bfloat16, device="cuda").normal_(0, wl.sigma, generator=gen)
               for t in wl.tensors]
        dst = [torch.empty(t.numel, dtype=torch.bfloat16, device="cuda") for t in wl.tensors]
        d = dict(
            src=src, dst=dst,
            src_tab=B.rs_tensor_table_create(plan, src), dst_tab=B.rs_tensor_table_create(plan, dst),
            dbuf=torch.empty(total, dtype=torch.bfloat16, device="cuda"),
            partials=torch.empty(W * S, dtype=torch.bfloat16, device="cuda").normal_(0, 1e-3, generator=gen),
            out=torch.empty(S, dtype=torch.float32, device="cuda"),
        )
        B.rs_pack(plan, d["src_tab"], d["dbuf"])
        if quant:
            # the gathered FP8 unit that AllGather would deliver: quantise every rank's shard once, untimed
            d["codes"] = torch.empty(total, dtype=torch.uint8, device="cuda")
            d["scales"] = torch.empty(max(nb, 1), dtype=torch.float32, device="cuda")
            B.rs_quantize(plan, -1, d["dbuf"], d["codes"], d["scales"])
            # rank views made once: the timed loop does no tensor bookkeeping
            d["shard"] = d["dbuf"][rank * S:(rank + 1) * S]
            d["shard_codes"] = d["codes"][rank * S:(rank + 1) * S]
            d["shard_scales"] = d["scales"][lo:hi]
        U.append(d)
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream()
    names = list(per_unit)

    # rank's shard of every unit in one launch: a single shard (10 MB here) cannot fill the GPU
    batch = (B.rs_shard_batch_create(plan, rank, [d["shard"] for d in U], [d["shard_codes"] for d in U],
                                     [d["shard_scales"] for d in U]) if quant else None)
    per_unit_names = [n for n in names if n != "block_quant"]

    def step(events=None, qevents=None):
        for ui, d in enumerate(U):
            ev = ([torch.cuda.Event(enable_timing=True) for _ in range(len(per_unit_names) + 1)]
                  if events is not None and ui % args.event_every == 0 else None)
            if ev:
                ev[0].record(stream)
            B.rs_pack(plan, d["src_tab"], d["dbuf"], stream)
            if ev:
                ev[1].record(stream)
            B.rs_reduce(plan, rank, d["partials"], S, d["out"], stream)
            if ev:
                ev[2].record(stream)
            if quant:
                B.rs_unpack(plan, d["codes"], d["scales"], d["dst_tab"], stream)
            else:
                B.rs_unpack_bf16(plan, d["dbuf"], d["dst_tab"], stream)
            if ev:
                ev[3].record(stream)
                events.append(ev)
        if quant:
            qe = [torch.cuda.Event(enable_timing=True) for _ in range(2)] if qevents is not None else None
            if qe:
                qe[0].record(stream)
            B.rs_quantize_batch(plan, batch, stream)
            if qe:
                qe[1].record(stream)
                qevents.append(qe)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events, qevents = [], []
    gc.collect()
    gc.disable()          # no collector pauses between launches inside the timed region
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(events, qevents)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    gc.enable()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    graph_ms = None
    if args.graph:
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            cap = torch.cuda.current_stream()
            for d in U:
                B.rs_pack(plan, d["src_tab"], d["dbuf"], cap)
                B.rs_reduce(plan, rank, d["partials"], S, d["out"], cap)
                if quant:
                    B.rs_unpack(plan, d["codes"], d["scales"], d["dst_tab"], cap)
                else:
                    B.rs_unpack_bf16(plan, d["dbuf"], d["dst_tab"], cap)
            if quant:
                B.rs_quantize_batch(plan, batch, cap)
        for _ in range(args.warmup):
            g.replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        for _ in range(args.steps):
            g.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - g0) * 1e3 / args.steps

    samples = {n: [] for n in names}          # event-to-event ms of every timed launch
    for ev in events:
        for i, n in enumerate(per_unit_names):
            samples[n].append(ev[i].elapsed_time(ev[i + 1]))
    launches = len(events)
    launch_bytes = dict(per_unit)
    if quant:   # one launch covers all units
        samples["block_quant"] = [a.elapsed_time(b) for a, b in qevents]
        launch_bytes["block_quant"] = units * per_unit["block_quant"]
    kern_ms = {n: sum(v) / len(v) for n, v in samples.items()}
    step_bytes = units * sum(per_unit.values())
    value = step_bytes / (ms_per_step * 1e-3) / 1e9

    kernels = {}
    for n in names:
        gbps = launch_bytes[n] / (kern_ms[n] * 1e-3) / 1e9
        ordered = sorted(samples[n])
        kernels[n] = {"ms": round(kern_ms[n], 4), "bytes": launch_bytes[n], "GBps": round(gbps, 1),
                      "frac_of_peak": round(gbps / HBM_PEAK_GBPS, 4), "launches_timed": len(ordered),
                      "median_ms": round(ordered[len(ordered) // 2], 4), "min_ms": round(ordered[0], 4)}
    if quant:
        kernels["block_quant"]["note"] = f"one launch over rank {rank}'s shard of all {units} unit(s)"

    # ---- extras outside the timed steps: all-shard quantisation and the plain-copy ceiling ----
    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        for i in range(reps):
            fn(i)
        b.record(stream)
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    # the same four launches back to back, without events between them: an event record costs a
    # few microseconds of stream time that the per-launch figures above attribute to the kernel
    b2b = {
        "ragged_pack": lambda i=0: B.rs_pack(plan, U[i % units]["src_tab"], U[i % units]["dbuf"], stream),
        "shard_reduce": lambda i=0: B.rs_reduce(plan, rank, U[i % units]["partials"], S, U[i % units]["out"], stream),
    }
    if quant:
        b2b["dequant_unpack"] = lambda i=0: B.rs_unpack(plan, U[i % units]["codes"], U[i % units]["scales"],
                                                        U[i % units]["dst_tab"], stream)
        b2b["block_quant"] = lambda i=0: B.rs_quantize_batch(plan, batch, stream)
    else:
        b2b["unpack_bf16"] = lambda i=0: B.rs_unpack_bf16(plan, U[i % units]["dbuf"], U[i % units]["dst_tab"], stream)
    for n_, fn_ in b2b.items():
        ms = timed(fn_, max(units, 8))
        kernels[n_]["back_to_back_ms"] = round(ms, 4)
        kernels[n_]["back_to_back_frac_of_peak"] = round(launch_bytes[n_] / ms / 1e6 / HBM_PEAK_GBPS, 4)

    if quant:
        one_ms = timed(lambda i=0: B.rs_quantize(plan, rank, U[i % units]["shard"], U[i % units]["shard_codes"],
                                                 U[i % units]["shard_scales"], stream), max(units, 8))
        kernels["block_quant_single_shard"] = {
            "ms": round(one_ms, 4), "bytes": per_unit["block_quant"],
            "GBps": round(per_unit["block_quant"] / one_ms / 1e6, 1),
            "frac_of_peak": round(per_unit["block_quant"] / one_ms / 1e6 / HBM_PEAK_GBPS, 4),
            "note": "one shard of one unit per launch: bounded by launch latency; not part of the timed step"}
        qa_bytes = 2 * E + total + 4 * nb
        qa_ms = timed(lambda i=0: B.rs_quantize(plan, -1, U[i % units]["dbuf"], U[i % units]["codes"],
                                                U[i % units]["scales"], stream), max(units, 8))
        kernels["block_quant_all_shards"] = {
            "ms": round(qa_ms, 4), "bytes": qa_bytes, "GBps": round(qa_bytes / qa_ms / 1e6, 1),
            "frac_of_peak": round(qa_bytes / qa_ms / 1e6 / HBM_PEAK_GBPS, 4),
            "note": "same kernel over all W shards of a unit in one launch; not part of the timed step"}
    if quant:   # reduce and quantise fused: the fp32 mean never reaches HBM
        rq_bytes = 2 * W * payload_r + S + 4 * (hi - lo)
        rq_ms = timed(lambda i=0: B.rs_reduce_quantize(plan, rank, U[i % units]["partials"], S,
                                                       U[i % units]["shard_codes"], U[i % units]["shard_scales"],
                                                       None, stream), max(units, 8))
        kernels["reduce_quantize"] = {
            "ms": round(rq_ms, 4), "bytes": rq_bytes, "GBps": round(rq_bytes / rq_ms / 1e6, 1),
            "frac_of_peak": round(rq_bytes / rq_ms / 1e6 / HBM_PEAK_GBPS, 4),
            "note": "shard_reduce + block_quant in one launch (codes and scales out, no fp32 mean); "
                    "not part of the timed step"}
        for d in U:   # the timed path's codes come from the packed parameters: restore them
            B.rs_quantize(plan, rank, d["shard"], d["shard_codes"], d["shard_scales"], stream)
    if quant:   # gathered FP8 unit straight into fp32 master copies (first 4 units: 4 bytes per element)
        f32_units = U[:min(units, 4)]
        for d in f32_units:
            d["dst32"] = [torch.empty(t.numel, dtype=torch.float32, device="cuda") for t in wl.tensors]
            d["dst32_tab"] = B.rs_tensor_table_create(plan, d["dst32"])
        nf = len(f32_units)
        uf_ms = timed(lambda i=0: B.rs_unpack_f32(plan, U[i % nf]["codes"], U[i % nf]["scales"], U[i % nf]["dst32_tab"],
                                                  stream), max(nf, 8))
        uf_bytes = E + 4 * nb + 4 * E
        kernels["unpack_f32"] = {"ms": round(uf_ms, 4), "bytes": uf_bytes, "GBps": round(uf_bytes / uf_ms / 1e6, 1),
                                 "frac_of_peak": round(uf_bytes / uf_ms / 1e6 / HBM_PEAK_GBPS, 4),
                                 "note": "dequant_unpack into fp32 tensors; not part of the timed step"}
        for d in f32_units:
            B.rs_tensor_table_destroy(d.pop("dst32_tab"))
            del d["dst32"]
    # group-level operators and the 8-bit Adam step (widening beyond the four timed kernels)
    group_bytes = {"pack_scaled": 2 * E + 2 * total, "group_add": 6 * E, "group_scale": 4 * E,
                   "group_zero": 2 * total}
    group_calls = {
        "pack_scaled": lambda i=0: B.rs_pack_scaled(plan, U[i % units]["src_tab"], 1.0 / W, U[i % units]["dbuf"], stream),
        "group_add": lambda i=0: B.rs_group_add(plan, U[i % units]["src_tab"], 1.0, U[i % units]["dbuf"], stream),
        "group_scale": lambda i=0: B.rs_group_scale(plan, 0.999, U[i % units]["dbuf"], stream),
        "group_zero": lambda i=0: B.rs_group_zero(plan, U[i % units]["dbuf"], stream),
    }
    for name in ("group_add", "group_scale", "pack_scaled", "group_zero"):   # ends with the buffer zeroed, then repacked
        ms = timed(group_calls[name], max(units, 8))
        kernels[name] = {"ms": round(ms, 4), "bytes": group_bytes[name], "GBps": round(group_bytes[name] / ms / 1e6, 1),
                         "frac_of_peak": round(group_bytes[name] / ms / 1e6 / HBM_PEAK_GBPS, 4),
                         "note": "group-level DBuffer operator; not part of the timed step"}
    for d in U:
        B.rs_pack(plan, d["src_tab"], d["dbuf"], stream)
    try:
        slo, shi = B.rs_plan_state_range(plan, rank)
    except B.RaggedShardError:
        slo = shi = None
    if slo is not None:
        for d in U:
            d["master"] = torch.empty(S, dtype=torch.float32, device="cuda").normal_(0, wl.sigma, generator=gen)
            d["param"] = torch.empty(S, dtype=torch.bfloat16, device="cuda")
            d["m_codes"] = torch.zeros(S, dtype=torch.int8, device="cuda")
            d["v_codes"] = torch.zeros(S, dtype=torch.uint8, device="cuda")
            d["m_absmax"] = torch.zeros(max(shi - slo, 1), dtype=torch.float32, device="cuda")
            d["v_absmax"] = torch.zeros(max(shi - slo, 1), dtype=torch.float32, device="cuda")
        hyper = B.rs_adam8_hyper(3e-4, 0.9, 0.95, 1e-8, 0.1, 2)

        def adam(i=0):
            d = U[i % units]
            B.rs_adam8_step(plan, rank, hyper, d["out"], d["master"], d["param"], d["m_codes"], d["v_codes"],
                            d["m_absmax"], d["v_absmax"], stream)
        for i in range(units):       # a first step so that the timed ones start from a non-trivial state
            adam(i)
        a_bytes = 18 * payload_r + 16 * (shi - slo)
        a_ms = timed(adam, max(units, 8))
        if units > 1:
            ab = B.rs_adam8_batch_create(plan, rank, *[[d[k] for d in U] for k in
                                                       ("out", "master", "param", "m_codes", "v_codes", "m_absmax", "v_absmax")])
            ab_ms = timed(lambda i=0: B.rs_adam8_step_batch(plan, ab, hyper, stream), 8)
            B.rs_adam8_batch_destroy(ab)
            kernels["adam8_step_batch"] = {
                "ms": round(ab_ms, 4), "bytes": units * a_bytes, "GBps": round(units * a_bytes / ab_ms / 1e6, 1),
                "frac_of_peak": round(units * a_bytes / ab_ms / 1e6 / HBM_PEAK_GBPS, 4),
                "note": f"the same step over rank {rank}'s shard of all {units} units in one launch"}
        kernels["adam8_step"] = {
            "ms": round(a_ms, 4), "bytes": a_bytes, "GBps": round(a_bytes / a_ms / 1e6, 1),
            "frac_of_peak": round(a_bytes / a_ms / 1e6 / HBM_PEAK_GBPS, 4),
            "note": f"AdamW with 8-bit 32x32-block moments on rank {rank}'s shard (fp32 grad and master, bf16 "
                    "param out, codes in place: 18 B per element); not part of the timed step"}
    nbytes = total * 2
    probe_dst = [d["dbuf"] for d in U[1:]] + [torch.empty(total, dtype=torch.bfloat16, device="cuda")]
    cp_ms = timed(lambda i=0: B.rs_copy_probe(probe_dst[i % units], U[i % units]["dbuf"], nbytes, stream),
                  max(units, 8))
    copy_gbps = 2 * nbytes / cp_ms / 1e6
    # the runtime's own device-to-device copy of the same buffers, as a second reference
    rt_ms = timed(lambda i=0: probe_dst[i % units].copy_(U[i % units]["dbuf"]), max(units, 8))
    runtime_copy_gbps = 2 * nbytes / rt_ms / 1e6

    dom = max(per_unit_names, key=lambda n: kern_ms[n])
    roof = {
        "bound": "hbm", "kernel": dom, "launches_timed": launches, "achieved": kernels[dom]["GBps"], "peak": HBM_PEAK_GBPS,
        "unit": "GB/s", "frac": round(kernels[dom]["GBps"] / HBM_PEAK_GBPS, 4),
        "traffic": PMC_TRAFFIC_CONFIG2.get(dom) if wl.index == 2 else None,
        "avg_launch_ms": kernels[dom]["ms"], "algorithmic_bytes_per_launch": per_unit[dom],
        "back_to_back_GBps": round(kernels[dom]["back_to_back_frac_of_peak"] * HBM_PEAK_GBPS, 1),
        "plain_copy_GBps": round(copy_gbps, 1), "runtime_dtod_copy_GBps": round(runtime_copy_gbps, 1),
    }
    result = {
        "metric": "HBM GB/s & % of peak: ragged_pack, shard_reduce, FP8 block_quant, unpack",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"configs[{wl.index - 1}]: {wl.name}, {units} unit(s) back to back", "world": W,
                   "shard_elems": S, "unit_elems": E, "dbuffer_elems": total, "rank": rank,
                   "blocks": "128x128 (2-D), 1x128 (1-D)", "bytes_per_step": step_bytes,
                   "arithmetic": "bf16 tensors and buffer, fp32 accumulation and scales, fp8-e4m3 codes"},
        "frac_of_hbm_peak": round(value / HBM_PEAK_GBPS, 4),
        "kernels": kernels,
        "roofline": roof,
    }
    # the paper's nearest figures, for context only: another system, another machine, per-iteration
    # times of the copies this path replaces and of the collectives around them (Table 1)
    result["paper_context"] = {
        "what": "FSDP2 baseline on GPT-OSS-120B, 64 x NVIDIA H800, bf16; ms per iteration, Shard(0) / Shard(1)",
        "copy_in_ms": [12.37, 23.14], "reduce_scatter_ms": [94.24, 95.36],
        "copy_out_ms": [5.22, 13.72], "all_gather_ms": [43.71, 44.35],
        "note": "no kernel-level GB/s is published, so vs_baseline is null"}
    if graph_ms is not None:
        result["graph_ms_per_step"] = round(graph_ms, 4)
        result["graph_GBps"] = round(step_bytes / (graph_ms * 1e-3) / 1e9, 1)
    if not args.no_cpu and wl.index == 2:
        result["cpu_baseline"] = cpu_baseline(wl)
        try:
            result["cpu_baseline_all_cores"] = cpu_baseline_all_cores(wl)
        except Exception as exc:       # no C compiler on the box: the numpy figure stands alone
            result["cpu_baseline_all_cores"] = {"error": str(exc)[:200]}
    print(json.dumps(result), flush=True)

    if batch:
        B.rs_shard_batch_destroy(batch)
    for d in U:
        B.rs_tensor_table_destroy(d["src_tab"])
        B.rs_tensor_table_destroy(d["dst_tab"])
    B.rs_plan_destroy(plan)


if __name__ == "__main__":
    main()
