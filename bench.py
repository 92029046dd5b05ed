#!/usr/bin/env python3
"""Benchmark of the RaggedShard / DBuffer hot path on one MI355X.

With no flags every configuration is timed in one process and ONE JSON line is printed: the
headline (`value`, `ms_per_step`, `roofline`, `cpu_baseline`, `config`) is the largest
configuration, the DeepSeek-V3-shaped MoE unit on 1024 ranks; `per_config` carries the same
figures for all five, and `min_frac_of_peak` is the smallest event-timed fraction of the 8 TB/s
HBM peak over (configurations 2-5) x (the four kernels).  Configuration 1 (the toy unit, 0.8 MB)
is launch-bound and is marked so.

A step is one pass of the whole path over one batch of synthetic input, all resident in HBM
before the timed region:
    per unit: ragged_pack (per-parameter tensors -> DBuffer), shard_reduce over the rank's region
    (W partials), dequant_unpack of the gathered FP8 unit (configuration 3: the bf16 unpack);
    then ONE block_quant launch over the rank's shard of every unit a rank holds: the 32 decoder
    units of configuration 2, and for the MoE configurations the rank's shard of as many units as
    the model has MoE layers (36 / 58; one unit's other buffers would not fit 32 times over).
    Configuration 2's regions are short (3.7 M elements, 68 us per reduce), so its 32 reduces
    are likewise one launch (rs_reduce_batch), after the per-unit pack and unpack launches.
HIP events on the launch stream bracket the launches inside the timed region; the same launches
are also timed back to back without events in between.  Further kernels of the library (fused
reduce + quantise, fp32 unpack, group operators, 8-bit Adam step, strided and rooted copies,
single-shard and all-shard block_quant) are timed outside the steps and never enter `value`.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload all|1..5] [--no-cpu] [--no-extras]
"""
from __future__ import annotations

import argparse
import gc
import glob
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X HBM3E, published
METRIC = "HBM GB/s & % of peak: ragged_pack, shard_reduce, FP8 block_quant, unpack"
FOUR = ("ragged_pack", "shard_reduce", "block_quant", "dequant_unpack")

# How many units' shards one block_quant launch covers in the step: a rank quantises its shard of
# every layer it holds.  Configuration 2 states 32 units; the MoE shapes stand for models with
# 36 (GPT-OSS-120B) and 58 (DeepSeek-V3) MoE layers.
QUANT_SHARDS = {1: 1, 2: 32, 4: 36, 5: 58}


def algorithmic_bytes(E, W, S, payload_r, nb_r, nb):
    """Bytes each op must move per unit (bf16 = 2, fp32 = 4, fp8 = 1)."""
    return {
        "ragged_pack": 2 * E + 2 * W * S,                    # read every tensor, write the whole DBuffer
        "shard_reduce": 2 * W * payload_r + 4 * S,           # W partials of the payload, fp32 shard out
        "block_quant": 2 * payload_r + S + 4 * nb_r,         # bf16 shard in, codes (padding zeroed) + scales out
        "dequant_unpack": E + 4 * nb + 2 * E,                # codes + scales in, bf16 tensors out
    }


def pmc_traffic(config_index, profiles_dir=None):
    """HBM bytes per launch of every operation of one configuration, read from the rocprofv3 --pmc
    summary under profiles/ (FETCH_SIZE and WRITE_SIZE runs, scaled by the plain-copy launch of
    known size).  {} when no summary covers the configuration."""
    d = profiles_dir or os.path.join(ROOT, "profiles")
    out = {}
    for path in sorted(glob.glob(os.path.join(d, f"pmc_hbm_traffic_bench_config{config_index}_*.md"))):
        cols = None
        for line in open(path):
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            if not line.startswith("|"):
                continue
            if cols is None:
                if "operation" in cells and "total MB" in cells:
                    cols = (cells.index("operation"), cells.index("total MB"))
                continue
            if set(cells[0]) <= set("-: "):
                continue
            try:
                out[cells[cols[0]]] = float(cells[cols[1]]) * 1e6
            except (ValueError, IndexError):
                pass
    return out


# ---- the CPU oracle, timed on a bounded sample of each configuration ---------------------------

# tensors of the sample (indices into the configuration's list) and the columns of the reduce sample
CPU_SAMPLE = {
    1: ([0, 1, 2, 3, 4, 5], None),             # the whole toy unit
    2: ([0, 1, 2, 3, 4, 5, 6, 7, 8], 1 << 20),  # the whole unit
    3: ([0, 2, 1], 1 << 20),
    4: ([4, 1, 6], 1 << 18),                   # router, wk, expert 0 down
    5: ([0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 768, 769], 1 << 16),   # four routed experts (128x128), two shared matrices (1x128 rows)
}


def _cpu_sample(wl, seed=1):
    import numpy as np
    from oracle import plan as OP
    from workloads import gen_param, gen_partial
    idx, cols = CPU_SAMPLE[wl.index]
    specs = [OP.TensorSpec(wl.tensors[t].rows, wl.tensors[t].cols, wl.tensors[t].mode) for t in idx]
    params = [gen_param(wl, seed, t) for t in idx]
    offsets, cur = [], 0
    for s in specs:                       # the sample's own little buffer: 16-byte-aligned starts
        offsets.append(cur)
        cur += -(-s.e // 16) * 16
    total = cur
    if cols is None:
        plan = OP.make_plan([OP.TensorSpec(t.rows, t.cols, t.mode) for t in wl.tensors], wl.world,
                            wl.align_bytes, wl.min_itemsize)
        cols = plan.S
        segs = plan.rank_segments(wl.rank)
    else:
        segs = [(0, 0, 0, cols)]
    parts = np.stack([gen_partial(wl, seed, w, cols) for w in range(wl.world)])
    return specs, params, offsets, total, parts, segs


def _cpu_report(wl, specs, total, parts, segs, secs, cores, kind):
    E_s = sum(s.e for s in specs)
    nb_s = sum(s.num_blocks for s in specs) if wl.quantised else 0
    payload = sum(s[3] for s in segs)
    moved = {"ragged_pack": 2 * E_s + 2 * total,
             "shard_reduce": 2 * wl.world * payload + 4 * parts.shape[1]}
    if wl.quantised:
        moved["block_quant"] = 3 * E_s + 4 * nb_s
        moved["dequant_unpack"] = 3 * E_s + 4 * nb_s
    else:
        moved["unpack_bf16"] = 4 * E_s
    t = sum(secs.values())
    return {"value": round(sum(moved.values()) / t / 1e9, 4), "unit": "GB/s", "cores": cores, "kind": kind,
            "sample": f"{len(specs)} tensors ({E_s} elem), reduce {wl.world}x{parts.shape[1]}; {t:.1f} s",
            "per_op_GBps": {k: round(moved[k] / secs[k] / 1e9, 4) for k in moved}}


def cpu_baseline(wl, seed=1):
    """The numpy oracle as it stands (one thread) on a bounded sample of the configuration: a few of
    its tensors through pack / quantise / dequantise and W partials of a stretch of the rank's region
    through the reduce."""
    from oracle import dbuffer as OD
    from oracle import fp8 as OF
    specs, params, offsets, total, parts, segs = _cpu_sample(wl, seed)
    secs = {}
    t0 = time.perf_counter()
    db = OD.ragged_pack(params, offsets, total)
    secs["ragged_pack"] = time.perf_counter() - t0
    t0 = time.perf_counter()
    OD.shard_reduce(parts, segs)
    secs["shard_reduce"] = time.perf_counter() - t0
    if wl.quantised:
        t0 = time.perf_counter()
        q = [OF.quantise_tensor(db[l:l + s.e], s) for s, l in zip(specs, offsets)]
        secs["block_quant"] = time.perf_counter() - t0
        t0 = time.perf_counter()
        for (c, sc), s in zip(q, specs):
            OF.dequantise_tensor(c, sc, s)
        secs["dequant_unpack"] = time.perf_counter() - t0
    else:
        t0 = time.perf_counter()
        OD.unpack_bf16(db, offsets, [s.e for s in specs])
        secs["unpack_bf16"] = time.perf_counter() - t0
    return _cpu_report(wl, specs, total, parts, segs, secs, 1, "oracle")


def cpu_baseline_all_cores(wl, seed=1):
    """The same sample through the plain-C / OpenMP statement of the oracle on every host core the
    process may use: context for the single-thread numpy figure, not a target."""
    from oracle import c_oracle as OC
    from oracle import dbuffer as OD
    from oracle import plan as OP
    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    OC.set_num_threads(cores)
    specs, params, offsets, total, parts, segs = _cpu_sample(wl, seed)

    def shape(s):
        return ((1, s.rows, 1, 128) if s.cols == 0 else
                (s.rows, s.cols, 128, 128) if s.mode == OP.BLOCK_128x128 else (s.rows, s.cols, 1, 128))
    secs = {}
    t0 = time.perf_counter()
    db = OC.ragged_pack(params, offsets, total)
    secs["ragged_pack"] = time.perf_counter() - t0
    t0 = time.perf_counter()
    OC.shard_reduce(parts, segs)
    secs["shard_reduce"] = time.perf_counter() - t0
    if wl.quantised:
        t0 = time.perf_counter()
        q = []
        for s, l in zip(specs, offsets):
            R, C, bh, bw = shape(s)
            q.append(OC.quantise_matrix(db[l:l + s.e].reshape(R, C), bh, bw) + (bh, bw))
        secs["block_quant"] = time.perf_counter() - t0
        t0 = time.perf_counter()
        for c, sc, bh, bw in q:
            OC.dequantise_matrix(c, sc, bh, bw)
        secs["dequant_unpack"] = time.perf_counter() - t0
    else:
        t0 = time.perf_counter()
        OD.unpack_bf16(db, offsets, [s.e for s in specs])
        secs["unpack_bf16"] = time.perf_counter() - t0
    return _cpu_report(wl, specs, total, parts, segs, secs, cores,
                       "oracle (plain C with OpenMP, the numpy oracle's cross-check)")


# ---- one configuration on the GPU ---------------------------------------------------------------

def bench_config(wl, args, torch, B):
    units = wl.units
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
    qshards = QUANT_SHARDS.get(wl.index, 1) if quant else 0

    # ---- synthetic inputs, resident in HBM ----
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1234 + wl.index)
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
    # the rank's shard of every unit it holds, for the one batched block_quant launch of the step
    Q = []
    if quant:
        for q in range(qshards):
            if q < units:
                Q.append((U[q]["shard"], U[q]["shard_codes"], U[q]["shard_scales"]))
            else:       # further layers: the shard alone (a unit's other buffers are not needed)
                Q.append((torch.empty(S, dtype=torch.bfloat16, device="cuda").normal_(0, wl.sigma, generator=gen),
                          torch.empty(S, dtype=torch.uint8, device="cuda"),
                          torch.empty(max(hi - lo, 1), dtype=torch.float32, device="cuda")))
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream()
    names = list(per_unit)
    batch = (B.rs_shard_batch_create(plan, rank, [q[0] for q in Q], [q[1] for q in Q], [q[2] for q in Q])
             if quant else None)
    # many units per step: their reduces are one launch too (the per-unit launch is timed outside)
    rbatch = (B.rs_partials_batch_create(plan, rank, [d["partials"] for d in U], S, [d["out"] for d in U])
              if units > 1 else None)
    batched_names = [n for n in names if n == "block_quant" or (n == "shard_reduce" and rbatch)]
    per_unit_names = [n for n in names if n not in batched_names]
    event_every = args.event_every if units > 1 else 1

    def step(events=None, qevents=None):
        for ui, d in enumerate(U):
            ev = ([torch.cuda.Event(enable_timing=True) for _ in range(len(per_unit_names) + 1)]
                  if events is not None and ui % event_every == 0 else None)
            k = 0
            if ev:
                ev[k].record(stream)
            B.rs_pack(plan, d["src_tab"], d["dbuf"], stream)
            k += 1
            if ev:
                ev[k].record(stream)
            if not rbatch:
                B.rs_reduce(plan, rank, d["partials"], S, d["out"], stream)
                k += 1
                if ev:
                    ev[k].record(stream)
            if quant:
                B.rs_unpack(plan, d["codes"], d["scales"], d["dst_tab"], stream)
            else:
                B.rs_unpack_bf16(plan, d["dbuf"], d["dst_tab"], stream)
            k += 1
            if ev:
                ev[k].record(stream)
                events.append(ev)
        qe = ([torch.cuda.Event(enable_timing=True) for _ in range(len(batched_names) + 1)]
              if qevents is not None and batched_names else None)
        k = 0
        if qe:
            qe[0].record(stream)
        if rbatch:
            B.rs_reduce_batch(plan, rbatch, stream)
            k += 1
            if qe:
                qe[k].record(stream)
        if quant:
            B.rs_quantize_batch(plan, batch, stream)
            k += 1
            if qe:
                qe[k].record(stream)
        if qe:
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

    samples = {n: [] for n in names}          # event-to-event ms of every timed launch
    for ev in events:
        for i, n in enumerate(per_unit_names):
            samples[n].append(ev[i].elapsed_time(ev[i + 1]))
    launch_bytes = dict(per_unit)
    for qe in qevents:      # the launches that cover many units at once
        for i, n in enumerate(batched_names):
            samples[n].append(qe[i].elapsed_time(qe[i + 1]))
    if quant:   # one launch covers the rank's shard of all qshards units
        launch_bytes["block_quant"] = qshards * per_unit["block_quant"]
    if rbatch:
        launch_bytes["shard_reduce"] = units * per_unit["shard_reduce"]
    kern_ms = {n: sum(v) / len(v) for n, v in samples.items()}
    step_bytes = units * sum(v for k, v in per_unit.items() if k not in batched_names) + sum(
        launch_bytes[k] for k in batched_names)
    value = step_bytes / (ms_per_step * 1e-3) / 1e9

    kernels = {}
    for n in names:
        gbps = launch_bytes[n] / (kern_ms[n] * 1e-3) / 1e9
        ordered = sorted(samples[n])
        kernels[n] = {"ms": round(kern_ms[n], 4), "bytes": launch_bytes[n], "GBps": round(gbps, 1),
                      "frac_of_peak": round(gbps / HBM_PEAK_GBPS, 4), "launches_timed": len(ordered),
                      "median_ms": round(ordered[len(ordered) // 2], 4), "min_ms": round(ordered[0], 4)}
    if quant:
        kernels["block_quant"]["note"] = f"one launch over rank {rank}'s shard of {qshards} unit(s)"
    if rbatch:
        kernels["shard_reduce"]["note"] = f"one launch over rank {rank}'s region of {units} units (rs_reduce_batch)"

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

    def entry(ms, nbytes, note=None):
        e = {"ms": round(ms, 4), "bytes": nbytes, "GBps": round(nbytes / ms / 1e6, 1),
             "frac_of_peak": round(nbytes / ms / 1e6 / HBM_PEAK_GBPS, 4)}
        if note:
            e["note"] = note
        return e

    reps = max(units, 8)
    # the same four launches back to back, without events between them: an event record costs a
    # few microseconds of stream time that the per-launch figures above attribute to the kernel
    b2b = {
        "ragged_pack": lambda i=0: B.rs_pack(plan, U[i % units]["src_tab"], U[i % units]["dbuf"], stream),
        "shard_reduce": ((lambda i=0: B.rs_reduce_batch(plan, rbatch, stream)) if rbatch else
                         (lambda i=0: B.rs_reduce(plan, rank, U[i % units]["partials"], S, U[i % units]["out"], stream))),
    }
    if quant:
        b2b["dequant_unpack"] = lambda i=0: B.rs_unpack(plan, U[i % units]["codes"], U[i % units]["scales"],
                                                        U[i % units]["dst_tab"], stream)
        b2b["block_quant"] = lambda i=0: B.rs_quantize_batch(plan, batch, stream)
    else:
        b2b["unpack_bf16"] = lambda i=0: B.rs_unpack_bf16(plan, U[i % units]["dbuf"], U[i % units]["dst_tab"], stream)
    for n_, fn_ in b2b.items():
        ms = timed(fn_, reps)
        kernels[n_]["back_to_back_ms"] = round(ms, 4)
        kernels[n_]["back_to_back_frac_of_peak"] = round(launch_bytes[n_] / ms / 1e6 / HBM_PEAK_GBPS, 4)

    if rbatch:
        ms = timed(lambda i=0: B.rs_reduce(plan, rank, U[i % units]["partials"], S, U[i % units]["out"], stream), reps)
        kernels["shard_reduce_per_unit"] = {
            "ms": round(ms, 4), "bytes": per_unit["shard_reduce"],
            "GBps": round(per_unit["shard_reduce"] / ms / 1e6, 1),
            "frac_of_peak": round(per_unit["shard_reduce"] / ms / 1e6 / HBM_PEAK_GBPS, 4),
            "note": "rs_reduce on one unit's region per launch, back to back; not in the step"}
    nbytes = total * 2
    probe_dst = torch.empty(total, dtype=torch.bfloat16, device="cuda")
    cp_ms = timed(lambda i=0: B.rs_copy_probe(probe_dst, U[i % units]["dbuf"], nbytes, stream), reps)
    copy_gbps = 2 * nbytes / cp_ms / 1e6
    # the runtime's own device-to-device copy of the same buffers, as a second reference
    rt_ms = timed(lambda i=0: probe_dst.copy_(U[i % units]["dbuf"]), reps)
    runtime_copy_gbps = 2 * nbytes / rt_ms / 1e6

    if quant and not args.no_extras:
        nq = len(Q)
        one_ms = timed(lambda i=0: B.rs_quantize(plan, rank, Q[i % nq][0], Q[i % nq][1], Q[i % nq][2], stream),
                       max(nq, 8))
        kernels["block_quant_single_shard"] = entry(
            one_ms, per_unit["block_quant"],
            "one shard of one unit per launch: bounded by launch latency (see plain_copy_same_bytes); not in the step")
        # what a launch of this size can reach at all: the plain copy moving the same number of bytes
        small = per_unit["block_quant"] // 32 * 16
        sm_ms = timed(lambda i=0: B.rs_copy_probe(probe_dst, U[0]["dbuf"], small, stream), 16)
        kernels["plain_copy_same_bytes"] = entry(
            sm_ms, 2 * small, "plain 16-byte copy kernel moving as many bytes as one single-shard block_quant launch")
        qa_bytes = 2 * E + total + 4 * nb
        qa_ms = timed(lambda i=0: B.rs_quantize(plan, -1, U[i % units]["dbuf"], U[i % units]["codes"],
                                                U[i % units]["scales"], stream), reps)
        kernels["block_quant_all_shards"] = entry(
            qa_ms, qa_bytes, "same kernel over all W shards of a unit in one launch; not in the step")
        # reduce and quantise fused: the fp32 mean never reaches HBM
        rq_bytes = 2 * W * payload_r + S + 4 * (hi - lo)
        rq_ms = timed(lambda i=0: B.rs_reduce_quantize(plan, rank, U[i % units]["partials"], S,
                                                       U[i % units]["shard_codes"], U[i % units]["shard_scales"],
                                                       None, stream), reps)
        kernels["reduce_quantize"] = entry(
            rq_ms, rq_bytes, "shard_reduce + block_quant in one launch (codes and scales out, no fp32 mean); not in the step")
        if rbatch and qshards == units:
            rqb_ms = timed(lambda i=0: B.rs_reduce_quantize_batch(plan, rbatch, batch, False, stream), 8)
            kernels["reduce_quantize_batch"] = entry(
                rqb_ms, units * rq_bytes,
                f"the same over rank {rank}'s region of all {units} units in one launch; not in the step")
        for d in U:   # the timed path's codes come from the packed parameters: restore them
            B.rs_quantize(plan, rank, d["shard"], d["shard_codes"], d["shard_scales"], stream)
        # gathered FP8 unit straight into fp32 master copies (first 4 units: 4 bytes per element)
        f32_units = U[:min(units, 4)]
        for d in f32_units:
            d["dst32"] = [torch.empty(t.numel, dtype=torch.float32, device="cuda") for t in wl.tensors]
            d["dst32_tab"] = B.rs_tensor_table_create(plan, d["dst32"])
        nf = len(f32_units)
        uf_ms = timed(lambda i=0: B.rs_unpack_f32(plan, U[i % nf]["codes"], U[i % nf]["scales"], U[i % nf]["dst32_tab"],
                                                  stream), max(nf, 8))
        kernels["unpack_f32"] = entry(uf_ms, E + 4 * nb + 4 * E, "dequant_unpack into fp32 tensors; not in the step")
        for d in f32_units:
            B.rs_tensor_table_destroy(d.pop("dst32_tab"))
            del d["dst32"]
    if not args.no_extras:
        # the unpack on regions gathered over a 2-D mesh (two groups; this group's regions are
        # every other S elements of a buffer twice the size)
        if quant:
            wide = torch.empty(2 * total, dtype=torch.uint8, device="cuda")
            wide.view(2 * W, S)[0::2].copy_(U[0]["codes"].view(W, S))
            ms = timed(lambda i=0: B.rs_unpack_strided(plan, wide, 2 * S, U[0]["scales"], U[0]["dst_tab"], stream), 8)
            kernels["unpack_strided"] = entry(ms, E + 4 * nb + 2 * E,
                                              "dequant_unpack of one of two groups of a mesh-gathered code buffer; not in the step")
        else:
            wide = torch.empty(2 * total, dtype=torch.bfloat16, device="cuda")
            wide.view(2 * W, S)[0::2].copy_(U[0]["dbuf"].view(W, S))
            ms = timed(lambda i=0: B.rs_unpack_bf16_strided(plan, wide, 2 * S, U[0]["dst_tab"], stream), 8)
            kernels["unpack_bf16_strided"] = entry(ms, 4 * E, "unpack_bf16 of one of two groups of a mesh-gathered "
                                                              "buffer; not in the step")
        del wide
        if wl.index == 3:
            # Algorithm 2's data path on these shapes: the balanced buffer P (128-row granularity) to
            # the rooted buffer Q (every matrix whole on the device SelectRoot gives it) and back,
            # one group copy each way
            from workloads import MODE_128x128, MODE_1x128
            pdesc = [(t.rows, t.cols, MODE_128x128 if t.cols else MODE_1x128) for t in wl.tensors]
            pplan = B.rs_plan_create(pdesc, W, wl.align_bytes, wl.min_itemsize)
            B.rs_plan_upload(pplan, 0)
            roots, _ = B.rs_select_roots(desc, W)
            roots = [r if r >= 0 else 0 for r in roots]
            qplan = B.rs_plan_create_rooted(desc, W, roots, wl.align_bytes, wl.min_itemsize)
            qoff = B.rs_plan_offsets(qplan)
            ptotal, qtotal = B.rs_plan_total_elems(pplan), B.rs_plan_total_elems(qplan)
            pbuf = torch.empty(ptotal, dtype=torch.bfloat16, device="cuda").normal_(0, wl.sigma, generator=gen)
            qbuf = torch.zeros(qtotal, dtype=torch.bfloat16, device="cuda")
            views = [qbuf[o:o + t.numel] for o, t in zip(qoff, wl.tensors)]
            vtab = B.rs_tensor_table_create(pplan, views)
            ms = timed(lambda i=0: B.rs_unpack_bf16(pplan, pbuf, vtab, stream), 16)
            kernels["redistribute_to_roots"] = entry(
                ms, 4 * E, f"P -> Q: balanced buffer ({ptotal} elem) into views of the rooted one ({qtotal} elem), "
                           "one unpack_bf16 launch; not in the step")
            ms = timed(lambda i=0: B.rs_pack(pplan, vtab, pbuf, stream), 16)
            kernels["redistribute_from_roots"] = entry(ms, 2 * E + 2 * ptotal, "Q -> P: one ragged_pack launch; not in the step")
            B.rs_tensor_table_destroy(vtab)
            B.rs_plan_destroy(pplan)
            B.rs_plan_destroy(qplan)
            del pbuf, qbuf, views
        # group-level operators (widening beyond the four timed kernels)
        group_bytes = {"pack_scaled": 2 * E + 2 * total, "group_add": 6 * E, "group_scale": 4 * E,
                       "group_zero": 2 * total}
        group_calls = {
            "pack_scaled": lambda i=0: B.rs_pack_scaled(plan, U[i % units]["src_tab"], 1.0 / W, U[i % units]["dbuf"], stream),
            "group_add": lambda i=0: B.rs_group_add(plan, U[i % units]["src_tab"], 1.0, U[i % units]["dbuf"], stream),
            "group_scale": lambda i=0: B.rs_group_scale(plan, 0.999, U[i % units]["dbuf"], stream),
            "group_zero": lambda i=0: B.rs_group_zero(plan, U[i % units]["dbuf"], stream),
        }
        for name in ("group_add", "group_scale", "pack_scaled", "group_zero"):   # ends with the buffer zeroed, then repacked
            ms = timed(group_calls[name], reps)
            kernels[name] = entry(ms, group_bytes[name], "group-level DBuffer operator; not in the step")
        for d in U:
            B.rs_pack(plan, d["src_tab"], d["dbuf"], stream)
        try:
            slo, shi = B.rs_plan_state_range(plan, rank)
        except B.RaggedShardError:
            slo = shi = None
        if slo is not None:
            # the 8-bit Adam step on the rank's shard of as many units as the block_quant launch covers
            na = max(qshards, 1)
            A = []
            for q in range(na):
                A.append(dict(
                    out=U[q]["out"] if q < units else torch.empty(S, dtype=torch.float32, device="cuda").normal_(0, 1e-3, generator=gen),
                    master=torch.empty(S, dtype=torch.float32, device="cuda").normal_(0, wl.sigma, generator=gen),
                    param=torch.empty(S, dtype=torch.bfloat16, device="cuda"),
                    m_codes=torch.zeros(S, dtype=torch.int8, device="cuda"),
                    v_codes=torch.zeros(S, dtype=torch.uint8, device="cuda"),
                    m_absmax=torch.zeros(max(shi - slo, 1), dtype=torch.float32, device="cuda"),
                    v_absmax=torch.zeros(max(shi - slo, 1), dtype=torch.float32, device="cuda")))
            hyper = B.rs_adam8_hyper(3e-4, 0.9, 0.95, 1e-8, 0.1, 2)

            def adam(i=0):
                d = A[i % na]
                B.rs_adam8_step(plan, rank, hyper, d["out"], d["master"], d["param"], d["m_codes"], d["v_codes"],
                                d["m_absmax"], d["v_absmax"], stream)
            for i in range(na):       # a first step so that the timed ones start from a non-trivial state
                adam(i)
            a_bytes = 18 * payload_r + 16 * (shi - slo)
            a_ms = timed(adam, max(na, 8))
            kernels["adam8_step"] = entry(
                a_ms, a_bytes, f"AdamW with 8-bit block-wise moments on rank {rank}'s shard of one unit (fp32 grad and "
                               "master, bf16 param out, codes in place: 18 B per element); not in the step")
            if na > 1:
                ab = B.rs_adam8_batch_create(plan, rank, *[[d[k] for d in A] for k in
                                                           ("out", "master", "param", "m_codes", "v_codes", "m_absmax", "v_absmax")])
                ab_ms = timed(lambda i=0: B.rs_adam8_step_batch(plan, ab, hyper, stream), 8)
                B.rs_adam8_batch_destroy(ab)
                kernels["adam8_step_batch"] = entry(
                    ab_ms, na * a_bytes, f"the same step over rank {rank}'s shard of {na} units in one launch")
            del A

    dom = max(per_unit_names, key=lambda n: kern_ms[n])     # the launch that takes longest of its kind
    traffic = pmc_traffic(wl.index)
    roof = {
        "bound": "hbm", "kernel": dom, "launches_timed": len(events), "achieved": kernels[dom]["GBps"],
        "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(kernels[dom]["GBps"] / HBM_PEAK_GBPS, 4),
        "traffic": traffic.get(dom),
        "avg_launch_ms": kernels[dom]["ms"], "algorithmic_bytes_per_launch": per_unit[dom],
        "back_to_back_GBps": round(kernels[dom]["back_to_back_frac_of_peak"] * HBM_PEAK_GBPS, 1),
        "plain_copy_GBps": round(copy_gbps, 1), "runtime_dtod_copy_GBps": round(runtime_copy_gbps, 1),
    }
    for n in kernels:
        if n in traffic:
            kernels[n]["pmc_traffic_bytes"] = traffic[n]
    result = {
        "workload": f"configs[{wl.index - 1}]: {wl.name}, {units} unit(s) per step"
                    + (f", block_quant over the rank's shard of {qshards} unit(s)" if quant else ""),
        "value": round(value, 1), "unit": "GB/s", "ms_per_step": round(ms_per_step, 4),
        "frac_of_hbm_peak": round(value / HBM_PEAK_GBPS, 4), "bytes_per_step": step_bytes,
        "world": W, "shard_elems": S, "unit_elems": E, "dbuffer_elems": total, "rank": rank,
        "launch_bound": wl.index == 1,
        "kernels": kernels, "roofline": roof,
    }
    if wl.index == 1 and not args.no_extras:
        # launch-bound: the same step captured once into a HIP graph and replayed (the entry points
        # only enqueue kernels, so a step is capturable as it stands)
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        with torch.cuda.stream(side):
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                stream_saved, stream = stream, side
                try:
                    step()
                finally:
                    stream = stream_saved
        torch.cuda.synchronize()
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        n_rep = 200
        t0 = time.perf_counter()
        for _ in range(n_rep):
            graph.replay()
        torch.cuda.synchronize()
        g_ms = (time.perf_counter() - t0) * 1e3 / n_rep
        result["graph_replay"] = {
            "ms_per_step": round(g_ms, 4), "GBps": round(step_bytes / (g_ms * 1e-3) / 1e9, 1),
            "note": "the step's launches captured into one HIP graph and replayed; not the headline figure"}
        del graph
    if wl.index == 1:
        result["note"] = ("the toy unit moves under 1 MB per launch: every kernel ends within the launch latency "
                          "(5-20 us), so its fractions say nothing about the kernels; it is here for completeness")

    if batch:
        B.rs_shard_batch_destroy(batch)
    if rbatch:
        B.rs_partials_batch_destroy(rbatch)
    for d in U:
        B.rs_tensor_table_destroy(d["src_tab"])
        B.rs_tensor_table_destroy(d["dst_tab"])
    B.rs_plan_destroy(plan)
    del U, Q, probe_dst
    gc.collect()
    torch.cuda.empty_cache()
    return result


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle legs")
    ap.add_argument("--no-extras", action="store_true", help="time the step's four kernels only")
    ap.add_argument("--event-every", type=int, default=4,
                    help="configuration 2: bracket the launches of every N-th unit with HIP events (1 = all); "
                         "events cost about 1.5 us per launch, so bracketing every launch slows the step by ~6 %%")
    ap.add_argument("--workload", default="all",
                    help="all (default: every configuration, headline on the largest) or one of 1-5")
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
    order = [5, 4, 3, 2, 1] if args.workload == "all" else [int(args.workload)]
    per_config = {}
    for idx in order:
        wl = WORKLOADS[idx]
        print(f"[bench] configuration {idx}: {wl.name}", file=sys.stderr, flush=True)
        r = bench_config(wl, args, torch, B)
        if not args.no_cpu:
            print(f"[bench] configuration {idx}: CPU oracle on its sample", file=sys.stderr, flush=True)
            r["cpu_baseline"] = cpu_baseline(wl)
            try:
                r["cpu_baseline_all_cores"] = cpu_baseline_all_cores(wl)
            except Exception as exc:       # no C compiler on the box: the numpy figure stands alone
                r["cpu_baseline_all_cores"] = {"error": str(exc)[:200]}
        per_config[str(idx)] = r

    head = per_config[str(order[0])]
    fracs = {f"{i}.{k}": per_config[i]["kernels"][k]["frac_of_peak"]
             for i in per_config if i != "1" for k in per_config[i]["kernels"]
             if k in FOUR or k == "unpack_bf16"}
    b2b = {f"{i}.{k}": per_config[i]["kernels"][k].get("back_to_back_frac_of_peak")
           for i in per_config if i != "1" for k in per_config[i]["kernels"]
           if k in FOUR or k == "unpack_bf16"}
    result = {
        "metric": METRIC,
        "value": head["value"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": head["workload"], "world": head["world"], "shard_elems": head["shard_elems"],
                   "unit_elems": head["unit_elems"], "dbuffer_elems": head["dbuffer_elems"], "rank": head["rank"],
                   "blocks": "128x128 (2-D), 1x128 (1-D and the shared expert's rows)",
                   "bytes_per_step": head["bytes_per_step"],
                   "arithmetic": "bf16 tensors and buffer, fp32 accumulation and scales, fp8-e4m3 codes"},
        "frac_of_hbm_peak": head["frac_of_hbm_peak"],
        "roofline": head["roofline"],
    }
    if "cpu_baseline" in head:
        result["cpu_baseline"] = head["cpu_baseline"]
        result["cpu_baseline_all_cores"] = head["cpu_baseline_all_cores"]
    if fracs:
        worst = min(fracs, key=fracs.get)
        result["min_frac_of_peak"] = {"value": fracs[worst], "where": worst,
                                      "back_to_back": min(v for v in b2b.values() if v is not None),
                                      "over": "configurations 2-5 x the step's four kernels, HIP-event timed"}
    result["kernels"] = head["kernels"]
    result["per_config"] = per_config
    # the paper's nearest figures, for context only: another system, another machine, per-iteration
    # times of the copies this path replaces and of the collectives around them (Table 1)
    result["paper_context"] = {
        "what": "FSDP2 baseline on GPT-OSS-120B, 64 x NVIDIA H800, bf16; ms per iteration, Shard(0) / Shard(1)",
        "copy_in_ms": [12.37, 23.14], "reduce_scatter_ms": [94.24, 95.36],
        "copy_out_ms": [5.22, 13.72], "all_gather_ms": [43.71, 44.35],
        "note": "no kernel-level GB/s is published, so vs_baseline is null"}
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
