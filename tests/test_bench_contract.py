"""The bench's contract: argument handling, the byte counts the GB/s figures rest on, the shape
of the CPU-oracle leg (no GPU), and the one JSON line of a short run (GPU)."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402
from oracle import plan as OP  # noqa: E402
from workloads import WORKLOADS  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode == 2 and r.stdout == ""
    assert "one GPU" in r.stderr and "--gpus must be 1" in r.stderr


def test_algorithmic_bytes_of_the_default_workload():
    """Llama-3-8B-shaped layer on 64 ranks: the figures every GB/s number divides by."""
    wl = WORKLOADS[2]
    specs = [OP.TensorSpec(t.rows, t.cols, t.mode) for t in wl.tensors]
    plan = OP.make_plan(specs, wl.world, wl.align_bytes, wl.min_itemsize)
    E, S, W = plan.payload, plan.S, wl.world
    assert (E, S) == (218_112_000, 3_670_016)
    segs = plan.rank_segments(wl.rank)
    payload_r = sum(s[3] for s in segs)
    lo, hi = plan.scale_range(wl.rank)
    nb = plan.scale_bases()[-1]
    got = bench.algorithmic_bytes(E, W, S, payload_r, hi - lo, nb)
    # pack: every tensor read once, the whole buffer written once (zeros included)
    assert got["ragged_pack"] == 436_224_000 + 469_762_048
    # reduce: 64 partials of the rank's payload in bf16, one fp32 region out
    assert got["shard_reduce"] == 64 * 2 * payload_r + 4 * 3_670_016
    # quantise one shard: bf16 payload in, one code byte per region element, 4 bytes per scale
    assert got["block_quant"] == 2 * payload_r + 3_670_016 + 4 * (hi - lo)
    # unpack: one code byte and two output bytes per element, every scale once
    assert got["dequant_unpack"] == 3 * 218_112_000 + 4 * 13_376 and nb == 13_376
    assert payload_r <= S


def test_cpu_baseline_leg_reports_what_the_contract_asks():
    out = bench.cpu_baseline(WORKLOADS[1])
    assert set(out) >= {"value", "unit", "cores", "kind", "sample"}
    assert out["kind"] == "oracle" and out["unit"] == "GB/s" and out["cores"] == 1 and out["value"] > 0
    assert set(out["per_op_GBps"]) == {"ragged_pack", "shard_reduce", "block_quant", "dequant_unpack"}


def test_traffic_figures_come_from_the_committed_counter_summaries(tmp_path):
    """roofline.traffic is read from profiles/pmc_hbm_traffic_bench_config<N>_*.md: every
    configuration with FP8 blocks lists the step's four kernels there, the figures are within a few
    per cent of the algorithmic bytes of the launch the bench times, and a table written by hand
    parses to the numbers in it."""
    for idx in (2, 3, 4, 5):
        wl = WORKLOADS[idx]
        got = bench.pmc_traffic(idx)
        step = ["ragged_pack", "shard_reduce", "block_quant", "dequant_unpack"] if idx != 3 else \
               ["ragged_pack", "shard_reduce", "unpack_bf16"]
        assert set(step) <= set(got), (idx, sorted(got))
        specs = [OP.TensorSpec(t.rows, t.cols, t.mode) for t in wl.tensors]
        plan = OP.make_plan(specs, wl.world, wl.align_bytes, wl.min_itemsize)
        payload_r = sum(s[3] for s in plan.rank_segments(wl.rank))
        pack = 2 * plan.payload + 2 * wl.world * plan.S
        assert 0.95 * pack <= got["ragged_pack"] <= 1.05 * pack, (idx, got["ragged_pack"], pack)
        one_reduce = 2 * wl.world * payload_r + 4 * plan.S
        ratio = got["shard_reduce"] / one_reduce          # a whole number of units per launch
        assert abs(ratio - round(ratio)) <= 0.05 * round(ratio) and round(ratio) >= 1, (idx, ratio)
    assert bench.pmc_traffic(1) == {} and bench.pmc_traffic(2, str(tmp_path)) == {}
    (tmp_path / "pmc_hbm_traffic_bench_config9_x.md").write_text(
        "# title\n\n| operation | kernel | fetch MB | write MB | total MB | algorithmic MB |\n"
        "|---|---|---|---|---|---|\n| a_b | k<1> | 1.5 | 2.25 | 3.75 | 3.7 |\n| c | k | x | y | n/a | 1 |\n\ntext | with | bars\n")
    assert bench.pmc_traffic(9, str(tmp_path)) == {"a_b": 3.75e6}


@pytest.mark.gpu
def test_short_run_prints_one_json_line_with_roofline(capsys, monkeypatch):
    monkeypatch.setattr(sys, "argv", ["bench.py", "--workload", "1", "--steps", "2", "--warmup", "1", "--no-cpu"])
    bench.main()
    lines = [l for l in capsys.readouterr().out.splitlines() if l.strip()]
    assert len(lines) == 1
    r = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
                "scaling", "vs_baseline", "dtype", "data", "config", "roofline", "kernels"):
        assert key in r, key
    assert r["n_gpus"] == 1 and r["steps"] == 2 and r["warmup"] == 1 and r["vs_baseline"] is None
    assert r["unit"] == "GB/s" and r["data"] == "synthetic" and "workload" in r["config"]
    roof = r["roofline"]
    assert roof["bound"] == "hbm" and roof["peak"] == 8000.0 and roof["unit"] == "GB/s"
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-3 and "traffic" in roof
    for name in ("ragged_pack", "shard_reduce", "block_quant", "dequant_unpack"):
        k = r["kernels"][name]
        assert k["ms"] > 0 and k["bytes"] > 0 and k["min_ms"] <= k["median_ms"]
