"""bench.py on the GPU, on the two small configurations (its functions called in this process): the result
carries what the contract asks for, the per-kernel durations add up to about the step, and the sweep mode lists
every chunk size the library takes."""
import argparse
import contextlib
import importlib.util
import io
import json
import os

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def _args(**kw):
    a = dict(gpus=1, steps=3, warmup=1, workload=None, chunk=None, impl="auto", d_tile=0, cpu_sample_heads=2,
             no_cpu_baseline=True, copy_calibration_mib=0, serial_kernels=False, gated=False, recompute_states=False,
             forward_only=False, all_configs=False, sweep=False, decode_batch=0)
    a.update(kw)
    return argparse.Namespace(**a)


def test_bench_line_small_forward_config():
    b = _bench()
    name = "cfg2_bf16_p2_T8192_d64_c128"
    print("bench.run_workload", name, flush=True)
    j = json.loads(json.dumps(b.run_workload(_args(workload=name), name, cpu=False)))    # what bench.py prints
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "kernels", "timing"):
        assert key in j, key
    assert j["n_gpus"] == 1 and j["steps"] == 3 and j["warmup"] == 1 and j["unit"] == "tokens/s" and j["dtype"] == "bf16"
    assert j["config"]["workload"] == name and j["config"]["pass"] == "fwd"
    assert abs(j["value"] - 4 * 8192 / (j["ms_per_step"] * 1e-3)) < 1e-6 * j["value"]     # tokens/s = B T / step
    rf = j["roofline"]
    assert rf["bound"] in ("hbm", "mfma", "alu") and rf["unit"] in ("GB/s", "TFLOP/s")
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-9 and 0.0 < rf["frac"] < 1.0
    assert rf["kernel"] in j["kernels"]
    # the matrix-core kernels ran (not the vector-ALU fallback), and back to back they take about a step
    assert "mfma_state_scan" in j["kernels"] and "mfma_fwd_chunk" in j["kernels"]
    serial = sum(k["avg_ms"] * k["launches_per_step"] for k in j["kernels"].values())
    assert 0.5 * j["timing"]["step_ms_median"] < serial < 1.5 * j["timing"]["step_ms_median"]


def test_bench_sweep_lists_every_chunk_size():
    b = _bench()
    name = "cfg1_f32_p2_T256_d16_c32"
    print("bench.sweep", name, flush=True)
    out = io.StringIO()
    with contextlib.redirect_stdout(out):
        b.sweep(_args(workload=name, steps=2, sweep=True), name)
    lines = [l for l in out.getvalue().splitlines() if l.strip()]
    assert len(lines) == 1                     # one JSON line on stdout
    j = json.loads(lines[0])
    asked = [r["chunk_requested"] for r in j["sweep"]]
    assert asked == [32, 64, 128, 256, 0]      # f32: the vector-ALU kernels take any chunk; 256 = the whole sequence
    assert all(r["step_ms_median"] > 0 for r in j["sweep"])
    best = min((r for r in j["sweep"] if r["chunk_requested"]), key=lambda r: r["step_ms_median"])
    assert j["best"]["chunk"] == best["chunk"]
