"""Host-side checks of bench.py (no GPU): the one-GPU contract, and the algorithmic FLOP / byte models that the
roofline figures are computed from, against numbers worked out by hand for the headline workload."""
import importlib.util
import math
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, cwd=ROOT)
    assert r.returncode != 0
    assert "one GPU" in r.stderr


def test_algorithmic_models_headline():
    b = _bench()
    w = dict(B=1, H=12, T=65536, d=64, p=2, chunk=128, dtype="bf16")
    D = 64 * 65 // 2                       # symmetric monomials of degree 2 in 64 variables (Lemma 4.2)
    assert D == math.comb(65, 2) == 2080
    fl, by = b.algorithmic_flops(w), b.algorithmic_bytes(w)
    n = 512
    state = 12 * (n - 1) * 128 * 2 * D * 65          # D x (v + 1) contraction for every token of the 511 chunks that use a state
    assert fl["update_state"] == fl["state_grad"] == fl["query_state"] == fl["dphi"] == state
    pairs = 12 * n * (128 * 129 // 2)                # causal (query, key) pairs inside the chunks
    assert fl["fwd_chunk"] == state + pairs * (2 * 64 + 2 * 65)
    assert fl["fwd_total"] == fl["update_state"] + fl["fwd_chunk"]
    states_bytes = 12 * (n - 1) * D * 65 * 2
    assert abs(states_bytes - 1.658e9) < 1e6          # the symmetric state; the tiled layout stores 36 x 64 x 68 per chunk
    tok = 12 * 65536 * 64 * 2
    assert by["update_state"] == states_bytes + 2 * tok
    assert by["fwd_chunk"] == states_bytes + 4 * tok + 12 * 65536 * 4
    # every kernel name the library reports for the matrix-core families has a role in both models
    for name, (role, peak) in b.KERNEL_ROLE.items():
        assert role in fl and role in by, name
        assert peak in (b.PEAK_BF16_MFMA_TFLOPS, b.PEAK_FP32_VECTOR_TFLOPS)
    assert b.PEAK_HBM_GBS == 8000.0 and b.PEAK_BF16_MFMA_TFLOPS == 2500.0


def test_algorithmic_models_scale_with_degree_and_head_size():
    b = _bench()
    w4 = dict(B=2, H=8, T=16384, d=32, p=4, chunk=128, dtype="bf16")
    assert math.comb(35, 4) == 52360
    assert b.algorithmic_flops(w4)["update_state"] == 16 * 127 * 128 * 2 * 52360 * 33
    w5 = dict(B=8, H=16, T=32768, d=128, p=2, chunk=256, dtype="bf16")
    assert b.algorithmic_bytes(w5)["query_state"] == 128 * 127 * 8256 * 129 * 2 + 128 * 32768 * 128 * 2 + 128 * 32768 * 129 * 4
