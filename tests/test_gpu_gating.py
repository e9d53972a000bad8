"""GPU parity of the gated layer (arXiv 2507.04239 Sec. 2 "Gating", App. E.2 / E.3) against the
float64 oracle, element by element, through the C ABI."""
import numpy as np
import pytest

from oracle import power_attn_oracle as orc
from paper_2507_04239_amd import inputs

from gpu_util import assert_close, run_fwd_bwd

pytestmark = pytest.mark.gpu

CASES = [
    # dtype, impl, p, B, H, T, d, chunk, normalize, scale, mean decay per step
    ("f32", "generic", 2, 1, 2, 256, 16, 32, True, 1.0, 0.02),
    ("f32", "generic", 4, 1, 1, 192, 8, 64, True, 0.8, 0.05),
    ("f32", "generic", 3, 2, 1, 96, 8, 32, False, 1.0, 0.02),
    ("f32", "generic", 2, 1, 1, 160, 12, 160, True, 1.0, 0.01),     # a single chunk: attention form only
    ("f32", "generic", 2, 1, 1, 130, 10, 26, False, 1.3, 0.3),      # strong decay, ragged sizes
    ("bf16", "generic", 2, 1, 2, 384, 32, 128, True, 1.0, 0.02),
    ("bf16", "generic", 4, 1, 1, 256, 16, 64, True, 1.0, 0.02),
    ("bf16", "generic", 2, 1, 1, 256, 32, 64, True, 1.0, 0.5),      # strong decay: the gate gradient is a small
    ("bf16", "generic", 4, 1, 1, 256, 16, 64, False, 1.0, 0.5),     # difference of sums that nearly cancel
    ("bf16", "mfma", 2, 1, 2, 512, 64, 128, True, 1.0, 0.02),
    ("bf16", "mfma", 2, 1, 1, 1024, 64, 256, True, 1.0, 0.01),     # two query blocks per chunk
    ("bf16", "mfma", 2, 1, 1, 128, 64, 128, True, 1.0, 0.05),      # a single chunk
    ("bf16", "mfma", 2, 1, 2, 768, 64, 128, True, 0.6, 0.1),       # scale != 1, stronger decay
    ("bf16", "mfma", 2, 1, 1, 512, 64, 128, False, 1.0, 0.02),     # un-normalised
    ("bf16", "mfma", 2, 1, 1, 1536, 64, 512, True, 1.0, 0.005),
    ("bf16", "mfma", 2, 1, 1, 4096, 64, 256, True, 1.0, 0.01),     # block ids of a chunk dealt out 8 apart
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "-".join(str(x) for x in c))
def test_gated_forward_backward(case):
    dtype, impl, p, B, H, T, d, chunk, normalize, scale, decay = case
    print("case", case, flush=True)
    seed = 7000 + CASES.index(case)
    Q, K, V, G = inputs.make_qkvg(B, H, T, d, seed=seed, dtype=dtype)
    lg = inputs.make_log_gates(B, H, T, seed + 500, decay)
    got = run_fwd_bwd(Q, K, V, G, p, chunk, dtype, normalize, scale, impl=impl, log_g=lg)
    if impl == "mfma":   # also with the states kept from the forward pass
        kept = run_fwd_bwd(Q, K, V, G, p, chunk, dtype, normalize, scale, impl=impl, log_g=lg, keep_state=True)
        for key in got:
            np.testing.assert_array_equal(kept[key], got[key], err_msg=f"keep_state changes {key}")
    O, Z = orc.fwd_bhtd(Q, K, V, p, None, normalize, scale, log_g=lg.astype(np.float64))
    dQ, dK, dV, dL = orc.bwd_bhtd(Q, K, V, G, p, None, normalize, scale, log_g=lg.astype(np.float64))
    assert_close(got, dict(O=O, Z=Z, dQ=dQ, dK=dK, dV=dV, dlog_g=dL), dtype, f"gated {case}")


def test_zero_log_gates_match_the_ungated_calls():
    Q, K, V, G = inputs.make_qkvg(1, 2, 256, 16, seed=7100, dtype="f32")
    zero = np.zeros((1, 2, 256), dtype=np.float32)
    a = run_fwd_bwd(Q, K, V, G, 2, 64, "f32", impl="generic", log_g=zero)
    b = run_fwd_bwd(Q, K, V, G, 2, 64, "f32", impl="generic")
    for key in ("O", "Z", "dQ", "dK", "dV"):
        np.testing.assert_allclose(a[key], b[key], rtol=1e-6, atol=1e-7)


def test_gated_and_ungated_entry_points_refuse_each_other():
    import ctypes
    import torch
    from paper_2507_04239_amd import binding
    lib = binding.load_library()
    prob = binding.make_problem(1, 1, 64, 16, 16, 2, 32, True, 1.0, "f32", "generic", False, True)
    x = torch.zeros(1, 1, 64, 16, device="cuda:0")
    z = torch.zeros(1, 1, 64, device="cuda:0")
    ws = torch.empty(max(binding.power_attn_workspace_bytes(prob, False), 256), dtype=torch.uint8, device="cuda:0")
    vp = lambda t: ctypes.c_void_p(t.data_ptr())
    st = lib.power_attn_fwd(ctypes.byref(prob), vp(x), vp(x), vp(x), vp(x), vp(z), vp(ws), ws.numel(), None)
    assert st == 1   # PA_ERR_INVALID_ARG: a gated problem through the un-gated call
    st = lib.power_attn_fwd_gated(ctypes.byref(prob), vp(x), vp(x), vp(x), None, vp(x), vp(z), vp(ws), ws.numel(), None)
    assert st == 1   # log_g missing
