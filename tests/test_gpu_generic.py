"""GPU parity of the generic (float32 vector-ALU) kernel family against the float64 oracle,
element by element, through the C ABI."""
import numpy as np
import pytest

from oracle import power_attn_oracle as orc
from paper_2507_04239_amd import inputs

from gpu_util import assert_close, run_fwd_bwd

pytestmark = pytest.mark.gpu


def _oracle_all(Q, K, V, G, p, normalize, scale):
    O, Z = orc.fwd_bhtd(Q, K, V, p, None, normalize, scale)
    dQ, dK, dV = orc.bwd_bhtd(Q, K, V, G, p, None, normalize, scale)
    return dict(O=O, Z=Z, dQ=dQ, dK=dK, dV=dV)


def test_config1_f32_forward():
    """fp32, p=2, B1 H1 T256 d16 chunk 32, normalised: the whole output against brute force."""
    w = inputs.WORKLOADS["cfg1_f32_p2_T256_d16_c32"]
    Q, K, V, _ = inputs.make_workload("cfg1_f32_p2_T256_d16_c32", with_grad=False)
    print("case cfg1", flush=True)
    got = run_fwd_bwd(Q, K, V, None, w["p"], w["chunk"], "f32", impl="generic", backward=False)
    O, Z = orc.fwd_bhtd(Q, K, V, w["p"], None)
    assert_close(got, dict(O=O, Z=Z), "f32", "cfg1 generic")


CASES = [
    # dtype, p, B, H, T, d, v, chunk, normalize, scale
    ("f32", 2, 1, 2, 256, 16, 16, 32, True, 1.0),
    ("f32", 2, 2, 1, 192, 64, 64, 64, True, 0.5),      # several LDS tiles per chunk, scale != 1
    ("f32", 4, 1, 2, 160, 8, 8, 32, True, 1.0),
    ("f32", 4, 1, 1, 96, 32, 32, 96, True, 1.3),       # one chunk only (pure attention form), 96-token tail pass
    ("f32", 3, 1, 2, 128, 12, 20, 16, False, 1.0),     # odd p, un-normalised, v != d, d not a multiple of 8
    ("f32", 1, 1, 1, 64, 8, 4, 8, False, 2.0),
    ("f32", 2, 1, 1, 40, 4, 4, 1, True, 1.0),          # chunk 1: pure recurrence
    ("bf16", 2, 1, 2, 256, 64, 64, 128, True, 1.0),
    ("bf16", 4, 1, 2, 256, 32, 32, 128, True, 1.0),
    ("bf16", 2, 1, 1, 512, 128, 128, 256, True, 1.0),
    ("f32", 2, 1, 1, 200, 24, 24, 100, False, 1.0),    # chunk not a multiple of the 64-token pass
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "-".join(str(x) for x in c))
def test_generic_full_tensors(case):
    dtype, p, B, H, T, d, v, chunk, normalize, scale = case
    print("case", case, flush=True)
    Q, K, V, G = inputs.make_qkvg(B, H, T, d, seed=2000 + CASES.index(case), dtype=dtype, v=v)
    got = run_fwd_bwd(Q, K, V, G, p, chunk, dtype, normalize, scale, impl="generic")
    want = _oracle_all(Q, K, V, G, p, normalize, scale)
    assert_close(got, want, dtype, f"generic {case}")


def test_zero_denominator_rows():
    Q, K, V, G = inputs.make_qkvg(1, 1, 64, 8, seed=5, dtype="f32")
    Q[0, 0, 10] = 0.0
    got = run_fwd_bwd(Q, K, V, G, 2, 16, "f32", impl="generic")
    assert (got["O"][0, 0, 10] == 0).all() and got["Z"][0, 0, 10] == 0
    want = _oracle_all(Q, K, V, G, 2, True, 1.0)
    assert_close(got, want, "f32", "zero-denominator row")


def test_invalid_arguments_are_rejected():
    import torch
    from paper_2507_04239_amd import PowerAttnError, power_attn_fwd
    q = torch.zeros(1, 1, 64, 8, device="cuda:0")
    with pytest.raises(PowerAttnError):
        power_attn_fwd(q, q, q, 2, 48)                   # chunk does not divide T
    with pytest.raises(PowerAttnError):
        power_attn_fwd(q, q, q, 3, 16, normalize=True)   # odd p cannot be normalised
    with pytest.raises(PowerAttnError):
        power_attn_fwd(q, q, q, 7, 16, normalize=False)  # no kernel for p = 7
    with pytest.raises(PowerAttnError):
        power_attn_fwd(q.cpu(), q.cpu(), q.cpu(), 2, 16)


def test_automatic_chunk_matches_the_explicit_one():
    import torch
    from gpu_util import to_dev, to_np
    from paper_2507_04239_amd import binding, power_attn_bwd, power_attn_fwd
    for (B, H, T, d, dtype) in ((1, 2, 1024, 64, "bf16"), (1, 1, 2048, 64, "bf16"), (1, 1, 512, 16, "f32")):
        Q, K, V, G = inputs.make_qkvg(B, H, T, d, seed=900 + T, dtype=dtype)
        prob = binding.make_problem(B, H, T, d, d, 2, 0, True, 1.0, dtype)
        c = binding.power_attn_resolved_chunk(prob)
        assert c > 0 and T % c == 0
        a = run_fwd_bwd(Q, K, V, G, 2, 0, dtype)
        b = run_fwd_bwd(Q, K, V, G, 2, c, dtype)
        for key in a:
            np.testing.assert_array_equal(a[key], b[key], err_msg=f"T={T} chunk 0 vs {c}: {key}")
