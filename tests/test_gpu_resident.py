"""GPU parity of the resident-state kernels (chunk states kept in registers, impl = "resident") against the
float64 oracle and against the kernels that store the chunk states."""
import numpy as np
import pytest

from oracle import power_attn_oracle as orc
from paper_2507_04239_amd import inputs

from gpu_util import assert_close, run_fwd_bwd

pytestmark = pytest.mark.gpu

# (B, H, T, chunk, scale): one segment (many heads), several segments (few heads, long), ragged segment split,
# several stages per chunk
FWD_CASES = [
    (1, 2, 512, 128, 1.0),
    (2, 3, 1024, 256, 1.0),
    (1, 1, 128 * 23, 128, 1.0),
    (1, 2, 128 * 40, 128, 0.7),
    (4, 24, 256, 128, 1.0),
    (1, 1, 384 * 5, 384, 1.0),
]


@pytest.mark.parametrize("B,H,T,chunk,scale", FWD_CASES)
def test_resident_forward(B, H, T, chunk, scale):
    Q, K, V, _ = inputs.make_qkvg(B, H, T, 64, seed=4000 + T + H, dtype="bf16", with_grad=False)
    print("case", (B, H, T, chunk, scale), flush=True)
    got = run_fwd_bwd(Q, K, V, None, 2, chunk, "bf16", scale=scale, impl="resident", backward=False)
    O, Z = orc.fwd_bhtd(Q, K, V, 2, chunk, True, scale)
    assert_close(got, dict(O=O, Z=Z), "bf16", f"resident fwd {(B, H, T, chunk, scale)}")


# d = 128: 68 pairs in 17 slabs per head, stages of 64 tokens
FWD_CASES_128 = [
    (1, 1, 512, 256, 1.0),
    (1, 2, 1024, 128, 1.0),
    (2, 2, 768, 256, 0.8),
    (1, 1, 256 * 9, 256, 1.0),
]


@pytest.mark.parametrize("B,H,T,chunk,scale", FWD_CASES_128)
def test_resident_forward_d128(B, H, T, chunk, scale):
    Q, K, V, _ = inputs.make_qkvg(B, H, T, 128, seed=4100 + T + H, dtype="bf16", with_grad=False)
    print("case d128", (B, H, T, chunk, scale), flush=True)
    got = run_fwd_bwd(Q, K, V, None, 2, chunk, "bf16", scale=scale, impl="resident", backward=False)
    O, Z = orc.fwd_bhtd(Q, K, V, 2, chunk, True, scale)
    assert_close(got, dict(O=O, Z=Z), "bf16", f"resident fwd d128 {(B, H, T, chunk, scale)}")


# forward + backward: (B, H, T, d, chunk, scale, keep_state)
BWD_CASES = [
    (1, 2, 512, 64, 128, 1.0, False),
    (1, 1, 128 * 23, 64, 128, 1.0, True),
    (2, 2, 1024, 64, 256, 0.7, True),
    (1, 1, 512, 128, 256, 1.0, False),
    (1, 2, 1024, 128, 128, 1.0, True),
    (1, 1, 256 * 7, 128, 256, 0.8, True),
]


@pytest.mark.parametrize("B,H,T,d,chunk,scale,keep", BWD_CASES)
def test_resident_forward_backward(B, H, T, d, chunk, scale, keep):
    Q, K, V, G = inputs.make_qkvg(B, H, T, d, seed=4200 + T + H + d, dtype="bf16")
    print("case bwd", (B, H, T, d, chunk, scale, keep), flush=True)
    got = run_fwd_bwd(Q, K, V, G, 2, chunk, "bf16", scale=scale, impl="resident", keep_state=keep)
    O, Z = orc.fwd_bhtd(Q, K, V, 2, chunk, True, scale)
    dQ, dK, dV = orc.bwd_bhtd(Q, K, V, G, 2, chunk, True, scale)
    assert_close(got, dict(O=O, Z=Z, dQ=dQ, dK=dK, dV=dV), "bf16", f"resident fwd+bwd {(B, H, T, d, chunk, scale, keep)}")
