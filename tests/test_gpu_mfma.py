"""GPU parity of the bf16 MFMA kernel family (p = 2) against the float64 oracle, element by
element, through the C ABI."""
import numpy as np
import pytest

from oracle import power_attn_oracle as orc
from paper_2507_04239_amd import inputs

from gpu_util import assert_close, run_fwd_bwd

pytestmark = pytest.mark.gpu

FWD_CASES = [
    # B, H, T, chunk, normalize, scale
    (1, 2, 512, 128, True, 1.0),
    (2, 1, 1024, 256, True, 1.0),      # two query blocks per chunk: unmasked + masked key blocks
    (1, 1, 128, 128, True, 1.0),       # a single chunk: attention form only
    (1, 3, 768, 128, True, 0.6),       # scale != 1, odd head count
    (1, 2, 512, 128, False, 1.0),      # un-normalised
    (1, 1, 1536, 512, True, 1.0),      # four query blocks per chunk
]


@pytest.mark.parametrize("case", FWD_CASES, ids=lambda c: "-".join(str(x) for x in c))
def test_mfma_forward_full_tensors(case):
    B, H, T, chunk, normalize, scale = case
    print("case", case, flush=True)
    Q, K, V, _ = inputs.make_qkvg(B, H, T, 64, seed=3000 + FWD_CASES.index(case), dtype="bf16", with_grad=False)
    got = run_fwd_bwd(Q, K, V, None, 2, chunk, "bf16", normalize, scale, impl="mfma", backward=False)
    O, Z = orc.fwd_bhtd(Q, K, V, 2, None, normalize, scale)
    assert_close(got, dict(O=O, Z=Z), "bf16", f"mfma fwd {case}")


BWD_CASES = [
    # B, H, T, chunk, normalize, scale
    (1, 2, 512, 128, True, 1.0),
    (1, 1, 1024, 256, True, 1.0),
    (1, 1, 128, 128, True, 1.0),
    (1, 2, 768, 128, True, 0.6),
    (1, 2, 512, 128, False, 1.0),
    (1, 1, 1536, 512, True, 1.0),
]


@pytest.mark.parametrize("keep_state", [False, True], ids=["recompute", "keep_state"])
@pytest.mark.parametrize("case", BWD_CASES, ids=lambda c: "-".join(str(x) for x in c))
def test_mfma_backward_full_tensors(case, keep_state):
    B, H, T, chunk, normalize, scale = case
    print("case", case, "keep_state", keep_state, flush=True)
    Q, K, V, G = inputs.make_qkvg(B, H, T, 64, seed=4000 + BWD_CASES.index(case), dtype="bf16")
    got = run_fwd_bwd(Q, K, V, G, 2, chunk, "bf16", normalize, scale, impl="mfma", keep_state=keep_state)
    O, Z = orc.fwd_bhtd(Q, K, V, 2, None, normalize, scale)
    dQ, dK, dV = orc.bwd_bhtd(Q, K, V, G, 2, None, normalize, scale)
    assert_close(got, dict(O=O, Z=Z, dQ=dQ, dK=dK, dV=dV), "bf16", f"mfma fwd+bwd {case}")
