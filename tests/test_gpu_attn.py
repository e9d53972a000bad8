"""GPU parity of the bf16 MFMA attention-form kernels (one chunk = the whole sequence; degrees 2, 3, 4,
head sizes 32, 64, 128) against the float64 oracle, element by element, through the C ABI."""
import numpy as np
import pytest

from oracle import power_attn_oracle as orc
from paper_2507_04239_amd import binding, inputs

from gpu_util import assert_close, run_fwd_bwd

pytestmark = pytest.mark.gpu

CASES = [
    # p, d, B, H, T, normalize, scale
    (4, 32, 1, 2, 512, True, 1.0),       # config 4's degree and head size
    (4, 32, 1, 1, 64, True, 1.0),        # a single tile: the diagonal only
    (4, 32, 2, 1, 320, True, 1.3),       # a block that is not full (320 = 256 + 64), scale != 1
    (2, 128, 1, 2, 512, True, 1.0),      # config 5's head size
    (2, 128, 1, 1, 192, True, 0.7),      # not a multiple of the block of either kernel
    (2, 128, 1, 1, 704, False, 1.0),     # un-normalised
    (2, 32, 1, 1, 384, True, 1.0),
    (4, 64, 1, 1, 448, True, 1.0),
    (4, 128, 1, 1, 256, True, 1.0),
    (3, 64, 1, 2, 384, False, 1.0),      # odd degree: signed weights, un-normalised only
    (3, 32, 1, 1, 128, False, 0.8),
    (3, 128, 1, 1, 320, False, 1.0),
    # sequence lengths that are not a multiple of the 64-row tile, nor of a wave's rows
    (2, 64, 1, 2, 333, True, 1.0),
    (4, 32, 1, 1, 65, True, 1.0),
    (2, 128, 1, 1, 271, True, 1.0),
    (2, 64, 1, 1, 17, True, 1.0),
    (3, 32, 2, 1, 100, False, 1.0),
    (2, 128, 1, 1, 1, True, 1.0),        # a single token
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "-".join(str(x) for x in c))
def test_attention_form_forward_backward(case):
    p, d, B, H, T, normalize, scale = case
    print("case", case, flush=True)
    prob = binding.make_problem(B, H, T, d, d, p, T, normalize, scale, "bf16", "mfma")
    assert binding.power_attn_supported(prob, True)
    assert binding.power_attn_state_rows(prob) == 0          # no state is built
    Q, K, V, G = inputs.make_qkvg(B, H, T, d, seed=7000 + CASES.index(case), dtype="bf16")
    got = run_fwd_bwd(Q, K, V, G, p, T, "bf16", normalize, scale, impl="mfma")
    O, Z = orc.fwd_bhtd(Q, K, V, p, None, normalize, scale)
    dQ, dK, dV = orc.bwd_bhtd(Q, K, V, G, p, None, normalize, scale)
    assert_close(got, dict(O=O, Z=Z, dQ=dQ, dK=dK, dV=dV), "bf16", f"attention form {case}")


def test_auto_chunk_picks_the_attention_form_for_other_shapes():
    """chunk = 0 with a degree / head size the chunked matrix-core kernels do not have: the library
    runs the attention form on the matrix cores rather than the chunked form on the vector ALUs."""
    for p, d in ((4, 32), (2, 128)):
        prob = binding.make_problem(1, 1, 2048, d, d, p, 0, True, 1.0, "bf16", "auto")
        assert binding.power_attn_resolved_chunk(prob) == 2048
    Q, K, V, G = inputs.make_qkvg(1, 1, 256, 32, seed=7100, dtype="bf16")
    got = run_fwd_bwd(Q, K, V, G, 4, 0, "bf16")
    O, Z = orc.fwd_bhtd(Q, K, V, 4, None, True, 1.0)
    dQ, dK, dV = orc.bwd_bhtd(Q, K, V, G, 4, None, True, 1.0)
    assert_close(got, dict(O=O, Z=Z, dQ=dQ, dK=dK, dV=dV), "bf16", "auto chunk, p = 4, d = 32")


def test_attention_form_zero_rows():
    """All-zero queries have Z = 0: O = 0 and no gradient through the row."""
    Q, K, V, G = inputs.make_qkvg(1, 1, 256, 32, seed=7200, dtype="bf16")
    Q[0, 0, 3] = 0
    Q[0, 0, 130] = 0
    K[0, 0, 70] = 0
    got = run_fwd_bwd(Q, K, V, G, 4, 256, "bf16", impl="mfma")
    O, Z = orc.fwd_bhtd(Q, K, V, 4, None, True, 1.0)
    dQ, dK, dV = orc.bwd_bhtd(Q, K, V, G, 4, None, True, 1.0)
    assert_close(got, dict(O=O, Z=Z, dQ=dQ, dK=dK, dV=dV), "bf16", "attention form zero rows")
    assert (got["O"][0, 0, 3] == 0).all() and (got["dQ"][0, 0, 3] == 0).all()


GATED_CASES = [
    # p, d, B, H, T, normalize, scale, mean decay per step
    (4, 32, 1, 2, 768, True, 1.0, 0.02),       # three blocks of 256 keys
    (2, 128, 1, 2, 512, True, 1.0, 0.02),      # four blocks of 128
    (2, 64, 1, 1, 640, True, 0.7, 0.05),
    (4, 64, 1, 1, 256, True, 1.0, 0.01),
    (3, 64, 1, 2, 384, False, 1.0, 0.03),      # un-normalised: the q . dq term of the gate gradient counts
    (2, 32, 2, 1, 256, False, 1.0, 0.5),       # strong decay: the factors underflow far from the diagonal
    (2, 32, 2, 1, 256, True, 1.0, 0.5),        # normalised: the rounding of O_i enters every e_ij = ghat_i . (v_j - O_i);
    (2, 32, 2, 1, 256, True, 1.0, 0.15),       # it cancels between the row term and the column terms of the gate gradient
    (2, 128, 1, 1, 128, True, 1.0, 0.02),      # a single block: no boundary sums
]


@pytest.mark.parametrize("case", GATED_CASES, ids=lambda c: "-".join(str(x) for x in c))
def test_gated_attention_form(case):
    """Per-timestep gates in the attention-form kernels: outputs, dQ, dK, dV and the gradient of the
    log-gates against the float64 oracle."""
    p, d, B, H, T, normalize, scale, decay = case
    print("case", case, flush=True)
    Q, K, V, G = inputs.make_qkvg(B, H, T, d, seed=7300 + GATED_CASES.index(case), dtype="bf16")
    lg = inputs.make_log_gates(B, H, T, 7400 + GATED_CASES.index(case), decay)
    prob = binding.make_problem(B, H, T, d, d, p, T, normalize, scale, "bf16", "mfma", False, True)
    assert binding.power_attn_supported(prob, True)
    got = run_fwd_bwd(Q, K, V, G, p, T, "bf16", normalize, scale, impl="mfma", log_g=lg)
    O, Z = orc.fwd_bhtd(Q, K, V, p, None, normalize, scale, log_g=lg)
    dQ, dK, dV, dL = orc.bwd_bhtd(Q, K, V, G, p, None, normalize, scale, log_g=lg)
    assert_close(got, dict(O=O, Z=Z, dQ=dQ, dK=dK, dV=dV, dlog_g=dL), "bf16", f"gated attention form {case}")


def test_gated_attention_form_long():
    """Gate gradient over many blocks (T = 8192, d = 128: 64 blocks): the part that crosses block
    boundaries comes from the block sums, not from a running sum over the sequence."""
    p, d, T = 2, 128, 8192
    Q, K, V, G = inputs.make_qkvg(1, 1, T, d, seed=7500, dtype="bf16")
    lg = inputs.make_log_gates(1, 1, T, 7501, 0.02)
    print("case gated attention form long", flush=True)
    got = run_fwd_bwd(Q, K, V, G, p, T, "bf16", impl="mfma", log_g=lg)
    lg64 = lg[0, 0].astype(np.float64)
    O, Z = orc.fwd_chunked_gated(Q[0, 0], K[0, 0], V[0, 0], lg64, p, 512)
    dQ, dK, dV, dL = orc.bwd_chunked_gated(Q[0, 0], K[0, 0], V[0, 0], lg64, G[0, 0], p, 512)
    assert_close({k: a[0, 0] for k, a in got.items()}, dict(O=O, Z=Z, dQ=dQ, dK=dK, dV=dV, dlog_g=dL), "bf16",
                 "gated attention form T = 8192")
