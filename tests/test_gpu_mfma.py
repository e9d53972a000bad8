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
    (1, 1, 4096, 256, True, 1.0),      # 32 blocks of 128 tokens: the blocks of a chunk are dealt out 8 ids apart
    (1, 1, 4096, 512, True, 1.0),      # the same with four blocks per chunk
    (1, 1, 3072, 384, True, 1.0),      # three blocks per chunk, 24 blocks: one full group of the dealing
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


def test_mfma_back_to_back_steps_share_workspace():
    """Two forward+backward steps with different inputs, queued one after the other on the same
    workspace without host synchronisation in between: the second forward pass overwrites states
    the first backward pass (which runs part of its kernels on a stream of the library's own)
    still reads unless the passes are ordered correctly."""
    import torch
    from paper_2507_04239_amd import binding, power_attn_bwd, power_attn_fwd
    from gpu_util import to_dev, to_np
    B, H, T, chunk = 1, 2, 1024, 128
    prob = binding.make_problem(B, H, T, 64, 64, 2, chunk, True, 1.0, "bf16", "mfma", True)
    ws = torch.empty(max(binding.power_attn_workspace_bytes(prob, True), 256), dtype=torch.uint8, device="cuda:0")
    steps = []
    for seed in (5001, 5002, 5003):
        Q, K, V, G = inputs.make_qkvg(B, H, T, 64, seed=seed, dtype="bf16")
        steps.append((Q, K, V, G, [to_dev(a, "bf16") for a in (Q, K, V, G)]))
    results = []
    for _, _, _, _, (tq, tk, tv, tg) in steps:   # no synchronisation between the steps
        O, Z = power_attn_fwd(tq, tk, tv, 2, chunk, impl="mfma", workspace=ws, keep_state=True)
        dQ, dK, dV = power_attn_bwd(tq, tk, tv, O, Z, tg, 2, chunk, impl="mfma", workspace=ws, keep_state=True)
        results.append(dict(O=O, Z=Z, dQ=dQ, dK=dK, dV=dV))
    torch.cuda.synchronize()
    for i, (Q, K, V, G, _) in enumerate(steps):
        O, Z = orc.fwd_bhtd(Q, K, V, 2, None, True, 1.0)
        dQ, dK, dV = orc.bwd_bhtd(Q, K, V, G, 2, None, True, 1.0)
        assert_close({k: to_np(t) for k, t in results[i].items()}, dict(O=O, Z=Z, dQ=dQ, dK=dK, dV=dV), "bf16",
                     f"mfma back-to-back step {i}")


def test_mfma_on_a_side_stream_of_the_caller():
    """The calls are queued on the caller's current stream, whichever that is."""
    import torch
    from gpu_util import to_dev, to_np
    from paper_2507_04239_amd import power_attn_bwd, power_attn_fwd
    Q, K, V, G = inputs.make_qkvg(1, 1, 512, 64, seed=5010, dtype="bf16")
    tq, tk, tv, tg = (to_dev(a, "bf16") for a in (Q, K, V, G))
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        O, Z = power_attn_fwd(tq, tk, tv, 2, 128, impl="mfma")
        dQ, dK, dV = power_attn_bwd(tq, tk, tv, O, Z, tg, 2, 128, impl="mfma")
    stream.synchronize()
    Oo, Zo = orc.fwd_bhtd(Q, K, V, 2, None, True, 1.0)
    dQo, dKo, dVo = orc.bwd_bhtd(Q, K, V, G, 2, None, True, 1.0)
    assert_close({k: to_np(t) for k, t in dict(O=O, Z=Z, dQ=dQ, dK=dK, dV=dV).items()},
                 dict(O=Oo, Z=Zo, dQ=dQo, dK=dKo, dV=dVo), "bf16", "mfma on a caller's side stream")


def test_mfma_zero_rows():
    """Queries that are all zero have Z = 0: O = 0 and no gradient flows through the row; zero keys
    and values contribute nothing."""
    Q, K, V, G = inputs.make_qkvg(1, 1, 384, 64, seed=5020, dtype="bf16")
    Q[0, 0, 5] = 0
    Q[0, 0, 200] = 0
    K[0, 0, 17] = 0
    V[0, 0, 130] = 0
    got = run_fwd_bwd(Q, K, V, G, 2, 128, "bf16", True, 1.0, impl="mfma")
    O, Z = orc.fwd_bhtd(Q, K, V, 2, None, True, 1.0)
    dQ, dK, dV = orc.bwd_bhtd(Q, K, V, G, 2, None, True, 1.0)
    assert_close(got, dict(O=O, Z=Z, dQ=dQ, dK=dK, dV=dV), "bf16", "mfma zero rows")
    assert (got["O"][0, 0, 5] == 0).all() and (got["dQ"][0, 0, 5] == 0).all()


RAGGED_CASES = [
    # B, H, T, chunk, normalize, gated
    (1, 2, 300, 128, True, False),       # 2 whole chunks + 44 tokens
    (2, 1, 517, 256, True, False),
    (1, 1, 129, 128, False, False),      # one token beyond a chunk
    (1, 2, 400, 128, True, True),
    (1, 1, 100, 128, True, False),       # shorter than one chunk
]


@pytest.mark.parametrize("keep_state", [False, True], ids=["recompute", "keep_state"])
@pytest.mark.parametrize("case", RAGGED_CASES, ids=lambda c: "-".join(str(x) for x in c))
def test_mfma_ragged_last_chunk(case, keep_state):
    """A sequence that is not a multiple of the chunk: the chunked kernels run it padded with zero
    rows; every output of the T real tokens against the oracle."""
    B, H, T, chunk, normalize, gated = case
    print("case", case, "keep_state", keep_state, flush=True)
    Q, K, V, G = inputs.make_qkvg(B, H, T, 64, seed=5100 + RAGGED_CASES.index(case), dtype="bf16")
    lg = inputs.make_log_gates(B, H, T, 5150 + RAGGED_CASES.index(case), 0.03) if gated else None
    got = run_fwd_bwd(Q, K, V, G, 2, chunk, "bf16", normalize, 1.0, impl="mfma", keep_state=keep_state, log_g=lg)
    O, Z = orc.fwd_bhtd(Q, K, V, 2, None, normalize, 1.0, log_g=lg)
    ref = orc.bwd_bhtd(Q, K, V, G, 2, None, normalize, 1.0, log_g=lg)
    want = dict(O=O, Z=Z, dQ=ref[0], dK=ref[1], dV=ref[2])
    if gated:
        want["dlog_g"] = ref[3]
    for k, a in got.items():
        assert a.shape[2] == T, k
    assert_close(got, want, "bf16", f"mfma ragged {case}")


def test_automatic_chunk_on_a_long_ragged_sequence():
    """chunk = 0 at a length that no chunk divides and that is too long for the attention form: the chunked
    kernels on the padded sequence; sampled rows by the definition."""
    from paper_2507_04239_amd import binding
    T = 8192 + 37
    prob = binding.make_problem(1, 1, T, 64, 64, 2, 0)
    assert binding.power_attn_resolved_chunk(prob) == 256
    Q, K, V, G = inputs.make_qkvg(1, 1, T, 64, seed=5200, dtype="bf16")
    got = run_fwd_bwd(Q, K, V, G, 2, 0, "bf16")
    q, k, v = (a[0, 0].astype(np.float64) for a in (Q, K, V))
    rows = [0, 255, 256, 4096, 8191, 8192, T - 2, T - 1]
    o_ref = np.stack([orc.fwd_row(q, k, v, i, 2)[0] for i in rows])
    dq_ref = np.stack([orc.bwd_dq_row(q, k, v, G[0, 0].astype(np.float64), i, 2) for i in rows])
    from gpu_util import TOL, rel_l2
    assert rel_l2(got["O"][0, 0][rows], o_ref) <= TOL["bf16"]
    assert rel_l2(got["dQ"][0, 0][rows], dq_ref) <= TOL["bf16"]
