"""GPU parity of the tiled chunked kernels (impl = "tiled": degree and tile width of the embedding as
parameters, chunk states in memory) against the float64 oracle, for every (p, d_tile, d) they are built for.
The reference is the definition (the oracle's attention form): the chunked form computes the same function
(App. A; the oracle's own chunked form is pinned to it on the CPU), and with the explicit state of 52360 rows
the oracle's chunked form of p = 4 takes a minute per case."""
import numpy as np
import pytest

from oracle import power_attn_oracle as orc
from paper_2507_04239_amd import inputs

from gpu_util import assert_close, run_fwd_bwd

pytestmark = pytest.mark.gpu

# (p, d_tile, d): tiles of 16, 64 and 256 rows; one and two features per side of a row's product
SHAPES = [
    (2, 4, 32), (2, 8, 32), (2, 16, 32), (3, 4, 32), (4, 2, 32), (4, 4, 32),
    (2, 4, 64), (2, 8, 64), (2, 16, 64), (3, 4, 64),
    (2, 8, 128),
]


@pytest.mark.parametrize("p,dt,d", SHAPES)
def test_tiled_forward_backward(p, dt, d):
    B, H, T, chunk = 1, 2, 512, 128
    norm = p % 2 == 0
    Q, K, V, G = inputs.make_qkvg(B, H, T, d, seed=5000 + 100 * p + dt + d, dtype="bf16")
    print("case", (p, dt, d), flush=True)
    got = run_fwd_bwd(Q, K, V, G, p, chunk, "bf16", normalize=norm, impl="tiled", d_tile=dt)
    O, Z = orc.fwd_bhtd(Q, K, V, p, None, norm, 1.0)
    dQ, dK, dV = orc.bwd_bhtd(Q, K, V, G, p, None, norm, 1.0)
    want = dict(O=O, Z=Z, dQ=dQ, dK=dK, dV=dV) if norm else dict(O=O, dQ=dQ, dK=dK, dV=dV)
    assert_close(got, want, "bf16", f"tiled {(p, dt, d)}")


# (p, d_tile, d, B, H, T, chunk, scale, keep_state): larger chunks, several heads, kept states, a scale
CASES = [
    (4, 4, 32, 2, 2, 1024, 256, 0.8, True),
    (4, 2, 32, 1, 3, 768, 128, 1.0, True),
    (3, 4, 32, 1, 2, 1024, 512, 0.7, False),
    (2, 8, 64, 1, 2, 1024, 256, 1.0, True),
    (3, 4, 64, 1, 1, 512, 128, 1.2, True),
    (4, 2, 32, 1, 2, 640, 128, 1.0, False),     # 2.5 blocks of the in-chunk kernels' 256 queries
    (2, 8, 32, 3, 5, 256, 128, 1.0, True),      # two chunks, odd head count
    (3, 4, 64, 1, 2, 2048, 256, 1.0, True),     # 816 tiles, 16 chunks
    (2, 16, 64, 2, 2, 2048, 128, 0.9, False),   # 256-row tiles
    (4, 4, 32, 1, 1, 4096, 128, 1.0, True),     # 32 chunks
    (2, 8, 128, 1, 2, 2048, 256, 0.8, True),    # d = 128: 136 tiles, two 128-token blocks per chunk
    (2, 8, 128, 2, 1, 4096, 256, 1.0, False),   # 16 blocks per head: the blocks of a chunk are dealt 8 apart
    (2, 8, 128, 2, 4, 512, 256, 1.0, True),     # a multiple of 8 heads: the scan keeps a head's workgroups on one XCD
    (4, 2, 32, 4, 4, 256, 128, 0.9, False),     # ... 16 heads, 243 workgroups each
    (3, 4, 64, 8, 1, 384, 128, 1.0, True),      # ... 8 heads, three chunks
]


@pytest.mark.parametrize("p,dt,d,B,H,T,chunk,scale,keep", CASES)
def test_tiled_shapes(p, dt, d, B, H, T, chunk, scale, keep):
    norm = p % 2 == 0
    Q, K, V, G = inputs.make_qkvg(B, H, T, d, seed=5100 + T + 10 * p + dt, dtype="bf16")
    print("case", (p, dt, d, B, H, T, chunk, scale, keep), flush=True)
    got = run_fwd_bwd(Q, K, V, G, p, chunk, "bf16", normalize=norm, scale=scale, impl="tiled", keep_state=keep, d_tile=dt)
    O, Z = orc.fwd_bhtd(Q, K, V, p, None, norm, scale)
    dQ, dK, dV = orc.bwd_bhtd(Q, K, V, G, p, None, norm, scale)
    want = dict(O=O, Z=Z, dQ=dQ, dK=dK, dV=dV) if norm else dict(O=O, dQ=dQ, dK=dK, dV=dV)
    assert_close(got, want, "bf16", f"tiled {(p, dt, d, B, H, T, chunk, scale, keep)}")


def test_automatic_choice_runs_the_tiled_kernels_for_degree_four():
    """The chunked form of p = 4, d = 32 with no family named: the state rows reported are those of the tiled
    embedding (3876 tiles of 16 rows at the default tile width 2), i.e. the matrix-core kernels run, not the
    vector-ALU family."""
    from paper_2507_04239_amd import binding
    prob = binding.make_problem(1, 2, 512, 32, 32, 4, 128, True, 1.0, "bf16", "auto")
    assert binding.power_attn_state_rows(prob) == 3876 * 16
    Q, K, V, G = inputs.make_qkvg(1, 2, 512, 32, seed=5200, dtype="bf16")
    got = run_fwd_bwd(Q, K, V, G, 4, 128, "bf16")
    O, Z = orc.fwd_bhtd(Q, K, V, 4, None, True, 1.0)
    dQ, dK, dV = orc.bwd_bhtd(Q, K, V, G, 4, None, True, 1.0)
    assert_close(got, dict(O=O, Z=Z, dQ=dQ, dK=dK, dV=dV), "bf16", "auto p=4 d=32")


def test_tiled_ragged_last_chunk():
    """A sequence that is not a multiple of the chunk runs padded with zero rows, as in the other chunked
    matrix-core kernels: p = 4, T = 1000 at chunk 128 (a last chunk of 104 tokens), kept states."""
    p, d, T, chunk = 4, 32, 1000, 128
    Q, K, V, G = inputs.make_qkvg(1, 2, T, d, seed=5300, dtype="bf16")
    got = run_fwd_bwd(Q, K, V, G, p, chunk, "bf16", impl="tiled", keep_state=True)
    O, Z = orc.fwd_bhtd(Q, K, V, p, None, True, 1.0)
    dQ, dK, dV = orc.bwd_bhtd(Q, K, V, G, p, None, True, 1.0)
    assert_close(got, dict(O=O, Z=Z, dQ=dQ, dK=dK, dV=dV), "bf16", "tiled ragged p=4 T=1000")


@pytest.mark.parametrize("p,dt", [(2, 8), (4, 4)])
def test_tiled_unnormalised_even_degree(p, dt):
    """normalize = 0 with an even degree: O is the numerator, Z is still returned, the backward pass has no
    normaliser terms."""
    Q, K, V, G = inputs.make_qkvg(1, 2, 512, 32, seed=5400 + p, dtype="bf16")
    got = run_fwd_bwd(Q, K, V, G, p, 128, "bf16", normalize=False, impl="tiled", d_tile=dt)
    O, Z = orc.fwd_bhtd(Q, K, V, p, None, False, 1.0)
    dQ, dK, dV = orc.bwd_bhtd(Q, K, V, G, p, None, False, 1.0)
    assert_close(got, dict(O=O, Z=Z, dQ=dQ, dK=dK, dV=dV), "bf16", f"tiled un-normalised p={p}")


@pytest.mark.parametrize("p,dt,d", [(2, 8, 32), (2, 16, 32), (4, 2, 32), (3, 4, 64), (2, 8, 128)])
def test_tiled_runs_are_bit_identical(p, dt, d):
    """No kernel of the family uses atomics or an order that depends on timing: two runs on the same inputs give
    the same bits.  (A d phi kernel that chained two kinds of MFMA instruction once returned values that differed
    from run to run in 16 lanes of a wave; this is the check that would have caught it without an oracle.)"""
    norm = p % 2 == 0
    Q, K, V, G = inputs.make_qkvg(1, 2, 512, d, seed=5400 + 10 * p + dt + d, dtype="bf16")
    print("case", (p, dt, d), flush=True)
    first = run_fwd_bwd(Q, K, V, G, p, 128, "bf16", normalize=norm, impl="tiled", d_tile=dt)
    for _ in range(3):
        again = run_fwd_bwd(Q, K, V, G, p, 128, "bf16", normalize=norm, impl="tiled", d_tile=dt)
        for k in first:
            assert np.array_equal(first[k], again[k]), (k, (p, dt, d))


@pytest.mark.parametrize("d,T", [(32, 4096 + 512 + 37), (128, 24576 + 256 + 5)])
def test_automatic_chunk_runs_the_tiled_kernels_on_long_sequences(d, T):
    """chunk = 0 at p = 2, d = 32 and d = 128, at a length beyond the attention form's reach that no chunk divides:
    chunk 256 on the tiled kernels, on the sequence padded with zero rows; sampled rows of O and dQ by the
    definition, every output finite."""
    from paper_2507_04239_amd import binding
    from gpu_util import TOL, rel_l2
    prob = binding.make_problem(1, 1, T, d, d, 2, 0)
    assert binding.power_attn_resolved_chunk(prob) == 256
    assert binding.power_attn_state_rows(prob) == (d // 8) * (d // 8 + 1) // 2 * 64
    Q, K, V, G = inputs.make_qkvg(1, 1, T, d, seed=5300 + d, dtype="bf16")
    print("case", (d, T), flush=True)
    got = run_fwd_bwd(Q, K, V, G, 2, 0, "bf16")
    q, k, v, g = (a[0, 0].astype(np.float64) for a in (Q, K, V, G))
    rows = [0, 255, 256, 2047, 4096, T - 300, T - 2, T - 1]
    o_ref = np.stack([orc.fwd_row(q, k, v, i, 2)[0] for i in rows])
    dq_ref = np.stack([orc.bwd_dq_row(q, k, v, g, i, 2) for i in rows])
    assert rel_l2(got["O"][0, 0][rows], o_ref) <= TOL["bf16"]
    assert rel_l2(got["dQ"][0, 0][rows], dq_ref) <= TOL["bf16"]
    for name in ("O", "Z", "dQ", "dK", "dV"):
        assert np.isfinite(got[name]).all(), name
