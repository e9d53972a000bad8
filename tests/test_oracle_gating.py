"""Pins for the oracle's gated forward and backward passes (arXiv 2507.04239 Sec. 2 "Gating",
gated update-state of App. E.2, discounted cumulative sum of App. E.3): a pure-Python brute
force written from the per-timestep definition, the reduction to the un-gated functions (which
have pins of their own) through the homogeneity of the power kernel, closed forms, invariances,
agreement of the attention, recurrent and chunked forms, finite differences."""
import math

import numpy as np
import pytest

from oracle import power_attn_oracle as orc


def _rand(T, d, v, seed, max_decay=0.6):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((T, d)) / np.sqrt(d), rng.standard_normal((T, d)) / np.sqrt(d),
            rng.standard_normal((T, v)), rng.standard_normal((T, v)), -rng.uniform(0.0, max_decay, size=T))


def _python_brute_force(Q, K, V, log_g, p, normalize, scale):
    """Scalar loops only: the weight of the pair (i, j) is s_ij^p times the product of the gates
    of the steps j+1 .. i.  Shares nothing with the oracle."""
    T, d, v = len(Q), len(Q[0]), len(V[0])
    gates = [math.exp(x) for x in log_g]
    out, zs = [], []
    for i in range(T):
        num, z = [0.0] * v, 0.0
        for j in range(i + 1):
            s = scale * sum(Q[i][a] * K[j][a] for a in range(d))
            w = 1.0
            for _ in range(p):
                w *= s
            for t in range(j + 1, i + 1):
                w *= gates[t]
            z += w
            for x in range(v):
                num[x] += w * V[j][x]
        zs.append(z)
        out.append([n / z for n in num] if normalize else num)
    return np.array(out), np.array(zs)


FORWARDS = {
    "quadratic": lambda Q, K, V, lg, p, nz, sc: orc.fwd_quadratic_gated(Q, K, V, lg, p, nz, sc),
    "recurrent": lambda Q, K, V, lg, p, nz, sc: orc.fwd_recurrent_gated(Q, K, V, lg, p, nz, sc),
    "chunk1": lambda Q, K, V, lg, p, nz, sc: orc.fwd_chunked_gated(Q, K, V, lg, p, 1, nz, sc),
    "chunk3": lambda Q, K, V, lg, p, nz, sc: orc.fwd_chunked_gated(Q, K, V, lg, p, 3, nz, sc),
    "chunkT": lambda Q, K, V, lg, p, nz, sc: orc.fwd_chunked_gated(Q, K, V, lg, p, len(Q), nz, sc),
    "rows": lambda Q, K, V, lg, p, nz, sc: tuple(
        np.array(x) for x in zip(*[orc.fwd_row_gated(Q, K, V, lg, i, p, nz, sc) for i in range(len(Q))])),
}


@pytest.mark.parametrize("p,normalize,scale", [(2, True, 1.0), (4, True, 0.7), (3, False, 1.3), (1, False, 1.0)])
@pytest.mark.parametrize("form", sorted(FORWARDS))
def test_gated_forward_vs_python_brute_force(form, p, normalize, scale):
    Q, K, V, _, lg = _rand(7, 3, 2, seed=10 + p)
    O_ref, Z_ref = _python_brute_force(Q.tolist(), K.tolist(), V.tolist(), lg.tolist(), p, normalize, scale)
    O, Z = FORWARDS[form](Q, K, V, lg, p, normalize, scale)
    np.testing.assert_allclose(O, O_ref, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(Z, Z_ref, rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("p,normalize", [(2, True), (4, True), (3, False)])
def test_no_decay_is_the_ungated_layer(p, normalize):
    Q, K, V, G, _ = _rand(9, 3, 2, seed=21)
    zero = np.zeros(9)
    O0, Z0 = orc.fwd_quadratic(Q, K, V, p, normalize, 0.9)
    for O, Z in (orc.fwd_quadratic_gated(Q, K, V, zero, p, normalize, 0.9), orc.fwd_chunked_gated(Q, K, V, zero, p, 4, normalize, 0.9)):
        np.testing.assert_allclose(O, O0, rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(Z, Z0, rtol=1e-12, atol=1e-14)
    ref = orc.bwd_quadratic(Q, K, V, G, p, normalize, 0.9)
    for got in (orc.bwd_quadratic_gated(Q, K, V, zero, G, p, normalize, 0.9), orc.bwd_chunked_gated(Q, K, V, zero, G, p, 4, normalize, 0.9)):
        for a, b in zip(got[:3], ref):
            np.testing.assert_allclose(a, b, rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("p,normalize", [(2, True), (4, True), (3, False), (1, False)])
def test_gating_is_a_rescaling_of_queries_and_keys(p, normalize):
    """(q.k)^p is homogeneous of degree p in q and in k, so exp(b_i - b_j) can be moved into the
    vectors: the gated layer equals the un-gated one on q_i exp(b_i / p), k_j exp(-b_j / p); its
    gradients follow by the chain rule.  The un-gated functions are pinned elsewhere."""
    Q, K, V, G, lg = _rand(10, 3, 2, seed=33 + p, max_decay=0.3)
    b = np.cumsum(lg)
    fq, fk = np.exp(b / p)[:, None], np.exp(-b / p)[:, None]
    O_ref, Z_ref = orc.fwd_quadratic(Q * fq, K * fk, V, p, normalize, 1.1)
    O, Z = orc.fwd_quadratic_gated(Q, K, V, lg, p, normalize, 1.1)
    np.testing.assert_allclose(O, O_ref, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(Z, Z_ref, rtol=1e-11, atol=1e-13)
    dQt, dKt, dV_ref = orc.bwd_quadratic(Q * fq, K * fk, V, G, p, normalize, 1.1)
    dQ, dK, dV, dlg = orc.bwd_quadratic_gated(Q, K, V, lg, G, p, normalize, 1.1)
    np.testing.assert_allclose(dQ, dQt * fq, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dK, dKt * fk, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dV, dV_ref, rtol=1e-10, atol=1e-12)
    # b enters only through the rescaling: dL/db_i = (q~_i . dq~_i - k~_i . dk~_i) / p, then the reverse running sum
    db = (((Q * fq) * dQt).sum(axis=1) - ((K * fk) * dKt).sum(axis=1)) / p
    np.testing.assert_allclose(dlg, np.cumsum(db[::-1])[::-1], rtol=1e-9, atol=1e-11)


def test_geometric_series_closed_form():
    """d = 1, q = k = v = 1, constant gate g: a_ij = g^(i-j), Z_i = (1 - g^(i+1)) / (1 - g); un-normalised
    O_i = Z_i; with v_j = j the numerator is sum_j g^(i-j) j."""
    T, g = 12, 0.8
    one = np.ones((T, 1))
    lg = np.full(T, math.log(g))
    O, Z = orc.fwd_quadratic_gated(one, one, one, lg, 2, False)
    want = (1 - g ** np.arange(1, T + 1)) / (1 - g)
    np.testing.assert_allclose(Z, want, rtol=1e-13)
    np.testing.assert_allclose(O[:, 0], want, rtol=1e-13)
    ramp = np.arange(T, dtype=float)[:, None]
    O, _ = orc.fwd_chunked_gated(one, one, ramp, lg, 2, 5, False)
    np.testing.assert_allclose(O[:, 0], [sum(g ** (i - j) * j for j in range(i + 1)) for i in range(T)], rtol=1e-13)


def test_strong_decay_and_first_gate():
    Q, K, V, G, lg = _rand(8, 3, 2, seed=5)
    # gates ~ 0: every row sees only itself
    O, _ = orc.fwd_quadratic_gated(Q, K, V, np.full(8, -80.0), 2, True)
    np.testing.assert_allclose(O, V, rtol=1e-12, atol=1e-12)
    # the first gate multiplies nothing (no step precedes token 0): no effect, zero gradient
    lg2 = lg.copy()
    lg2[0] -= 1.7
    for a, b in zip(orc.fwd_quadratic_gated(Q, K, V, lg, 2, True), orc.fwd_quadratic_gated(Q, K, V, lg2, 2, True)):
        np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-14)
    for nz in (True, False):
        dlg = orc.bwd_quadratic_gated(Q, K, V, lg, G, 2, nz)[3]
        assert abs(dlg[0]) <= 1e-12 * max(1.0, np.abs(dlg).max())
    # a gate only affects pairs that straddle it: rows before it are unchanged
    lg3 = lg.copy()
    lg3[5] -= 0.9
    O3, _ = orc.fwd_quadratic_gated(Q, K, V, lg3, 2, True)
    O0, _ = orc.fwd_quadratic_gated(Q, K, V, lg, 2, True)
    np.testing.assert_allclose(O3[:5], O0[:5], rtol=1e-13)
    assert np.abs(O3[5:] - O0[5:]).max() > 1e-3


@pytest.mark.parametrize("p,d", [(2, 4), (3, 3), (4, 3)])
def test_gated_chunked_equals_attention_form_for_every_chunk_size(p, d):
    Q, K, V, G, lg = _rand(13, d, 3, seed=40 + p)
    nz = p % 2 == 0
    O_ref, Z_ref = orc.fwd_quadratic_gated(Q, K, V, lg, p, nz)
    ref = orc.bwd_quadratic_gated(Q, K, V, lg, G, p, nz)
    for c in range(1, 15):
        O, Z = orc.fwd_chunked_gated(Q, K, V, lg, p, c, nz)
        np.testing.assert_allclose(O, O_ref, rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(Z, Z_ref, rtol=1e-10, atol=1e-12)
        for a, b in zip(orc.bwd_chunked_gated(Q, K, V, lg, G, p, c, nz), ref):
            np.testing.assert_allclose(a, b, rtol=1e-9, atol=1e-11)


def _loss(Q, K, V, G, lg, p, normalize, scale):
    O, _ = _python_brute_force(Q.tolist(), K.tolist(), V.tolist(), lg.tolist(), p, normalize, scale)
    return float((O * G).sum())


@pytest.mark.parametrize("p,normalize,scale", [(2, True, 1.0), (4, True, 0.8), (2, False, 1.2), (3, False, 1.0)])
def test_gated_backward_vs_finite_differences(p, normalize, scale):
    """Central differences of the loss evaluated by the pure-Python brute force, for every input
    including the log-gates."""
    Q, K, V, G, lg = _rand(6, 3, 2, seed=60 + p)
    got = orc.bwd_quadratic_gated(Q, K, V, lg, G, p, normalize, scale)
    h = 1e-6
    for which, grad in zip(range(4), got):
        arrs = [Q.copy(), K.copy(), V.copy(), lg.copy()]
        num = np.zeros_like(arrs[which])
        for idx in np.ndindex(arrs[which].shape):
            keep = arrs[which][idx]
            arrs[which][idx] = keep + h
            up = _loss(arrs[0], arrs[1], arrs[2], G, arrs[3], p, normalize, scale)
            arrs[which][idx] = keep - h
            dn = _loss(arrs[0], arrs[1], arrs[2], G, arrs[3], p, normalize, scale)
            arrs[which][idx] = keep
            num[idx] = (up - dn) / (2 * h)
        np.testing.assert_allclose(grad, num, rtol=2e-6, atol=2e-8)


def test_bhtd_wrappers_with_gates():
    rng = np.random.default_rng(3)
    Q, K = rng.standard_normal((2, 2, 2, 6, 3)) / 2
    V, G = rng.standard_normal((2, 2, 2, 6, 2))
    lg = -rng.uniform(0, 0.4, size=(2, 2, 6))
    O, Z = orc.fwd_bhtd(Q, K, V, 2, None, True, 1.0, log_g=lg)
    Oc, Zc = orc.fwd_bhtd(Q, K, V, 2, 4, True, 1.0, log_g=lg)
    np.testing.assert_allclose(O, Oc, rtol=1e-11)
    O11, Z11 = orc.fwd_quadratic_gated(Q[1, 1], K[1, 1], V[1, 1], lg[1, 1], 2)
    np.testing.assert_allclose(O[1, 1], O11, rtol=1e-13)
    out = orc.bwd_bhtd(Q, K, V, G, 2, 4, True, 1.0, log_g=lg)
    assert len(out) == 4 and out[3].shape == lg.shape
    ref = orc.bwd_quadratic_gated(Q[0, 1], K[0, 1], V[0, 1], lg[0, 1], G[0, 1], 2)
    for a, b in zip(out, ref):
        np.testing.assert_allclose(a[0, 1], b, rtol=1e-9, atol=1e-12)
