"""Pins for the oracle's forward and backward passes: a hand-computed fixture, pure-Python
brute force, closed forms and invariances of the definition (arXiv 2507.04239 Sec. 4 Eq. (7),
Sec. 2 "Normalization"), chunked == attention form (App. A), finite differences."""
import numpy as np
import pytest

from oracle import power_attn_oracle as orc

HAND_Q = np.array([[1.0, 0.0], [1.0, 1.0], [0.0, 2.0]])
HAND_K = np.array([[1.0, 2.0], [2.0, -1.0], [1.0, 1.0]])
HAND_V = np.array([[1.0, 0.0], [0.0, 1.0], [2.0, 2.0]])

FORWARDS = {
    "quadratic": lambda Q, K, V, p, nz, sc: orc.fwd_quadratic(Q, K, V, p, nz, sc),
    "chunk1": lambda Q, K, V, p, nz, sc: orc.fwd_chunked(Q, K, V, p, 1, nz, sc),
    "chunk2": lambda Q, K, V, p, nz, sc: orc.fwd_chunked(Q, K, V, p, 2, nz, sc),
    "chunkT": lambda Q, K, V, p, nz, sc: orc.fwd_chunked(Q, K, V, p, Q.shape[0], nz, sc),
    "recurrent": lambda Q, K, V, p, nz, sc: orc.fwd_recurrent(Q, K, V, p, nz, sc),
}


@pytest.mark.parametrize("form", sorted(FORWARDS))
def test_hand_example(golden_table, form):
    for p, nz, row, o0, o1, z in golden_table("hand_example_T3_d2.txt"):
        O, Z = FORWARDS[form](HAND_Q, HAND_K, HAND_V, int(p), bool(int(nz)), 1.0)
        np.testing.assert_allclose(O[int(row)], [float(o0), float(o1)], rtol=1e-13, atol=1e-13)
        np.testing.assert_allclose(Z[int(row)], float(z), rtol=1e-13)


def _python_brute_force(Q, K, V, p, normalize, scale):
    """Scalar loops only, written from Eq. (7); shares nothing with the oracle."""
    T, d = len(Q), len(Q[0])
    v = len(V[0])
    out, zs = [], []
    for i in range(T):
        num = [0.0] * v
        z = 0.0
        for j in range(i + 1):
            s = 0.0
            for a in range(d):
                s += Q[i][a] * K[j][a]
            s *= scale
            w = 1.0
            for _ in range(p):
                w *= s
            z += w
            for x in range(v):
                num[x] += w * V[j][x]
        zs.append(z)
        out.append([n / z for n in num] if normalize else num)
    return np.array(out), np.array(zs)


def _rand(T, d, v, seed):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((T, d)) / np.sqrt(d), rng.standard_normal((T, d)) / np.sqrt(d),
            rng.standard_normal((T, v)))


@pytest.mark.parametrize("p,normalize,scale", [(2, True, 1.0), (4, True, 0.7), (3, False, 1.3), (1, False, 1.0), (2, False, 2.0)])
@pytest.mark.parametrize("form", sorted(FORWARDS))
def test_forward_vs_python_brute_force(form, p, normalize, scale):
    Q, K, V = _rand(7, 3, 2, seed=p * 11 + int(normalize))
    O_want, Z_want = _python_brute_force(Q.tolist(), K.tolist(), V.tolist(), p, normalize, scale)
    O, Z = FORWARDS[form](Q, K, V, p, normalize, scale)
    np.testing.assert_allclose(O, O_want, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(Z, Z_want, rtol=1e-10, atol=1e-13)


def test_p1_unnormalized_is_causal_linear_attention():
    # degree 1 without normalisation is plain linear attention with phi = identity (Sec. 2 Eq. (5))
    Q, K, V = _rand(33, 5, 4, seed=1)
    want = np.tril(Q @ K.T) @ V
    for form in FORWARDS.values():
        np.testing.assert_allclose(form(Q, K, V, 1, False, 1.0)[0], want, rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("p", [2, 4])
def test_closed_forms_and_invariances(p):
    T, d, v = 40, 6, 5
    Q, K, V = _rand(T, d, v, seed=p)
    O, Z = orc.fwd_quadratic(Q, K, V, p, True)
    # first token attends only to itself: O_0 = V_0
    np.testing.assert_allclose(O[0], V[0], rtol=1e-12)
    # even p: all scores positive, rows are convex combinations of earlier values
    assert (Z > 0).all()
    assert (O.max(axis=0) <= V.max(axis=0) + 1e-12).all() and (O.min(axis=0) >= V.min(axis=0) - 1e-12).all()
    # constant values give that constant back
    c = np.tile(np.array([[1.5, -2.0, 0.25, 3.0, 7.0]]), (T, 1))
    np.testing.assert_allclose(orc.fwd_quadratic(Q, K, c, p, True)[0], c, rtol=1e-12)
    # scaling q or k by a constant cancels in the normalised output (Z scales by alpha^p)
    O2, Z2 = orc.fwd_quadratic(-3.0 * Q, K, V, p, True)
    np.testing.assert_allclose(O2, O, rtol=1e-10)
    np.testing.assert_allclose(Z2, 3.0 ** p * Z, rtol=1e-10)
    np.testing.assert_allclose(orc.fwd_quadratic(Q, K, V, p, True, scale=0.37)[0], O, rtol=1e-10)
    # joint orthogonal rotation of q and k leaves every score unchanged
    R, _ = np.linalg.qr(np.random.default_rng(9).standard_normal((d, d)))
    np.testing.assert_allclose(orc.fwd_quadratic(Q @ R, K @ R, V, p, True)[0], O, rtol=1e-9, atol=1e-12)
    # causality: changing token 25 leaves rows < 25 untouched and changes row 25
    K2, V2 = K.copy(), V.copy()
    K2[25] += 1.0
    V2[25] -= 2.0
    O3 = orc.fwd_quadratic(Q, K2, V2, p, True)[0]
    np.testing.assert_array_equal(O3[:25], O[:25])
    assert np.abs(O3[25] - O[25]).max() > 1e-3
    # independent one-line evaluation in float64 torch on the CPU
    import torch
    tq, tk, tv = (torch.from_numpy(a) for a in (Q, K, V))
    A = torch.tril((tq @ tk.T) ** p)
    np.testing.assert_allclose(O, ((A @ tv) / A.sum(1, keepdim=True)).numpy(), rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("p,d", [(2, 4), (3, 3), (4, 3)])
def test_chunked_equals_attention_form_for_every_chunk_size(p, d):
    # App. A: the chunked form equals the attention form when the initial state is zero
    T, v = 24, 3
    Q, K, V = _rand(T, d, v, seed=50 + p)
    normalize = p % 2 == 0
    O_want, Z_want = orc.fwd_quadratic(Q, K, V, p, normalize)
    for c in [1, 2, 3, 4, 5, 6, 7, 8, 12, 24, 100]:          # divisors, ragged tails, c > T
        O, Z = orc.fwd_chunked(Q, K, V, p, c, normalize)
        np.testing.assert_allclose(O, O_want, rtol=1e-9, atol=1e-12)
        np.testing.assert_allclose(Z, Z_want, rtol=1e-9, atol=1e-13)


def test_row_function_equals_full_forward():
    Q, K, V = _rand(30, 4, 3, seed=77)
    O, Z = orc.fwd_quadratic(Q, K, V, 2, True, 0.9)
    for i in (0, 1, 17, 29):
        o, z = orc.fwd_row(Q, K, V, i, 2, True, 0.9)
        np.testing.assert_array_equal(o, O[i])
        assert z == Z[i]


def test_zero_denominator_convention():
    Q, K, V = _rand(6, 3, 2, seed=5)
    Q[2] = 0.0                                  # row 2 scores are all exactly zero
    G = np.random.default_rng(6).standard_normal((6, 2))
    for O, Z in (orc.fwd_quadratic(Q, K, V, 2, True), orc.fwd_chunked(Q, K, V, 2, 2, True)):
        assert Z[2] == 0.0 and (O[2] == 0.0).all() and np.isfinite(O).all()
    for dQ, dK, dV in (orc.bwd_quadratic(Q, K, V, G, 2, True), orc.bwd_chunked(Q, K, V, G, 2, 2, True)):
        assert np.isfinite(dQ).all() and np.isfinite(dK).all() and np.isfinite(dV).all()
        assert (dQ[2] == 0.0).all()


# ------------------------------------------------------------------------------------------
# backward
# ------------------------------------------------------------------------------------------

def _loss(Q, K, V, G, p, normalize, scale):
    O, _ = _python_brute_force(Q.tolist(), K.tolist(), V.tolist(), p, normalize, scale)
    return float((O * G).sum())


def _finite_difference_grads(Q, K, V, G, p, normalize, scale, h=1e-6):
    grads = []
    for which in range(3):
        arrs = [Q, K, V]
        g = np.zeros_like(arrs[which])
        for idx in np.ndindex(*arrs[which].shape):
            plus = [a.copy() for a in arrs]
            minus = [a.copy() for a in arrs]
            plus[which][idx] += h
            minus[which][idx] -= h
            g[idx] = (_loss(*plus, G, p, normalize, scale) - _loss(*minus, G, p, normalize, scale)) / (2 * h)
        grads.append(g)
    return grads


BACKWARDS = {
    "quadratic": lambda Q, K, V, G, p, nz, sc: orc.bwd_quadratic(Q, K, V, G, p, nz, sc),
    "chunk1": lambda Q, K, V, G, p, nz, sc: orc.bwd_chunked(Q, K, V, G, p, 1, nz, sc),
    "chunk3": lambda Q, K, V, G, p, nz, sc: orc.bwd_chunked(Q, K, V, G, p, 3, nz, sc),
    "chunkT": lambda Q, K, V, G, p, nz, sc: orc.bwd_chunked(Q, K, V, G, p, 8, nz, sc),
}


@pytest.mark.parametrize("p,normalize,scale", [(2, True, 1.0), (4, True, 0.8), (2, False, 1.2), (3, False, 1.0), (4, False, 1.0)])
def test_backward_vs_finite_differences(p, normalize, scale):
    # the loss is evaluated by the pure-Python brute force, not by the oracle
    T, d, v = 8, 3, 2
    Q, K, V = _rand(T, d, v, seed=300 + p)
    Q, K = Q * 1.5, K * 1.5
    G = np.random.default_rng(301).standard_normal((T, v))
    fd = _finite_difference_grads(Q, K, V, G, p, normalize, scale)
    for name, bwd in BACKWARDS.items():
        got = bwd(Q, K, V, G, p, normalize, scale)
        for g, w, what in zip(got, fd, "QKV"):
            err = np.abs(g - w).max() / max(1.0, np.abs(w).max())
            assert err < 2e-7, (name, what, err)


@pytest.mark.parametrize("p", [2, 4])
def test_backward_structure(p):
    T, d, v = 20, 4, 3
    Q, K, V = _rand(T, d, v, seed=400 + p)
    rng = np.random.default_rng(401)
    G1, G2 = rng.standard_normal((T, v)), rng.standard_normal((T, v))
    # every gradient is linear in the upstream gradient
    a = orc.bwd_quadratic(Q, K, V, G1, p, True)
    b = orc.bwd_quadratic(Q, K, V, G2, p, True)
    c = orc.bwd_quadratic(Q, K, V, 2.0 * G1 - 3.0 * G2, p, True)
    for x, y, z in zip(a, b, c):
        np.testing.assert_allclose(z, 2.0 * x - 3.0 * y, rtol=1e-9, atol=1e-12)
    # normalised output is invariant to the scale of q_i and of all k: q_i . dQ_i = 0, sum_j k_j . dK_j = 0
    dQ, dK, dV = a
    assert np.abs((Q * dQ).sum(axis=1)).max() < 1e-11 * max(1.0, np.abs(dQ).max())
    assert abs((K * dK).sum()) < 1e-11 * max(1.0, np.abs(dK).max())
    # rows of the attention weights sum to one: sum_j dV_j = sum_i G_i
    np.testing.assert_allclose(dV.sum(axis=0), G1.sum(axis=0), rtol=1e-10)
    # constant values: output does not depend on q, k at all
    Vc = np.ones((T, v)) * 0.7
    dQc, dKc, _ = orc.bwd_quadratic(Q, K, Vc, G1, p, True)
    assert np.abs(dQc).max() < 1e-12 and np.abs(dKc).max() < 1e-12
    # last token's key/value only meet the last query
    s = float(Q[-1] @ K[-1])
    np.testing.assert_allclose(dV[-1], (s ** p) * G1[-1] / orc.fwd_row(Q, K, V, T - 1, p)[1], rtol=1e-10)


@pytest.mark.parametrize("p,normalize", [(2, True), (4, True), (3, False)])
def test_chunked_and_sampled_backward_agree_with_quadratic(p, normalize):
    T, d, v = 36, 4, 3
    Q, K, V = _rand(T, d, v, seed=500 + p)
    G = np.random.default_rng(501).standard_normal((T, v))
    want = orc.bwd_quadratic(Q, K, V, G, p, normalize, 0.9)
    for c in (1, 4, 5, 12, 36):
        got = orc.bwd_chunked(Q, K, V, G, p, c, normalize, 0.9)
        for g, w in zip(got, want):
            np.testing.assert_allclose(g, w, rtol=1e-8, atol=1e-11)
    O, Z = orc.fwd_quadratic(Q, K, V, p, normalize, 0.9)
    for i in (0, 9, 35):
        np.testing.assert_allclose(orc.bwd_dq_row(Q, K, V, G, i, p, normalize, 0.9), want[0][i], rtol=1e-9, atol=1e-12)
        dk, dv = orc.bwd_dkdv_col(Q, K, V, G, O, Z, i, p, normalize, 0.9)
        np.testing.assert_allclose(dk, want[1][i], rtol=1e-9, atol=1e-12)
        np.testing.assert_allclose(dv, want[2][i], rtol=1e-9, atol=1e-12)


def test_dq_row_at_saved_forward_results():
    """bwd_dq_row(saved=(O_i, Z_i)): with the exact forward results it is the default; with Z_i doubled and
    O_i kept, Ghat and gz halve and so does the row (the row is linear in 1 / Z_i at fixed O_i); with O_i moved
    by delta the row moves by -(G_i . delta) / Z_i times the gradient of Z_i, i.e. of sum_j s_ij^p (pinned
    against finite differences of that sum taken with the forward row sampler)."""
    T, d, v, p = 20, 4, 3, 4
    Q, K, V = _rand(T, d, v, seed=900)
    G = np.random.default_rng(901).standard_normal((T, v))
    i = 13
    O_i, Z_i = orc.fwd_row(Q, K, V, i, p)
    base = orc.bwd_dq_row(Q, K, V, G, i, p)
    np.testing.assert_allclose(orc.bwd_dq_row(Q, K, V, G, i, p, saved=(O_i, Z_i)), base, rtol=1e-13)
    np.testing.assert_allclose(orc.bwd_dq_row(Q, K, V, G, i, p, saved=(O_i, 2.0 * Z_i)), 0.5 * base, rtol=1e-12)
    delta = np.array([0.3, -0.2, 0.1])
    moved = orc.bwd_dq_row(Q, K, V, G, i, p, saved=(O_i + delta, Z_i))
    dZ = np.zeros(d)
    h = 1e-6
    for a in range(d):
        Qp, Qm = Q.copy(), Q.copy()
        Qp[i, a] += h
        Qm[i, a] -= h
        dZ[a] = (orc.fwd_row(Qp, K, V, i, p)[1] - orc.fwd_row(Qm, K, V, i, p)[1]) / (2 * h)
    np.testing.assert_allclose(moved - base, -(G[i] @ delta) / Z_i * dZ, rtol=1e-6, atol=1e-9)


def test_bhtd_wrappers_loop_over_heads():
    rng = np.random.default_rng(8)
    Q, K, V, G = (rng.standard_normal((2, 3, 10, 4)) * 0.5 for _ in range(4))
    O, Z = orc.fwd_bhtd(Q, K, V, 2, chunk=5)
    dQ, dK, dV = orc.bwd_bhtd(Q, K, V, G, 2, chunk=5)
    o, z = orc.fwd_quadratic(Q[1, 2], K[1, 2], V[1, 2], 2)
    np.testing.assert_allclose(O[1, 2], o, rtol=1e-10)
    np.testing.assert_allclose(Z[1, 2], z, rtol=1e-10)
    g = orc.bwd_quadratic(Q[1, 2], K[1, 2], V[1, 2], G[1, 2], 2)
    for got, w in zip((dQ[1, 2], dK[1, 2], dV[1, 2]), g):
        np.testing.assert_allclose(got, w, rtol=1e-8, atol=1e-12)
