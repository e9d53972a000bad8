"""Pins of the oracle's single-token decode step (Sec. 2 Eq. (6)): stepping through a sequence must
reproduce the definition of power attention row by row, written out here in plain Python."""
import math

import numpy as np
import pytest

from oracle import power_attn_oracle as orc


def _definition_row(Q, K, V, log_g, i, p, scale, normalize):
    """O_i, Z_i by the definition with the product of gates, pure Python."""
    num = [0.0] * len(V[0])
    den = 0.0
    for j in range(i + 1):
        s = scale * sum(float(a) * float(b) for a, b in zip(Q[i], K[j]))
        w = s ** p
        for t in range(j + 1, i + 1):
            w *= math.exp(float(log_g[t])) if log_g is not None else 1.0
        den += w
        for c in range(len(num)):
            num[c] += w * float(V[j][c])
    if normalize:
        return [x / den if den != 0.0 else 0.0 for x in num], den
    return num, den


@pytest.mark.parametrize("p,d,v,normalize,gated,scale", [
    (2, 4, 3, True, False, 1.0), (2, 5, 2, True, True, 0.7), (3, 3, 2, False, False, 1.0),
    (3, 4, 4, False, True, 1.3), (4, 3, 3, True, True, 1.0), (1, 4, 2, False, False, 1.0),
])
def test_stepping_reproduces_the_definition(p, d, v, normalize, gated, scale):
    rng = np.random.default_rng(100 * p + d)
    T = 9
    Q, K, V = rng.normal(size=(T, d)), rng.normal(size=(T, d)), rng.normal(size=(T, v))
    lg = -rng.uniform(0.0, 0.7, size=T) if gated else None
    S = orc.decode_state_init(d, v, p)
    assert S.shape == (math.comb(d + p - 1, p), v + 1) and not S.any()
    for i in range(T):
        S, o, z = orc.decode_step(S, Q[i], K[i], V[i], p, normalize, scale, None if lg is None else lg[i])
        o_ref, z_ref = _definition_row(Q, K, V, lg, i, p, scale, normalize)
        np.testing.assert_allclose(z, z_ref, rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(o, o_ref, rtol=1e-7, atol=1e-10)   # the quotient of two sums that may nearly cancel


def test_first_step_closed_form():
    """With an empty state the token sees only itself: z = (scale q.k)^p and, normalised, o = v exactly;
    the first gate multiplies an empty state and cannot matter."""
    q, k, v = np.array([0.5, -1.0, 2.0]), np.array([1.5, 0.25, -0.5]), np.array([3.0, -4.0])
    for lg in (None, -2.0):
        S, o, z = orc.decode_step(orc.decode_state_init(3, 2, 2), q, k, v, 2, True, 0.5, lg)
        assert z == pytest.approx((0.5 * (0.75 - 0.25 - 1.0)) ** 2)
        np.testing.assert_allclose(o, v, rtol=1e-12)
        # the state is phi(k) [v, 1]^T: its normaliser column alone recovers |k|^(2p) against phi(k)
        np.testing.assert_allclose(orc.spow(k, 2) @ S[:, -1], (k @ k) ** 2, rtol=1e-12)


def test_a_dropped_gate_or_a_step_that_skips_itself_is_caught():
    """Planted mistakes: forgetting the decay of the old state, or reading the state before the update."""
    rng = np.random.default_rng(5)
    T, d, v, p = 6, 3, 2, 2
    Q, K, V = rng.normal(size=(T, d)), rng.normal(size=(T, d)), rng.normal(size=(T, v))
    lg = -rng.uniform(0.2, 0.9, size=T)
    S = orc.decode_state_init(d, v, p)
    S_nogate = S.copy()
    for i in range(T):
        S_prev = S
        S, o, z = orc.decode_step(S, Q[i], K[i], V[i], p, True, 1.0, lg[i])
        S_nogate, o_ng, _ = orc.decode_step(S_nogate, Q[i], K[i], V[i], p, True, 1.0, None)
        z_before = orc.spow(Q[i], p) @ S_prev[:, -1]
        if i > 0:
            assert not np.allclose(o, o_ng)
            assert not np.isclose(z, z_before)
    o_ref, z_ref = _definition_row(Q, K, V, lg, T - 1, p, 1.0, True)
    np.testing.assert_allclose(o, o_ref, rtol=1e-9)


def test_matches_the_recurrent_form_of_the_whole_sequence():
    rng = np.random.default_rng(8)
    T, d, v, p = 12, 6, 5, 2
    Q, K, V = rng.normal(size=(T, d)), rng.normal(size=(T, d)), rng.normal(size=(T, v))
    O_ref, Z_ref = orc.fwd_quadratic(Q, K, V, p)
    S = orc.decode_state_init(d, v, p)
    for i in range(T):
        S, o, z = orc.decode_step(S, Q[i], K[i], V[i], p)
        np.testing.assert_allclose(o, O_ref[i], rtol=1e-9, atol=1e-12)
        np.testing.assert_allclose(z, Z_ref[i], rtol=1e-10)
