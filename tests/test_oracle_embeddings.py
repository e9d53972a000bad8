"""Pins for the oracle's embeddings: the paper's printed numbers, its worked examples and
the inner-product identities of Lemma 4.1 / 4.2 (arXiv 2507.04239, Sec. 4)."""
import itertools
import math

import numpy as np
import pytest

from oracle import power_attn_oracle as orc


def test_table3_state_sizes(golden_table):
    for p, tp, sp, savings in golden_table("table3_state_sizes.txt"):
        p, tp, sp = int(p), int(tp), int(sp)
        assert orc.dim_tpow(64, p) == tp
        assert orc.dim_spow(64, p) == sp
        printed = float(savings.rstrip("%"))
        exact = 100.0 * (1.0 - sp / tp)
        # the paper prints the saving cut to a whole percent (one decimal in the last row)
        assert 0.0 <= exact - printed < (0.1 if "." in savings else 1.0)


def test_growth_factors_quoted_in_text():
    # Sec. 4: head size 64 -> state grows by about 32 (p=2), 700 (p=3), 12000 (p=4)
    assert round(orc.dim_spow(64, 2) / 64) in (32, 33)
    assert abs(orc.dim_spow(64, 3) / 64 - 700) / 700 < 0.03
    assert abs(orc.dim_spow(64, 4) / 64 - 12000) / 12000 < 0.01


def test_fig5_counts(golden_table):
    want = {k: int(n) for k, n in golden_table("fig5_tile_counts.txt")}
    x = np.arange(1.0, 7.0)
    assert orc.tpow(x, 2).size == want["tpow"] == orc.dim_tpow(6, 2)
    assert orc.spow(x, 2).size == want["spow"] == orc.dim_spow(6, 2)
    assert orc.tspow(x, 2, 2).size == want["tspow"] == orc.dim_tspow(6, 2, 2)


def test_benchmark_config_dims():
    # D values named with the benchmark configurations
    assert orc.dim_spow(16, 2) == 136
    assert orc.dim_spow(64, 2) == 2080
    assert orc.dim_spow(32, 4) == 52360
    assert orc.dim_spow(128, 2) == 8256


def test_spow_worked_examples():
    # Sec. 4, examples after Lemma 4.2 (order included)
    x1, x2 = 1.7, -0.3
    np.testing.assert_allclose(orc.spow(np.array([x1, x2]), 2),
                               [x1 * x1, math.sqrt(2) * x1 * x2, x2 * x2], rtol=1e-15)
    np.testing.assert_allclose(orc.spow(np.array([x1, x2]), 3),
                               [x1 ** 3, math.sqrt(3) * x1 * x1 * x2, math.sqrt(3) * x1 * x2 * x2, x2 ** 3],
                               rtol=1e-15)


def test_tpow_order_and_values():
    # Lemma 4.1: rows x_1..x_1, x_1..x_2, ..., x_d..x_d  (row-major multi-index order)
    x = np.array([2.0, 3.0, 5.0])
    want = [x[i] * x[j] * x[k] for i, j, k in itertools.product(range(3), repeat=3)]
    np.testing.assert_array_equal(orc.tpow(x, 3), want)
    assert orc.tpow(x, 1).tolist() == x.tolist()


def test_ndmi_is_lexicographic_and_complete():
    for n, p in [(1, 3), (4, 2), (3, 4), (5, 3)]:
        got = [tuple(r) for r in orc.ndmi(n, p)]
        brute = sorted(t for t in itertools.product(range(n), repeat=p) if list(t) == sorted(t))
        assert got == brute
        assert len(got) == math.comb(n + p - 1, p)


def test_multiplicity_counts_orderings():
    for row in [(0, 0), (0, 1), (1, 1, 2), (0, 1, 2, 3), (2, 2, 2, 2), (0, 0, 1, 1), (0, 1, 1, 1)]:
        assert orc.multiplicity(row) == len(set(itertools.permutations(row)))


@pytest.mark.parametrize("d,p", [(1, 1), (1, 4), (2, 2), (3, 3), (4, 4), (5, 2), (6, 5), (8, 3), (7, 6)])
def test_inner_product_identities(d, p):
    rng = np.random.default_rng(100 * d + p)
    q, k = rng.standard_normal(d), rng.standard_normal(d)
    want = float(q @ k) ** p
    tol = 1e-12 * max(1.0, abs(want), float(np.linalg.norm(q) * np.linalg.norm(k)) ** p)
    if d ** p <= 300000:
        assert abs(orc.tpow(q, p) @ orc.tpow(k, p) - want) < tol          # Lemma 4.1
    assert abs(orc.spow(q, p) @ orc.spow(k, p) - want) < tol              # Lemma 4.2 (2)
    assert orc.spow(q, p).size == math.comb(d + p - 1, p)                 # Lemma 4.2 (1)


@pytest.mark.parametrize("d,p,dt", [(6, 2, 2), (8, 2, 4), (8, 3, 2), (8, 4, 2), (12, 3, 4), (16, 2, 8), (4, 2, 4), (4, 3, 1)])
def test_tspow_identity_and_dim(d, p, dt):
    rng = np.random.default_rng(7 * d + p + dt)
    q, k = rng.standard_normal(d), rng.standard_normal(d)
    want = float(q @ k) ** p
    eq, ek = orc.tspow(q, p, dt), orc.tspow(k, p, dt)
    assert eq.size == orc.dim_tspow(d, p, dt) == math.comb(d // dt + p - 1, p) * dt ** p
    assert abs(eq @ ek - want) < 1e-12 * max(1.0, abs(want), (np.linalg.norm(q) * np.linalg.norm(k)) ** p)
    # d_tile = d is TPOW, d_tile = 1 is SPOW (the two ends TSPOW interpolates between)
    np.testing.assert_allclose(orc.tspow(q, p, d), orc.tpow(q, p), rtol=1e-14)
    np.testing.assert_allclose(orc.tspow(q, p, 1), orc.spow(q, p), rtol=1e-14)


def test_tspow_without_weights_would_break_identity():
    # documents why the tile weight is needed: dropping it changes the inner product
    rng = np.random.default_rng(3)
    q, k = rng.standard_normal(4), rng.standard_normal(4)
    blocks_q, blocks_k = [], []
    for a, b in orc.ndmi(2, 2):
        blocks_q.append(np.outer(q[2 * a:2 * a + 2], q[2 * b:2 * b + 2]).ravel())
        blocks_k.append(np.outer(k[2 * a:2 * a + 2], k[2 * b:2 * b + 2]).ravel())
    unweighted = np.concatenate(blocks_q) @ np.concatenate(blocks_k)
    assert abs(unweighted - (q @ k) ** 2) > 1e-3


@pytest.mark.parametrize("d,p", [(2, 2), (3, 3), (4, 4), (5, 2)])
def test_spow_jacobian_matches_finite_differences(d, p):
    rng = np.random.default_rng(d * 10 + p)
    x = rng.standard_normal((3, d))
    g = rng.standard_normal((3, orc.dim_spow(d, p)))
    got = orc.spow_jacobian_transpose_apply(x, g, p)
    h = 1e-6
    for t in range(3):
        for a in range(d):
            xp, xm = x.copy(), x.copy()
            xp[t, a] += h
            xm[t, a] -= h
            fd = ((orc.spow(xp[t], p) - orc.spow(xm[t], p)) / (2 * h)) @ g[t]
            assert abs(fd - got[t, a]) < 1e-7 * max(1.0, abs(fd))
