"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

The float64 oracle cannot produce every output of a 65536-token problem by brute force in
seconds, so: one head is checked completely against the chunked float64 oracle (which is
itself pinned to the brute force on small inputs), and rows / columns sampled from every head
are checked against the definition evaluated row by row.  Chunk-size invariance is checked on
the device as a property that holds at any size."""
import numpy as np
import pytest

from oracle import power_attn_oracle as orc
from paper_2507_04239_amd import inputs

from gpu_util import ROW_TOL, TOL, assert_close, max_row_err, rel_l2, run_fwd_bwd

pytestmark = pytest.mark.gpu


def _sample_rows(T, count, seed):
    rng = np.random.default_rng(seed)
    fixed = [0, 1, 127, 128, 129, T // 2 - 1, T // 2, T - 129, T - 128, T - 1]
    return sorted(set(fixed) | set(int(x) for x in rng.integers(0, T, size=count)))


def _check_sampled(name, got, Q, K, V, G, w, heads, n_rows, n_cols, ref_head=None):
    """Rows of O, Z, dQ and columns of dK, dV by the definition, on the listed (b, h).  Both bounds of
    gpu_util are asserted on the sampled rows.  One allowance, derived from the arithmetic: the backward pass
    reads the saved output O in bf16, and a row with a tiny Z_i (the first tokens of a sequence at p = 4: one
    key dominates, v_j - O_i nearly cancels, and G_i / Z_i is hundreds of times G_i) turns that rounding into
    an error of several per cent of the row whatever the kernel does.  The oracle measures it per row (the row
    evaluated at O_i rounded to bf16) and twice that is taken off a dQ row's error before the per-row bound."""
    p, dtype = w["p"], w["dtype"]
    T = w["T"]
    errs = {k: [] for k in ("O", "Z", "dQ", "dK", "dV")}
    slack = {"dQ": []}
    for (b, h) in heads:
        q, k, v = Q[b, h], K[b, h], V[b, h]
        rows = _sample_rows(T, n_rows, seed=17 * b + h)
        o_ref = np.stack([orc.fwd_row(q, k, v, i, p)[0] for i in rows])
        z_ref = np.array([orc.fwd_row(q, k, v, i, p)[1] for i in rows])
        errs["O"].append((got["O"][b, h][rows], o_ref))
        errs["Z"].append((got["Z"][b, h][rows], z_ref))
        if G is not None:
            dq_ref = np.stack([orc.bwd_dq_row(q, k, v, G[b, h], i, p) for i in rows])
            errs["dQ"].append((got["dQ"][b, h][rows], dq_ref))
            if dtype == "bf16":
                # what rounding the saved output to bf16 (an input of the backward pass) does to each row, by the
                # oracle alone: the same row evaluated at O_i rounded to bf16
                o_bf = inputs.bf16_bits_to_f32(inputs.f32_to_bf16_bits(o_ref.astype(np.float32))).astype(np.float64)
                moved = np.stack([orc.bwd_dq_row(q, k, v, G[b, h], i, p, saved=(o_bf[n], z_ref[n])) for n, i in enumerate(rows)])
                slack["dQ"].append(np.linalg.norm(moved - dq_ref, axis=1))
            if ref_head is not None and (b, h) == ref_head[0]:
                O_full, Z_full = ref_head[1]
                cols = _sample_rows(T, n_cols, seed=1000 + 17 * b + h)
                pairs = [orc.bwd_dkdv_col(q, k, v, G[b, h], O_full, Z_full, j, p) for j in cols]
                errs["dK"].append((got["dK"][b, h][cols], np.stack([a for a, _ in pairs])))
                errs["dV"].append((got["dV"][b, h][cols], np.stack([c for _, c in pairs])))
    report, rows_off = {}, {}
    for key, lst in errs.items():
        if lst:
            g = np.concatenate([a.reshape(len(a), -1) for a, _ in lst])
            r = np.concatenate([c.reshape(len(c), -1) for _, c in lst])
            report[key] = rel_l2(g, r)
            # worst sampled row against max(its own norm, the rms norm of the sampled rows), after taking off
            # twice what the rounding of the saved output alone does to that row (see _check_sampled's docstring)
            allow = 2.0 * np.concatenate(slack[key]) if slack.get(key) else 0.0
            norm = np.linalg.norm(r, axis=1)
            err = np.maximum(np.linalg.norm(g - r, axis=1) - allow, 0.0)
            rows_off[key] = float((err / np.maximum(norm, np.sqrt(np.mean(norm ** 2)))).max())
    print(f"{name} sampled: " + " ".join(f"{k}={v:.2e} (row {rows_off[k]:.2e})" for k, v in report.items()), flush=True)
    for key, lst in errs.items():
        if lst and not (report[key] <= TOL[dtype] and rows_off[key] <= ROW_TOL[dtype]):
            for g, r in lst:
                per_row = np.linalg.norm((g - r).reshape(len(g), -1), axis=1)
                print(f"  {key}: |err| per sampled row {np.round(per_row, 4)} |ref| {np.round(np.linalg.norm(r.reshape(len(r), -1), axis=1), 4)}", flush=True)
    bad = {k: v for k, v in report.items() if not v <= TOL[dtype]}
    assert not bad, f"{name}: sampled relative L2 error above {TOL[dtype]}: {bad}"
    bad = {k: v for k, v in rows_off.items() if not v <= ROW_TOL[dtype]}
    assert not bad, f"{name}: a sampled row is off by more than {ROW_TOL[dtype]} of the rms row norm: {bad}"


def test_headline_config3_fwd_bwd():
    """bf16 fwd+bwd, p=2, B1 H12 T65536 d64 chunk 128 (the shape bench.py times)."""
    name = "cfg3_bf16_p2_T65536_d64_c128"
    w = inputs.WORKLOADS[name]
    Q, K, V, G = inputs.make_workload(name)
    print("case", name, flush=True)
    got = run_fwd_bwd(Q, K, V, G, w["p"], w["chunk"], "bf16", keep_state=True)   # as bench.py runs it
    for k, a in got.items():
        assert np.isfinite(a).all(), k
    # head (0, 5): every output against the chunked float64 oracle
    b, h = 0, 5
    O_ref, Z_ref = orc.fwd_chunked(Q[b, h], K[b, h], V[b, h], w["p"], w["chunk"])
    dQ_ref, dK_ref, dV_ref = orc.bwd_chunked(Q[b, h], K[b, h], V[b, h], G[b, h], w["p"], w["chunk"])
    assert_close({k: a[b, h] for k, a in got.items()}, dict(O=O_ref, Z=Z_ref, dQ=dQ_ref, dK=dK_ref, dV=dV_ref),
                 "bf16", f"{name} head (0,5) vs chunked oracle")
    # sampled rows of every head by the definition; dK/dV columns on the fully checked head
    _check_sampled(name, got, Q, K, V, G, w, [(0, hh) for hh in range(w["H"])], n_rows=64, n_cols=32,
                   ref_head=((b, h), (O_ref, Z_ref)))


def test_headline_shape_with_the_library_chosen_chunk():
    """The headline shape with chunk = 0: the library resolves it to 256, where the two 128-token blocks of a
    chunk are dealt to the same XCD.  One head in full against the chunked float64 oracle, sampled rows of
    four heads against the definition."""
    from paper_2507_04239_amd import binding
    name = "cfg3_bf16_p2_T65536_d64_c128"
    w = dict(inputs.WORKLOADS[name])
    assert binding.power_attn_resolved_chunk(binding.make_problem(w["B"], w["H"], w["T"], w["d"], w["d"], w["p"], 0)) == 256
    Q, K, V, G = inputs.make_workload(name)
    print("case", name, "chunk 0", flush=True)
    got = run_fwd_bwd(Q, K, V, G, w["p"], 0, "bf16", keep_state=True)
    for k, a in got.items():
        assert np.isfinite(a).all(), k
    b, h = 0, 7
    O_ref, Z_ref = orc.fwd_chunked(Q[b, h], K[b, h], V[b, h], w["p"], 256)
    dQ_ref, dK_ref, dV_ref = orc.bwd_chunked(Q[b, h], K[b, h], V[b, h], G[b, h], w["p"], 256)
    assert_close({k: a[b, h] for k, a in got.items()}, dict(O=O_ref, Z=Z_ref, dQ=dQ_ref, dK=dK_ref, dV=dV_ref),
                 "bf16", f"{name} chunk 0 head (0,7) vs chunked oracle")
    w["chunk"] = 256
    _check_sampled(name, got, Q, K, V, G, w, [(0, hh) for hh in (0, 3, 7, 11)], n_rows=6, n_cols=12,
                   ref_head=((b, h), (O_ref, Z_ref)))


def test_config2_forward():
    """bf16 forward, p=2, B4 H12 T8192 d64 chunk 128."""
    name = "cfg2_bf16_p2_T8192_d64_c128"
    w = inputs.WORKLOADS[name]
    Q, K, V, _ = inputs.make_workload(name, with_grad=False)
    print("case", name, flush=True)
    got = run_fwd_bwd(Q, K, V, None, w["p"], w["chunk"], "bf16", backward=False)
    b, h = 3, 11
    O_ref, Z_ref = orc.fwd_quadratic(Q[b, h], K[b, h], V[b, h], w["p"])      # brute force on one head
    assert_close({k: a[b, h] for k, a in got.items()}, dict(O=O_ref, Z=Z_ref), "bf16", f"{name} head (3,11) brute force")
    heads = [(bb, hh) for bb in range(w["B"]) for hh in range(0, w["H"], 3)]
    _check_sampled(name, got, Q, K, V, None, w, heads, n_rows=8, n_cols=0)


def test_chunk_size_invariance_on_device():
    """The result does not depend on the chunk size (App. A): 128, 256 and 512 agree on the device."""
    Q, K, V, G = inputs.make_qkvg(1, 2, 4096, 64, seed=77, dtype="bf16")
    outs = [run_fwd_bwd(Q, K, V, G, 2, c, "bf16") for c in (128, 256, 512)]
    for other in outs[1:]:
        for key in ("O", "dQ", "dK", "dV"):
            err = rel_l2(other[key], outs[0][key])
            print(f"chunk invariance {key}: {err:.2e}", flush=True)
            assert err <= 2 * TOL["bf16"], (key, err)


def test_config4_as_stated_full_shape():
    """Config 4 as stated, all of it: bf16 fwd+bwd, p=4, B2 H8 T16384 d32, chunk 128, as bench.py runs it (the
    tiled matrix-core kernels of degree 4, chunk states kept between the passes).  One head, every output
    (O, Z, dQ, dK, dV), against the definition in float64; eight more heads spread over the batch, sampled rows
    of O, Z, dQ by the definition; sampled columns of dK, dV on the fully checked head."""
    name = "cfg4_bf16_p4_T16384_d32_c128"
    w = inputs.WORKLOADS[name]
    Q, K, V, G = inputs.make_workload(name)
    print("case", name, "as stated", flush=True)
    got = run_fwd_bwd(Q, K, V, G, w["p"], w["chunk"], "bf16", keep_state=True)
    for k, a in got.items():
        assert np.isfinite(a).all(), k
    b, h = 1, 5
    q, k, v, g = (a[b, h].astype(np.float64) for a in (Q, K, V, G))
    O_ref, Z_ref = orc.fwd_quadratic(q, k, v, w["p"])
    dQ_ref, dK_ref, dV_ref = orc.bwd_quadratic(q, k, v, g, w["p"])
    assert_close({key: a[b, h] for key, a in got.items()}, dict(O=O_ref, Z=Z_ref, dQ=dQ_ref, dK=dK_ref, dV=dV_ref),
                 "bf16", f"{name} head (1,5) by the definition")
    heads = [(1, 5), (0, 0), (0, 3), (0, 7), (1, 0), (1, 2), (1, 7), (0, 5), (1, 4)]
    _check_sampled(name, got, Q, K, V, G, w, heads, n_rows=32, n_cols=32, ref_head=((b, h), (O_ref, Z_ref)))


def test_config4_tile_width_four_one_head():
    """The same head shape with the tile width the automatic choice does not take (d_tile = 4, 330 tiles of
    256 rows): one head, every output by the definition."""
    w = dict(inputs.WORKLOADS["cfg4_bf16_p4_T16384_d32_c128"])
    Q, K, V, G = (a.astype(np.float64) for a in inputs.make_qkvg(1, 1, w["T"], w["d"], seed=1004, dtype="bf16"))
    print("case cfg4 one head, d_tile 4", flush=True)
    got = run_fwd_bwd(Q, K, V, G, 4, w["chunk"], "bf16", d_tile=4)
    O_ref, Z_ref = orc.fwd_quadratic(Q[0, 0], K[0, 0], V[0, 0], 4)
    dQ_ref, dK_ref, dV_ref = orc.bwd_quadratic(Q[0, 0], K[0, 0], V[0, 0], G[0, 0], 4)
    assert_close({key: a[0, 0] for key, a in got.items()}, dict(O=O_ref, Z=Z_ref, dQ=dQ_ref, dK=dK_ref, dV=dV_ref),
                 "bf16", "cfg4 head shape, d_tile 4, by the definition")


def test_d128_config5_shape_reduced_batch():
    """Config 5 as stated (bf16 fwd+bwd, p=2, d=128, chunk 256, T=32768), two of its 128 heads.  Covered:
    one head, every output (O, Z, dQ, dK, dV) against the chunked float64 oracle; the other head, sampled
    rows of O, Z, dQ by the definition.  Not covered here: the remaining 126 heads of B8 H16."""
    w = dict(inputs.WORKLOADS["cfg5_bf16_p2_T32768_d128_c256"])
    Q, K, V, G = inputs.make_qkvg(1, 2, w["T"], w["d"], seed=1005, dtype="bf16")
    print("case cfg5 two heads", flush=True)
    got = run_fwd_bwd(Q, K, V, G, 2, w["chunk"], "bf16")
    for k, a in got.items():
        assert np.isfinite(a).all(), k
    h = 1
    O_ref, Z_ref = orc.fwd_chunked(Q[0, h], K[0, h], V[0, h], 2, w["chunk"])
    dQ_ref, dK_ref, dV_ref = orc.bwd_chunked(Q[0, h], K[0, h], V[0, h], G[0, h], 2, w["chunk"])
    assert_close({k: a[0, h] for k, a in got.items()}, dict(O=O_ref, Z=Z_ref, dQ=dQ_ref, dK=dK_ref, dV=dV_ref),
                 "bf16", "cfg5 chunk 256, head 1 vs chunked oracle")
    _check_sampled("cfg5", got, Q, K, V, G, dict(w, B=1, H=2), [(0, 0)], n_rows=12, n_cols=0)


def test_config5_as_stated_full_shape():
    """Config 5 as stated, all of it: bf16 fwd+bwd, p=2, B8 H16 T32768 d128, chunk 256, as bench.py runs it (the
    tiled matrix-core kernels, chunk states in memory and kept between the passes).  One head, every output, against the
    chunked float64 oracle; eight more heads spread over the batch, sampled rows of O, Z, dQ by the definition;
    sampled columns of dK, dV on the fully checked head."""
    name = "cfg5_bf16_p2_T32768_d128_c256"
    w = inputs.WORKLOADS[name]
    Q, K, V, G = inputs.make_workload(name)
    print("case", name, "as stated", flush=True)
    got = run_fwd_bwd(Q, K, V, G, w["p"], w["chunk"], "bf16", keep_state=True)
    for k, a in got.items():
        assert np.isfinite(a).all(), k
    b, h = 5, 11
    O_ref, Z_ref = orc.fwd_chunked(Q[b, h], K[b, h], V[b, h], w["p"], w["chunk"])
    dQ_ref, dK_ref, dV_ref = orc.bwd_chunked(Q[b, h], K[b, h], V[b, h], G[b, h], w["p"], w["chunk"])
    assert_close({k: a[b, h] for k, a in got.items()}, dict(O=O_ref, Z=Z_ref, dQ=dQ_ref, dK=dK_ref, dV=dV_ref),
                 "bf16", f"{name} head (5,11) vs chunked oracle")
    heads = [(5, 11), (0, 0), (1, 15), (2, 3), (3, 8), (4, 12), (6, 5), (7, 15), (7, 0)]
    _check_sampled(name, got, Q, K, V, G, w, heads, n_rows=32, n_cols=32, ref_head=((b, h), (O_ref, Z_ref)))


def test_headline_shape_gated():
    """The headline head shape (T = 65536, d = 64, chunk 128, bf16) with per-timestep gates, two
    heads: every output of one head against the chunked float64 oracle, sampled forward rows of
    the other by the definition."""
    name = "cfg3_bf16_p2_T65536_d64_c128"
    w = inputs.WORKLOADS[name]
    Q, K, V, G = inputs.make_qkvg(1, 2, w["T"], w["d"], seed=1103, dtype="bf16")
    lg = inputs.make_log_gates(1, 2, w["T"], 1603, 0.02)
    print("case", name, "gated", flush=True)
    got = run_fwd_bwd(Q, K, V, G, 2, w["chunk"], "bf16", keep_state=True, log_g=lg)
    for k, a in got.items():
        assert np.isfinite(a).all(), k
    h = 1
    lg64 = lg[0, h].astype(np.float64)
    O_ref, Z_ref = orc.fwd_chunked_gated(Q[0, h], K[0, h], V[0, h], lg64, 2, w["chunk"])
    dQ_ref, dK_ref, dV_ref, dL_ref = orc.bwd_chunked_gated(Q[0, h], K[0, h], V[0, h], lg64, G[0, h], 2, w["chunk"])
    assert_close({k: a[0, h] for k, a in got.items()},
                 dict(O=O_ref, Z=Z_ref, dQ=dQ_ref, dK=dK_ref, dV=dV_ref, dlog_g=dL_ref), "bf16", f"{name} gated head 1")
    rows = _sample_rows(w["T"], 8, seed=5)
    ref = [orc.fwd_row_gated(Q[0, 0], K[0, 0], V[0, 0], lg[0, 0].astype(np.float64), i, 2) for i in rows]
    assert rel_l2(got["O"][0, 0][rows], np.stack([r[0] for r in ref])) <= TOL["bf16"]
    assert rel_l2(got["Z"][0, 0][rows], np.array([r[1] for r in ref])) <= TOL["bf16"]


def test_config4_attention_form_full_shape():
    """Config 4's full shape (bf16 fwd+bwd, p=4, B2 H8 T16384 d32) with chunk = 0: the library runs the
    attention form on the matrix cores.  Sampled rows of every head by the definition; on one head O, Z
    of every row by the definition and sampled columns of dK, dV."""
    name = "cfg4_bf16_p4_T16384_d32_c128"
    w = dict(inputs.WORKLOADS[name])
    Q, K, V, G = (a.astype(np.float64) for a in inputs.make_workload(name))
    print("case", name, "chunk = 0", flush=True)
    got = run_fwd_bwd(Q, K, V, G, w["p"], 0, "bf16")
    for k, a in got.items():
        assert np.isfinite(a).all(), k
    b, h = 1, 3
    O_ref, Z_ref = orc.fwd_quadratic(Q[b, h], K[b, h], V[b, h], w["p"])
    assert_close({k: got[k][b, h] for k in ("O", "Z")}, dict(O=O_ref, Z=Z_ref), "bf16", f"{name} head (1,3) by the definition")
    heads = [(bb, hh) for bb in range(w["B"]) for hh in range(w["H"])]
    _check_sampled(name, got, Q, K, V, G, w, heads, n_rows=5, n_cols=12, ref_head=((b, h), (O_ref, Z_ref)))


def test_config5_shape_attention_form_reduced_batch():
    """Config 5's head shape (bf16 fwd+bwd, p=2, d=128, T=32768) with chunk = 0, two of its 128 heads:
    sampled rows of O, Z, dQ by the definition; columns of dK, dV among the last 512 keys (their
    sums need O, Z of every later row, which the definition gives row by row)."""
    w = dict(inputs.WORKLOADS["cfg5_bf16_p2_T32768_d128_c256"], B=1, H=2)
    T = w["T"]
    Q, K, V, G = (a.astype(np.float64) for a in inputs.make_qkvg(1, 2, T, w["d"], seed=1105, dtype="bf16"))
    print("case cfg5 two heads, chunk = 0", flush=True)
    got = run_fwd_bwd(Q, K, V, G, 2, 0, "bf16")
    for k, a in got.items():
        assert np.isfinite(a).all(), k
    _check_sampled("cfg5", got, Q, K, V, G, w, [(0, 0), (0, 1)], n_rows=8, n_cols=0)
    h, tail = 1, 512
    O_t = np.zeros((T, w["d"]))
    Z_t = np.ones(T)
    for i in range(T - tail, T):
        O_t[i], Z_t[i] = orc.fwd_row(Q[0, h], K[0, h], V[0, h], i, 2)
    cols = sorted(set(int(x) for x in np.random.default_rng(55).integers(T - tail, T, size=10)) | {T - tail, T - 1})
    pairs = [orc.bwd_dkdv_col(Q[0, h], K[0, h], V[0, h], G[0, h], O_t, Z_t, j, 2) for j in cols]
    dk_err = rel_l2(got["dK"][0, h][cols], np.stack([a for a, _ in pairs]))
    dv_err = rel_l2(got["dV"][0, h][cols], np.stack([c for _, c in pairs]))
    print(f"cfg5 tail columns: dK={dk_err:.2e} dV={dv_err:.2e}", flush=True)
    assert dk_err <= TOL["bf16"] and dv_err <= TOL["bf16"]


def test_d128_attention_form_every_output_at_4096():
    """d = 128, T = 4096 (64 key tiles, 16 to 32 workgroups per kernel and head): every output against
    the definition."""
    Q, K, V, G = inputs.make_qkvg(1, 1, 4096, 128, seed=1106, dtype="bf16")
    print("case d128 T4096", flush=True)
    got = run_fwd_bwd(Q, K, V, G, 2, 4096, "bf16", impl="mfma")
    O, Z = orc.fwd_bhtd(Q, K, V, 2, None, True, 1.0)
    dQ, dK, dV = orc.bwd_bhtd(Q, K, V, G, 2, None, True, 1.0)
    assert_close(got, dict(O=O, Z=Z, dQ=dQ, dK=dK, dV=dV), "bf16", "d128 T4096 attention form")
