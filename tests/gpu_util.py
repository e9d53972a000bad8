"""Helpers of the GPU parity tests: move seeded inputs to the device, run the library
through its binding, compare with the float64 oracle."""
import numpy as np

TOL = {"f32": 1e-4, "bf16": 2e-2}   # relative L2 error per tensor (the bar the benchmark names)
# Per-row bound: no single row (one token's vector, or one scalar of Z / dlog_g) may be off by more than
# this fraction of its own norm or of the root-mean-square row norm of the reference, whichever is
# larger (gradient rows are heavy-tailed: a few are many times the typical size, and their rounding
# error grows with them).  The tensor-level bar alone lets one entirely wrong row of a 4096-row tensor
# through (sqrt(1/4096) = 1.6e-2); a wrong row scores about 1 here, one that is 30 % off about 0.3.
# Rounding alone reaches up to ten times the tensor-level error in the worst row (observed on the GPU:
# bf16 up to 4.2e-2 at 3-5e-3 per tensor, f32 2e-6), so the limit sits at 2.5 x the tensor-level bar.
ROW_TOL = {"f32": 2.5e-4, "bf16": 5e-2}


def rel_l2(got, want):
    want = np.asarray(want, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    den = np.linalg.norm(want)
    return float(np.linalg.norm(got - want) / den) if den > 0 else float(np.linalg.norm(got))


def max_over_rms(got, want):
    want = np.asarray(want, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    rms = np.sqrt(np.mean(want ** 2))
    return float(np.abs(got - want).max() / rms) if rms > 0 else float(np.abs(got).max())


def max_row_err(got, want):
    """max_i |got_i - want_i|_2 / max(|want_i|_2, rms_i |want_i|_2) over the rows (last axis = one row;
    1-D: every element is a row)."""
    want = np.asarray(want, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    if want.ndim <= 1:
        want, got = want.reshape(-1, 1), got.reshape(-1, 1)
    else:
        want, got = want.reshape(-1, want.shape[-1]), got.reshape(-1, got.shape[-1])
    norm = np.sqrt(np.sum(want ** 2, axis=1))
    rms = np.sqrt(np.mean(norm ** 2))
    err = np.sqrt(np.sum((got - want) ** 2, axis=1))
    return float((err / np.maximum(norm, rms)).max()) if rms > 0 else float(err.max())


def to_dev(a, dtype):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def to_np(t):
    return t.detach().float().cpu().numpy()


def run_fwd_bwd(Q, K, V, G, p, chunk, dtype, normalize=True, scale=1.0, impl="auto", backward=True,
                keep_state=False, log_g=None, d_tile=0):
    """-> dict of numpy arrays O, Z (and dQ, dK, dV; dlog_g when log_g is given) computed by the HIP
    library.  keep_state: the backward pass reuses the chunk states the forward pass left in a
    shared workspace."""
    import torch
    from paper_2507_04239_amd import binding, power_attn_bwd, power_attn_fwd
    tq, tk, tv = (to_dev(a, dtype) for a in (Q, K, V))
    tl = None if log_g is None else torch.from_numpy(np.ascontiguousarray(log_g, dtype=np.float32)).to("cuda:0")
    ws = None
    if keep_state:
        B, H, T, d = Q.shape
        prob = binding.make_problem(B, H, T, d, V.shape[3], p, chunk, normalize, scale, dtype, impl, True, log_g is not None, d_tile)
        ws = torch.empty(max(binding.power_attn_workspace_bytes(prob, True), 256), dtype=torch.uint8, device="cuda:0")
    O, Z = power_attn_fwd(tq, tk, tv, p, chunk, normalize, scale, impl, workspace=ws, keep_state=keep_state, log_g=tl,
                          d_tile=d_tile)
    out = {"O": O, "Z": Z}
    if backward:
        tg = to_dev(G, dtype)
        res = power_attn_bwd(tq, tk, tv, O, Z, tg, p, chunk, normalize, scale, impl, workspace=ws,
                             keep_state=keep_state, log_g=tl, d_tile=d_tile)
        out.update(dQ=res[0], dK=res[1], dV=res[2])
        if log_g is not None:
            out.update(dlog_g=res[3])
    torch.cuda.synchronize()
    return {k: to_np(t) for k, t in out.items()}


def assert_close(got: dict, want: dict, dtype: str, what: str, factor: float = 1.0):
    """Every tensor of `want`: relative L2 error within the tolerance AND no single row further off
    than the per-row bound."""
    tol = TOL[dtype] * factor
    row_tol = ROW_TOL[dtype] * factor
    report = {}
    for name, w in want.items():
        g = got[name]
        assert np.isfinite(g).all(), f"{what}: {name} has non-finite values"
        report[name] = (rel_l2(g, w), max_row_err(g, w))
    print(f"{what}: " + " ".join(f"{k}: l2={a:.2e} row={b:.2e}" for k, (a, b) in report.items()), flush=True)
    bad = {k: e for k, e in report.items() if not e[0] <= tol}
    assert not bad, f"{what}: relative L2 error above {tol}: {bad}"
    bad = {k: e for k, e in report.items() if not e[1] <= row_tol}
    assert not bad, f"{what}: a row is off by more than {row_tol} of the rms row norm: {bad}"
    return report
