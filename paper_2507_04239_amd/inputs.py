"""Seeded synthetic inputs for power attention, shared by the tests, the benchmark and
the smoke check.  This module holds no arithmetic of the method itself: it only draws
random numbers, rounds them to the storage dtype and names the workload shapes.

Recipe (all five workloads): q, k ~ N(0,1) * d^-1/2, v ~ N(0,1), upstream gradient
dY ~ N(0,1), iid, layout [B, H, T, d] row-major, value width v = d.  Values are drawn in
float32 from numpy's PCG64 with one independent stream per tensor, then (for bf16
workloads) rounded to nearest-even bf16, so both the GPU and the CPU checker see
exactly the same representable numbers.
"""
from __future__ import annotations

import numpy as np

# name -> problem description; "position" is the 1-based place in the benchmark's config list
WORKLOADS = {
    "cfg1_f32_p2_T256_d16_c32":   dict(position=1, B=1, H=1,  T=256,   d=16,  p=2, chunk=32,  dtype="f32",  backward=False),
    "cfg2_bf16_p2_T8192_d64_c128": dict(position=2, B=4, H=12, T=8192,  d=64,  p=2, chunk=128, dtype="bf16", backward=False),
    "cfg3_bf16_p2_T65536_d64_c128": dict(position=3, B=1, H=12, T=65536, d=64,  p=2, chunk=128, dtype="bf16", backward=True),
    "cfg4_bf16_p4_T16384_d32_c128": dict(position=4, B=2, H=8,  T=16384, d=32,  p=4, chunk=128, dtype="bf16", backward=True),
    "cfg5_bf16_p2_T32768_d128_c256": dict(position=5, B=8, H=16, T=32768, d=128, p=2, chunk=256, dtype="bf16", backward=True),
}
HEADLINE = "cfg3_bf16_p2_T65536_d64_c128"
# Not one of the paper's benchmark configurations: a shape for timing the degree the paper names beside 2 and 4
# (p = 3, d_tile = 4, Sec. 4.1.1).  Odd degree: un-normalised.  bench.py takes it by name; --all-configs does not run it.
EXTRA_WORKLOADS = {
    "extra_bf16_p3_T16384_d64_c128": dict(position=6, B=1, H=4, T=16384, d=64, p=3, chunk=128, dtype="bf16", backward=True,
                                          normalize=False),
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round-to-nearest-even; NaN stays NaN."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounded = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)
    nan = np.isnan(x)
    out = rounded.astype(np.uint16)
    if nan.any():
        out = np.where(nan, np.uint16(0x7FC0), out)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float32, exact."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_dtype(x: np.ndarray, dtype: str) -> np.ndarray:
    """float32 array holding exactly the values representable in ``dtype``."""
    x = np.asarray(x, dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(x))
    raise ValueError(f"unknown dtype {dtype!r}")


def make_qkvg(B: int, H: int, T: int, d: int, seed: int, dtype: str = "bf16", v: int | None = None,
              with_grad: bool = True):
    """Draw (Q, K, V, dY) as float32 arrays that hold dtype-representable values.
    dY is None when ``with_grad`` is false.  Four independent PCG64 streams are spawned
    from ``seed`` (q, k, v, dY in that order)."""
    v = d if v is None else v
    streams = [np.random.Generator(np.random.PCG64(s)) for s in np.random.SeedSequence(seed).spawn(4)]
    qk_scale = np.float32(d ** -0.5)
    Q = streams[0].standard_normal((B, H, T, d), dtype=np.float32) * qk_scale
    K = streams[1].standard_normal((B, H, T, d), dtype=np.float32) * qk_scale
    V = streams[2].standard_normal((B, H, T, v), dtype=np.float32)
    G = streams[3].standard_normal((B, H, T, v), dtype=np.float32) if with_grad else None
    Q, K, V = (round_to_dtype(a, dtype) for a in (Q, K, V))
    if G is not None:
        G = round_to_dtype(G, dtype)
    return Q, K, V, G


def make_workload(name: str, with_grad: bool | None = None):
    """Inputs of a named workload; the seed is 1000 + its position."""
    w = WORKLOADS[name] if name in WORKLOADS else EXTRA_WORKLOADS[name]
    wg = w["backward"] if with_grad is None else with_grad
    return make_qkvg(w["B"], w["H"], w["T"], w["d"], 1000 + w["position"], w["dtype"], with_grad=wg)


def make_log_gates(B, H, T, seed, mean_decay=0.02):
    """Seeded log-gates [B, H, T], float32, <= 0: log g_t = -mean_decay * e_t with e_t exponential
    of mean 1 (most steps keep nearly everything, a few forget a lot), as a learned per-head,
    per-timestep gate would give.  Both the oracle and the library read these float32 values."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return (-mean_decay * rng.exponential(1.0, size=(B, H, T))).astype(np.float32)
