#!/usr/bin/env python3
"""Benchmark of the power-attention hot path on one MI355X.

A step is one forward + one backward pass of the chunked causal power-attention layer over
one batch of the headline workload (p=2, d=64, T=65536, B=1, H=12, chunk=128, bf16,
normalised), inputs resident in HBM.  Prints ONE JSON line: tokens/s, the roofline figure of
the dominant kernel (timed with HIP events inside the library), and the float64 CPU oracle
timed on a bounded sample of the same workload.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_MFMA_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_FP32_VECTOR_TFLOPS = 157.3  # MI355X fp32 vector


def algorithmic_flops(w):
    """Algorithmic FLOPs per launch of every kernel (all heads), multiply-add = 2, with the
    symmetric dimension D = C(d+p-1, p): padding, masked tiles and recomputation earn nothing."""
    B, H, T, d, p, c = w["B"], w["H"], w["T"], w["d"], w["p"], w["chunk"]
    v = d
    BH, n = B * H, T // c
    D = math.comb(d + p - 1, p)
    state = BH * (n - 1) * c * 2 * D * (v + 1)           # one D x (v+1) contraction over the chunks that use it
    pairs = BH * n * c * (c + 1) // 2
    f = {
        "update_state": state,
        "fwd_chunk": state + pairs * (2 * d + 2 * (v + 1)),
        "state_grad": state,
        "bwd_dq": state + pairs * (4 * d + 2 * v + 2),
        "bwd_dkdv": state + BH * (n - 1) * c * 2 * D * v + pairs * (2 * d + 2 * v),
        "bwd_dk": state + pairs * 2 * d,
        "bwd_dv": BH * (n - 1) * c * 2 * D * v + pairs * 2 * v,
    }
    f["recompute"] = 0   # the backward pass rebuilds the chunk states: executed, not credited
    f["fwd_total"] = f["update_state"] + f["fwd_chunk"]
    f["bwd_total"] = f["state_grad"] + f["bwd_dq"] + f["bwd_dkdv"]
    return f


# kernel name (as the library reports it) -> (key in algorithmic_flops, credited?, peak TFLOP/s)
KERNEL_ROLE = {
    "generic_state_scan": ("update_state", PEAK_FP32_VECTOR_TFLOPS),
    "generic_fwd_chunk": ("fwd_chunk", PEAK_FP32_VECTOR_TFLOPS),
    "generic_state_scan_reverse": ("state_grad", PEAK_FP32_VECTOR_TFLOPS),
    "generic_bwd_dq": ("bwd_dq", PEAK_FP32_VECTOR_TFLOPS),
    "generic_bwd_dkdv": ("bwd_dkdv", PEAK_FP32_VECTOR_TFLOPS),
    "mfma_state_scan": ("update_state", PEAK_BF16_MFMA_TFLOPS),
    "mfma_state_scan_bwd": ("recompute", PEAK_BF16_MFMA_TFLOPS),
    "mfma_fwd_chunk": ("fwd_chunk", PEAK_BF16_MFMA_TFLOPS),
    "mfma_state_grad_scan": ("state_grad", PEAK_BF16_MFMA_TFLOPS),
    "mfma_bwd_dq": ("bwd_dq", PEAK_BF16_MFMA_TFLOPS),
    "mfma_bwd_dk": ("bwd_dk", PEAK_BF16_MFMA_TFLOPS),
    "mfma_bwd_dv": ("bwd_dv", PEAK_BF16_MFMA_TFLOPS),
}


def cpu_baseline(w, sample_tokens):
    """The float64 oracle (chunked form, forward + backward) on one head, first `sample_tokens`
    tokens of the workload; its cost per token does not depend on the position."""
    import numpy as np
    from oracle import power_attn_oracle as orc
    from paper_2507_04239_amd import inputs
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:
        cores = 1
    Q, K, V, G = inputs.make_qkvg(1, 1, sample_tokens, w["d"], seed=1000 + w["position"], dtype=w["dtype"])
    t0 = time.perf_counter()
    orc.bwd_chunked(Q[0, 0], K[0, 0], V[0, 0], G[0, 0], w["p"], w["chunk"])   # runs the forward pass inside
    dt = time.perf_counter() - t0
    # one head of H: a token of the whole job costs H such head-tokens
    return {"value": sample_tokens / (dt * w["H"]), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"fwd+bwd of 1 of {w['H']} heads over the first {sample_tokens} of {w['T']} tokens "
                      f"({dt:.1f} s), scaled by 1/{w['H']}", "seconds": dt}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=None, help="name from paper_2507_04239_amd.inputs.WORKLOADS")
    ap.add_argument("--impl", default="auto", choices=["auto", "generic", "mfma"])
    ap.add_argument("--cpu-sample-tokens", type=int, default=32768)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--recompute-states", action="store_true",
                    help="backward pass rebuilds the chunk states instead of reusing the forward pass's workspace")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build measures one GPU only (the path shards over batch and heads with no "
                 "communication); run with --gpus 1")

    import torch
    from paper_2507_04239_amd import binding, inputs, power_attn_bwd, power_attn_fwd

    name = args.workload or inputs.HEADLINE
    w = inputs.WORKLOADS[name]
    dev = torch.device("cuda:0")
    tdt = torch.bfloat16 if w["dtype"] == "bf16" else torch.float32
    Q, K, V, G = inputs.make_workload(name, with_grad=True)
    tq, tk, tv, tg = (torch.from_numpy(a).to(dev).to(tdt) for a in (Q, K, V, G))
    del Q, K, V, G
    p, chunk = w["p"], w["chunk"]
    keep = not args.recompute_states
    prob = binding.make_problem(w["B"], w["H"], w["T"], w["d"], w["d"], p, chunk, True, 1.0, w["dtype"], args.impl, keep)
    ws_bytes = max(binding.power_attn_workspace_bytes(prob, True), binding.power_attn_workspace_bytes(prob, False))
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)
    O = torch.empty_like(tv)
    Z = torch.empty(tq.shape[:3], dtype=torch.float32, device=dev)
    grads = (torch.empty_like(tq), torch.empty_like(tk), torch.empty_like(tv))

    def step():
        power_attn_fwd(tq, tk, tv, p, chunk, impl=args.impl, workspace=ws, out=O, out_z=Z, keep_state=keep)
        power_attn_bwd(tq, tk, tv, O, Z, tg, p, chunk, impl=args.impl, workspace=ws, out=grads, keep_state=keep)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    tokens = w["B"] * w["T"]

    # per-kernel durations from HIP events recorded by the library on the launch stream
    binding.profile_begin()
    for _ in range(args.steps):
        step()
    kernels = binding.profile_end()
    fl = algorithmic_flops(w)
    per_kernel = {}
    for kname, (launches, ms_total) in kernels.items():
        per_kernel[kname] = {"launches_per_step": launches / args.steps, "avg_ms": ms_total / launches}
    credited = {k: v for k, v in kernels.items() if k in KERNEL_ROLE}
    dom = max(credited, key=lambda k: credited[k][1])
    role, peak = KERNEL_ROLE[dom]
    dom_ms = credited[dom][1] / credited[dom][0]
    achieved = fl[role] / (dom_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma" if peak == PEAK_BF16_MFMA_TFLOPS else "alu", "kernel": dom, "achieved": achieved,
                "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak, "traffic": None,
                "avg_kernel_ms": dom_ms, "algorithmic_flops_per_launch": fl[role]}
    total_alg = fl["fwd_total"] + fl["bwd_total"]
    out = {
        "metric": "power-attention fwd+bwd tokens/sec at p=2,d=64,T=64k; % bf16 MFMA peak",
        "value": tokens / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w["dtype"], "data": "synthetic",
        "config": {"workload": name, "B": w["B"], "H": w["H"], "T": w["T"], "d": w["d"], "p": p, "chunk": chunk,
                   "normalize": True, "pass": "fwd+bwd", "impl": args.impl, "keep_state": keep,
                   "state_rows": binding.power_attn_state_rows(prob)},
        "step_algorithmic_tflop": total_alg / 1e12,
        "step_frac_of_bf16_mfma_peak": total_alg / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS,
        "roofline": roofline,
        "kernels": per_kernel,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, min(args.cpu_sample_tokens, w["T"]))
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
