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
PEAK_HBM_GBS = 8000.0            # MI355X HBM3E


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
    # resident-state kernels: a walk does the update and one contraction with the state in one launch
    f["walk_fwd"] = 2 * state                                             # update-state + query-state
    f["walk_dq"] = state                                                  # d phi(q); rebuilding S is executed, not credited
    f["walk_dv"] = state + BH * (n - 1) * c * 2 * D * v                   # state gradient + its read-out
    f["walk_dk"] = state                                                  # d phi(k); R is credited to the dV walk
    f["chunk_fwd"] = pairs * (2 * d + 2 * (v + 1))
    f["chunk_dq"] = pairs * (4 * d + 2 * v + 2)
    f["chunk_dkdv"] = pairs * (2 * d + 2 * v)
    # tiled kernels: each state contraction is a launch of its own, the in-chunk parts run on the chunk_* kernels
    f["query_state"] = state
    f["dphi"] = state
    f["dv_readout"] = BH * (n - 1) * c * 2 * D * v
    f["recompute"] = 0   # a backward pass that rebuilds the chunk states: executed, not credited
    f["fwd_total"] = f["update_state"] + f["fwd_chunk"]
    f["bwd_total"] = f["state_grad"] + f["bwd_dq"] + f["bwd_dkdv"]
    return f


def algorithmic_bytes(w):
    """Algorithmic HBM bytes per launch of every kernel (all heads): the n - 1 chunk states a
    pass needs, D x (v+1) each in the storage type, written (scans) or read (per-chunk kernels)
    once, plus the token rows the kernel reads and writes once.  Padding of the tiled embedding,
    feature-major copies and re-reads earn nothing."""
    B, H, T, d, p, c = w["B"], w["H"], w["T"], w["d"], w["p"], w["chunk"]
    v = d
    BH, n = B * H, T // c
    e = 2 if w["dtype"] == "bf16" else 4
    D = math.comb(d + p - 1, p)
    states = BH * (n - 1) * D * (v + 1) * e
    tok = BH * T * d * e                 # one [T, d] operand of every head
    return {
        "update_state": states + 2 * tok,            # K, V in
        "fwd_chunk": states + 4 * tok + BH * T * 4,  # Q, K, V in; O, Z out
        "state_grad": states + 2 * tok + BH * T * 4,  # Q, ghat, gz in
        "bwd_dq": states + 5 * tok + BH * T * 4,     # Q, K, V, ghat, gz in; dQ out
        "bwd_dkdv": states + 6 * tok + BH * T * 4,   # Q, K, V, ghat, gz in; dK, dV out; R once
        "bwd_dk": states + 5 * tok + BH * T * 4,
        "bwd_dv": states + 4 * tok,                  # Q, K, ghat in; dV out
        "recompute": 0,
        # resident-state kernels: no state leaves the chip; what is credited is the token rows in and the
        # result out (the per-slab float32 partial results they exchange are overhead)
        "walk_fwd": 3 * tok + BH * T * v * 4, "walk_dq": 4 * tok + BH * T * d * 4,
        "walk_dv": 3 * tok + BH * T * v * 4, "walk_dk": 4 * tok + BH * T * d * 4,
        "chunk_fwd": 4 * tok + BH * T * 4, "chunk_dq": 5 * tok + BH * T * 4, "chunk_dkdv": 7 * tok + BH * T * 4,
        # tiled kernels: the states once, the token rows in, the float32 result out
        "query_state": states + tok + BH * T * (v + 1) * 4, "dphi": states + 2 * tok + BH * T * d * 4,
        "dv_readout": states + tok + BH * T * v * 4,
    }


# kernel name (as the library reports it) -> (key in the two models above, compute peak in TFLOP/s)
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
    "mfma_bwd_dkdv": ("bwd_dkdv", PEAK_BF16_MFMA_TFLOPS),
    "mfma_bwd_dk": ("bwd_dk", PEAK_BF16_MFMA_TFLOPS),
    "mfma_bwd_dv": ("bwd_dv", PEAK_BF16_MFMA_TFLOPS),
    "res_state_walk": ("walk_fwd", PEAK_BF16_MFMA_TFLOPS),
    "res_state_totals": ("recompute", PEAK_BF16_MFMA_TFLOPS),
    "res_grad_totals": ("recompute", PEAK_BF16_MFMA_TFLOPS),
    "res_dq_walk": ("walk_dq", PEAK_BF16_MFMA_TFLOPS),
    "res_dv_walk": ("walk_dv", PEAK_BF16_MFMA_TFLOPS),
    "res_dk_walk": ("walk_dk", PEAK_BF16_MFMA_TFLOPS),
    "tiled_state_scan": ("update_state", PEAK_BF16_MFMA_TFLOPS),
    "tiled_state_scan_bwd": ("recompute", PEAK_BF16_MFMA_TFLOPS),
    "tiled_query_state": ("query_state", PEAK_BF16_MFMA_TFLOPS),
    "tiled_state_grad_scan": ("state_grad", PEAK_BF16_MFMA_TFLOPS),
    "tiled_dq": ("dphi", PEAK_BF16_MFMA_TFLOPS),
    "tiled_dk": ("dphi", PEAK_BF16_MFMA_TFLOPS),
    "tiled_dv": ("dv_readout", PEAK_BF16_MFMA_TFLOPS),
    "mfma_fwd_chunk_partial": ("chunk_fwd", PEAK_BF16_MFMA_TFLOPS),
    "chunk_fwd": ("chunk_fwd", PEAK_BF16_MFMA_TFLOPS),
    "chunk_bwd_dq": ("chunk_dq", PEAK_BF16_MFMA_TFLOPS),
    "chunk_bwd_dkdv": ("chunk_dkdv", PEAK_BF16_MFMA_TFLOPS),
    # attention form (one chunk, no state): the same formulas with n = 1
    "attn_fwd": ("fwd_chunk", PEAK_BF16_MFMA_TFLOPS),
    "attn_bwd_dq": ("bwd_dq", PEAK_BF16_MFMA_TFLOPS),
    "attn_bwd_dkdv": ("bwd_dkdv", PEAK_BF16_MFMA_TFLOPS),
}


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter summary of this
    workload (a line `TRAFFIC <workload> <kernel> <bytes>`), or None."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        f = line.split()
        if len(f) == 4 and f[0] == "TRAFFIC" and f[1] == workload and f[2] == kernel:
            return float(f[3])
    return None


def traffic_source():
    """The line of profiles/hbm_traffic.txt that says which commit its counters were taken at."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    for line in open(path):
        if line.startswith("COMMIT"):
            return line.strip()
    return "profiles/hbm_traffic.txt (commit not recorded)"


def cpu_baseline(w, heads):
    """The float64 oracle (chunked form, forward + backward) on the first `heads` heads of the
    workload, whole sequence."""
    from oracle import power_attn_oracle as orc
    from paper_2507_04239_amd import inputs
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:
        cores = 1
    heads = max(1, min(heads, w["B"] * w["H"]))
    Q, K, V, G = inputs.make_qkvg(1, heads, w["T"], w["d"], seed=1000 + w["position"], dtype=w["dtype"])
    t0 = time.perf_counter()
    for h in range(heads):
        orc.bwd_chunked(Q[0, h], K[0, h], V[0, h], G[0, h], w["p"], w["chunk"])   # runs the forward pass inside
    dt = time.perf_counter() - t0
    # `heads` of the B*H heads of the job: a token of the whole job costs H head-tokens
    return {"value": heads * w["T"] / (dt * w["H"]), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"fwd+bwd of {heads} of {w['B'] * w['H']} heads, all {w['T']} tokens ({dt:.1f} s), "
                      f"scaled by {heads}/{w['H']}", "seconds": dt}


def decode_bench(args, name, w):
    """One decode step = one new token for each of --decode-batch sequences, all heads; the state
    (D x (v+1) float32 per head) is read and written once per step."""
    import torch
    from paper_2507_04239_amd import binding
    B, H, d, p = args.decode_batch, w["H"], w["d"], w["p"]
    dev = torch.device("cuda:0")
    tdt = torch.bfloat16 if w["dtype"] == "bf16" else torch.float32
    prob = binding.make_problem(B, H, 1, d, d, p, 1, True, 1.0, w["dtype"], "auto", False, args.gated)
    state = binding.power_attn_decode_init(prob)
    g = torch.Generator(device=dev)
    g.manual_seed(2000 + w["position"])
    q = (torch.randn((B, H, d), device=dev, generator=g) * d ** -0.5).to(tdt)
    k = (torch.randn((B, H, d), device=dev, generator=g) * d ** -0.5).to(tdt)
    v = torch.randn((B, H, d), device=dev, generator=g).to(tdt)
    lg = -0.02 * torch.rand((B, H), device=dev, generator=g) if args.gated else None
    o = torch.empty_like(v)
    z = torch.empty((B, H), dtype=torch.float32, device=dev)

    def step():
        binding.power_attn_decode_step(prob, q, k, v, state, lg, out=o, out_z=z)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    binding.profile_begin()
    for _ in range(args.steps):
        step()
    kernels = binding.profile_end()
    D = math.comb(d + p - 1, p)
    alg_bytes = 2 * B * H * D * (d + 1) * 4                 # the state, read and written once
    kms = kernels["decode_step"][1] / kernels["decode_step"][0]
    achieved = alg_bytes / (kms * 1e-3) / 1e9
    print(json.dumps({
        "metric": "power-attention decode tokens/sec (one token per sequence and step, state resident)",
        "value": B / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32 state, " + w["dtype"] + " tokens",
        "data": "synthetic",
        "config": {"workload": name + " head shape, decode", "B": B, "H": H, "d": d, "p": p, "state_rows": D, "gated": args.gated},
        "roofline": {"bound": "hbm", "kernel": "decode_step", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": achieved / PEAK_HBM_GBS, "traffic": None, "avg_kernel_ms": kms,
                     "algorithmic_bytes_per_launch": alg_bytes},
        "kernels": {n: {"launches_per_step": l / args.steps, "avg_ms": t / l} for n, (l, t) in kernels.items()},
    }), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=None, help="name from paper_2507_04239_amd.inputs.WORKLOADS (the paper's five configurations) or EXTRA_WORKLOADS")
    ap.add_argument("--chunk", type=int, default=None,
                    help="chunk size instead of the workload's own; 0 lets the library choose (attention form or chunked)")
    ap.add_argument("--impl", default="auto", choices=["auto", "generic", "mfma", "resident", "tiled"])
    ap.add_argument("--d-tile", type=int, default=0, help="tile width of the embedding for the tiled kernels (0: their default)")
    ap.add_argument("--cpu-sample-heads", type=int, default=2, help="heads the CPU oracle is timed on")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB (a dispatch of known size, for scaling "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--serial-kernels", action="store_true",
                    help="run every step with the library's per-kernel events on, i.e. kernels back to back with no "
                         "overlap between streams (for a rocprofv3 kernel trace whose averages are each kernel's own)")
    ap.add_argument("--gated", action="store_true",
                    help="time the gated layer (per-timestep log-gates, mean decay 0.02 per step) instead of the headline one")
    ap.add_argument("--recompute-states", action="store_true",
                    help="backward pass rebuilds the chunk states instead of reusing the forward pass's workspace")
    ap.add_argument("--forward-only", action="store_true", help="time the forward pass alone")
    ap.add_argument("--all-configs", action="store_true",
                    help="run the five benchmark configurations as stated, one JSON line each")
    ap.add_argument("--sweep", action="store_true",
                    help="time the workload at every chunk size (128 ... 1024, and the whole sequence) and tile width "
                         "the library takes for it, plus its own choice (chunk 0); one JSON line with the table")
    ap.add_argument("--decode-batch", type=int, default=0,
                    help="instead of the training step: time the single-token decode step of the workload's head shape "
                         "on this many sequences (state resident in HBM)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build measures one GPU only (the path shards over batch and heads with no "
                 "communication); run with --gpus 1")

    from paper_2507_04239_amd import inputs
    if args.decode_batch > 0:
        name = args.workload or inputs.HEADLINE
        return decode_bench(args, name, dict(inputs.WORKLOADS[name] if name in inputs.WORKLOADS else inputs.EXTRA_WORKLOADS[name]))
    if args.sweep:
        return sweep(args, args.workload or inputs.HEADLINE)
    if args.all_configs:
        # every benchmark configuration as stated, one JSON line each (the headline one carries the CPU baseline)
        for name in sorted(inputs.WORKLOADS, key=lambda n: inputs.WORKLOADS[n]["position"]):
            out = run_workload(args, name, cpu=(name == inputs.HEADLINE and not args.no_cpu_baseline))
            print(json.dumps(out), flush=True)
        return
    name = args.workload or inputs.HEADLINE
    print(json.dumps(run_workload(args, name, cpu=not args.no_cpu_baseline)), flush=True)


def sweep(args, name):
    """Chunk size x tile width (Sec. 4.1.1, Fig. 6(c)'s study): every combination the library takes for the workload,
    the attention form (one chunk) and the library's own choice, HIP-event median per step."""
    import copy
    from paper_2507_04239_amd import binding, inputs
    w = inputs.WORKLOADS[name] if name in inputs.WORKLOADS else inputs.EXTRA_WORKLOADS[name]
    with_bwd = bool(w.get("backward", True)) and not args.forward_only
    rows, seen = [], set()
    sizes = (32, 64, 128, 256, 512, 1024) if w["dtype"] == "f32" else (128, 256, 512, 1024)   # (bf16 below 128: vector ALUs only)
    chunks = [c for c in sizes if w["T"] % c == 0 and c < w["T"]] + [w["T"], 0]
    for chunk in chunks:
        for dt in (0, 2, 4, 8, 16):
            prob = binding.make_problem(w["B"], w["H"], w["T"], w["d"], w["d"], w["p"], chunk, w.get("normalize", True), 1.0, w["dtype"],
                                        args.impl, not args.recompute_states, args.gated, dt)
            if not binding.power_attn_supported(prob, with_bwd):
                continue
            key = (binding.power_attn_resolved_chunk(prob), dt, binding.power_attn_state_rows(prob)) if chunk else ("auto", dt)
            if key in seen or (chunk == 0 and dt) or (dt == {2: 8, 3: 4, 4: 2}.get(w["p"]) and (chunk, "tiled") in seen):
                continue   # (the tile width named is the one the tiled kernels just ran with by default)
            seen.add(key)
            a = copy.copy(args)
            a.chunk, a.d_tile, a.serial_kernels = chunk, dt, False
            out = run_workload(a, name, cpu=False)
            rows.append({"chunk_requested": chunk, "chunk": out["config"]["chunk"], "d_tile": dt,
                         "state_rows": out["config"]["state_rows"], "step_ms_median": out["timing"]["step_ms_median"],
                         "fwd_ms_median": out["timing"]["fwd_ms_median"], "kernels": sorted(out["kernels"])})
            if dt == 0 and any(k.startswith("tiled") for k in out["kernels"]):
                seen.add((chunk, "tiled"))
            print(f"# chunk {chunk} d_tile {dt}: {rows[-1]['step_ms_median']:.3f} ms", file=sys.stderr, flush=True)
    best = min((r for r in rows if r["chunk_requested"]), key=lambda r: r["step_ms_median"])
    print(json.dumps({"metric": "power-attention step time over chunk size and tile width", "unit": "ms", "workload": name,
                      "pass": "fwd+bwd" if with_bwd else "fwd", "impl": args.impl, "steps": args.steps, "warmup": args.warmup,
                      "best": {k: best[k] for k in ("chunk", "d_tile", "step_ms_median")}, "sweep": rows}), flush=True)


def event_times(step, steps):
    """Milliseconds of `steps` calls of step(), each bracketed by a pair of HIP events on the current stream
    (the stream the library launches on; its side stream is forked from and joined back into it)."""
    import torch
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for e0, e1 in ev:
        e0.record()
        step()
        e1.record()
    torch.cuda.synchronize()
    return sorted(e0.elapsed_time(e1) for e0, e1 in ev)


def run_workload(args, name, cpu):
    import torch
    from paper_2507_04239_amd import binding, inputs, power_attn_bwd, power_attn_fwd

    w = dict(inputs.WORKLOADS[name] if name in inputs.WORKLOADS else inputs.EXTRA_WORKLOADS[name])
    norm = bool(w.get("normalize", True))
    oracle_chunk = w["chunk"]
    if args.chunk is not None:
        w["chunk"] = args.chunk
    dev = torch.device("cuda:0")
    tdt = torch.bfloat16 if w["dtype"] == "bf16" else torch.float32
    Q, K, V, G = inputs.make_workload(name, with_grad=True)
    tq, tk, tv, tg = (torch.from_numpy(a).to(dev).to(tdt) for a in (Q, K, V, G))
    del Q, K, V, G
    p, chunk = w["p"], w["chunk"]
    keep = not args.recompute_states
    tl = None
    if args.gated:
        tl = torch.from_numpy(inputs.make_log_gates(w["B"], w["H"], w["T"], 1500 + w["position"])).to(dev)
    prob = binding.make_problem(w["B"], w["H"], w["T"], w["d"], w["d"], p, chunk, norm, 1.0, w["dtype"], args.impl, keep,
                                args.gated, args.d_tile)
    w["chunk"] = binding.power_attn_resolved_chunk(prob)      # what the library runs (differs when 0 was asked for)
    ws_bytes = max(binding.power_attn_workspace_bytes(prob, True), binding.power_attn_workspace_bytes(prob, False))
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)
    O = torch.empty_like(tv)
    Z = torch.empty(tq.shape[:3], dtype=torch.float32, device=dev)
    grads = (torch.empty_like(tq), torch.empty_like(tk), torch.empty_like(tv))

    with_bwd = bool(w.get("backward", True)) and not args.forward_only    # configs 1 and 2 are forward-only

    def fwd():
        power_attn_fwd(tq, tk, tv, p, chunk, normalize=norm, impl=args.impl, workspace=ws, out=O, out_z=Z, keep_state=keep,
                       log_g=tl, d_tile=args.d_tile)

    def bwd():
        power_attn_bwd(tq, tk, tv, O, Z, tg, p, chunk, normalize=norm, impl=args.impl, workspace=ws, out=grads, keep_state=keep,
                       log_g=tl, d_tile=args.d_tile)

    def step():
        fwd()
        if with_bwd:
            bwd()

    if args.serial_kernels:
        binding.profile_begin()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    if args.serial_kernels:
        binding.profile_end()
    tokens = w["B"] * w["T"]

    # the same steps again, each one between a pair of HIP events; then the two passes on their own
    ev_step = event_times(step, args.steps)
    ev_fwd = event_times(fwd, args.steps)
    ev_bwd = event_times(bwd, args.steps) if with_bwd else None
    med = lambda xs: xs[len(xs) // 2]
    timing = {"clock": "hip events on the launch stream, per step", "step_ms_median": med(ev_step), "step_ms_min": ev_step[0],
              "step_ms_max": ev_step[-1], "fwd_ms_median": med(ev_fwd), "fwd_ms_min": ev_fwd[0]}
    if ev_bwd:
        timing.update({"bwd_ms_median": med(ev_bwd), "bwd_ms_min": ev_bwd[0]})

    if args.copy_calibration_mib > 0:
        src = torch.empty(args.copy_calibration_mib << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # per-kernel durations from HIP events recorded by the library on the launch stream; while
    # they are recorded the library runs its kernels back to back (no overlap between streams)
    binding.profile_begin()
    for _ in range(args.steps):
        step()
    kernels = binding.profile_end()
    fl, by = algorithmic_flops(w), algorithmic_bytes(w)
    per_kernel = {}
    for kname, (launches, ms_total) in kernels.items():
        per_kernel[kname] = {"launches_per_step": launches / args.steps, "avg_ms": ms_total / launches}
        if kname in KERNEL_ROLE:
            role, peak = KERNEL_ROLE[kname]
            sec = ms_total / launches * 1e-3
            per_kernel[kname].update({"tflops": fl[role] / sec / 1e12, "frac_compute_peak": fl[role] / sec / 1e12 / peak,
                                      "hbm_gbs": by[role] / sec / 1e9, "frac_hbm_peak": by[role] / sec / 1e9 / PEAK_HBM_GBS})
    # The dominant kernel, and the roof that bounds it: the one whose lower bound on its time is larger.
    credited = {k: v for k, v in kernels.items() if k in KERNEL_ROLE and KERNEL_ROLE[k][0] != "recompute"}
    dom = max(credited, key=lambda k: credited[k][1])
    role, peak = KERNEL_ROLE[dom]
    dom_ms = credited[dom][1] / credited[dom][0]
    t_compute = fl[role] / (peak * 1e12)
    t_hbm = by[role] / (PEAK_HBM_GBS * 1e9)
    traffic = measured_traffic(name, dom)
    if t_hbm >= t_compute:
        achieved = by[role] / (dom_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": achieved / PEAK_HBM_GBS, "traffic": traffic, "avg_kernel_ms": dom_ms,
                    "algorithmic_bytes_per_launch": by[role], "algorithmic_flops_per_launch": fl[role],
                    "frac_of_compute_peak": fl[role] / (dom_ms * 1e-3) / 1e12 / peak}
    else:
        achieved = fl[role] / (dom_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma" if peak == PEAK_BF16_MFMA_TFLOPS else "alu", "kernel": dom, "achieved": achieved,
                    "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak, "traffic": traffic,
                    "avg_kernel_ms": dom_ms, "algorithmic_flops_per_launch": fl[role],
                    "algorithmic_bytes_per_launch": by[role]}
    roofline["traffic_source"] = traffic_source() if traffic is not None else None
    total_alg = fl["fwd_total"] + (fl["bwd_total"] if with_bwd else 0)
    out = {
        "metric": "power-attention fwd+bwd tokens/sec at p=2,d=64,T=64k; % bf16 MFMA peak",
        "value": tokens / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w["dtype"], "data": "synthetic",
        "config": {"workload": name, "B": w["B"], "H": w["H"], "T": w["T"], "d": w["d"], "p": p, "chunk": w["chunk"],
                   "chunk_requested": chunk, "normalize": norm, "pass": "fwd+bwd" if with_bwd else "fwd", "impl": args.impl, "d_tile": args.d_tile, "keep_state": keep, "serial_kernels": args.serial_kernels, "gated": args.gated,
                   "state_rows": binding.power_attn_state_rows(prob)},
        "timing": timing,
        "step_algorithmic_tflop": total_alg / 1e12,
        "step_frac_of_bf16_mfma_peak": total_alg / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS,
        "roofline": roofline,
        "kernels": per_kernel,
    }
    if cpu:
        out["cpu_baseline"] = cpu_baseline(dict(w, chunk=oracle_chunk), args.cpu_sample_heads)
    del ws, tq, tk, tv, tg, O, Z, grads
    torch.cuda.empty_cache()
    return out


if __name__ == "__main__":
    main()
