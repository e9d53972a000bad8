"""GPU parity of the single-token decode step against the float64 oracle, through the C ABI: a
sequence is fed token by token and every step's output is compared; the state left behind is
compared with the oracle's (the device keeps the integer multiplicity of each monomial on the state,
the oracle its square root on both sides: S_dev[r] = sqrt(m_r) S_oracle[r])."""
import numpy as np
import pytest

from oracle import power_attn_oracle as orc
from paper_2507_04239_amd import binding, inputs

from gpu_util import TOL, rel_l2, to_dev, to_np

pytestmark = pytest.mark.gpu

CASES = [
    # dtype, p, B, H, T, d, normalize, scale, gated
    ("f32", 2, 1, 2, 40, 16, True, 1.0, False),
    ("f32", 2, 2, 1, 24, 64, True, 0.8, True),
    ("bf16", 2, 1, 3, 48, 64, True, 1.0, False),       # the headline head shape
    ("bf16", 2, 1, 2, 32, 64, True, 1.0, True),
    ("f32", 4, 1, 1, 20, 16, True, 1.0, True),
    ("bf16", 4, 1, 2, 16, 32, True, 1.0, False),       # config 4's head shape: 52360 state rows
    ("f32", 3, 1, 2, 24, 24, False, 1.0, False),       # odd degree, un-normalised
    ("bf16", 2, 1, 1, 12, 128, True, 1.0, False),      # config 5's head shape: two column passes per row
    ("f32", 1, 1, 1, 16, 8, False, 1.0, True),         # degree 1: gated linear attention
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "-".join(str(x) for x in c))
def test_decode_steps_match_the_oracle(case):
    import torch
    dtype, p, B, H, T, d, normalize, scale, gated = case
    print("case", case, flush=True)
    Q, K, V, _ = inputs.make_qkvg(B, H, T, d, seed=8000 + CASES.index(case), dtype=dtype, with_grad=False)
    lg = inputs.make_log_gates(B, H, T, 8100 + CASES.index(case), 0.1) if gated else None
    prob = binding.make_problem(B, H, 1, d, d, p, 1, normalize, scale, dtype, "auto", False, gated)
    state = binding.power_attn_decode_init(prob)
    tq, tk, tv = (to_dev(a, dtype) for a in (Q, K, V))
    tl = None if lg is None else torch.from_numpy(np.ascontiguousarray(lg)).to("cuda:0")
    outs, zs = [], []
    for t in range(T):
        o, z = binding.power_attn_decode_step(prob, tq[:, :, t].contiguous(), tk[:, :, t].contiguous(),
                                              tv[:, :, t].contiguous(), state,
                                              None if tl is None else tl[:, :, t].contiguous())
        outs.append(o)
        zs.append(z)
    torch.cuda.synchronize()
    got_o = np.stack([to_np(o) for o in outs], axis=2)       # [B, H, T, v]
    got_z = np.stack([to_np(z) for z in zs], axis=2)         # [B, H, T]
    ref_o, ref_z = np.zeros_like(got_o, dtype=np.float64), np.zeros_like(got_z, dtype=np.float64)
    D = orc.dim_spow(d, p)
    S_ref = np.zeros((B, H, D, d + 1))
    for b in range(B):
        for h in range(H):
            S = orc.decode_state_init(d, d, p)
            for t in range(T):
                S, ref_o[b, h, t], ref_z[b, h, t] = orc.decode_step(S, Q[b, h, t], K[b, h, t], V[b, h, t], p, normalize, scale,
                                                                    None if lg is None else lg[b, h, t])
            S_ref[b, h] = S
    # Numerator and denominator are sums over the expanded dimension whose terms cancel down to
    # (q.k)^p; in float32 each is accurate relative to the size of those terms, not to its own value.
    # So: the denominator and the numerator o z are compared as they are, and the quotient on the rows
    # whose denominator is not far below the typical one (a first token with a tiny score is not).
    ez = rel_l2(got_z, ref_z)
    en = rel_l2(got_o * got_z[..., None], ref_o * ref_z[..., None]) if normalize else rel_l2(got_o, ref_o)
    well = np.abs(ref_z) >= 0.05 * np.median(np.abs(ref_z)) if normalize else np.ones_like(ref_z, dtype=bool)
    assert well.mean() > 0.6
    eo = rel_l2(got_o[well], ref_o[well])
    # the state itself: float32 words at the start of the buffer, S [BH][D][v] then gamma [BH][D]
    words = state.view(torch.float32)
    S_dev = to_np(words[: B * H * D * d]).reshape(B, H, D, d)
    off_gam = ((B * H * D * d * 4 + 255) // 256 * 256) // 4
    gam_dev = to_np(words[off_gam: off_gam + B * H * D]).reshape(B, H, D)
    sq = np.sqrt(np.array([orc.multiplicity(r) for r in orc.ndmi(d, p)], dtype=np.float64))
    es = rel_l2(S_dev, S_ref[..., :d] * sq[None, None, :, None])
    eg = rel_l2(gam_dev, S_ref[..., d] * sq[None, None, :])
    print(f"decode {case}: o={eo:.2e} ({well.sum()} of {well.size} rows) numerator={en:.2e} z={ez:.2e} state={es:.2e} gamma={eg:.2e}",
          flush=True)
    assert eo <= TOL[dtype] and ez <= TOL[dtype] and en <= TOL[dtype]
    assert es <= TOL[dtype] and eg <= TOL[dtype]


def test_decode_agrees_with_the_whole_sequence_call():
    """Token by token, the decode step returns the rows the forward call returns for the sequence."""
    import torch
    from paper_2507_04239_amd import power_attn_fwd
    B, H, T, d = 1, 2, 256, 64
    Q, K, V, _ = inputs.make_qkvg(B, H, T, d, seed=8200, dtype="bf16", with_grad=False)
    tq, tk, tv = (to_dev(a, "bf16") for a in (Q, K, V))
    O, Z = power_attn_fwd(tq, tk, tv, 2, 128)
    prob = binding.make_problem(B, H, 1, d, d, 2, 1, True, 1.0, "bf16")
    state = binding.power_attn_decode_init(prob)
    for t in range(T):
        o, z = binding.power_attn_decode_step(prob, tq[:, :, t].contiguous(), tk[:, :, t].contiguous(), tv[:, :, t].contiguous(), state)
        if t in (0, 1, 127, 128, 200, 255):
            torch.cuda.synchronize()
            assert rel_l2(to_np(o), to_np(O[:, :, t])) <= TOL["bf16"], t
            assert rel_l2(to_np(z), to_np(Z[:, :, t])) <= TOL["bf16"], t


def test_decode_refusals():
    import torch
    prob = binding.make_problem(1, 1, 1, 16, 16, 2, 1, True, 1.0, "f32")
    need = binding.power_attn_decode_state_bytes(prob)
    assert need > 0
    small = torch.empty(need - 256, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(binding.PowerAttnError):
        binding.power_attn_decode_init(prob, small)
    odd = binding.make_problem(1, 1, 1, 16, 16, 3, 1, True, 1.0, "f32")          # odd degree cannot be normalised
    assert binding.power_attn_decode_state_bytes(odd) == 0
    state = binding.power_attn_decode_init(prob)
    x = torch.zeros(1, 1, 16, device="cuda:0")
    with pytest.raises(binding.PowerAttnError):                                   # gates given to an un-gated problem
        binding.power_attn_decode_step(prob, x, x, x, state, torch.zeros(1, 1, device="cuda:0"))


ABSORB_CASES = [
    # dtype, p, B, H, T, d, normalize, gated
    ("bf16", 2, 1, 2, 200, 64, True, False),
    ("bf16", 2, 1, 2, 77, 64, True, True),
    ("f32", 4, 1, 1, 50, 16, True, True),
    ("bf16", 2, 1, 1, 40, 128, True, False),
    ("f32", 3, 2, 1, 33, 24, False, False),
]


@pytest.mark.parametrize("case", ABSORB_CASES, ids=lambda c: "-".join(str(x) for x in c))
def test_absorbing_a_prompt_equals_stepping_through_it(case):
    """The hand-over from a prompt: the state after power_attn_decode_absorb is the oracle's state after
    stepping through the same tokens, also when the prompt arrives in two pieces, and the next decode
    step returns the oracle's output."""
    import torch
    dtype, p, B, H, T, d, normalize, gated = case
    print("case", case, flush=True)
    Q, K, V, _ = inputs.make_qkvg(B, H, T + 1, d, seed=8300 + ABSORB_CASES.index(case), dtype=dtype, with_grad=False)
    lg = inputs.make_log_gates(B, H, T + 1, 8400 + ABSORB_CASES.index(case), 0.05) if gated else None
    tq, tk, tv = (to_dev(a, dtype) for a in (Q, K, V))
    tl = None if lg is None else torch.from_numpy(np.ascontiguousarray(lg)).to("cuda:0")

    def absorb(lo, hi, state):
        prob = binding.make_problem(B, H, hi - lo, d, d, p, 1, normalize, 1.0, dtype, "auto", False, gated)
        return binding.power_attn_decode_absorb(prob, tk[:, :, lo:hi].contiguous(), tv[:, :, lo:hi].contiguous(), state,
                                                None if tl is None else tl[:, :, lo:hi].contiguous())

    prob1 = binding.make_problem(B, H, 1, d, d, p, 1, normalize, 1.0, dtype, "auto", False, gated)
    whole = absorb(0, T, binding.power_attn_decode_init(prob1))
    pieces = absorb(T // 3, T, absorb(0, T // 3, binding.power_attn_decode_init(prob1)))
    D = orc.dim_spow(d, p)
    n_s = B * H * D * d
    off_gam = ((n_s * 4 + 255) // 256 * 256) // 4
    sq = np.sqrt(np.array([orc.multiplicity(r) for r in orc.ndmi(d, p)], dtype=np.float64))
    S_ref = np.zeros((B, H, D, d + 1))
    o_ref, z_ref = np.zeros((B, H, d)), np.zeros((B, H))
    for b in range(B):
        for h in range(H):
            S = orc.decode_state_init(d, d, p)
            for t in range(T):
                S, _, _ = orc.decode_step(S, Q[b, h, t], K[b, h, t], V[b, h, t], p, normalize, 1.0, None if lg is None else lg[b, h, t])
            S_ref[b, h] = S
            _, o_ref[b, h], z_ref[b, h] = orc.decode_step(S, Q[b, h, T], K[b, h, T], V[b, h, T], p, normalize, 1.0,
                                                          None if lg is None else lg[b, h, T])
    for name, state in (("whole", whole), ("two pieces", pieces)):
        words = state.view(torch.float32)
        S_dev = to_np(words[:n_s]).reshape(B, H, D, d)
        gam_dev = to_np(words[off_gam: off_gam + B * H * D]).reshape(B, H, D)
        es = rel_l2(S_dev, S_ref[..., :d] * sq[None, None, :, None])
        eg = rel_l2(gam_dev, S_ref[..., d] * sq[None, None, :])
        print(f"absorb {case} {name}: state={es:.2e} gamma={eg:.2e}", flush=True)
        assert es <= 1e-5 and eg <= 1e-5          # float32 sums of exactly representable inputs
    o, z = binding.power_attn_decode_step(prob1, tq[:, :, T].contiguous(), tk[:, :, T].contiguous(), tv[:, :, T].contiguous(), whole,
                                          None if tl is None else tl[:, :, T].contiguous())
    torch.cuda.synchronize()
    ez = rel_l2(to_np(z), z_ref)
    en = rel_l2(to_np(o) * to_np(z)[..., None], o_ref * z_ref[..., None]) if normalize else rel_l2(to_np(o), o_ref)
    print(f"absorb {case}: next step numerator={en:.2e} z={ez:.2e}", flush=True)
    assert ez <= TOL[dtype] and en <= TOL[dtype]


@pytest.mark.parametrize("gated", [False, True], ids=["plain", "gated"])
def test_prompt_through_the_matrix_core_scan(gated):
    """bf16, p = 2, d = 64, a prompt of a multiple of 128 tokens: with a workspace the hand-over runs the
    state scan on the matrix cores.  Its sums are rounded to bf16 once (2^-9 per entry); state and next
    decode step against the oracle, and against the float32 hand-over."""
    import torch
    B, H, T, d, p = 1, 3, 640, 64, 2
    Q, K, V, _ = inputs.make_qkvg(B, H, T + 1, d, seed=8600 + int(gated), dtype="bf16", with_grad=False)
    lg = inputs.make_log_gates(B, H, T + 1, 8610, 0.03) if gated else None
    tq, tk, tv = (to_dev(a, "bf16") for a in (Q, K, V))
    tl = None if lg is None else torch.from_numpy(np.ascontiguousarray(lg)).to("cuda:0")
    prob = binding.make_problem(B, H, T, d, d, p, 1, True, 1.0, "bf16", "auto", False, gated)
    prob1 = binding.make_problem(B, H, 1, d, d, p, 1, True, 1.0, "bf16", "auto", False, gated)
    assert binding.power_attn_decode_absorb_workspace_bytes(prob) > 0
    assert binding.power_attn_decode_absorb_workspace_bytes(binding.make_problem(B, H, T + 1, d, d, p, 1)) == 0
    kk, vv = tk[:, :, :T].contiguous(), tv[:, :, :T].contiguous()
    ll = None if tl is None else tl[:, :, :T].contiguous()
    fast = binding.power_attn_decode_absorb(prob, kk, vv, binding.power_attn_decode_init(prob1), ll, fast=True)
    slow = binding.power_attn_decode_absorb(prob, kk, vv, binding.power_attn_decode_init(prob1), ll, fast=False)
    # a second prompt on top of the first: the old state decays across it
    fast = binding.power_attn_decode_absorb(prob, kk, vv, fast, ll, fast=True)
    slow = binding.power_attn_decode_absorb(prob, kk, vv, slow, ll, fast=False)
    D = orc.dim_spow(d, p)
    n_s = B * H * D * d
    off_gam = ((n_s * 4 + 255) // 256 * 256) // 4
    wf, wsl = fast.view(torch.float32), slow.view(torch.float32)
    e_s = rel_l2(to_np(wf[:n_s]), to_np(wsl[:n_s]))
    e_g = rel_l2(to_np(wf[off_gam: off_gam + B * H * D]), to_np(wsl[off_gam: off_gam + B * H * D]))
    print(f"scan hand-over vs float32 hand-over: state={e_s:.2e} gamma={e_g:.2e}", flush=True)
    assert e_s <= 5e-3 and e_g <= 5e-3
    o, z = binding.power_attn_decode_step(prob1, tq[:, :, T].contiguous(), tk[:, :, T].contiguous(), tv[:, :, T].contiguous(), fast,
                                          None if tl is None else tl[:, :, T].contiguous())
    torch.cuda.synchronize()
    o_ref, z_ref = np.zeros((B, H, d)), np.zeros((B, H))
    for h in range(H):
        S = orc.decode_state_init(d, d, p)
        for rep in range(2):
            for t in range(T):
                S, _, _ = orc.decode_step(S, Q[0, h, t], K[0, h, t], V[0, h, t], p, True, 1.0, None if lg is None else lg[0, h, t])
        _, o_ref[0, h], z_ref[0, h] = orc.decode_step(S, Q[0, h, T], K[0, h, T], V[0, h, T], p, True, 1.0,
                                                      None if lg is None else lg[0, h, T])
    assert rel_l2(to_np(z), z_ref) <= TOL["bf16"]
    assert rel_l2(to_np(o) * to_np(z)[..., None], o_ref * z_ref[..., None]) <= TOL["bf16"]


@pytest.mark.parametrize("fast", [False, True], ids=["float32", "scan"])
def test_prefill_then_decode_continues_the_sequence(fast):
    """power_attn_fwd on a prompt, the prompt handed to a decode state, then decode steps: every
    decoded row equals the row power_attn_fwd returns for the longer sequence."""
    import torch
    from paper_2507_04239_amd import power_attn_fwd
    B, H, T, extra, d = 1, 2, 512, 128, 64
    Q, K, V, _ = inputs.make_qkvg(B, H, T + extra, d, seed=8500, dtype="bf16", with_grad=False)
    tq, tk, tv = (to_dev(a, "bf16") for a in (Q, K, V))
    O_all, Z_all = power_attn_fwd(tq, tk, tv, 2, 128)
    prob_prompt = binding.make_problem(B, H, T, d, d, 2, 1, True, 1.0, "bf16")
    prob1 = binding.make_problem(B, H, 1, d, d, 2, 1, True, 1.0, "bf16")
    state = binding.power_attn_decode_init(prob1)
    binding.power_attn_decode_absorb(prob_prompt, tk[:, :, :T].contiguous(), tv[:, :, :T].contiguous(), state, fast=fast)
    for t in range(T, T + extra):
        o, z = binding.power_attn_decode_step(prob1, tq[:, :, t].contiguous(), tk[:, :, t].contiguous(), tv[:, :, t].contiguous(), state)
        if t in (T, T + 1, T + 63, T + extra - 1):
            torch.cuda.synchronize()
            assert rel_l2(to_np(o), to_np(O_all[:, :, t])) <= TOL["bf16"], t
            assert rel_l2(to_np(z), to_np(Z_all[:, :, t])) <= TOL["bf16"], t
