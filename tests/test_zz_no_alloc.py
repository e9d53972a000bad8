"""power_attn_fwd_static (the entry point that allocates nothing) against power_attn_fwd, through the C ABI:
two calls in a row on the library's static scratch, the second on a smaller input."""
import ctypes

import numpy as np
import pytest

from paper_2507_04239_amd import binding, inputs

from gpu_util import TOL, ROW_TOL, max_row_err, rel_l2

pytestmark = pytest.mark.gpu


def _both(lib, B, H, T, d, p, chunk, dtype, impl, seed):
    import torch
    Q, K, V, _ = inputs.make_qkvg(B, H, T, d, seed=seed, dtype=dtype, with_grad=False)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    tq, tk, tv = (torch.from_numpy(a).to("cuda:0").to(tdt) for a in (Q, K, V))
    prob = binding.make_problem(B, H, T, d, d, p, chunk, True, 1.0, dtype, impl)
    need = lib.power_attn_workspace_bytes(ctypes.byref(prob), 0)
    assert need <= lib.power_attn_static_scratch_bytes()
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda:0")
    outs = []
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    for static in (False, True):
        # outputs start as NaN: whatever the call leaves unwritten shows up
        O = torch.full_like(tv, float("nan"))
        Z = torch.full((B, H, T), float("nan"), dtype=torch.float32, device="cuda:0")
        args = [ctypes.byref(prob)] + [ctypes.c_void_p(t.data_ptr()) for t in (tq, tk, tv, O, Z)]
        if static:
            st = lib.power_attn_fwd_static(*args, stream)
        else:
            st = lib.power_attn_fwd(*args, ctypes.c_void_p(ws.data_ptr()), need, stream)
        assert st == 0, (static, st, lib.power_attn_last_hip_error())
        torch.cuda.synchronize()
        outs.append((O.float().cpu().numpy(), Z.cpu().numpy()))
    return outs


@pytest.mark.parametrize("dtype,impl,chunk,shapes", [
    ("bf16", "mfma", 128, [(1, 2, 1024, 64), (1, 1, 256, 64)]),      # chunked matrix-core kernels: states in the scratch
    ("f32", "generic", 32, [(1, 2, 512, 16), (1, 1, 96, 16)]),       # vector-ALU family
])
def test_static_scratch_matches_workspace_call(dtype, impl, chunk, shapes):
    lib = binding.load_library()
    for n, (B, H, T, d) in enumerate(shapes):      # second call: smaller input, on the scratch the first left behind
        print("case", dtype, impl, (B, H, T, d), "call", n, flush=True)
        (O_ws, Z_ws), (O_st, Z_st) = _both(lib, B, H, T, d, 2, chunk, dtype, impl, seed=300 + n)
        assert np.isfinite(O_st).all() and np.isfinite(Z_st).all()
        # the same kernels on the same inputs: identical up to the order of the generic family's float atomics
        for got, want in ((O_st, O_ws), (Z_st, Z_ws)):
            assert rel_l2(got, want) <= TOL[dtype] and max_row_err(got, want) <= ROW_TOL[dtype]
        if impl == "mfma":
            assert np.array_equal(O_st, O_ws) and np.array_equal(Z_st, Z_ws)


def test_static_scratch_refuses_what_does_not_fit():
    import torch
    lib = binding.load_library()
    prob = binding.make_problem(1, 12, 65536, 64, 64, 2, 128, True, 1.0, "bf16", "mfma")
    assert lib.power_attn_workspace_bytes(ctypes.byref(prob), 0) > lib.power_attn_static_scratch_bytes()
    x = torch.zeros(8, device="cuda:0")
    p = ctypes.c_void_p(x.data_ptr())
    assert lib.power_attn_fwd_static(ctypes.byref(prob), p, p, p, p, p, None) == 3   # PA_ERR_WORKSPACE; nothing launched
