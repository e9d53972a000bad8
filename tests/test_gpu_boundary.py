"""Boundary behaviour on the GPU: calls from several host threads, misaligned pointers, run-to-run repeatability."""
import ctypes
import threading

import numpy as np
import pytest

from oracle import power_attn_oracle as orc
from paper_2507_04239_amd import binding, inputs

from gpu_util import TOL, rel_l2, run_fwd_bwd

pytestmark = pytest.mark.gpu


def test_two_host_threads_on_two_streams():
    """The library keeps its side stream, error text and profiling records per host thread: two threads, each on
    a stream, workspace and tensors of its own, run forward + backward at the same time and both match the oracle."""
    import torch
    from paper_2507_04239_amd import power_attn_bwd, power_attn_fwd
    cases = [(1, 2, 1024, 64, 128, 901), (1, 2, 768, 64, 128, 902)]
    results, errors = [None, None], []

    def work(i):
        try:
            B, H, T, d, chunk, seed = cases[i]
            Q, K, V, G = inputs.make_qkvg(B, H, T, d, seed=seed, dtype="bf16")
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                tq, tk, tv, tg = (torch.from_numpy(a).to("cuda:0").to(torch.bfloat16) for a in (Q, K, V, G))
                for _ in range(3):      # several rounds, so that the two threads' calls really interleave
                    O, Z = power_attn_fwd(tq, tk, tv, 2, chunk, impl="mfma")
                    dQ, dK, dV = power_attn_bwd(tq, tk, tv, O, Z, tg, 2, chunk, impl="mfma")
                stream.synchronize()
            binding.load_library().power_attn_release_thread()
            results[i] = (Q, K, V, G, chunk, [t.float().cpu().numpy() for t in (O, dQ, dK, dV)])
        except Exception as e:   # noqa: BLE001
            errors.append(e)

    threads = [threading.Thread(target=work, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    for Q, K, V, G, chunk, (O, dQ, dK, dV) in results:
        O_ref, _ = orc.fwd_bhtd(Q, K, V, 2, chunk)
        ref = orc.bwd_bhtd(Q, K, V, G, 2, chunk)
        for got, want in ((O, O_ref), (dQ, ref[0]), (dK, ref[1]), (dV, ref[2])):
            assert rel_l2(got, want) <= TOL["bf16"]


def test_misaligned_tensor_pointer_is_refused():
    """Tensor pointers must be 16-byte aligned: a misaligned one is an invalid argument, and nothing is launched."""
    import torch
    lib = binding.load_library()
    B, H, T, d = 1, 1, 256, 64
    prob = binding.make_problem(B, H, T, d, d, 2, 128, True, 1.0, "bf16", "mfma")
    need = lib.power_attn_workspace_bytes(ctypes.byref(prob), 0)
    ws = torch.empty(need + 256, dtype=torch.uint8, device="cuda:0")
    buf = torch.zeros(B * H * T * d + 8, dtype=torch.bfloat16, device="cuda:0")
    good = ctypes.c_void_p(buf.data_ptr())
    bad = ctypes.c_void_p(buf.data_ptr() + 2)          # one bf16 element off
    Z = torch.empty(B * H * T, dtype=torch.float32, device="cuda:0")
    z = ctypes.c_void_p(Z.data_ptr())
    w = ctypes.c_void_p(ws.data_ptr())
    assert lib.power_attn_fwd(ctypes.byref(prob), bad, good, good, good, z, w, need, None) == 1     # PA_ERR_INVALID_ARG
    assert lib.power_attn_fwd(ctypes.byref(prob), good, good, good, bad, z, w, need, None) == 1
    assert lib.power_attn_fwd(ctypes.byref(prob), good, good, good, good, z, ctypes.c_void_p(ws.data_ptr() + 16), need, None) == 3
    torch.cuda.synchronize()


@pytest.mark.parametrize("impl,d,chunk", [("mfma", 64, 128), ("mfma", 64, 512), ("resident", 64, 128), ("resident", 128, 256),
                                          ("mfma", 128, 0)])
def test_matrix_core_kernels_repeat_bit_for_bit(impl, d, chunk):
    """Every sum of the matrix-core kernels is taken in a fixed order (no float atomics): two runs on the same
    inputs give identical bits in every output."""
    Q, K, V, G = inputs.make_qkvg(1, 2, 1024, d, seed=950 + d, dtype="bf16")
    a = run_fwd_bwd(Q, K, V, G, 2, chunk, "bf16", impl=impl)
    b = run_fwd_bwd(Q, K, V, G, 2, chunk, "bf16", impl=impl)
    for key in a:
        assert np.array_equal(a[key], b[key]), key


def test_generic_family_forward_repeats_and_backward_is_order_dependent_within_tolerance():
    """The vector-ALU family's forward pass has a fixed summation order.  Its dQ / dK kernels add the Jacobian terms
    with LDS float atomics, whose order is not fixed: two runs may differ in the last bits, by far less than the
    float32 tolerance."""
    Q, K, V, G = inputs.make_qkvg(1, 1, 256, 16, seed=951, dtype="f32")
    a = run_fwd_bwd(Q, K, V, G, 2, 32, "f32", impl="generic")
    b = run_fwd_bwd(Q, K, V, G, 2, 32, "f32", impl="generic")
    assert np.array_equal(a["O"], b["O"]) and np.array_equal(a["Z"], b["Z"]) and np.array_equal(a["dV"], b["dV"])
    for key in ("dQ", "dK"):
        assert rel_l2(a[key], b[key]) <= 1e-6, key
