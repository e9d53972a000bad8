"""ctypes binding of libpower_attn.so: argument marshalling only.

The functions mirror the C ABI (include/power_attn.h): ``power_attn_fwd`` and
``power_attn_bwd`` take torch tensors that live on the GPU, pass their device pointers
and the current HIP stream to the library, and allocate the output tensors and the
workspace with torch.  No arithmetic of the method happens here.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libpower_attn.so"

PA_DTYPE_F32, PA_DTYPE_BF16 = 0, 1
PA_IMPL_AUTO, PA_IMPL_GENERIC, PA_IMPL_MFMA, PA_IMPL_RESIDENT, PA_IMPL_TILED = 0, 1, 2, 3, 4
_IMPL = {"auto": PA_IMPL_AUTO, "generic": PA_IMPL_GENERIC, "mfma": PA_IMPL_MFMA, "resident": PA_IMPL_RESIDENT,
         "tiled": PA_IMPL_TILED}

EXPORTED_SYMBOLS = (
    "power_attn_workspace_bytes",
    "power_attn_supported",
    "power_attn_decode_state_bytes",
    "power_attn_decode_init",
    "power_attn_decode_absorb",
    "power_attn_decode_absorb_workspace_bytes",
    "power_attn_decode_step",
    "power_attn_fwd",
    "power_attn_fwd_static",
    "power_attn_static_scratch_bytes",
    "power_attn_bwd",
    "power_attn_fwd_gated",
    "power_attn_bwd_gated",
    "power_attn_state_rows",
    "power_attn_resolved_chunk",
    "power_attn_status_string",
    "power_attn_last_hip_error",
    "power_attn_release_thread",
    "power_attn_profile_begin",
    "power_attn_profile_end",
)


class PowerAttnError(RuntimeError):
    pass


class PaProblem(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int), ("H", ctypes.c_int), ("T", ctypes.c_int), ("d", ctypes.c_int),
                ("v", ctypes.c_int), ("p", ctypes.c_int), ("chunk", ctypes.c_int), ("normalize", ctypes.c_int),
                ("scale", ctypes.c_float), ("dtype", ctypes.c_int), ("impl", ctypes.c_int),
                ("keep_state", ctypes.c_int), ("gated", ctypes.c_int), ("d_tile", ctypes.c_int)]


class PaKernelTime(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char * 48), ("launches", ctypes.c_int), ("ms_total", ctypes.c_float)]


_lib = None


def library_path() -> str:
    return os.path.join(_HERE, _LIB_NAME)


def load_library():
    """Load the HIP library built in-tree; a missing library is an error (there is no
    fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise PowerAttnError(f"{path} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'`")
    # torch first: it brings a HIP runtime of its own, and the library has to end up on the runtime
    # that owns the tensors' device context.  Loaded the other way round, every launch of the library
    # fails with "no ROCm-capable device is detected".
    import torch  # noqa: F401
    lib = ctypes.CDLL(path)
    P = ctypes.POINTER(PaProblem)
    vp = ctypes.c_void_p
    lib.power_attn_workspace_bytes.restype = ctypes.c_size_t
    lib.power_attn_workspace_bytes.argtypes = [P, ctypes.c_int]
    lib.power_attn_supported.restype = ctypes.c_int
    lib.power_attn_supported.argtypes = [P, ctypes.c_int]
    lib.power_attn_resolved_chunk.restype = ctypes.c_int
    lib.power_attn_resolved_chunk.argtypes = [P]
    lib.power_attn_state_rows.restype = ctypes.c_longlong
    lib.power_attn_state_rows.argtypes = [P]
    lib.power_attn_decode_state_bytes.restype = ctypes.c_size_t
    lib.power_attn_decode_state_bytes.argtypes = [P]
    lib.power_attn_decode_init.restype = ctypes.c_int
    lib.power_attn_decode_init.argtypes = [P, vp, ctypes.c_size_t, vp]
    lib.power_attn_decode_absorb.restype = ctypes.c_int
    lib.power_attn_decode_absorb.argtypes = [P, vp, vp, vp, vp, ctypes.c_size_t, vp, ctypes.c_size_t, vp]
    lib.power_attn_decode_absorb_workspace_bytes.restype = ctypes.c_size_t
    lib.power_attn_decode_absorb_workspace_bytes.argtypes = [P]
    lib.power_attn_decode_step.restype = ctypes.c_int
    lib.power_attn_decode_step.argtypes = [P, vp, vp, vp, vp, vp, ctypes.c_size_t, vp, vp, vp]
    lib.power_attn_fwd.restype = ctypes.c_int
    lib.power_attn_fwd.argtypes = [P, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.power_attn_fwd_static.restype = ctypes.c_int
    lib.power_attn_fwd_static.argtypes = [P, vp, vp, vp, vp, vp, vp]
    lib.power_attn_static_scratch_bytes.restype = ctypes.c_size_t
    lib.power_attn_static_scratch_bytes.argtypes = []
    lib.power_attn_bwd.restype = ctypes.c_int
    lib.power_attn_bwd.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.power_attn_fwd_gated.restype = ctypes.c_int
    lib.power_attn_fwd_gated.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.power_attn_bwd_gated.restype = ctypes.c_int
    lib.power_attn_bwd_gated.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.power_attn_status_string.restype = ctypes.c_char_p
    lib.power_attn_status_string.argtypes = [ctypes.c_int]
    lib.power_attn_last_hip_error.restype = ctypes.c_char_p
    lib.power_attn_last_hip_error.argtypes = []
    lib.power_attn_release_thread.restype = None
    lib.power_attn_release_thread.argtypes = []
    lib.power_attn_profile_begin.restype = ctypes.c_int
    lib.power_attn_profile_begin.argtypes = []
    lib.power_attn_profile_end.restype = ctypes.c_int
    lib.power_attn_profile_end.argtypes = [ctypes.POINTER(PaKernelTime), ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
    _lib = lib
    return lib


def _check(lib, status: int, what: str):
    if status != 0:
        detail = lib.power_attn_last_hip_error().decode() if status == 4 else ""
        raise PowerAttnError(f"{what}: {lib.power_attn_status_string(status).decode()} (status {status}) {detail}")


def make_problem(B, H, T, d, v, p, chunk, normalize=True, scale=1.0, dtype="bf16", impl="auto",
                 keep_state=False, gated=False, d_tile=0) -> PaProblem:
    return PaProblem(B, H, T, d, v, p, chunk, int(bool(normalize)), float(scale),
                     PA_DTYPE_BF16 if dtype == "bf16" else PA_DTYPE_F32, _IMPL[impl], int(bool(keep_state)),
                     int(bool(gated)), int(d_tile))


def _problem_of(Q, V, p, chunk, normalize, scale, impl, keep_state=False, gated=False, d_tile=0) -> PaProblem:
    import torch
    if Q.dim() != 4 or V.dim() != 4:
        raise PowerAttnError("tensors must be [B, H, T, d]")
    if Q.dtype == torch.bfloat16:
        dtype = "bf16"
    elif Q.dtype == torch.float32:
        dtype = "f32"
    else:
        raise PowerAttnError(f"unsupported dtype {Q.dtype}")
    B, H, T, d = Q.shape
    return make_problem(B, H, T, d, V.shape[3], p, chunk, normalize, scale, dtype, impl, keep_state, gated, d_tile)


def _dev_ptr(t, like=None, name="tensor"):
    if not t.is_cuda:
        raise PowerAttnError(f"{name} must be on the GPU")
    if not t.is_contiguous():
        raise PowerAttnError(f"{name} must be contiguous")
    if like is not None and (t.dtype != like.dtype or t.device != like.device):
        raise PowerAttnError(f"{name} must match the dtype and device of Q")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def power_attn_workspace_bytes(prob: PaProblem, for_backward: bool) -> int:
    return int(load_library().power_attn_workspace_bytes(ctypes.byref(prob), int(for_backward)))


def power_attn_supported(prob: PaProblem, for_backward: bool) -> bool:
    return int(load_library().power_attn_supported(ctypes.byref(prob), int(for_backward))) == 0


def power_attn_resolved_chunk(prob: PaProblem) -> int:
    return int(load_library().power_attn_resolved_chunk(ctypes.byref(prob)))


def power_attn_state_rows(prob: PaProblem) -> int:
    return int(load_library().power_attn_state_rows(ctypes.byref(prob)))


def _workspace(lib, prob, for_backward, workspace, device):
    import torch
    need = int(lib.power_attn_workspace_bytes(ctypes.byref(prob), int(for_backward)))
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=device)
    if workspace.numel() * workspace.element_size() < need:
        raise PowerAttnError(f"workspace holds {workspace.numel() * workspace.element_size()} bytes, {need} needed")
    return workspace, need


def _gate_ptr(log_g, Q, name):
    import torch
    if not log_g.is_cuda or not log_g.is_contiguous() or log_g.dtype != torch.float32 or tuple(log_g.shape) != tuple(Q.shape[:3]):
        raise PowerAttnError(f"{name} must be a contiguous float32 [B, H, T] tensor on the GPU")
    return ctypes.c_void_p(log_g.data_ptr())


def power_attn_fwd(Q, K, V, p: int, chunk: int, normalize: bool = True, scale: float = 1.0, impl: str = "auto",
                   workspace=None, out=None, out_z=None, keep_state: bool = False, log_g=None, d_tile: int = 0):
    """Forward pass on the current stream.  Returns (O, Z): O like V, Z float32 [B, H, T].
    keep_state=True needs a caller-provided workspace that is then handed, untouched, to
    power_attn_bwd(..., keep_state=True).  log_g (float32 [B, H, T], <= 0) switches gating on."""
    import torch
    lib = load_library()
    for t, name in ((Q, "Q"), (K, "K"), (V, "V")):
        _dev_ptr(t, None, name)
    prob = _problem_of(Q, V, p, chunk, normalize, scale, impl, keep_state, log_g is not None, d_tile)
    if keep_state and workspace is None:
        raise PowerAttnError("keep_state=True needs a workspace that outlives the call")
    _check(lib, lib.power_attn_supported(ctypes.byref(prob), 0), "power_attn_fwd")
    with torch.cuda.device(Q.device):
        O = torch.empty_like(V) if out is None else out
        Z = torch.empty(Q.shape[:3], dtype=torch.float32, device=Q.device) if out_z is None else out_z
        workspace, need = _workspace(lib, prob, False, workspace, Q.device)
        if log_g is None:
            st = lib.power_attn_fwd(ctypes.byref(prob), _dev_ptr(Q, name="Q"), _dev_ptr(K, Q, "K"), _dev_ptr(V, Q, "V"),
                                    _dev_ptr(O, Q, "O"), ctypes.c_void_p(Z.data_ptr()),
                                    ctypes.c_void_p(workspace.data_ptr()), need, _stream())
        else:
            st = lib.power_attn_fwd_gated(ctypes.byref(prob), _dev_ptr(Q, name="Q"), _dev_ptr(K, Q, "K"),
                                          _dev_ptr(V, Q, "V"), _gate_ptr(log_g, Q, "log_g"), _dev_ptr(O, Q, "O"),
                                          ctypes.c_void_p(Z.data_ptr()), ctypes.c_void_p(workspace.data_ptr()), need,
                                          _stream())
    _check(lib, st, "power_attn_fwd")
    return O, Z


def power_attn_fwd_static(Q, K, V, O, Z, p: int, chunk: int, normalize: bool = True, scale: float = 1.0, impl: str = "auto"):
    """power_attn_fwd on the library's own static scratch: the caller passes the outputs O (like V) and
    Z (float32 [B, H, T]) too, and neither this wrapper nor the call allocates anything."""
    lib = load_library()
    prob = _problem_of(Q, V, p, chunk, normalize, scale, impl)
    st = lib.power_attn_fwd_static(ctypes.byref(prob), _dev_ptr(Q, name="Q"), _dev_ptr(K, Q, "K"), _dev_ptr(V, Q, "V"),
                                   _dev_ptr(O, Q, "O"), ctypes.c_void_p(Z.data_ptr()), _stream())
    _check(lib, st, "power_attn_fwd_static")
    return O, Z


def power_attn_bwd(Q, K, V, O, Z, dO, p: int, chunk: int, normalize: bool = True, scale: float = 1.0,
                   impl: str = "auto", workspace=None, out=None, keep_state: bool = False, log_g=None, d_tile: int = 0):
    """Backward pass on the current stream.  Returns (dQ, dK, dV), or (dQ, dK, dV, dlog_g) when
    log_g is given."""
    import torch
    lib = load_library()
    for t, name in ((Q, "Q"), (K, "K"), (V, "V"), (dO, "dO")):
        _dev_ptr(t, None, name)
    prob = _problem_of(Q, V, p, chunk, normalize, scale, impl, keep_state, log_g is not None, d_tile)
    if keep_state and workspace is None:
        raise PowerAttnError("keep_state=True needs the workspace the forward pass used")
    _check(lib, lib.power_attn_supported(ctypes.byref(prob), 1), "power_attn_bwd")
    with torch.cuda.device(Q.device):
        if out is None:
            dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
        else:
            dQ, dK, dV = out
        workspace, need = _workspace(lib, prob, True, workspace, Q.device)
        o_ptr = _dev_ptr(O, Q, "O") if O is not None else ctypes.c_void_p(0)
        z_ptr = ctypes.c_void_p(Z.data_ptr()) if Z is not None else ctypes.c_void_p(0)
        if log_g is None:
            st = lib.power_attn_bwd(ctypes.byref(prob), _dev_ptr(Q, name="Q"), _dev_ptr(K, Q, "K"), _dev_ptr(V, Q, "V"),
                                    o_ptr, z_ptr, _dev_ptr(dO, Q, "dO"), _dev_ptr(dQ, Q, "dQ"), _dev_ptr(dK, Q, "dK"),
                                    _dev_ptr(dV, Q, "dV"), ctypes.c_void_p(workspace.data_ptr()), need, _stream())
        else:
            dlog_g = torch.empty(Q.shape[:3], dtype=torch.float32, device=Q.device)
            st = lib.power_attn_bwd_gated(ctypes.byref(prob), _dev_ptr(Q, name="Q"), _dev_ptr(K, Q, "K"),
                                          _dev_ptr(V, Q, "V"), _gate_ptr(log_g, Q, "log_g"), o_ptr, z_ptr,
                                          _dev_ptr(dO, Q, "dO"), _dev_ptr(dQ, Q, "dQ"), _dev_ptr(dK, Q, "dK"),
                                          _dev_ptr(dV, Q, "dV"), ctypes.c_void_p(dlog_g.data_ptr()),
                                          ctypes.c_void_p(workspace.data_ptr()), need, _stream())
    _check(lib, st, "power_attn_bwd")
    if log_g is not None:
        return dQ, dK, dV, dlog_g
    return dQ, dK, dV


def profile_begin():
    lib = load_library()
    _check(lib, lib.power_attn_profile_begin(), "power_attn_profile_begin")


def profile_end(max_entries: int = 64):
    """-> {kernel name: (launches, total ms)} for the kernels launched since profile_begin()."""
    lib = load_library()
    arr = (PaKernelTime * max_entries)()
    n = ctypes.c_int(0)
    _check(lib, lib.power_attn_profile_end(arr, max_entries, ctypes.byref(n)), "power_attn_profile_end")
    return {arr[i].name.decode(): (int(arr[i].launches), float(arr[i].ms_total)) for i in range(n.value)}


def power_attn_decode_state_bytes(prob: PaProblem) -> int:
    return int(load_library().power_attn_decode_state_bytes(ctypes.byref(prob)))


def power_attn_decode_init(prob: PaProblem, state=None):
    """-> the initialised (empty) state of a decode session: a uint8 tensor on the current device
    (allocated here unless one of sufficient size is passed in)."""
    import torch
    lib = load_library()
    need = int(lib.power_attn_decode_state_bytes(ctypes.byref(prob)))
    if need == 0:
        raise PowerAttnError("power_attn_decode_init: invalid or unsupported problem")
    if state is None:
        state = torch.empty(need, dtype=torch.uint8, device=torch.device("cuda", torch.cuda.current_device()))
    _check(lib, lib.power_attn_decode_init(ctypes.byref(prob), _dev_ptr(state, name="state"), state.numel(), _stream()),
           "power_attn_decode_init")
    return state


def power_attn_decode_absorb_workspace_bytes(prob: PaProblem) -> int:
    return int(load_library().power_attn_decode_absorb_workspace_bytes(ctypes.byref(prob)))


def power_attn_decode_absorb(prob: PaProblem, K, V, state, log_g=None, fast: bool = True):
    """Feeds the prompt K [B, H, T, d], V [B, H, T, v] (prob.T = T) into the state, as T decode steps
    would, without outputs.  fast: give the library the workspace its matrix-core path asks for, where
    it has one (sums rounded to bf16 once); else the float32 kernel runs."""
    import torch
    lib = load_library()
    lg = None if log_g is None else _dev_ptr(log_g, name="log_g")
    need = int(lib.power_attn_decode_absorb_workspace_bytes(ctypes.byref(prob))) if fast else 0
    ws = torch.empty(need, dtype=torch.uint8, device=K.device) if need > 0 else None
    _check(lib, lib.power_attn_decode_absorb(ctypes.byref(prob), _dev_ptr(K, name="K"), _dev_ptr(V, K, "V"), lg,
                                             _dev_ptr(state, name="state"), state.numel(),
                                             None if ws is None else _dev_ptr(ws, name="workspace"), need, _stream()),
           "power_attn_decode_absorb")
    return state


def power_attn_decode_step(prob: PaProblem, q, k, v, state, log_g=None, out=None, out_z=None):
    """One token for every (batch, head): q, k [B, H, d], v [B, H, v] -> (o [B, H, v], z [B, H]); the
    state is updated in place."""
    import torch
    lib = load_library()
    o = out if out is not None else torch.empty_like(v)
    z = out_z if out_z is not None else torch.empty(v.shape[:2], dtype=torch.float32, device=v.device)
    lg = None if log_g is None else _dev_ptr(log_g, name="log_g")
    _check(lib, lib.power_attn_decode_step(ctypes.byref(prob), _dev_ptr(q, name="q"), _dev_ptr(k, q, "k"), _dev_ptr(v, q, "v"), lg,
                                           _dev_ptr(state, name="state"), state.numel(), _dev_ptr(o, q, "o"),
                                           _dev_ptr(z, name="z"), _stream()), "power_attn_decode_step")
    return o, z
