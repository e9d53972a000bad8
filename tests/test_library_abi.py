"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header declares,
validates arguments and sizes workspaces without touching a GPU."""
import ctypes
import os
import re

import pytest

from paper_2507_04239_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.library_path()):
        import __graft_entry__ as g
        g.build()
    return binding.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "power_attn.h")).read()
    declared = set(re.findall(r"\b(power_attn_\w+)\s*\(", header))
    assert declared == set(binding.EXPORTED_SYMBOLS)
    for sym in declared:
        assert getattr(lib, sym) is not None


def test_status_strings(lib):
    assert lib.power_attn_status_string(0) == b"ok"
    assert b"workspace" in lib.power_attn_status_string(3)


def test_validation_and_sizes(lib):
    ok = binding.make_problem(1, 1, 256, 16, 16, 2, 32, dtype="f32")
    assert lib.power_attn_supported(ctypes.byref(ok), 1) == 0
    assert binding.power_attn_state_rows(ok) == 136
    assert binding.power_attn_workspace_bytes(ok, True) > binding.power_attn_workspace_bytes(ok, False) > 0
    # a ragged last chunk is a valid request, but only the chunked matrix-core kernels take it
    ragged = binding.make_problem(1, 1, 256, 16, 16, 2, 48)
    assert lib.power_attn_supported(ctypes.byref(ragged), 0) == 2
    assert binding.power_attn_workspace_bytes(ragged, False) == 0
    ragged_mfma = binding.make_problem(1, 2, 300, 64, 64, 2, 128)
    assert lib.power_attn_supported(ctypes.byref(ragged_mfma), 1) == 0
    whole = binding.make_problem(1, 2, 384, 64, 64, 2, 128)
    assert binding.power_attn_workspace_bytes(ragged_mfma, True) > binding.power_attn_workspace_bytes(whole, True) > 0
    odd_p = binding.make_problem(1, 1, 256, 16, 16, 3, 32, normalize=True)
    assert lib.power_attn_supported(ctypes.byref(odd_p), 0) == 1
    odd_p_unnorm = binding.make_problem(1, 1, 256, 16, 16, 3, 32, normalize=False)
    assert lib.power_attn_supported(ctypes.byref(odd_p_unnorm), 1) == 0
    big_p = binding.make_problem(1, 1, 256, 16, 16, 8, 32)
    assert lib.power_attn_supported(ctypes.byref(big_p), 0) == 2
    # null pointers are rejected before anything is launched (no GPU needed to see that)
    assert lib.power_attn_fwd(ctypes.byref(ok), None, None, None, None, None, None, 0, None) == 1
    assert lib.power_attn_fwd(None, None, None, None, None, None, None, 0, None) == 1
    # a real-looking call with no workspace is refused with the workspace status
    fake = ctypes.c_void_p(256)
    assert lib.power_attn_fwd(ctypes.byref(ok), fake, fake, fake, fake, None, None, 0, None) == 3


def test_state_rows_match_the_embedding_dimension(lib):
    import math
    for d, p in [(16, 2), (32, 4), (12, 3)]:
        pr = binding.make_problem(1, 1, 64, d, d, p, 32, normalize=(p % 2 == 0), impl="generic")
        assert binding.power_attn_state_rows(pr) == math.comb(d + p - 1, p)


def test_automatic_chunk_choice():
    """chunk = 0 lets the library choose (host logic only): the attention form (one chunk) for short
    sequences, the chunked form beyond; an explicit chunk is returned unchanged."""
    from paper_2507_04239_amd import binding
    mk = binding.make_problem
    rc = binding.power_attn_resolved_chunk
    assert rc(mk(1, 12, 65536, 64, 64, 2, 128)) == 128
    assert rc(mk(1, 12, 65536, 64, 64, 2, 0)) == 256          # bf16, p = 2, d = 64: measured best chunk
    assert rc(mk(1, 12, 65536 + 128, 64, 64, 2, 0)) == 128    # 256 does not divide T
    assert rc(mk(1, 12, 65536 + 5, 64, 64, 2, 0)) == 256      # ragged: chunked all the same, the sequence is padded
    assert rc(mk(1, 12, 3000, 64, 64, 2, 0)) == 3000          # short and ragged: attention form, any length
    assert rc(mk(4, 12, 4096, 64, 64, 2, 0)) == 4096          # short: attention form
    assert rc(mk(4, 12, 8192, 64, 64, 2, 0)) == 256
    assert rc(mk(4, 12, 4096, 64, 64, 2, 0, gated=True)) == 256
    assert rc(mk(4, 12, 2048, 64, 64, 2, 0, gated=True)) == 2048
    assert rc(mk(4, 12, 512, 64, 64, 2, 0)) == 512
    # d = 128, p = 2: the tiled chunked kernels from about 24k tokens on (not gated: they take no gates)
    assert rc(mk(8, 16, 32768, 128, 128, 2, 0)) == 256
    assert rc(mk(8, 16, 16384, 128, 128, 2, 0)) == 16384
    assert rc(mk(8, 16, 32768, 128, 128, 2, 0, gated=True)) == 32768
    assert rc(mk(8, 16, 32768, 128, 128, 4, 0)) == 32768
    # d = 32, p = 2: the tiled chunked kernels beyond 4096 tokens
    assert rc(mk(4, 8, 8192, 32, 32, 2, 0)) == 256
    assert rc(mk(4, 8, 4096, 32, 32, 2, 0)) == 4096
    assert rc(mk(4, 8, 8192, 32, 32, 2, 0, gated=True)) == 8192     # (they take no gates)
    # p = 3, d = 64: chunked matrix-core kernels exist (tiled), the attention form is the faster one at these lengths
    assert rc(mk(1, 4, 16384, 64, 64, 3, 0, normalize=False)) == 16384
    # p = 4, d = 32: the state is 52360 x 33 per head, the attention form stays cheaper far beyond 16k tokens
    assert rc(mk(2, 8, 16384, 32, 32, 4, 0, dtype="bf16")) == 16384
    # float32, small head: state 136 x 17; chunked from a few hundred tokens on
    assert rc(mk(1, 1, 64, 16, 16, 2, 0, dtype="f32")) == 64
    assert rc(mk(1, 1, 4096, 16, 16, 2, 0, dtype="f32")) == 64   # generic kernels: measured best chunk
    assert rc(mk(1, 1, 96, 16, 16, 2, 0, dtype="f32", impl="generic")) == 96
    assert rc(mk(1, 1, 4000, 16, 16, 2, 0, dtype="f32")) == 32   # largest power of two <= 64 dividing T
    assert binding.power_attn_workspace_bytes(mk(1, 12, 65536, 64, 64, 2, 0), False) == \
        binding.power_attn_workspace_bytes(mk(1, 12, 65536, 64, 64, 2, 256), False)
    assert rc(mk(1, 1, 100, 16, 16, 2, 7)) == 7                  # an explicit chunk is returned as it is ...
    assert not binding.power_attn_supported(mk(1, 1, 100, 16, 16, 2, 7), False)   # ... supported or not
    assert rc(mk(1, 1, 100, 16, 16, 2, -1)) == 0                 # invalid


def test_tiled_kernels_host_logic():
    """Which problems the tiled matrix-core kernels (degree and tile width as parameters) take, the state rows
    of their embedding C(d / d_tile + p - 1, p) d_tile^p (Sec. 4.1.1), and when the automatic choice runs them."""
    import math
    from paper_2507_04239_amd import binding
    mk, ok, rows = binding.make_problem, binding.power_attn_supported, binding.power_attn_state_rows

    def tspow_rows(d, p, dt):
        return math.comb(d // dt + p - 1, p) * dt ** p

    for (p, dt, d) in [(2, 4, 32), (2, 8, 32), (2, 16, 32), (3, 4, 32), (4, 2, 32), (4, 4, 32),
                       (2, 4, 64), (2, 8, 64), (2, 16, 64), (3, 4, 64)]:
        pr = mk(1, 2, 1024, d, d, p, 128, normalize=(p % 2 == 0), impl="tiled", d_tile=dt)
        assert ok(pr, True) and ok(pr, False), (p, dt, d)
        assert rows(pr) == tspow_rows(d, p, dt), (p, dt, d)
    # the default widths: 8, 4, 2 for p = 2, 3, 4
    assert rows(mk(1, 2, 1024, 32, 32, 2, 128, impl="tiled")) == tspow_rows(32, 2, 8)
    assert rows(mk(1, 2, 1024, 32, 32, 3, 128, normalize=False, impl="tiled")) == tspow_rows(32, 3, 4) == 7680
    assert rows(mk(1, 2, 1024, 32, 32, 4, 128, impl="tiled")) == tspow_rows(32, 4, 2) == 62016
    # config 4 as stated with no family named: the tiled kernels, not the vector-ALU family (52360 rows there)
    assert rows(mk(2, 8, 16384, 32, 32, 4, 128)) == 62016
    assert rows(mk(2, 8, 16384, 32, 32, 4, 128, d_tile=4)) == 84480
    assert rows(mk(2, 8, 16384, 32, 32, 4, 128, impl="generic")) == 52360
    # a tile width is a request for these kernels: p = 2, d = 64 otherwise runs the d_tile = 8 family of its own
    assert rows(mk(1, 12, 65536, 64, 64, 2, 128)) == 2304
    assert rows(mk(1, 12, 65536, 64, 64, 2, 128, d_tile=4)) == tspow_rows(64, 2, 4) == 2176
    assert rows(mk(1, 12, 65536, 64, 64, 2, 128, d_tile=16)) == 2560
    # not taken: widths that are not built, one chunk, chunks that are not a multiple of 128, gates, float32, d = 128 beyond p = 2 with width 8
    assert not ok(mk(1, 2, 1024, 32, 32, 4, 128, d_tile=8), True)
    assert not ok(mk(1, 2, 1024, 32, 32, 4, 128, d_tile=3), True)
    assert not ok(mk(1, 2, 1024, 32, 32, 4, 1024, impl="tiled"), True)
    assert not ok(mk(1, 2, 1024, 32, 32, 4, 64, impl="tiled"), True)
    assert not ok(mk(1, 2, 1024, 32, 32, 4, 128, impl="tiled", gated=True), True)
    assert not ok(mk(1, 2, 1024, 32, 32, 4, 128, impl="tiled", dtype="f32"), True)
    assert ok(mk(1, 2, 1024, 128, 128, 2, 128, impl="tiled"), True)
    assert rows(mk(1, 2, 1024, 128, 128, 2, 128, impl="tiled")) == tspow_rows(128, 2, 8) == 8704
    assert not ok(mk(1, 2, 1024, 128, 128, 2, 128, d_tile=4), True)
    assert not ok(mk(1, 2, 1024, 128, 128, 3, 128, impl="tiled", normalize=False), True)
    assert ok(mk(1, 2, 1024, 32, 32, 4, 128, gated=True), True)           # automatic: the vector-ALU family takes it
    assert rows(mk(1, 2, 1024, 32, 32, 4, 128, gated=True)) == 52360
    assert not ok(mk(1, 2, 1024, 32, 32, 4, 128, d_tile=-1), True)        # invalid


def test_support_matrix_host_logic():
    """Which problems the matrix-core kernels take (host logic only, nothing is launched)."""
    from paper_2507_04239_amd import binding
    mk, ok, rows = binding.make_problem, binding.power_attn_supported, binding.power_attn_state_rows
    # chunked form: p = 2, d = 64, chunk a multiple of 128
    assert ok(mk(1, 2, 1024, 64, 64, 2, 128, impl="mfma"), True)
    assert rows(mk(1, 2, 1024, 64, 64, 2, 128, impl="mfma")) == 36 * 64            # tiled embedding, d_tile = 8
    assert not ok(mk(1, 2, 1024, 64, 64, 2, 64, impl="mfma"), True)
    # d = 128 chunked: the tiled kernels (136 tiles of 64 rows); the resident-state kernels when asked for by name
    assert ok(mk(1, 2, 1024, 128, 128, 2, 256, impl="mfma"), True)
    assert rows(mk(1, 2, 1024, 128, 128, 2, 256, impl="mfma")) == 136 * 64
    assert ok(mk(1, 2, 1024, 64, 64, 2, 128, impl="resident"), True)
    assert ok(mk(1, 2, 1024, 128, 128, 2, 256, impl="resident"), True)
    assert not ok(mk(1, 2, 1024, 64, 64, 2, 64, impl="resident"), True)            # chunk a multiple of 128
    assert not ok(mk(1, 2, 1024, 32, 32, 4, 128, impl="resident"), True)           # p = 2 only
    assert not ok(mk(1, 2, 1024, 64, 64, 2, 128, impl="resident", gated=True), True)
    assert ok(mk(1, 2, 1024, 128, 128, 2, 256, impl="auto"), True)                 # ... the generic family runs it
    assert rows(mk(1, 2, 1024, 128, 128, 2, 256)) == 8704                          # auto: the tiled embedding (Sec. 4.1.1)
    assert rows(mk(1, 2, 1024, 128, 128, 2, 256, impl="generic")) == 8256          # C(129, 2), Lemma 4.2
    # attention form: one chunk, degrees 2-4, head sizes 32 / 64 / 128, any length
    for p, d in ((2, 32), (3, 64), (4, 128), (4, 32)):
        assert ok(mk(1, 1, 1000, d, d, p, 1000, normalize=(p % 2 == 0), impl="mfma"), True), (p, d)
        assert rows(mk(1, 1, 1000, d, d, p, 1000, normalize=(p % 2 == 0), impl="mfma")) == 0
    assert not ok(mk(1, 1, 1024, 48, 48, 2, 1024, impl="mfma"), True)
    assert not ok(mk(1, 1, 1024, 64, 32, 2, 1024, impl="mfma"), True)              # d != v
    # with gates the sequence has to be a multiple of the dK / dV kernel's key block
    assert ok(mk(1, 1, 1024, 128, 128, 2, 1024, impl="mfma", gated=True), True)
    assert not ok(mk(1, 1, 1000, 128, 128, 2, 1000, impl="mfma", gated=True), True)
    assert ok(mk(1, 1, 1000, 128, 128, 2, 1000, impl="auto", gated=True), True)    # generic
    assert not ok(mk(1, 1, 128, 32, 32, 4, 128, impl="mfma", gated=True), True)    # d = 32: blocks of 256 keys
    assert ok(mk(1, 1, 256, 32, 32, 4, 256, impl="mfma", gated=True), True)
    # f32 never runs on the MFMA kernels
    assert not ok(mk(1, 1, 256, 64, 64, 2, 128, dtype="f32", impl="mfma"), True)


def test_decode_state_size_host_logic():
    from paper_2507_04239_amd import binding
    import math
    for (B, H, d, p) in ((1, 12, 64, 2), (2, 3, 32, 4), (1, 1, 128, 2)):
        prob = binding.make_problem(B, H, 1, d, d, p, 1)
        D = math.comb(d + p - 1, p)
        need = binding.power_attn_decode_state_bytes(prob)
        assert need >= B * H * D * (d + 1) * 4          # the float32 state itself
        assert need <= B * H * D * (d + 1) * 4 + D * 8 + B * H * ((D + 127) // 128) * (d + 1) * 4 + 5 * 256
    assert binding.power_attn_decode_state_bytes(binding.make_problem(1, 1, 1, 200, 200, 2, 1)) == 0   # head size above 128
    assert binding.power_attn_decode_state_bytes(binding.make_problem(1, 1, 1, 16, 16, 5, 1, normalize=False)) == 0
