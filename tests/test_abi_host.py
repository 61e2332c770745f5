"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every function the
header declares, sizes workspaces, and turns bad arguments into status codes before any launch."""
import ctypes
import os
import re

import pytest

from paper_2404_07904_amd import binding
from paper_2404_07904_amd.binding import hgrn2_shape

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OK, E_NULL, E_SHAPE, E_UNSUP, E_WS, E_HIP = range(6)
FAKE = ctypes.c_void_p(0x10000)          # never dereferenced: every call below fails validation first
FAKE_WS = ctypes.c_void_p(0x100000)      # 256-byte aligned


def declared_functions():
    text = open(os.path.join(ROOT, "include", "hgrn2.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hgr[nu][12]_[a-z0-9_]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    lib = binding.lib()
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS), (names, binding.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings():
    for code in range(6):
        s = binding.status_string(code)
        assert isinstance(s, str) and s
    assert binding.status_string(0) == "ok"
    assert "unknown" in binding.status_string(99)


def shape(B=2, H=3, N=100, dk=64, dv=64, chunk=0, io=1, gate=1, layout=0):
    return hgrn2_shape(B, H, N, dk, dv, chunk, io, gate, layout)


def test_workspace_sizes():
    s = shape(B=8, H=16, N=2048, dk=128, dv=128)
    one = 8 * 16 * 32 * 128 * 128 * 2
    assert binding.hgrn2_fwd_workspace_bytes(s) == one
    # backward: the forward states; the two runs per sequence of the reverse walk need nothing more
    assert binding.hgrn2_bwd_workspace_bytes(s) == one
    assert binding.hgrn2_saved_states_bytes(s) == one
    assert binding.hgrn2_bwd_saved_workspace_bytes(s, False) == 0
    s32 = shape(B=1, H=1, N=256, io=0, gate=0)
    assert binding.hgrn2_fwd_workspace_bytes(s32) == 4 * 64 * 64 * 4
    assert binding.hgrn2_bwd_workspace_bytes(s32) == 4 * 64 * 64 * 4   # fp32 backward: heads of 64 x 64 only
    assert binding.hgrn2_bwd_workspace_bytes(shape(B=1, H=1, N=256, dk=128, dv=128, io=0, gate=0)) == 0
    assert binding.hgrn2_fwd_workspace_bytes(shape(N=65)) == 2 * 3 * 2 * 64 * 64 * 2   # ragged: 2 chunks
    assert binding.hgrn2_fwd_workspace_bytes(shape(N=0)) == 0
    assert binding.hgrn2_fwd_workspace_bytes(shape(dk=96)) == 0
    # few long sequences are walked in runs: per run an fp32 state and a decay vector on top
    long = shape(B=2, H=16, N=16384, dk=128, dv=128)
    one = 32 * 256 * 128 * 128 * 2
    assert binding.hgrn2_fwd_workspace_bytes(long) == one + 32 * 8 * (128 * 128 + 128) * 4      # 8 runs forward
    # backward: forward states in 8 runs; reverse walk in 8 runs of 32 chunks, boundaries from 28 sub-runs of 8 chunks
    assert binding.hgrn2_bwd_workspace_bytes(long) == (one + 32 * 8 * (128 * 128 + 128) * 4
                                                       + 32 * 28 * (128 * 128 + 128) * 4 + 32 * 128 * 128 * 4)


def test_small_gate_mode_workspace_and_support():
    """chunk = 16 / 32, equal lengths: chunks of that many tokens, so the workspace of a sequence of
    64 / chunk times as many tokens and nothing else; packed batches alike."""
    s = shape(B=2, H=3, N=200, dk=64, dv=128, chunk=16)
    inner = shape(B=2, H=3, N=13 * 64, dk=64, dv=128)           # 13 blocks of 16 tokens, a chunk each
    assert binding.hgrn2_fwd_workspace_bytes(s) == binding.hgrn2_fwd_workspace_bytes(inner) == 2 * 3 * 13 * 64 * 128 * 2
    assert binding.hgrn2_bwd_workspace_bytes(s) == binding.hgrn2_bwd_workspace_bytes(inner)
    assert binding.hgrn2_saved_states_bytes(s) == 2 * 3 * 13 * 64 * 128 * 2
    lib = binding.lib()
    sp = ctypes.byref(s)
    big = 1 << 40
    assert binding.hgrn2_bwd_gated_workspace_bytes(s) == binding.hgrn2_bwd_gated_workspace_bytes(inner)
    assert lib.hgrn2_fwd_gated(sp, FAKE, FAKE, None, FAKE, None, FAKE, None, FAKE_WS, big, None) == E_NULL      # beta missing
    # packed batches: the tables and the states of at most 200 // 16 + 2 chunks of 16 tokens per head
    sv = shape(B=2, H=3, N=200, dk=64, dv=128, layout=1, chunk=16)
    tables = binding.hgrn2_fwd_varlen_workspace_bytes(shape(B=2, H=3, N=200, dk=64, dv=128, layout=1)) - 5 * 3 * 64 * 128 * 2
    assert binding.hgrn2_fwd_varlen_workspace_bytes(sv) == tables + 14 * 3 * 64 * 128 * 2
    # not offered for the stage calls
    assert lib.hgrn2_state_sweep(sp, 0, None, FAKE, FAKE, None, None, FAKE_WS, big, None) == E_UNSUP
    assert lib.hgrn2_fwd(sp, FAKE, FAKE, FAKE, None, FAKE, None, FAKE_WS, 1024, None) == E_WS
    assert lib.hgrn2_fwd(sp, None, FAKE, FAKE, None, FAKE, None, FAKE_WS, big, None) == E_NULL
    assert lib.hgrn2_fwd(ctypes.byref(shape(chunk=48)), FAKE, FAKE, FAKE, None, FAKE, None, FAKE_WS, big, None) == E_UNSUP
    # reference rows every 32 tokens: 7 blocks of 32 tokens, a chunk each
    s32 = shape(B=2, H=3, N=200, dk=64, dv=128, chunk=32)
    assert binding.hgrn2_fwd_workspace_bytes(s32) == binding.hgrn2_fwd_workspace_bytes(shape(B=2, H=3, N=7 * 64, dk=64, dv=128))


def test_chunk_length_chosen_on_the_device_sizes_and_support():
    """chunk = HGRN2_CHUNK_AUTO: workspaces and kept states are those of the alternative with most chunks (16
    tokens per chunk) plus 256 bytes for the flags; equal-length entry points only; chunk = 8 likewise."""
    AUTO = -1
    a, s16, s8 = (shape(B=2, H=3, N=200, dk=64, dv=128, chunk=c) for c in (AUTO, 16, 8))
    assert binding.hgrn2_fwd_workspace_bytes(a) == 256 + binding.hgrn2_fwd_workspace_bytes(s16)
    assert binding.hgrn2_bwd_workspace_bytes(a) == 256 + binding.hgrn2_bwd_workspace_bytes(s16)
    assert binding.hgrn2_bwd_gated_workspace_bytes(a) == 256 + binding.hgrn2_bwd_gated_workspace_bytes(s16)
    assert binding.hgrn2_saved_states_bytes(a) == 256 + binding.hgrn2_saved_states_bytes(s16)
    assert binding.hgrn2_bwd_saved_workspace_bytes(a, False) == binding.hgrn2_bwd_saved_workspace_bytes(s16, False)
    assert binding.hgrn2_saved_states_bytes(s8) == 2 * 3 * 25 * 64 * 128 * 2          # 25 chunks of 8 tokens
    lib = binding.lib()
    big = 1 << 40
    ap = ctypes.byref(a)
    assert lib.hgrn2_fwd(ap, FAKE, FAKE, FAKE, None, FAKE, None, FAKE_WS, binding.hgrn2_fwd_workspace_bytes(s16), None) == E_WS
    assert lib.hgrn2_fwd(ap, None, FAKE, FAKE, None, FAKE, None, FAKE_WS, big, None) == E_NULL
    assert lib.hgrn2_bwd(ap, FAKE, FAKE, FAKE, None, FAKE, None, FAKE, None, FAKE, None, FAKE_WS, big, None) == E_NULL
    assert lib.hgrn2_bwd(ap, FAKE, FAKE, FAKE, None, FAKE, None, FAKE, FAKE, FAKE, None, FAKE_WS, 1024, None) == E_WS
    assert lib.hgrn2_fwd_saving(ap, FAKE, FAKE, None, FAKE, None, FAKE, None, FAKE_WS, binding.hgrn2_saved_states_bytes(s16),
                                FAKE_WS, big, None) == E_WS
    bad = shape(B=2, H=3, N=200, dk=96, dv=128, chunk=AUTO)
    assert binding.hgrn2_fwd_workspace_bytes(bad) == 0
    assert lib.hgrn2_fwd(ctypes.byref(bad), FAKE, FAKE, FAKE, None, FAKE, None, FAKE_WS, big, None) == E_UNSUP
    assert lib.hgrn2_fwd(ctypes.byref(shape(chunk=-2)), FAKE, FAKE, FAKE, None, FAKE, None, FAKE_WS, big, None) == E_SHAPE
    # not offered: the stage calls
    assert lib.hgrn2_state_sweep(ap, 0, None, FAKE, FAKE, None, None, FAKE_WS, big, None) == E_SHAPE
    # packed batches: the workspace of the alternative with most chunks plus the flags; every alternative keeps its
    # states and tables in a place of its own
    sv, sv64, sv32, sv16 = (shape(B=2, H=3, N=200, dk=64, dv=128, layout=1, chunk=c) for c in (AUTO, 0, 32, 16))
    assert binding.hgrn2_fwd_varlen_workspace_bytes(sv) == 256 + binding.hgrn2_fwd_varlen_workspace_bytes(sv16)
    assert binding.hgrn2_bwd_varlen_workspace_bytes(sv) == 256 + binding.hgrn2_bwd_varlen_workspace_bytes(sv16)
    assert binding.hgrn2_saved_states_varlen_bytes(sv) == 256 + sum(binding.hgrn2_saved_states_varlen_bytes(x) for x in (sv64, sv32, sv16))
    assert lib.hgrn2_fwd_varlen(ctypes.byref(sv), FAKE, FAKE, FAKE, None, FAKE, None, FAKE, None, FAKE_WS,
                                binding.hgrn2_fwd_varlen_workspace_bytes(sv16), None) == E_WS
    assert lib.hgrn2_fwd_varlen(ctypes.byref(sv), FAKE, None, FAKE, None, FAKE, None, FAKE, None, FAKE_WS, big, None) == E_NULL


def call_fwd(s, q=FAKE, f=FAKE, v=FAKE, h0=None, o=FAKE, hT=None, ws=FAKE_WS, ws_bytes=1 << 40):
    return binding.lib().hgrn2_fwd(ctypes.byref(s) if s is not None else None, q, f, v, h0, o, hT, ws, ws_bytes, None)


def call_bwd(s, q=FAKE, f=FAKE, v=FAKE, go=FAKE, gq=FAKE, gf=FAKE, gv=FAKE, ws=FAKE_WS, ws_bytes=1 << 40):
    return binding.lib().hgrn2_bwd(ctypes.byref(s) if s is not None else None, q, f, v, None, go, None, gq, gf, gv,
                                   None, ws, ws_bytes, None)


def test_fwd_argument_errors():
    assert call_fwd(None) == E_NULL
    assert call_fwd(shape(B=-1)) == E_SHAPE
    assert call_fwd(shape(N=-5)) == E_SHAPE
    assert call_fwd(shape(dk=0)) == E_SHAPE
    assert call_fwd(shape(io=7)) == E_SHAPE
    assert call_fwd(shape(B=1 << 20, H=1 << 20)) == E_SHAPE
    assert call_fwd(shape(dk=96)) == E_UNSUP
    assert call_fwd(shape(dv=256)) == E_UNSUP
    assert call_fwd(shape(chunk=48)) == E_UNSUP
    assert call_fwd(shape(), q=None) == E_NULL
    assert call_fwd(shape(), o=None) == E_NULL
    assert call_fwd(shape(), ws=None) == E_WS
    assert call_fwd(shape(), ws_bytes=1000) == E_WS
    assert call_fwd(shape(), ws=ctypes.c_void_p(0x100010)) == E_WS
    # nothing to do: no sequences at all
    assert call_fwd(shape(B=0), q=None, f=None, v=None, o=None, ws=None, ws_bytes=0) == OK


def test_bwd_argument_errors():
    assert call_bwd(None) == E_NULL
    assert call_bwd(shape(io=0, dk=128)) == E_UNSUP  # fp32 storage in the backward pass: heads of 64 x 64 only
    assert call_bwd(shape(io=0, dv=128)) == E_UNSUP
    assert call_bwd(shape(dk=32)) == E_UNSUP
    assert call_bwd(shape(), go=None) == E_NULL
    assert call_bwd(shape(), gf=None) == E_NULL
    assert call_bwd(shape(), ws_bytes=binding.hgrn2_bwd_workspace_bytes(shape()) - 1) == E_WS
    assert call_bwd(shape(B=0), q=None, f=None, v=None, go=None, gq=None, gf=None, gv=None, ws=None, ws_bytes=0) == OK


def test_step_argument_errors():
    step = binding.lib().hgrn2_step
    assert step(-1, 1, 64, 64, 1, 1, FAKE, FAKE, FAKE, FAKE, FAKE, None) == E_SHAPE
    assert step(1, 1, 64, 64, 3, 1, FAKE, FAKE, FAKE, FAKE, FAKE, None) == E_SHAPE
    assert step(1, 1, 48, 64, 1, 1, FAKE, FAKE, FAKE, FAKE, FAKE, None) == E_UNSUP
    assert step(1, 1, 64, 64, 1, 1, FAKE, FAKE, FAKE, None, FAKE, None) == E_NULL
    assert step(0, 4, 64, 64, 1, 1, None, None, None, None, None, None) == OK
    gated = binding.lib().hgrn2_step_gated
    assert gated(1, 1, 64, 64, 1, 1, FAKE, FAKE, None, FAKE, FAKE, FAKE, None) == E_NULL       # beta missing
    assert gated(1, 1, 48, 64, 1, 1, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None) == E_UNSUP
    assert gated(0, 4, 64, 64, 1, 1, None, None, None, None, None, None, None) == OK


def test_stage_entry_point_errors():
    lib = binding.lib()
    s = shape()
    assert lib.hgrn2_state_sweep(ctypes.byref(s), 5, FAKE, FAKE, FAKE, None, None, FAKE_WS, 1 << 40, None) == E_SHAPE
    assert lib.hgrn2_state_sweep(ctypes.byref(s), 2, None, FAKE, FAKE, None, None, FAKE_WS, 1 << 40, None) == E_NULL
    assert lib.hgrn2_state_sweep(ctypes.byref(s), 0, None, FAKE, FAKE, None, None, FAKE_WS, 10, None) == E_WS
    s32 = shape(io=0, gate=0, dk=128)
    assert lib.hgrn2_state_sweep(ctypes.byref(s32), 1, None, FAKE, FAKE, None, None, FAKE_WS, 1 << 40, None) == E_UNSUP
    s32 = shape(io=0, gate=0)
    assert lib.hgrn2_bwd_chunk_grads(ctypes.byref(s32), FAKE, FAKE, FAKE, FAKE, FAKE_WS, FAKE_WS, FAKE, FAKE, FAKE, None) == E_UNSUP
    assert lib.hgrn2_fwd_readout(ctypes.byref(s), FAKE, FAKE, FAKE, None, FAKE, None) == E_NULL
    assert lib.hgrn2_bwd_chunk_grads(ctypes.byref(s), FAKE, FAKE, FAKE, FAKE, FAKE_WS, ctypes.c_void_p(0x100008),
                                     FAKE, FAKE, FAKE, None) == E_WS


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(RuntimeError):
        binding.lib()


# ------------------------------------------------------------------ gate formed inside the kernels
def test_gated_workspace_and_error_codes():
    lib = binding.lib()
    s = shape(B=8, H=16, N=2048, dk=128, dv=128)
    one = 8 * 16 * 32 * 128 * 128 * 2
    partials = 8 * 16 * 32 * 8 * 128 * 4 + 8 * 16 * 128 * 4     # per-wave rows of every chunk, then 8 slice sums per head
    assert binding.hgrn2_bwd_gated_workspace_bytes(s) == binding.hgrn2_bwd_workspace_bytes(s) + partials
    assert binding.hgrn2_bwd_gated_workspace_bytes(shape(dk=96)) == 0
    big = 1 << 40
    fwd = lambda s_, q=FAKE, z=FAKE, beta=FAKE, v=FAKE, o=FAKE, ws=FAKE_WS, n=big: lib.hgrn2_fwd_gated(
        ctypes.byref(s_) if s_ is not None else None, q, z, beta, v, None, o, None, ws, n, None)
    assert fwd(None) == E_NULL
    assert fwd(shape(), beta=None) == E_NULL
    assert fwd(shape(), z=None) == E_NULL
    assert fwd(shape(dk=96)) == E_UNSUP
    assert fwd(shape(), n=16) == E_WS
    bwd = lambda s_, beta=FAKE, gz=FAKE, gb=FAKE, ws=FAKE_WS, n=big: lib.hgrn2_bwd_gated(
        ctypes.byref(s_), FAKE, FAKE, beta, FAKE, None, FAKE, None, FAKE, gz, gb, FAKE, None, ws, n, None)
    assert bwd(shape(), beta=None) == E_NULL
    assert bwd(shape(), gb=None) == E_NULL
    assert bwd(shape(), gz=None) == E_NULL
    assert bwd(shape(io=0, gate=0, dk=128)) == E_UNSUP
    need = binding.hgrn2_bwd_gated_workspace_bytes(shape())
    assert bwd(shape(), n=need - 1) == E_WS
    assert bwd(shape(), ws=ctypes.c_void_p(0x100010)) == E_WS
    assert lib.hgrn2_min_gate_product(ctypes.byref(shape()), FAKE, None, None, None) == E_NULL
    assert lib.hgrn2_min_gate_product(ctypes.byref(shape()), None, None, FAKE, None) == E_NULL
    assert lib.hgrn2_min_gate_product(ctypes.byref(shape(dk=96)), FAKE, None, FAKE, None) == E_UNSUP
    assert lib.hgrn2_cumax(-1, 4, FAKE, FAKE, None) == E_SHAPE
    assert lib.hgrn2_cumax(3, 4, None, FAKE, None) == E_NULL
    assert lib.hgrn2_cumax(0, 4, None, None, None) == OK


def test_layout_field():
    assert call_fwd(shape(layout=1), ws_bytes=16) == E_WS          # a valid layout gets as far as the workspace check
    assert call_fwd(shape(layout=2)) == E_SHAPE
    assert call_fwd(shape(layout=-1)) == E_SHAPE
    assert binding.hgrn2_fwd_workspace_bytes(shape(layout=1)) == binding.hgrn2_fwd_workspace_bytes(shape())


def test_hgrn1_workspace_and_error_codes():
    lib = binding.lib()
    fwd_d_limit = lambda: lib.hgrn1_fwd(1, 4, (1 << 20) + 128, 1, 1, FAKE, FAKE, FAKE, None, FAKE, None, FAKE_WS, 1 << 40, None)
    # one saved state per 16-token segment (whole 256-token blocks) plus one row of grad_beta shares per sequence
    assert binding.hgrn1_workspace_bytes(8, 2048, 2048) == (8 * 128 * 2048 + 8 * 2048) * 4
    assert binding.hgrn1_workspace_bytes(1, 257, 128) == (2 * 16 * 128 + 128) * 4
    assert binding.hgrn1_workspace_bytes(1, 513, 128) == (3 * 16 * 128 + 128) * 4
    assert fwd_d_limit() == E_SHAPE
    assert binding.hgrn1_workspace_bytes(8, 2048, 100) == 0
    big = 1 << 40
    fwd = lambda B=2, N=100, d=256, io=1, gate=1, f=FAKE, y=FAKE, ws=FAKE_WS, n=big: lib.hgrn1_fwd(
        B, N, d, io, gate, f, FAKE, FAKE, None, y, None, ws, n, None)
    assert fwd(B=-1) == E_SHAPE
    assert fwd(d=100) == E_UNSUP
    assert fwd(io=0) == E_UNSUP
    assert fwd(f=None) == E_NULL
    assert fwd(y=None) == E_NULL
    assert fwd(n=16) == E_WS
    bwd = lambda d=256, gf=FAKE, n=big: lib.hgrn1_bwd(2, 100, d, 1, 1, FAKE, FAKE, FAKE, None, FAKE, None, gf, FAKE,
                                                      FAKE, None, FAKE_WS, n, None)
    assert bwd(d=96) == E_UNSUP
    assert bwd(gf=None) == E_NULL
    assert bwd(n=16) == E_WS
    # the forms that take the pre-activations of Eq. 1 and the lower bounds of Eq. 2
    fwd_act = lambda d=256, beta=FAKE, n=big: lib.hgrn1_fwd_act(2, 100, d, 1, 1, FAKE, FAKE, FAKE, beta, None, FAKE, None,
                                                                FAKE_WS, n, None)
    assert fwd_act(beta=None) == E_NULL
    assert fwd_act(d=100) == E_UNSUP
    assert fwd_act(n=16) == E_WS
    bwd_act = lambda beta=FAKE, gb=FAKE, n=big: lib.hgrn1_bwd_act(2, 100, 256, 1, 1, FAKE, FAKE, FAKE, beta, None, FAKE, None,
                                                                  FAKE, FAKE, FAKE, gb, None, FAKE_WS, n, None)
    assert bwd_act(beta=None) == E_NULL
    assert bwd_act(gb=None) == E_NULL
    assert bwd_act(n=16) == E_WS


def test_varlen_workspace_and_error_codes():
    lib = binding.lib()
    s = shape(B=6, H=3, N=1000, dk=64, dv=64, layout=1)
    table = 256 + 768                                        # 4 * 7 ints, rounded up; 2 ints for each of the 256 // 3 spans of the reverse walk + 2, rounded up
    states = (1000 // 64 + 6) * 3 * 64 * 64 * 2              # worst split of 1000 tokens into 6 sequences
    assert binding.hgrn2_fwd_varlen_workspace_bytes(s) == table + states
    partials = (1000 // 64 + 6) * 3 * 8 * 64 * 4 + 8 * 3 * 64 * 4     # per-wave shares of grad_beta of every chunk slot, then 8 slice sums per head
    assert binding.hgrn2_bwd_varlen_workspace_bytes(s) == table + 2 * states + partials
    assert binding.hgrn2_fwd_varlen_workspace_bytes(shape(B=6, H=3, N=1000, layout=0)) == 0      # packed tokens are token-major
    # two documents in 32768 tokens of 16 heads are cut like 2 x 16384: 8 runs of 32 chunks per document,
    # planned for the mean length; R bounds the runs of any split of the tokens
    lp = shape(B=2, H=16, N=32768, dk=128, dv=128, layout=1)
    r256 = lambda x: (x + 255) // 256 * 256
    st = (32768 // 64 + 2) * 16 * 128 * 128 * 2
    Rf = 2 + (512 + 2) // 32 + 1
    groups = lambda R: 0                                     # a batch cut into runs is not walked in groups ...
    spans = 256                                              # ... but the reverse walk takes 16 spans per head of the runs' chunks (2 ints each + 2)
    assert binding.hgrn2_fwd_varlen_workspace_bytes(lp) == (256 + r256(4 * (Rf + 1) * 4 + 3 * 4) + groups(Rf) + st
                                                            + Rf * 16 * (128 * 128 + 128) * 4)
    Rb = Rf
    assert binding.hgrn2_bwd_varlen_workspace_bytes(lp) == (256 + r256(4 * (Rb + 1) * 4 + 3 * 4) + spans + 2 * st
                                                            + 2 * Rb * 16 * 128 * 128 * 4 + Rb * 16 * 128 * 4
                                                            + (32768 // 64 + 2) * 16 * 8 * 128 * 4 + 8 * 16 * 128 * 4)
    big = 1 << 40
    fwd = lambda s_, cu=FAKE, q=FAKE, o=FAKE, ws=FAKE_WS, n=big: lib.hgrn2_fwd_varlen(
        ctypes.byref(s_) if s_ is not None else None, cu, q, FAKE, None, FAKE, None, o, None, ws, n, None)
    assert fwd(None) == E_NULL
    assert fwd(shape(layout=0)) == E_SHAPE
    assert fwd(shape(layout=1, dk=96)) == E_UNSUP
    assert fwd(s, cu=None) == E_NULL
    assert fwd(s, q=None) == E_NULL
    assert fwd(s, n=table + states - 1) == E_WS
    assert fwd(s, ws=None) == E_WS
    assert fwd(shape(B=0, layout=1), cu=None, q=None, o=None, ws=None, n=0) == OK
    # many short sequences are walked in groups: 16 per head at H = 16, two ints per group and two more
    many = shape(B=40, H=16, N=4096, dk=128, dv=128, layout=1)
    st40 = (4096 // 64 + 40) * 16 * 128 * 128 * 2
    assert binding.hgrn2_fwd_varlen_workspace_bytes(many) == r256(4 * 41 * 4) + r256((2 * 16 + 2) * 4) + st40
    bwd = lambda s_, cu=FAKE, gq=FAKE, ws=FAKE_WS, n=big, beta=None, gb=None: lib.hgrn2_bwd_varlen(
        ctypes.byref(s_), cu, FAKE, FAKE, beta, FAKE, None, FAKE, None, gq, FAKE, gb, FAKE, None, ws, n, None)
    assert bwd(s, beta=FAKE, gb=None) == E_NULL                 # lower bounds given: their gradient must have a place
    assert bwd(shape(layout=1, io=0, gate=0)) == E_UNSUP
    assert bwd(s, cu=None) == E_NULL
    assert bwd(s, gq=None) == E_NULL
    assert bwd(s, n=table + 2 * states + partials - 1) == E_WS
    # the training pair: one slot per chunk for the kept states, then the tables as the backward pass lays
    # them out (it builds none of its own then); checked before the call proper
    assert binding.hgrn2_saved_states_varlen_bytes(s) == states + table
    assert binding.hgrn2_saved_states_varlen_bytes(many) == st40 + r256(4 * 41 * 4) + r256((2 * 16 + 2) * 4)
    assert binding.hgrn2_saved_states_varlen_bytes(shape(B=6, H=3, N=1000, layout=0)) == 0
    fwd_s = lambda s_, cu=FAKE, q=FAKE, sv=FAKE_WS, sn=big, ws=FAKE_WS, n=big: lib.hgrn2_fwd_varlen_saving(
        ctypes.byref(s_), cu, q, FAKE, None, FAKE, None, FAKE, None, sv, sn, ws, n, None)
    bwd_s = lambda s_, cu=FAKE, gq=FAKE, sv=FAKE_WS, sn=big, ws=FAKE_WS, n=big: lib.hgrn2_bwd_varlen_saved(
        ctypes.byref(s_), cu, FAKE, FAKE, None, FAKE, None, sv, sn, FAKE, None, gq, FAKE, None, FAKE, None, ws, n, None)
    for call in (fwd_s, bwd_s):
        assert call(shape(layout=0)) == E_SHAPE
        assert call(shape(layout=1, io=0, gate=0)) == E_UNSUP        # the shapes the backward pass takes
        assert call(shape(B=6, H=3, N=1000, dk=64, dv=64, layout=1, chunk=48)) == E_UNSUP
        assert call(s, sv=None) == E_WS
        assert call(s, sn=states + table - 1) == E_WS
        assert call(s, cu=None) == E_NULL
        assert call(s, ws=None) == E_WS
    assert fwd_s(s, q=None) == E_NULL
    assert bwd_s(s, gq=None) == E_NULL
    assert fwd_s(s, n=table + states - 1) == E_WS
    assert bwd_s(s, n=table + 2 * states + partials - 1) == E_WS


def test_packed_gate_probe_error_codes():
    lib = binding.lib()
    s = shape(B=3, H=2, N=500, layout=1)
    assert binding.lib().hgrn2_min_gate_product_varlen_workspace_bytes(ctypes.byref(s)) == 256
    call = lambda s_, cu=FAKE, f=FAKE, out=FAKE, ws=FAKE_WS, n=1 << 20: lib.hgrn2_min_gate_product_varlen(
        ctypes.byref(s_), cu, f, None, out, ws, n, None)
    assert call(shape(B=3, H=2, N=500, layout=0)) == E_SHAPE            # packed tokens are token-major
    assert call(s, out=None) == E_NULL
    assert call(s, cu=None) == E_NULL
    assert call(s, f=None) == E_NULL
    assert call(s, ws=None) == E_WS
    assert call(s, n=255) == E_WS
    assert call(shape(B=3, H=2, N=500, layout=1, chunk=48)) == E_UNSUP


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asked for more it says so and exits before touching a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header compiles as C99 with warnings as errors, and a C program
    that takes the address of every declared function links against the library."""
    import subprocess
    hdr = os.path.join(ROOT, "include", "hgrn2.h")
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c", hdr])
    src = tmp_path / "use.c"
    names = declared_functions()
    src.write_text('#include "hgrn2.h"\n#include <stdio.h>\nint main(void) {\n    const void* fns[] = {%s};\n'
                   '    printf("%%d\\n", (int)(sizeof fns / sizeof fns[0]));\n    return fns[0] == 0;\n}\n'
                   % ", ".join("(const void*)%s" % n for n in names))
    exe = tmp_path / "use"
    libdir = os.path.dirname(binding.LIB_PATH)
    subprocess.check_call(["gcc", "-std=gnu99", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe),
                           "-L", libdir, "-l:" + os.path.basename(binding.LIB_PATH), "-Wl,-rpath," + libdir,
                           "-Wl,--allow-shlib-undefined"])
    out = subprocess.run([str(exe)], capture_output=True, text=True)
    assert out.returncode == 0 and int(out.stdout) == len(names)
