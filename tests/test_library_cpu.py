"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every symbol the header declares, reproduces the hand-written chunk tables
bit-exactly and turns bad arguments into error codes before any GPU work."""
import ctypes
import os
import re

import pytest
import torch

from oracle import cref
from paper_2601_04342_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "rehyat.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rehyat_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = binding.library()
    names = declared_functions()
    assert len(names) >= 10
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names
    assert binding.version() >= 100
    assert binding.status_string(0) == "ok"
    for code in (-1, -2, -3, -4, -5):
        assert binding.status_string(code) not in ("ok", "unknown status code")


def test_chunk_plan_bit_exact_against_hand_tables(plan_cases):
    for (T, HW, chunk, overlap), rows in plan_cases:
        got = binding.chunk_plan(T, HW, chunk, overlap)
        assert got.dtype == torch.int64
        assert got.tolist() == rows, (T, HW, chunk, overlap)


@pytest.mark.parametrize("T,HW,chunk,overlap", [(21, 1560, 1, 0), (21, 1560, 2, 0),
                                                (21, 1560, 3, 0), (21, 1560, 3, 1),
                                                (41, 1560, 1, 0), (21, 3600, 1, 0),
                                                (161, 600, 7, 3), (1, 1, 1, 0)])
def test_chunk_plan_equals_oracle_plan(T, HW, chunk, overlap):
    got = binding.chunk_plan(T, HW, chunk, overlap).numpy()
    want = cref.chunk_plan(T, HW, chunk, overlap)
    assert (got == want).all()


def test_chunk_plan_errors():
    lib = binding.library()
    n = ctypes.c_int(0)
    assert lib.rehyat_chunk_plan(4, 4, 1, 0, None, None) == binding.E_NULL
    for bad in ((0, 4, 1, 0), (4, 0, 1, 0), (4, 4, 0, 0), (4, 4, 1, -1)):
        assert lib.rehyat_chunk_plan(*bad, None, ctypes.byref(n)) == binding.E_SHAPE


def test_workspace_size_is_independent_of_video_length():
    # the signature has no T, HW or chunk: constant memory in video duration
    # (section 3.3, point 3); it scales with B*H only
    a = binding.workspace_bytes(1, 12, 128)
    assert a > 0 and a % 256 == 0
    assert binding.workspace_bytes(2, 12, 128) == pytest.approx(2 * a, rel=1e-3)
    assert binding.workspace_bytes(1, 12, 64) < a
    assert binding.workspace_bytes(1, 12, 96) == 0
    assert binding.workspace_bytes(0, 12, 128) == 0
    assert binding.workspace_bytes(1, 12, 128, dprime=128) == 0


A = 0x1000   # a non-null, 16-byte aligned fake device pointer (never dereferenced)


def _phi(hidden=128, dprime=128, degree=2, act=0, fill=A):
    p = binding.PhiParams()
    for n in ("w1_q", "b1_q", "w2_q", "b2_q", "w1_k", "b1_k", "w2_k", "b2_k"):
        setattr(p, n, fill)
    p.hidden, p.dprime, p.degree, p.act = hidden, dprime, degree, act
    return p


def test_forward_argument_validation_without_gpu():
    """Every rejected call returns before touching the device (the fake
    non-null pointers below are never dereferenced)."""
    lib = binding.library()
    ok = _phi()
    fwd = lambda *a: lib.rehyat_forward(*a)
    P = ctypes.byref
    assert fwd(None, A, A, P(ok), A, 1, 2, 4, 8, 64, 1, None) == binding.E_NULL
    assert fwd(A, A, A, P(ok), None, 1, 2, 4, 8, 64, 1, None) == binding.E_NULL
    assert fwd(A, A, A, None, A, 1, 2, 4, 8, 64, 1, None) == binding.E_NULL
    assert fwd(A, A, A, P(_phi(fill=None)), A, 1, 2, 4, 8, 64, 1, None) == binding.E_NULL
    for bad in ((0, 2, 4, 8, 64, 1), (1, 0, 4, 8, 64, 1), (1, 2, 0, 8, 64, 1),
                (1, 2, 4, 0, 64, 1), (1, 2, 4, 8, 64, 0), (1, 2, 4, 8, 0, 1),
                (1, 2, 70000, 70000, 64, 1)):
        assert fwd(A, A, A, P(ok), A, *bad, None) == binding.E_SHAPE, bad
    # one softmax window of 2^31 bytes or more per head; more workgroups than an int counts
    assert fwd(A, A, A, P(ok), A, 1, 2, 64, 1 << 18, 128, 64, None) == binding.E_SHAPE
    assert fwd(A, A, A, P(ok), A, 60000, 1, 4, 1 << 22, 128, 1, None) == binding.E_SHAPE
    assert fwd(A, A, A, P(ok), A, 1, 2, 4, 8, 32, 1, None) == binding.E_UNSUPPORTED
    assert fwd(A, A, A, P(_phi(hidden=64)), A, 1, 2, 4, 8, 64, 1, None) == binding.E_UNSUPPORTED
    assert fwd(A, A, A, P(_phi(degree=4)), A, 1, 2, 4, 8, 64, 1, None) == binding.E_UNSUPPORTED
    assert fwd(A, A, A, P(_phi(degree=3)), A, 1, 2, 4, 8, 64, 1, None) == binding.E_SHAPE
    assert fwd(A, A, A, P(_phi(act=1)), A, 1, 2, 4, 8, 64, 1, None) == binding.E_UNSUPPORTED
    ex = lambda *a: lib.rehyat_forward_ex(*a)
    base = (A, A, A, P(ok), A, 1, 2, 4, 8, 64, 1)
    assert ex(*base, -1, 1, 0, None, None) == binding.E_SHAPE       # negative overlap
    assert ex(*base, 0, 2, 0, None, None) == binding.E_SHAPE
    assert ex(*base, 0, 1, 7, None, None) == binding.E_SHAPE        # unknown stabiliser
    st = lambda *a: lib.rehyat_state(*a)
    assert st(None, A, P(ok), A, A, 1, 2, 4, 8, 64, 2, None) == binding.E_NULL
    assert st(A, A, P(ok), A, A, 1, 2, 4, 8, 64, 5, None) == binding.E_SHAPE
    assert st(A, A, P(ok), A, A, 1, 2, 4, 8, 64, -1, None) == binding.E_SHAPE
    # rehyat_step(q_t, k_win, v_win, phi, S, z, out_t, B, H, d, n_q, n_win, n_absorb, stab, stream)
    sp = lambda *a: lib.rehyat_step(*a)
    assert sp(A, A, A, P(ok), A, None, A, 1, 2, 64, 8, 16, 8, 0, None) == binding.E_NULL
    assert sp(A, None, A, P(ok), A, A, A, 1, 2, 64, 8, 16, 8, 0, None) == binding.E_NULL
    assert sp(A, A, A, None, A, A, A, 1, 2, 64, 8, 16, 8, 0, None) == binding.E_NULL
    assert sp(A, A, A, P(ok), A, A, A, 1, 2, 64, 8, 16, 17, 0, None) == binding.E_SHAPE   # absorbs more than the window
    assert sp(A, A, A, P(ok), A, A, A, 1, 2, 64, 8, 16, -1, 0, None) == binding.E_SHAPE
    assert sp(A, A, A, P(ok), A, A, A, 1, 2, 64, 0, 16, 8, 0, None) == binding.E_SHAPE
    assert sp(A, A, A, P(ok), A, A, A, 1, 2, 64, 8, 0, 0, 0, None) == binding.E_SHAPE
    assert sp(A, A, A, P(ok), A, A, A, 1, 2, 64, 8, 16, 8, 3, None) == binding.E_SHAPE    # unknown stabiliser
    assert sp(A, A, A, P(ok), A, A, A, 1, 2, 96, 8, 16, 8, 0, None) == binding.E_UNSUPPORTED


def test_set_workspace_rejects_misaligned_pointer():
    lib = binding.library()
    assert lib.rehyat_set_workspace(0x1001, 1 << 20) == binding.E_WORKSPACE
    assert lib.rehyat_set_workspace(0x1000, 0) == binding.E_WORKSPACE
    assert lib.rehyat_set_workspace(None, 0) == binding.OK
    assert lib.rehyat_profile_read(None, None) == binding.E_NULL


def test_binding_rejects_wrong_tensor_types():
    q = torch.zeros(1, 2, 8, 64)
    with pytest.raises(TypeError):
        binding.forward(q, q, q, {}, 2, 4, 1)


def test_chunk_longer_than_the_video_is_one_chunk():
    """chunk >= T is one chunk, also at the largest int (no overflow in the chunk count)."""
    big = 2**31 - 1
    for chunk, overlap in ((big, 0), (big, big), (22, 5), (21, 0)):
        got = binding.chunk_plan(21, 1560, chunk, overlap)
        assert got.tolist() == [[0, 32760, 0, 32760, 0]], (chunk, overlap)
    # overlap beyond the video clips to the first frame
    assert binding.chunk_plan(4, 10, 1, big).tolist() == [[0, 10, 0, 10, 0], [10, 20, 0, 20, 0],
                                                          [20, 30, 0, 30, 0], [30, 40, 0, 40, 0]]


def test_misaligned_tensor_pointers_are_rejected():
    lib = binding.library()
    ok = _phi()
    P = ctypes.byref
    for bad in ((A + 2, A, A, A), (A, A + 8, A, A), (A, A, A + 4, A), (A, A, A, A + 2)):
        q, k, v, out = bad
        assert lib.rehyat_forward(q, k, v, P(ok), out, 1, 2, 4, 8, 64, 1, None) == binding.E_SHAPE
    w = _phi()
    w.w2_k = A + 8
    assert lib.rehyat_forward(A, A, A, P(w), A, 1, 2, 4, 8, 64, 1, None) == binding.E_SHAPE
    b = _phi()
    b.b1_q = A + 2
    assert lib.rehyat_forward(A, A, A, P(b), A, 1, 2, 4, 8, 64, 1, None) == binding.E_SHAPE


def test_per_call_workspace_validation():
    lib = binding.library()
    ok = _phi()
    P = ctypes.byref
    need = binding.workspace_bytes(1, 2, 64)
    args = (A, A, A, P(ok), A, 1, 2, 4, 8, 64, 1, 0, 1, 0)
    assert lib.rehyat_forward_ws(*args, None, need, None) == binding.E_NULL
    assert lib.rehyat_forward_ws(*args, A + 16, need, None) == binding.E_WORKSPACE     # misaligned
    assert lib.rehyat_forward_ws(*args, A, need - 1, None) == binding.E_WORKSPACE      # too small
    assert lib.rehyat_forward_ws(None, A, A, P(ok), A, 1, 2, 4, 8, 64, 1, 0, 1, 0, A, need,
                                 None) == binding.E_NULL


def test_caller_owned_workspace_is_never_replaced():
    """A caller-set workspace that is too small makes the call fail; the library does
    not allocate one of its own behind the caller's back."""
    lib = binding.library()
    ok = _phi()
    try:
        assert lib.rehyat_set_workspace(A, 4096) == binding.OK
        rc = lib.rehyat_forward(A, A, A, ctypes.byref(ok), A, 1, 2, 4, 8, 64, 1, None)
        assert rc == binding.E_WORKSPACE
        rc = lib.rehyat_state(A, A, ctypes.byref(ok), A, A, 1, 2, 4, 8, 64, 2, None)
        assert rc == binding.E_WORKSPACE
    finally:
        assert lib.rehyat_set_workspace(None, 0) == binding.OK


def test_noalloc_entry_point_limits():
    lib = binding.library()
    big = _phi(hidden=256, dprime=256)
    P = ctypes.byref
    # more (batch, head) pairs than the fixed scratch array can hold one chunk state for
    assert lib.rehyat_forward_noalloc(A, A, A, P(big), A, 17, 12, 4, 8, 128, 1, None) == binding.E_WORKSPACE
    assert lib.rehyat_forward_noalloc(None, A, A, P(big), A, 1, 12, 4, 8, 128, 1, None) == binding.E_NULL
    assert lib.rehyat_forward_noalloc(A, A, A, P(big), A, 1, 12, 4, 8, 128, 0, None) == binding.E_SHAPE


def test_phi_backward_validation_and_workspace_size():
    """rehyat_phi_backward rejects bad arguments before any GPU work; its workspace grows
    with the token count (activations are kept token by token) and is 0 for rejected sizes."""
    lib = binding.library()
    ok = _phi()
    P = ctypes.byref
    g = binding.PhiGrads(*([A] * 8))
    wsb = lambda *a: lib.rehyat_phi_backward_workspace_bytes(*a)
    need = wsb(1, 2, 4, 8, 64, 1)
    assert need > 0 and need % 256 == 0
    assert wsb(1, 2, 8, 8, 64, 1) > need                 # more tokens, more workspace
    assert wsb(1, 2, 4, 8, 64, 9) == wsb(1, 2, 4, 8, 64, 4)   # chunk clamps to T
    assert wsb(1, 2, 4, 8, 96, 1) == 0 and wsb(0, 2, 4, 8, 64, 1) == 0
    assert wsb(1, 2, 2000, 1, 64, 1) == 0                # more chunks than the entry point takes
    bw = lambda *a: lib.rehyat_phi_backward(*a)
    #   q, k, v, phi, grad_out, out, saved, grads, B, H, T, HW, d, chunk, overlap, ws, ws_bytes, stream
    base = (1, 2, 4, 8, 64, 1, 0)
    assert bw(A, A, A, P(ok), None, A, None, P(g), *base, A, need, None) == binding.E_NULL
    assert bw(A, A, A, P(ok), A, A, None, None, *base, A, need, None) == binding.E_NULL
    assert bw(None, A, A, P(ok), A, A, None, P(g), *base, A, need, None) == binding.E_NULL
    assert bw(A, A, A, P(ok), A, A, None, P(g), *base, None, need, None) == binding.E_NULL
    gn = binding.PhiGrads(*([A] * 8))
    gn.b2_k = None
    assert bw(A, A, A, P(ok), A, A, None, P(gn), *base, A, need, None) == binding.E_NULL
    gm = binding.PhiGrads(*([A] * 8))
    gm.w1_q = A + 2
    assert bw(A, A, A, P(ok), A, A, None, P(gm), *base, A, need, None) == binding.E_SHAPE
    assert bw(A, A, A, P(ok), A + 8, A, None, P(g), *base, A, need, None) == binding.E_SHAPE      # grad_out misaligned
    assert bw(A, A, A, P(ok), A, A, None, P(g), *base, A + 16, need, None) == binding.E_WORKSPACE
    assert bw(A, A, A, P(ok), A, A, None, P(g), *base, A, need - 1, None) == binding.E_WORKSPACE
    assert bw(A, A, A, P(ok), A, A, None, P(g), 1, 2, 4, 8, 64, 1, -1, A, need, None) == binding.E_SHAPE
    assert bw(A, A, A, P(ok), A, A, None, P(g), 1, 2, 2000, 1, 64, 1, 0, A, 1 << 40, None) == binding.E_UNSUPPORTED
    assert bw(A, A, A, P(ok), A, A, None, P(g), 1, 2, 4, 8, 32, 1, 0, A, need, None) == binding.E_UNSUPPORTED
    sv = binding.ForwardSaved(A, A)
    assert bw(A, A, A, P(ok), A, None, P(sv), P(g), *base, A, need, None) == binding.E_NULL   # saved needs out
    assert bw(A, A, A, P(ok), A, A, P(binding.ForwardSaved(A, None)), P(g), *base, A, need, None) == binding.E_NULL
    assert bw(A, A, A, P(ok), A, A, P(binding.ForwardSaved(A + 2, A)), P(g), *base, A, need, None) == binding.E_SHAPE
    # N at or beyond 2^31 / (4 d): tile offsets of the token-major buffers would not fit 32 bits
    assert bw(A, A, A, P(ok), A, A, None, P(g), 1, 1, 1 << 12, 1 << 11, 64, 1 << 12, 0, A, 1 << 40, None) == binding.E_SHAPE


def test_xcd_mask_hook_validation():
    """The measurement hook takes any mask with a low bit set and refuses one with none;
    setting it launches nothing."""
    lib = binding.library()
    assert lib.rehyat_debug_set_xcd_mask(0) == binding.E_SHAPE
    assert lib.rehyat_debug_set_xcd_mask(0x100) == binding.E_SHAPE
    assert lib.rehyat_debug_set_xcd_mask(0x01) == binding.OK
    assert lib.rehyat_debug_set_xcd_mask(0xFF) == binding.OK
