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


def _phi(hidden=128, dprime=128, degree=2, act=0, fill=1):
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
    assert fwd(None, 1, 1, P(ok), 1, 1, 2, 4, 8, 64, 1, None) == binding.E_NULL
    assert fwd(1, 1, 1, P(ok), None, 1, 2, 4, 8, 64, 1, None) == binding.E_NULL
    assert fwd(1, 1, 1, None, 1, 1, 2, 4, 8, 64, 1, None) == binding.E_NULL
    assert fwd(1, 1, 1, P(_phi(fill=None)), 1, 1, 2, 4, 8, 64, 1, None) == binding.E_NULL
    for bad in ((0, 2, 4, 8, 64, 1), (1, 0, 4, 8, 64, 1), (1, 2, 0, 8, 64, 1),
                (1, 2, 4, 0, 64, 1), (1, 2, 4, 8, 64, 0), (1, 2, 4, 8, 0, 1),
                (1, 2, 70000, 70000, 64, 1)):
        assert fwd(1, 1, 1, P(ok), 1, *bad, None) == binding.E_SHAPE, bad
    # one softmax window of 2^31 bytes or more per head; more workgroups than an int counts
    assert fwd(1, 1, 1, P(ok), 1, 1, 2, 64, 1 << 18, 128, 64, None) == binding.E_SHAPE
    assert fwd(1, 1, 1, P(ok), 1, 60000, 1, 4, 1 << 22, 128, 1, None) == binding.E_SHAPE
    assert fwd(1, 1, 1, P(ok), 1, 1, 2, 4, 8, 32, 1, None) == binding.E_UNSUPPORTED
    assert fwd(1, 1, 1, P(_phi(hidden=64)), 1, 1, 2, 4, 8, 64, 1, None) == binding.E_UNSUPPORTED
    assert fwd(1, 1, 1, P(_phi(degree=4)), 1, 1, 2, 4, 8, 64, 1, None) == binding.E_UNSUPPORTED
    assert fwd(1, 1, 1, P(_phi(degree=3)), 1, 1, 2, 4, 8, 64, 1, None) == binding.E_SHAPE
    assert fwd(1, 1, 1, P(_phi(act=1)), 1, 1, 2, 4, 8, 64, 1, None) == binding.E_UNSUPPORTED
    ex = lambda *a: lib.rehyat_forward_ex(*a)
    base = (1, 1, 1, P(ok), 1, 1, 2, 4, 8, 64, 1)
    assert ex(*base, -1, 1, 0, None, None) == binding.E_SHAPE       # negative overlap
    assert ex(*base, 0, 2, 0, None, None) == binding.E_SHAPE
    assert ex(*base, 0, 1, 7, None, None) == binding.E_SHAPE        # unknown stabiliser
    st = lambda *a: lib.rehyat_state(*a)
    assert st(None, 1, P(ok), 1, 1, 1, 2, 4, 8, 64, 2, None) == binding.E_NULL
    assert st(1, 1, P(ok), 1, 1, 1, 2, 4, 8, 64, 5, None) == binding.E_SHAPE
    assert st(1, 1, P(ok), 1, 1, 1, 2, 4, 8, 64, -1, None) == binding.E_SHAPE
    # rehyat_step(q_t, k_win, v_win, phi, S, z, out_t, B, H, d, n_q, n_win, n_absorb, stab, stream)
    sp = lambda *a: lib.rehyat_step(*a)
    assert sp(1, 1, 1, P(ok), 1, None, 1, 1, 2, 64, 8, 16, 8, 0, None) == binding.E_NULL
    assert sp(1, None, 1, P(ok), 1, 1, 1, 1, 2, 64, 8, 16, 8, 0, None) == binding.E_NULL
    assert sp(1, 1, 1, None, 1, 1, 1, 1, 2, 64, 8, 16, 8, 0, None) == binding.E_NULL
    assert sp(1, 1, 1, P(ok), 1, 1, 1, 1, 2, 64, 8, 16, 17, 0, None) == binding.E_SHAPE   # absorbs more than the window
    assert sp(1, 1, 1, P(ok), 1, 1, 1, 1, 2, 64, 8, 16, -1, 0, None) == binding.E_SHAPE
    assert sp(1, 1, 1, P(ok), 1, 1, 1, 1, 2, 64, 0, 16, 8, 0, None) == binding.E_SHAPE
    assert sp(1, 1, 1, P(ok), 1, 1, 1, 1, 2, 64, 8, 0, 0, 0, None) == binding.E_SHAPE
    assert sp(1, 1, 1, P(ok), 1, 1, 1, 1, 2, 64, 8, 16, 8, 3, None) == binding.E_SHAPE    # unknown stabiliser
    assert sp(1, 1, 1, P(ok), 1, 1, 1, 1, 2, 96, 8, 16, 8, 0, None) == binding.E_UNSUPPORTED


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
