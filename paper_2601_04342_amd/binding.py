"""Thin ctypes binding of the C-ABI library ``librehyat.so``.

Argument marshalling only: every step of the operator runs in the library's HIP
kernels.  torch is used for device memory and streams.  There is no fallback:
if the library is missing or cannot be loaded, importing a symbol from it
raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librehyat.so")

OK = 0
E_NULL, E_SHAPE, E_UNSUPPORTED, E_WORKSPACE, E_HIP = -1, -2, -3, -4, -5
STAB_ROWMAX, STAB_NONE = 0, 1

# every symbol include/rehyat.h declares
EXPORTS = ("rehyat_chunk_plan", "rehyat_workspace_bytes", "rehyat_set_workspace",
           "rehyat_forward", "rehyat_forward_ex", "rehyat_forward_ws", "rehyat_forward_noalloc",
           "rehyat_step", "rehyat_state", "rehyat_shutdown",
           "rehyat_phi_backward", "rehyat_phi_backward_workspace_bytes",
           "rehyat_status_string", "rehyat_version", "rehyat_last_hip_error",
           "rehyat_attn_kernel_name",
           "rehyat_profile_enable", "rehyat_profile_read", "rehyat_debug_set_xcd_mask")


class PhiParams(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("w1_q", "b1_q", "w2_q", "b2_q", "w1_k", "b1_k", "w2_k", "b2_k")] + [
        ("hidden", ctypes.c_int32), ("dprime", ctypes.c_int32),
        ("degree", ctypes.c_int32), ("act", ctypes.c_int32)]


class DebugOut(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("m", "nS", "aS", "nL", "aL")]


class PhiGrads(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("w1_q", "b1_q", "w2_q", "b2_q", "w1_k", "b1_k", "w2_k", "b2_k")]


class ForwardSaved(ctypes.Structure):
    _fields_ = [("nS", ctypes.c_void_p), ("nL", ctypes.c_void_p)]


BACKWARD_MAX_CHUNKS = 1024


class RehyatError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        lib = _load()
        msg = lib.rehyat_status_string(code).decode()
        hip = lib.rehyat_last_hip_error().decode()
        super().__init__(f"{where} failed: {code} ({msg}){' [' + hip + ']' if hip else ''}")


_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2601_04342_amd.build` "
            "(there is no CPU or PyTorch fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, ci = ctypes.c_void_p, ctypes.c_int
    lib.rehyat_chunk_plan.restype = ci
    lib.rehyat_chunk_plan.argtypes = [ci, ci, ci, ci, ctypes.POINTER(ctypes.c_int64),
                                      ctypes.POINTER(ci)]
    lib.rehyat_workspace_bytes.restype = ctypes.c_size_t
    lib.rehyat_workspace_bytes.argtypes = [ci, ci, ci, ci]
    lib.rehyat_set_workspace.restype = ci
    lib.rehyat_set_workspace.argtypes = [vp, ctypes.c_size_t]
    lib.rehyat_forward.restype = ci
    lib.rehyat_forward.argtypes = [vp, vp, vp, ctypes.POINTER(PhiParams), vp,
                                   ci, ci, ci, ci, ci, ci, vp]
    lib.rehyat_forward_ex.restype = ci
    lib.rehyat_forward_ex.argtypes = [vp, vp, vp, ctypes.POINTER(PhiParams), vp,
                                      ci, ci, ci, ci, ci, ci, ci, ci, ci,
                                      ctypes.POINTER(DebugOut), vp]
    lib.rehyat_forward_ws.restype = ci
    lib.rehyat_forward_ws.argtypes = [vp, vp, vp, ctypes.POINTER(PhiParams), vp,
                                      ci, ci, ci, ci, ci, ci, ci, ci, ci,
                                      vp, ctypes.c_size_t, vp]
    lib.rehyat_forward_noalloc.restype = ci
    lib.rehyat_forward_noalloc.argtypes = [vp, vp, vp, ctypes.POINTER(PhiParams), vp,
                                           ci, ci, ci, ci, ci, ci, vp]
    lib.rehyat_step.restype = ci
    lib.rehyat_step.argtypes = [vp, vp, vp, ctypes.POINTER(PhiParams), vp, vp, vp,
                                ci, ci, ci, ci, ci, ci, ci, vp]
    lib.rehyat_state.restype = ci
    lib.rehyat_state.argtypes = [vp, vp, ctypes.POINTER(PhiParams), vp, vp,
                                 ci, ci, ci, ci, ci, ci, vp]
    lib.rehyat_phi_backward_workspace_bytes.restype = ctypes.c_size_t
    lib.rehyat_phi_backward_workspace_bytes.argtypes = [ci, ci, ci, ci, ci, ci]
    lib.rehyat_phi_backward.restype = ci
    lib.rehyat_phi_backward.argtypes = [vp, vp, vp, ctypes.POINTER(PhiParams), vp, vp,
                                        ctypes.POINTER(ForwardSaved), ctypes.POINTER(PhiGrads),
                                        ci, ci, ci, ci, ci, ci, ci, vp, ctypes.c_size_t, vp]
    lib.rehyat_shutdown.restype = ci
    lib.rehyat_shutdown.argtypes = []
    lib.rehyat_status_string.restype = ctypes.c_char_p
    lib.rehyat_status_string.argtypes = [ci]
    lib.rehyat_version.restype = ci
    lib.rehyat_version.argtypes = []
    lib.rehyat_last_hip_error.restype = ctypes.c_char_p
    lib.rehyat_last_hip_error.argtypes = []
    lib.rehyat_attn_kernel_name.restype = ctypes.c_char_p
    lib.rehyat_attn_kernel_name.argtypes = [ci]
    lib.rehyat_profile_enable.restype = ci
    lib.rehyat_profile_enable.argtypes = [ci]
    lib.rehyat_debug_set_xcd_mask.restype = ci
    lib.rehyat_debug_set_xcd_mask.argtypes = [ctypes.c_uint]
    lib.rehyat_profile_read.restype = ci
    lib.rehyat_profile_read.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ci)]
    _lib = lib
    return lib


def library():
    """The loaded ctypes library (raises if it is not built)."""
    return _load()


def version():
    return _load().rehyat_version()


def attn_kernel_name(d):
    return _load().rehyat_attn_kernel_name(d).decode()


def status_string(code):
    return _load().rehyat_status_string(code).decode()


def chunk_plan(T, HW, chunk, overlap=0):
    """[n_chunks, 5] int64 tensor of (q_lo, q_hi, s_lo, s_hi, l_hi) rows."""
    lib = _load()
    n = ctypes.c_int(0)
    rc = lib.rehyat_chunk_plan(T, HW, chunk, overlap, None, ctypes.byref(n))
    if rc != OK:
        raise RehyatError(rc, "rehyat_chunk_plan")
    table = torch.zeros(n.value, 5, dtype=torch.int64)
    rc = lib.rehyat_chunk_plan(T, HW, chunk, overlap,
                               ctypes.cast(table.data_ptr(), ctypes.POINTER(ctypes.c_int64)),
                               ctypes.byref(n))
    if rc != OK:
        raise RehyatError(rc, "rehyat_chunk_plan")
    return table


def workspace_bytes(B, H, d, dprime=None):
    return _load().rehyat_workspace_bytes(B, H, d, 2 * d if dprime is None else dprime)


def set_workspace(tensor):
    """Hand a caller-owned CUDA byte tensor to the library (None to undo)."""
    lib = _load()
    if tensor is None:
        rc = lib.rehyat_set_workspace(None, 0)
    else:
        rc = lib.rehyat_set_workspace(tensor.data_ptr(), tensor.numel() * tensor.element_size())
    if rc != OK:
        raise RehyatError(rc, "rehyat_set_workspace")


def shutdown():
    rc = _load().rehyat_shutdown()
    if rc != OK:
        raise RehyatError(rc, "rehyat_shutdown")


KERNEL_KINDS = ("state", "prefix", "attn")


def profile_enable(on=True):
    rc = _load().rehyat_profile_enable(1 if on else 0)
    if rc != OK:
        raise RehyatError(rc, "rehyat_profile_enable")


def debug_set_xcd_mask(mask):
    """Measurement hook (timing only): attention workgroups on XCDs whose bit is clear exit at once."""
    rc = _load().rehyat_debug_set_xcd_mask(int(mask))
    if rc != OK:
        raise RehyatError(rc, "rehyat_debug_set_xcd_mask")


def profile_read():
    """{kind: (total_ms, launches)} since the last read; waits for the events."""
    ms = (ctypes.c_double * 3)()
    n = (ctypes.c_int * 3)()
    rc = _load().rehyat_profile_read(ms, n)
    if rc != OK:
        raise RehyatError(rc, "rehyat_profile_read")
    return {k: (ms[i], n[i]) for i, k in enumerate(KERNEL_KINDS)}


def phi_to_device(phi, device="cuda"):
    """dict of fp32 CPU tensors -> dict of device tensors in the library's dtypes
    (weights bf16, biases fp32)."""
    out = {}
    for name, t in phi.items():
        dt = torch.bfloat16 if name.startswith("w") else torch.float32
        out[name] = t.to(device=device, dtype=dt).contiguous()
    return out


def _phi_struct(phi, d):
    for name, t in phi.items():
        want = torch.bfloat16 if name.startswith("w") else torch.float32
        if t.dtype != want or not t.is_cuda or not t.is_contiguous():
            raise TypeError(f"phi[{name}] must be a contiguous CUDA {want} tensor")
    H, hidden, dd = phi["w1_q"].shape
    dprime = phi["w2_q"].shape[1]
    if dd != d:
        raise ValueError("phi weights do not match the head dimension")
    for s in ("q", "k"):
        if (phi[f"w1_{s}"].shape != (H, hidden, d) or phi[f"b1_{s}"].shape != (H, hidden)
                or phi[f"w2_{s}"].shape != (H, dprime, hidden)
                or phi[f"b2_{s}"].shape != (H, dprime)):
            raise ValueError("inconsistent phi parameter shapes")
    p = PhiParams()
    for name in ("w1_q", "b1_q", "w2_q", "b2_q", "w1_k", "b1_k", "w2_k", "b2_k"):
        setattr(p, name, phi[name].data_ptr())
    p.hidden, p.dprime, p.degree, p.act = hidden, dprime, 2, 0
    return p, H


def _check_qkv(q, k, v):
    for t in (q, k, v):
        if t.dtype != torch.bfloat16 or not t.is_cuda or not t.is_contiguous() or t.dim() != 4:
            raise TypeError("q, k, v must be contiguous CUDA bf16 tensors [B, H, N, d]")
    if k.shape != q.shape or v.shape != q.shape:
        raise ValueError("q, k, v shapes differ")


def forward(q, k, v, phi, T, HW, chunk, out=None, overlap=0, causal=True,
            stab_mode=STAB_ROWMAX, debug=False, stream=None, plain=False, workspace=None,
            noalloc=False):
    """Hybrid attention forward.  q, k, v: CUDA bf16 [B, H, T*HW, d].

    Returns ``out`` (bf16, same shape), or ``(out, components)`` with
    ``debug=True`` where components is a dict of fp32 tensors m, nS, aS, nL, aL.
    ``plain=True`` calls ``rehyat_forward`` (no extra knobs) instead of
    ``rehyat_forward_ex``; ``workspace`` (a CUDA byte tensor) calls
    ``rehyat_forward_ws``; ``noalloc=True`` calls ``rehyat_forward_noalloc``.
    """
    lib = _load()
    _check_qkv(q, k, v)
    B, H, N, d = q.shape
    if N != T * HW:
        raise ValueError("N != T*HW")
    p, Hp = _phi_struct(phi, d)
    if Hp != H:
        raise ValueError("phi head count differs from q")
    if out is None:
        out = torch.empty_like(q)
    s = torch.cuda.current_stream() if stream is None else stream
    sp = ctypes.c_void_p(s.cuda_stream)
    if plain or noalloc:
        fn, name = ((lib.rehyat_forward_noalloc, "rehyat_forward_noalloc") if noalloc
                    else (lib.rehyat_forward, "rehyat_forward"))
        rc = fn(q.data_ptr(), k.data_ptr(), v.data_ptr(), ctypes.byref(p),
                out.data_ptr(), B, H, T, HW, d, chunk, sp)
        if rc != OK:
            raise RehyatError(rc, name)
        return out
    if workspace is not None:
        rc = lib.rehyat_forward_ws(q.data_ptr(), k.data_ptr(), v.data_ptr(), ctypes.byref(p),
                                   out.data_ptr(), B, H, T, HW, d, chunk, overlap,
                                   int(bool(causal)), stab_mode, workspace.data_ptr(),
                                   workspace.numel() * workspace.element_size(), sp)
        if rc != OK:
            raise RehyatError(rc, "rehyat_forward_ws")
        return out
    comps, dbg = None, None
    if debug:
        f32 = dict(device=q.device, dtype=torch.float32)
        comps = dict(m=torch.zeros(B, H, N, **f32), nS=torch.zeros(B, H, N, **f32),
                     aS=torch.zeros(B, H, N, d, **f32), nL=torch.zeros(B, H, N, **f32),
                     aL=torch.zeros(B, H, N, d, **f32))
        dbg = DebugOut(*(comps[n].data_ptr() for n in ("m", "nS", "aS", "nL", "aL")))
    rc = lib.rehyat_forward_ex(q.data_ptr(), k.data_ptr(), v.data_ptr(), ctypes.byref(p),
                               out.data_ptr(), B, H, T, HW, d, chunk, overlap,
                               int(bool(causal)), stab_mode,
                               ctypes.byref(dbg) if dbg is not None else None, sp)
    if rc != OK:
        raise RehyatError(rc, "rehyat_forward_ex")
    return (out, comps) if debug else out


def step(q_t, k_win, v_win, phi, S, z, n_absorb, out=None, stab_mode=STAB_ROWMAX, stream=None):
    """One chunk of the chunk-wise RNN (Eq. 14-18).  q_t: CUDA bf16 [B, H, n_q, d];
    k_win, v_win: [B, H, n_win, d], the softmax window oldest token first; S
    [B, H, D', d] and z [B, H, D'] fp32 are read for the read-out and then
    advanced in place by the first ``n_absorb`` window tokens.  Returns y_t."""
    lib = _load()
    for t in (q_t, k_win, v_win):
        if t.dtype != torch.bfloat16 or not t.is_cuda or not t.is_contiguous() or t.dim() != 4:
            raise TypeError("q_t, k_win, v_win must be contiguous CUDA bf16 tensors [B, H, n, d]")
    if k_win.shape != v_win.shape or k_win.shape[:2] != q_t.shape[:2] or k_win.shape[3] != q_t.shape[3]:
        raise ValueError("q_t / k_win / v_win shapes are inconsistent")
    B, H, n_q, d = q_t.shape
    n_win = k_win.shape[2]
    p, _ = _phi_struct(phi, d)
    for t, shape in ((S, (B, H, p.dprime, d)), (z, (B, H, p.dprime))):
        if t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous() or tuple(t.shape) != shape:
            raise TypeError(f"state tensors must be contiguous CUDA fp32 of shape {shape}")
    if out is None:
        out = torch.empty_like(q_t)
    elif out.shape != q_t.shape or out.dtype != torch.bfloat16 or not out.is_contiguous():
        raise TypeError("out must match q_t")
    s = torch.cuda.current_stream() if stream is None else stream
    rc = lib.rehyat_step(q_t.data_ptr(), k_win.data_ptr(), v_win.data_ptr(), ctypes.byref(p),
                         S.data_ptr(), z.data_ptr(), out.data_ptr(), B, H, d, n_q, n_win,
                         int(n_absorb), stab_mode, ctypes.c_void_p(s.cuda_stream))
    if rc != OK:
        raise RehyatError(rc, "rehyat_step")
    return out


def state(k, v, phi, T, HW, upto_frames, stream=None):
    """(S [B,H,D',d] fp32, z [B,H,D'] fp32) after absorbing the first
    ``upto_frames`` latent frames (Eq. 14-15, 17-18)."""
    lib = _load()
    _check_qkv(k, k, v)
    B, H, N, d = k.shape
    p, _ = _phi_struct(phi, d)
    S = torch.empty(B, H, p.dprime, d, device=k.device, dtype=torch.float32)
    z = torch.empty(B, H, p.dprime, device=k.device, dtype=torch.float32)
    s = torch.cuda.current_stream() if stream is None else stream
    rc = lib.rehyat_state(k.data_ptr(), v.data_ptr(), ctypes.byref(p), S.data_ptr(),
                          z.data_ptr(), B, H, T, HW, d, upto_frames,
                          ctypes.c_void_p(s.cuda_stream))
    if rc != OK:
        raise RehyatError(rc, "rehyat_state")
    return S, z


def phi_backward_workspace_bytes(B, H, T, HW, d, chunk):
    return _load().rehyat_phi_backward_workspace_bytes(B, H, T, HW, d, chunk)


def phi_backward(q, k, v, phi, grad_out, T, HW, chunk, overlap=0, workspace=None, out=None,
                 grads=None, stream=None, saved=None):
    """Gradients of a loss w.r.t. the parameters of phi_q and phi_k for a given
    ``grad_out`` = dL/dy_hat (CUDA bf16 [B, H, T*HW, d]): one step of the distillation of
    Eq. 19.  Returns ``(grads, y_hat)``: a dict of eight fp32 CUDA tensors shaped like the
    parameters, and the output of the recomputed forward pass.  ``workspace`` is a CUDA
    byte tensor of at least ``phi_backward_workspace_bytes`` bytes (allocated here if
    None).  ``saved`` = (out, nS, nL) from ``forward(..., debug=True)`` on the same arguments
    skips the attention kernel of the recomputation."""
    lib = _load()
    _check_qkv(q, k, v)
    if grad_out.shape != q.shape or grad_out.dtype != torch.bfloat16 or not grad_out.is_cuda \
            or not grad_out.is_contiguous():
        raise TypeError("grad_out must be a contiguous CUDA bf16 tensor shaped like q")
    B, H, N, d = q.shape
    if N != T * HW:
        raise ValueError("N != T*HW")
    p, Hp = _phi_struct(phi, d)
    if Hp != H:
        raise ValueError("phi head count differs from q")
    if workspace is None:
        need = lib.rehyat_phi_backward_workspace_bytes(B, H, T, HW, d, chunk)
        if need == 0:
            raise RehyatError(E_UNSUPPORTED, "rehyat_phi_backward_workspace_bytes")
        workspace = torch.empty(need, device=q.device, dtype=torch.uint8)
    sv = None
    if saved is not None:
        out, nS, nL = saved
        for t in (nS, nL):
            if t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous() or t.shape != q.shape[:3]:
                raise TypeError("saved nS, nL must be contiguous CUDA fp32 tensors [B, H, N]")
        if out.shape != q.shape or out.dtype != torch.bfloat16 or not out.is_contiguous():
            raise TypeError("saved out must match q")
        sv = ForwardSaved(nS.data_ptr(), nL.data_ptr())
    if out is None:
        out = torch.empty_like(q)
    if grads is None:
        grads = {n: torch.empty(t.shape, device=q.device, dtype=torch.float32) for n, t in phi.items()}
    g = PhiGrads()
    for name in ("w1_q", "b1_q", "w2_q", "b2_q", "w1_k", "b1_k", "w2_k", "b2_k"):
        t = grads[name]
        if t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous() or t.shape != phi[name].shape:
            raise TypeError(f"grads[{name}] must be a contiguous CUDA fp32 tensor shaped like phi[{name}]")
        setattr(g, name, t.data_ptr())
    s = torch.cuda.current_stream() if stream is None else stream
    rc = lib.rehyat_phi_backward(q.data_ptr(), k.data_ptr(), v.data_ptr(), ctypes.byref(p),
                                 grad_out.data_ptr(), out.data_ptr(),
                                 ctypes.byref(sv) if sv is not None else None, ctypes.byref(g),
                                 B, H, T, HW, d, chunk, overlap, workspace.data_ptr(),
                                 workspace.numel() * workspace.element_size(),
                                 ctypes.c_void_p(s.cuda_stream))
    if rc != OK:
        raise RehyatError(rc, "rehyat_phi_backward")
    return grads, out
