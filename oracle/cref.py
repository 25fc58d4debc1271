"""TEST INFRASTRUCTURE: ctypes front end of the C oracle (``rehyat_oracle.c``).

Argument marshalling only; every number is computed by the C file, in fp64.
"""
import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rehyat_oracle.c")
_LIB = os.path.join(_HERE, "librehyat_oracle.so")
_lib = None


def build(force=False):
    """Compile the C oracle with gcc (host only, OpenMP)."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c99", "-Wall",
           _SRC, "-o", _LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int64)
        lib.rehyat_oracle_chunk_plan.restype = ctypes.c_int
        lib.rehyat_oracle_chunk_plan.argtypes = [ctypes.c_int] * 4 + [
            ip, ctypes.POINTER(ctypes.c_int)]
        lib.rehyat_oracle_phi.restype = ctypes.c_int
        lib.rehyat_oracle_phi.argtypes = [dp, ctypes.c_int64, ctypes.c_int, dp, dp,
                                          dp, dp, ctypes.c_int, ctypes.c_int,
                                          ctypes.c_int, dp]
        lib.rehyat_oracle_forward.restype = ctypes.c_int
        lib.rehyat_oracle_forward.argtypes = ([dp] * 11 + [ctypes.c_int] * 12
                                              + [ip, ctypes.c_int64] + [dp] * 6)
        lib.rehyat_oracle_state.restype = ctypes.c_int
        lib.rehyat_oracle_state.argtypes = [dp, dp, ctypes.c_int64, ctypes.c_int,
                                            dp, dp, dp, dp, ctypes.c_int,
                                            ctypes.c_int, ctypes.c_int, dp, dp]
        _lib = lib
    return _lib


def _d(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


@dataclass
class Components:
    """The five terms of Eq. 5-9 for each evaluated query row."""
    out: np.ndarray   # [B, H, R, d]
    m: np.ndarray     # [B, H, R]   row maximum of the softmax exponents
    nS: np.ndarray    # [B, H, R]
    aS: np.ndarray    # [B, H, R, d]
    nL: np.ndarray    # [B, H, R]
    aL: np.ndarray    # [B, H, R, d]


def chunk_plan(T, HW, chunk, overlap=0):
    """[n_chunks, 5] int64 rows (q_lo, q_hi, s_lo, s_hi, l_hi); Eq. 12-13."""
    lib = _load()
    n = ctypes.c_int(0)
    rc = lib.rehyat_oracle_chunk_plan(T, HW, chunk, overlap, None, ctypes.byref(n))
    if rc != 0:
        raise ValueError("bad chunk-plan arguments")
    table = np.zeros((n.value, 5), dtype=np.int64)
    rc = lib.rehyat_oracle_chunk_plan(
        T, HW, chunk, overlap, table.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
        ctypes.byref(n))
    assert rc == 0
    return table


def phi(x, w1, b1, w2, b2, degree=2):
    """Feature map of one head: x [n, d] -> [n, D']."""
    lib = _load()
    x, xp = _d(x)
    w1, w1p = _d(w1)
    b1, b1p = _d(b1)
    w2, w2p = _d(w2)
    b2, b2p = _d(b2)
    n, d = x.shape
    hidden, dprime = w1.shape[0], w2.shape[0]
    assert w1.shape == (hidden, d) and w2.shape == (dprime, hidden)
    assert b1.shape == (hidden,) and b2.shape == (dprime,)
    out = np.zeros((n, dprime), dtype=np.float64)
    rc = lib.rehyat_oracle_phi(xp, n, d, w1p, b1p, w2p, b2p, hidden, dprime, degree,
                               out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    if rc != 0:
        raise ValueError(f"rehyat_oracle_phi failed: {rc}")
    return out


def forward(q, k, v, phi_params, T, HW, chunk, overlap=0, causal=True, stab=0,
            rows=None, degree=2):
    """Hybrid attention in the chunk-recurrent form (Eq. 14-18).

    q, k, v: [B, H, N, d]; phi_params: dict with w1_q, b1_q, w2_q, b2_q, w1_k,
    b1_k, w2_k, b2_k (leading H axis).  rows: optional sorted token indices.
    Returns ``Components``.
    """
    lib = _load()
    q, qp = _d(q)
    k, kp = _d(k)
    v, vp = _d(v)
    B, H, N, d = q.shape
    assert k.shape == q.shape and v.shape == q.shape and N == T * HW
    names = ["w1_q", "b1_q", "w2_q", "b2_q", "w1_k", "b1_k", "w2_k", "b2_k"]
    arrs, ptrs = zip(*[_d(phi_params[n]) for n in names])
    hidden, dprime = arrs[0].shape[1], arrs[2].shape[1]
    for w1, b1, w2, b2 in (arrs[:4], arrs[4:]):
        assert w1.shape == (H, hidden, d) and b1.shape == (H, hidden)
        assert w2.shape == (H, dprime, hidden) and b2.shape == (H, dprime)
    if rows is None:
        R, rp, nr = N, None, 0
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        R, nr = len(rows), len(rows)
        rp = rows.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))
    res = Components(out=np.zeros((B, H, R, d)), m=np.zeros((B, H, R)),
                     nS=np.zeros((B, H, R)), aS=np.zeros((B, H, R, d)),
                     nL=np.zeros((B, H, R)), aL=np.zeros((B, H, R, d)))
    P = lambda a: a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))
    rc = lib.rehyat_oracle_forward(qp, kp, vp, *ptrs, hidden, dprime, degree, B, H,
                                   T, HW, d, chunk, overlap, int(bool(causal)),
                                   int(stab), rp, nr, P(res.out), P(res.m),
                                   P(res.nS), P(res.aS), P(res.nL), P(res.aL))
    if rc != 0:
        raise ValueError(f"rehyat_oracle_forward failed: {rc}")
    return res


def state(k, v, upto, w1, b1, w2, b2, degree=2):
    """RNN state (S [D', d], z [D']) after absorbing tokens [0, upto) of one head."""
    lib = _load()
    k, kp = _d(k)
    v, vp = _d(v)
    w1, w1p = _d(w1)
    b1, b1p = _d(b1)
    w2, w2p = _d(w2)
    b2, b2p = _d(b2)
    d = k.shape[1]
    hidden, dprime = w1.shape[0], w2.shape[0]
    S = np.zeros((dprime, d))
    z = np.zeros(dprime)
    P = lambda a: a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))
    rc = lib.rehyat_oracle_state(kp, vp, int(upto), d, w1p, b1p, w2p, b2p, hidden,
                                 dprime, degree, P(S), P(z))
    if rc != 0:
        raise ValueError(f"rehyat_oracle_state failed: {rc}")
    return S, z
