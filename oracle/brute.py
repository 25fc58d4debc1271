"""TEST INFRASTRUCTURE: brute-force hybrid attention, numpy fp64, O(N^2).

The definition of section 3.2 written out token by token: for every query i,
build its softmax set and its linear set explicitly (Eq. 10-13), then sum
Eq. 6-9 over them and divide (Eq. 5).  No chunk state, no recurrence, no
blocking: the point is that a reader can check it against the paper by eye, and
that it shares nothing with the chunk-recurrent C oracle it is used to pin.
"""
import numpy as np


def phi_map(x, w1, b1, w2, b2, degree=2):
    """phi(x) = [psi_1^1, psi_2^2, ..., psi_P^P] ("Characterization of phi").

    x [n, d]; w1 [h, d]; b1 [h]; w2 [D', h]; b2 [D'].  The embedding network is
    a two-layer per-head MLP (appendix, "Training Details"); ReLU keeps every
    psi, and hence phi, non-negative as section 3.1 requires.
    """
    x = np.asarray(x, dtype=np.float64)
    u = np.maximum(x @ np.asarray(w1, np.float64).T + np.asarray(b1, np.float64), 0.0)
    psi = np.maximum(u @ np.asarray(w2, np.float64).T + np.asarray(b2, np.float64), 0.0)
    parts = np.split(psi, degree, axis=-1)
    return np.concatenate([p ** (i + 1) for i, p in enumerate(parts)], axis=-1)


def token_sets(i, T, HW, chunk, overlap, causal):
    """(softmax set, linear set) of query token i as index arrays.

    N' = chunk*HW tokens per chunk, t = chunk of i.  Softmax set (Eq. 12):
    max(t*N' - overlap*HW, 0) <= j < (t+1)*N' (clipped to N for a short last
    chunk).  Linear set: j below the window start (Eq. 13) when causal, else
    every token not in the softmax set (Eq. 11-12).
    """
    N = T * HW
    Np = chunk * HW
    t = i // Np
    lo = max(t * Np - overlap * HW, 0)
    hi = min((t + 1) * Np, N)
    allj = np.arange(N)
    in_s = (allj >= lo) & (allj < hi)
    if causal:
        in_l = allj < lo
    else:
        in_l = ~in_s
    return allj[in_s], allj[in_l]


def forward(q, k, v, phi_params, T, HW, chunk, overlap=0, causal=True, stab=0,
            degree=2):
    """Returns dict(out, m, nS, aS, nL, aL) with shapes [B,H,N,(d)]."""
    q = np.asarray(q, np.float64)
    k = np.asarray(k, np.float64)
    v = np.asarray(v, np.float64)
    B, H, N, d = q.shape
    assert N == T * HW
    out = np.zeros((B, H, N, d))
    m = np.zeros((B, H, N))
    nS = np.zeros((B, H, N))
    nL = np.zeros((B, H, N))
    aS = np.zeros((B, H, N, d))
    aL = np.zeros((B, H, N, d))
    for b in range(B):
        for h in range(H):
            fq = phi_map(q[b, h], phi_params["w1_q"][h], phi_params["b1_q"][h],
                         phi_params["w2_q"][h], phi_params["b2_q"][h], degree)
            fk = phi_map(k[b, h], phi_params["w1_k"][h], phi_params["b1_k"][h],
                         phi_params["w2_k"][h], phi_params["b2_k"][h], degree)
            for i in range(N):
                js, jl = token_sets(i, T, HW, chunk, overlap, causal)
                e = (k[b, h, js] @ q[b, h, i]) / np.sqrt(d)     # exponents
                c = e.max() if stab == 0 else 0.0               # stabiliser c_t
                w = np.exp(e - c)
                a_s = w @ v[b, h, js]                           # Eq. 6
                n_s = w.sum()                                   # Eq. 8
                sim = fk[jl] @ fq[i]                            # phi_q(q_i).phi_k(k_j)
                a_l = sim @ v[b, h, jl]                         # Eq. 7
                n_l = sim.sum()                                 # Eq. 9
                out[b, h, i] = (a_s + a_l) / (n_s + n_l)        # Eq. 5
                m[b, h, i], nS[b, h, i], nL[b, h, i] = e.max(), n_s, n_l
                aS[b, h, i], aL[b, h, i] = a_s, a_l
    return dict(out=out, m=m, nS=nS, aS=aS, nL=nL, aL=aL)
