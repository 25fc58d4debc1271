"""TEST INFRASTRUCTURE: gradients of the hybrid attention output with respect to the
feature-map parameters phi_q, phi_k -- what one step of the attention distillation
of section 3.4 (Eq. 19) needs -- in numpy fp64.

Eq. 19 trains only phi_q and phi_k of a block so that the student output y_hat matches
the teacher's: phi <- phi - eta * grad_phi E|y - y_hat|.  For one sample the gradient of
any loss L is fixed by G = dL/dy_hat (for the L1 loss of Eq. 19, G = sign(y_hat - y) /
count); this module returns dL/d(w1_q, b1_q, w2_q, b2_q, w1_k, b1_k, w2_k, b2_k) for a
given G by the chain rule through Eq. 5-9 with the causal sets of Eq. 13, written out
chunk by chunk with plain matrix products: no suffix sums, no fusion.

With the row-maximum stabiliser the softmax terms a^S, n^S do not depend on phi, so

    y_i   = (a^S_i + Phi_q,i S_t) / (n^S_i + Phi_q,i . z_t)            Eq. 5, 16
    S_t   = sum_{j in T^L_t} Phi_k,j v_j^T ,  z_t = sum_{j in T^L_t} Phi_k,j   Eq. 14-18
    dL/d(a^L_i) = G_i / den_i ,   dL/d(n^L_i) = -(G_i . y_i) / den_i ,  den_i = n^S_i + n^L_i
    dL/dPhi_q,i = S_t (dL/da^L_i) + z_t dL/dn^L_i
    dL/dS_t = sum_{i in chunk t} Phi_q,i (dL/da^L_i)^T ,  dL/dz_t = sum_i Phi_q,i dL/dn^L_i
    dL/dPhi_k,j = sum_{t : j in T^L_t} ( dL/dS_t v_j + dL/dz_t )

followed by the backward pass of the two-layer map phi = [psi_1, psi_2^2],
psi = relu(W2 u + b2), u = relu(W1 x + b1) ("Characterization of phi", appendix
"Training Details").  The stabiliser reading (per-row maximum) and the ReLU are the
readings of the forward oracle; "parity unpinned" applies to them exactly as there.
This function itself is pinned by central finite differences of the forward oracle and,
entry by entry, by reverse-mode differentiation of the token-by-token definition
(tests/test_oracle_grad_pins.py).

ReLU gates are 0/1 decisions taken by floating point.  A kernel that keeps the hidden
activations U in bf16 takes the second layer's gates (psi > 0) on slightly different
values than fp64 does, and a gate that flips changes an entry of the gradient by its whole
contribution, not by a rounding error.  `hidden_round="bf16"` makes this oracle take those
decisions in the kernel's precision: U is rounded to the nearest-even bf16 value right after
the first layer and everything downstream (forward and backward) uses the rounded U.  The
default (None) is the exact fp64 chain that the finite-difference pins check; the option
changes no formula, only the values of U.
"""
import numpy as np


def round_to_bf16(x):
    """Nearest-even bf16 value of each element (via fp32), returned as fp64."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    bits = f.view(np.uint32).astype(np.uint64)
    bits = (bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000
    return bits.astype(np.uint32).view(np.float32).astype(np.float64).reshape(np.shape(x))


def _mlp_forward(x, w1, b1, w2, b2, hidden_round=None):
    pre1 = x @ w1.T + b1
    u = np.maximum(pre1, 0.0)
    if hidden_round == "bf16":
        u = round_to_bf16(u)
    elif hidden_round is not None:
        raise ValueError("hidden_round must be None or 'bf16'")
    pre2 = u @ w2.T + b2
    psi = np.maximum(pre2, 0.0)
    half = psi.shape[1] // 2
    phi = np.concatenate([psi[:, :half], psi[:, half:] ** 2], axis=1)
    return u, psi, phi


def _mlp_backward(x, w1, w2, u, psi, dphi):
    """Gradients of sum(dphi * phi(x)) w.r.t. w1, b1, w2, b2 (degree-2 map, ReLU)."""
    half = psi.shape[1] // 2
    dpsi = dphi.copy()
    dpsi[:, half:] *= 2.0 * psi[:, half:]
    dpsi *= (psi > 0.0)
    dw2 = dpsi.T @ u
    db2 = dpsi.sum(axis=0)
    du = (dpsi @ w2) * (u > 0.0)
    dw1 = du.T @ x
    db1 = du.sum(axis=0)
    return dw1, db1, dw2, db2


def chunk_sets(T, HW, chunk, overlap):
    """Per chunk (q_lo, q_hi, s_lo, s_hi, l_hi) from section 3.2's layout, Eq. 12 and Eq. 13."""
    rows = []
    f0 = 0
    while f0 < T:
        f1 = min(f0 + chunk, T)
        q_lo, q_hi = f0 * HW, f1 * HW
        s_lo = max(q_lo - overlap * HW, 0)
        rows.append((q_lo, q_hi, s_lo, q_hi, s_lo))
        f0 = f1
    return rows


def phi_backward(q, k, v, phi_params, G, T, HW, chunk, overlap=0, hidden_round=None):
    """q, k, v, G: [B, H, N, d]; phi_params: dict of the eight tensors with a leading
    head axis.  Returns (grads dict of the same eight shapes, y_hat [B, H, N, d])."""
    q, k, v, G = (np.asarray(a, np.float64) for a in (q, k, v, G))
    P = {n: np.asarray(a, np.float64) for n, a in phi_params.items()}
    B, H, N, d = q.shape
    assert N == T * HW
    grads = {n: np.zeros_like(a) for n, a in P.items()}
    y_all = np.zeros_like(q)
    sets = chunk_sets(T, HW, chunk, overlap)
    for b in range(B):
        for h in range(H):
            uq, psiq, Fq = _mlp_forward(q[b, h], P["w1_q"][h], P["b1_q"][h], P["w2_q"][h], P["b2_q"][h], hidden_round)
            uk, psik, Fk = _mlp_forward(k[b, h], P["w1_k"][h], P["b1_k"][h], P["w2_k"][h], P["b2_k"][h], hidden_round)
            dFq = np.zeros_like(Fq)
            dFk = np.zeros_like(Fk)
            for (q_lo, q_hi, s_lo, s_hi, l_hi) in sets:
                Q = q[b, h, q_lo:q_hi]
                Kw, Vw = k[b, h, s_lo:s_hi], v[b, h, s_lo:s_hi]
                s = Q @ Kw.T / np.sqrt(d)
                m = s.max(axis=1, keepdims=True)
                p = np.exp(s - m)
                nS = p.sum(axis=1)
                aS = p @ Vw
                S = Fk[:l_hi].T @ v[b, h, :l_hi]          # [D', d]   (Eq. 14-18)
                z = Fk[:l_hi].sum(axis=0)                # [D']
                aL = Fq[q_lo:q_hi] @ S
                nL = Fq[q_lo:q_hi] @ z
                den = nS + nL
                y = (aS + aL) / den[:, None]
                y_all[b, h, q_lo:q_hi] = y
                g = G[b, h, q_lo:q_hi]
                daL = g / den[:, None]                   # dL/d a^L_i
                dnL = -(g * y).sum(axis=1) / den         # dL/d n^L_i
                dFq[q_lo:q_hi] = daL @ S.T + dnL[:, None] * z[None, :]
                dS = Fq[q_lo:q_hi].T @ daL               # [D', d]
                dz = Fq[q_lo:q_hi].T @ dnL               # [D']
                if l_hi > 0:
                    dFk[:l_hi] += v[b, h, :l_hi] @ dS.T + dz[None, :]
            gq = _mlp_backward(q[b, h], P["w1_q"][h], P["w2_q"][h], uq, psiq, dFq)
            gk = _mlp_backward(k[b, h], P["w1_k"][h], P["w2_k"][h], uk, psik, dFk)
            for name, val in zip(("w1_q", "b1_q", "w2_q", "b2_q"), gq):
                grads[name][h] += val
            for name, val in zip(("w1_k", "b1_k", "w2_k", "b2_k"), gk):
                grads[name][h] += val
    return grads, y_all
