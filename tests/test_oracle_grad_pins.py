"""Pins of the gradient oracle (oracle/grad.py: dL/dphi for the distillation step of
section 3.4, Eq. 19) against things other than itself: central finite differences
of the independent C forward oracle, the L1 loss of Eq. 19 itself, and cases
whose gradient is known in closed form.  No GPU."""
import numpy as np
import pytest

from oracle import brute, cref, grad

NAMES = ("w1_q", "b1_q", "w2_q", "b2_q", "w1_k", "b1_k", "w2_k", "b2_k")


def make(B, H, T, HW, d, hidden, dprime, seed, scale=0.6):
    rng = np.random.default_rng(seed)
    N = T * HW
    q, k, v = (rng.standard_normal((B, H, N, d)) for _ in range(3))
    shapes = {"w1": (H, hidden, d), "b1": (H, hidden), "w2": (H, dprime, hidden), "b2": (H, dprime)}
    phi = {n: rng.standard_normal(shapes[n[:2]]) * scale for n in NAMES}
    G = rng.standard_normal((B, H, N, d))
    return q, k, v, phi, G


def loss_forward(q, k, v, phi, G, T, HW, chunk, overlap):
    """sum(G * y_hat) with y_hat from the C oracle of the forward pass."""
    return float((cref.forward(q, k, v, phi, T, HW, chunk, overlap=overlap).out * G).sum())


def fd_entries(rng, arr, n):
    idx = [tuple(rng.integers(0, s) for s in arr.shape) for _ in range(n)]
    return list(dict.fromkeys(idx))


@pytest.mark.parametrize("T,HW,chunk,overlap", [(4, 5, 1, 0), (5, 4, 2, 0), (5, 4, 2, 1), (6, 3, 1, 2)])
def test_gradients_match_central_differences_of_the_forward_oracle(T, HW, chunk, overlap):
    B, H, d, hidden, dprime = 2, 2, 6, 10, 8
    q, k, v, phi, G = make(B, H, T, HW, d, hidden, dprime, seed=T * 100 + chunk * 10 + overlap)
    grads, y = grad.phi_backward(q, k, v, phi, G, T, HW, chunk, overlap)
    ref = cref.forward(q, k, v, phi, T, HW, chunk, overlap=overlap).out
    assert np.abs(y - ref).max() <= 1e-11 * max(1.0, np.abs(ref).max())   # same forward
    rng = np.random.default_rng(7)
    eps = 1e-6
    checked = 0
    for name in NAMES:
        scale = max(np.abs(grads[name]).max(), 1e-12)
        for idx in fd_entries(rng, phi[name], 7):
            p_hi = {n: a.copy() for n, a in phi.items()}
            p_lo = {n: a.copy() for n, a in phi.items()}
            p_hi[name][idx] += eps
            p_lo[name][idx] -= eps
            fd = (loss_forward(q, k, v, p_hi, G, T, HW, chunk, overlap)
                  - loss_forward(q, k, v, p_lo, G, T, HW, chunk, overlap)) / (2 * eps)
            assert abs(fd - grads[name][idx]) <= 2e-6 * scale + 1e-9, (name, idx, fd, grads[name][idx])
            checked += 1
    assert checked >= 40


def test_l1_distillation_loss_of_eq_19():
    """Eq. 19: L = mean |y - y_hat| over the block output; its gradient is the gradient for
    G = sign(y_hat - y) / count.  Checked by differencing the L1 loss itself, evaluated with
    the brute-force definition of the forward pass."""
    B, H, T, HW, d, hidden, dprime, chunk = 1, 2, 4, 4, 6, 8, 6, 1
    q, k, v, phi, _ = make(B, H, T, HW, d, hidden, dprime, seed=3)
    teacher = np.random.default_rng(4).standard_normal(q.shape)   # stands in for the softmax teacher's output
    y = brute.forward(q, k, v, phi, T, HW, chunk)["out"]
    G = np.sign(y - teacher) / y.size
    grads, _ = grad.phi_backward(q, k, v, phi, G, T, HW, chunk)

    def l1(p):
        return float(np.abs(teacher - brute.forward(q, k, v, p, T, HW, chunk)["out"]).mean())

    rng = np.random.default_rng(5)
    eps = 1e-7   # small enough that no |.| or ReLU kink is crossed for these entries
    for name in NAMES:
        scale = max(np.abs(grads[name]).max(), 1e-12)
        for idx in fd_entries(rng, phi[name], 4):
            p_hi = {n: a.copy() for n, a in phi.items()}
            p_lo = {n: a.copy() for n, a in phi.items()}
            p_hi[name][idx] += eps
            p_lo[name][idx] -= eps
            fd = (l1(p_hi) - l1(p_lo)) / (2 * eps)
            assert abs(fd - grads[name][idx]) <= 1e-5 * scale + 1e-10, (name, idx)


def test_one_chunk_has_no_linear_part_hence_zero_gradient():
    """chunk >= T: every output is plain softmax attention (Eq. 2), independent of phi."""
    q, k, v, phi, G = make(1, 2, 3, 5, 6, 8, 6, seed=11)
    grads, _ = grad.phi_backward(q, k, v, phi, G, 3, 5, 3)
    for name in NAMES:
        assert np.abs(grads[name]).max() == 0.0


def test_gradient_is_linear_in_the_upstream_gradient():
    q, k, v, phi, G1 = make(1, 2, 4, 4, 6, 8, 6, seed=12)
    G2 = np.random.default_rng(13).standard_normal(G1.shape)
    g1, _ = grad.phi_backward(q, k, v, phi, G1, 4, 4, 1)
    g2, _ = grad.phi_backward(q, k, v, phi, G2, 4, 4, 1)
    g3, _ = grad.phi_backward(q, k, v, phi, 2.0 * G1 - 0.5 * G2, 4, 4, 1)
    for name in NAMES:
        want = 2.0 * g1[name] - 0.5 * g2[name]
        assert np.abs(g3[name] - want).max() <= 1e-11 * max(1.0, np.abs(want).max())


def test_dead_feature_and_first_chunk_queries_get_no_gradient():
    """A feature whose pre-activation is negative for every token has zero gradient in its
    row of w2 and its bias; queries of chunk 0 have an empty linear set, so with a single
    linear-set chunk the query map only sees chunk-1 queries."""
    q, k, v, phi, G = make(1, 1, 2, 6, 6, 8, 6, seed=14)
    phi["b2_k"][0, 2] = -1e6
    phi["b2_q"][0, 4] = -1e6
    grads, _ = grad.phi_backward(q, k, v, phi, G, 2, 6, 1)
    assert np.abs(grads["w2_k"][0, 2]).max() == 0.0 and grads["b2_k"][0, 2] == 0.0
    assert np.abs(grads["w2_q"][0, 4]).max() == 0.0 and grads["b2_q"][0, 4] == 0.0
    # zeroing the upstream gradient on chunk 1 leaves nothing that depends on phi
    G0 = G.copy()
    G0[:, :, 6:] = 0.0
    g0, _ = grad.phi_backward(q, k, v, phi, G0, 2, 6, 1)
    for name in NAMES:
        assert np.abs(g0[name]).max() == 0.0


def test_bf16_rounding_helper_and_hidden_round_option():
    """round_to_bf16 against hand-worked bit patterns (nearest, ties to even), and the
    hidden_round option: identical results when U is already representable in bf16."""
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -9, 1.0 + 3 * 2.0 ** -9,
                  1.0 + 2.0 ** -7 + 2.0 ** -8, -2.5, 0.0, 1e-3])
    got = grad.round_to_bf16(x)        # bf16 keeps 7 fraction bits: spacing 2^-7 in [1, 2)
    assert got[0] == 1.0 and got[5] == -2.5 and got[6] == 0.0
    assert got[1] == 1.0                      # exactly half way: ties to the even mantissa
    assert got[2] == 1.0                      # below half way
    assert got[3] == 1.0 + 2.0 ** -7          # above half way
    assert got[4] == 1.0 + 2.0 ** -6          # half way again, the even neighbour is the upper one
    assert abs(got[7] - 1e-3) <= 2.0 ** -8 * 1e-3
    # a first layer whose outputs are small integers: rounding changes nothing
    rng = np.random.default_rng(21)
    B, H, T, HW, d, hidden, dprime = 1, 1, 3, 4, 4, 6, 4
    q = rng.integers(-2, 3, (B, H, T * HW, d)).astype(float)
    k = rng.integers(-2, 3, (B, H, T * HW, d)).astype(float)
    v = rng.standard_normal((B, H, T * HW, d))
    phi = {"w1_q": rng.integers(-1, 2, (H, hidden, d)).astype(float), "b1_q": np.zeros((H, hidden)),
           "w2_q": rng.standard_normal((H, dprime, hidden)) * 0.3, "b2_q": rng.standard_normal((H, dprime)) * 0.1,
           "w1_k": rng.integers(-1, 2, (H, hidden, d)).astype(float), "b1_k": np.zeros((H, hidden)),
           "w2_k": rng.standard_normal((H, dprime, hidden)) * 0.3, "b2_k": rng.standard_normal((H, dprime)) * 0.1}
    G = rng.standard_normal(q.shape)
    g0, y0 = grad.phi_backward(q, k, v, phi, G, T, HW, 1)
    g1, y1 = grad.phi_backward(q, k, v, phi, G, T, HW, 1, hidden_round="bf16")
    assert np.array_equal(y0, y1)
    for name in NAMES:
        assert np.array_equal(g0[name], g1[name])


@pytest.mark.parametrize("T,HW,chunk,overlap", [(4, 5, 1, 0), (5, 4, 2, 1), (6, 3, 2, 0)])
def test_every_entry_against_reverse_mode_differentiation_of_the_definition(T, HW, chunk, overlap):
    """Eq. 5-9 with the sets of Eq. 12-13 written token by token in torch (fp64) and
    differentiated by torch's reverse mode: every entry of all eight gradients, not a sample.
    The library routine knows nothing of the chunk-wise derivation in oracle/grad.py."""
    import torch
    B, H, d, hidden, dprime = 1, 2, 6, 10, 8
    q, k, v, phi, G = make(B, H, T, HW, d, hidden, dprime, seed=77 + T)
    tq, tk, tv, tG = (torch.tensor(a, dtype=torch.float64) for a in (q, k, v, G))
    tp = {n: torch.tensor(a, dtype=torch.float64, requires_grad=True) for n, a in phi.items()}

    def fmap(x, s, h):
        u = torch.relu(tp[f"w1_{s}"][h] @ x + tp[f"b1_{s}"][h])
        psi = torch.relu(tp[f"w2_{s}"][h] @ u + tp[f"b2_{s}"][h])
        half = dprime // 2
        return torch.cat([psi[:half], psi[half:] ** 2])

    loss = torch.zeros((), dtype=torch.float64)
    N = T * HW
    for b in range(B):
        for h in range(H):
            fk = [fmap(tk[b, h, j], "k", h) for j in range(N)]
            for i in range(N):
                t = i // (chunk * HW)
                q_lo = t * chunk * HW
                q_hi = min((t + 1) * chunk, T) * HW
                s_lo = max(q_lo - overlap * HW, 0)
                scores = torch.stack([tq[b, h, i] @ tk[b, h, j] for j in range(s_lo, q_hi)]) / d ** 0.5
                w = torch.exp(scores - scores.max())
                num = (w[:, None] * tv[b, h, s_lo:q_hi]).sum(0)
                den = w.sum()
                if s_lo > 0:
                    fq = fmap(tq[b, h, i], "q", h)
                    lw = torch.stack([fq @ fk[j] for j in range(s_lo)])
                    num = num + (lw[:, None] * tv[b, h, :s_lo]).sum(0)
                    den = den + lw.sum()
                loss = loss + (tG[b, h, i] * num / den).sum()
    loss.backward()
    grads, _ = grad.phi_backward(q, k, v, phi, G, T, HW, chunk, overlap)
    for name in NAMES:
        want = tp[name].grad.numpy()
        assert np.abs(grads[name] - want).max() <= 1e-10 * max(1.0, np.abs(want).max()), name
