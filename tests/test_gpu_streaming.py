"""GPU parity of the streaming step entry point (the literal chunk-wise RNN of
section 3.3, Eq. 14-18): chunks are fed one at a time, the caller keeps the
state and the K/V window, and the concatenated outputs must equal the oracle's
forward pass over the whole sequence; the state after every step must equal
the oracle's state over the tokens that have left the window."""
import numpy as np
import pytest
import torch

from oracle import cref
from paper_2601_04342_amd import binding, synth
from tests import parity

pytestmark = pytest.mark.gpu


def stream(dq, dk, dv, dphi, T, HW, chunk, overlap, stab=0, absorb_all_at_end=False, on_step=None,
           state_offset=0):
    """Drive rehyat_step over the chunks of a sequence; returns (out, S, z).  `state_offset`
    floats are skipped in front of S, so that it is only 4-byte aligned."""
    B, H, N, d = dq.shape
    plan = binding.chunk_plan(T, HW, chunk, overlap).tolist()
    S = torch.zeros(state_offset + B * H * 2 * d * d, device="cuda")[state_offset:].view(B, H, 2 * d, d)
    z = torch.zeros(B, H, 2 * d, device="cuda")
    out = torch.empty_like(dq)
    for t, (q_lo, q_hi, s_lo, s_hi, l_hi) in enumerate(plan):
        assert l_hi == s_lo
        if t + 1 < len(plan):
            n_absorb = plan[t + 1][2] - s_lo
        else:
            n_absorb = (s_hi - s_lo) if absorb_all_at_end else 0
        y = binding.step(dq[:, :, q_lo:q_hi].contiguous(), dk[:, :, s_lo:s_hi].contiguous(),
                         dv[:, :, s_lo:s_hi].contiguous(), dphi, S, z, n_absorb, stab_mode=stab)
        out[:, :, q_lo:q_hi] = y
        if on_step is not None:
            torch.cuda.synchronize()
            on_step(t, s_lo + n_absorb, S, z)
    torch.cuda.synchronize()
    return out, S, z


def check_state(k, v, phi, upto, S, z, label):
    for h in range(k.shape[1]):
        Sr, zr = cref.state(k[0, h].double().numpy(), v[0, h].double().numpy(), upto,
                            *(phi[n][h].double().numpy() for n in ("w1_k", "b1_k", "w2_k", "b2_k")))
        assert np.abs(S[0, h].cpu().numpy() - Sr).max() <= 6e-3 * max(np.abs(Sr).max(), 1e-30) + 1e-30, label
        assert np.abs(z[0, h].cpu().numpy() - zr).max() <= 3e-3 * max(np.abs(zr).max(), 1e-30) + 1e-30, label


@pytest.mark.parametrize("B,H,T,HW,d,chunk,overlap,stab,gain", [
    (1, 2, 4, 64, 64, 1, 0, 0, 8.0),      # the tiny configuration
    (1, 2, 7, 100, 128, 2, 1, 0, 3.0),    # overlap, short last chunk, ragged tiles
    (2, 3, 9, 37, 64, 3, 2, 0, 4.0),      # window of chunk + 2 frames, batch of two
    (1, 2, 6, 150, 128, 1, 3, 1, 2.0),    # overlap longer than the chunk, stabiliser off
    (1, 1, 5, 200, 128, 5, 0, 0, 1.0),    # a single chunk: plain softmax, nothing absorbed
])
def test_streaming_equals_forward(B, H, T, HW, d, chunk, overlap, stab, gain):
    print(f"[gpu-test] streaming B{B} H{H} T{T} HW{HW} d{d} chunk{chunk} ov{overlap} stab{stab}", flush=True)
    q, k, v = synth.make_qkv(B, H, T * HW, d, seed=21)
    phi = synth.make_phi(H, d, seed=22, gain=gain)
    dq, dk, dv, dphi = parity.to_device(q, k, v, phi)

    def on_step(t, upto, S, z):
        if B == 1:
            check_state(k, v, phi, upto, S, z, f"state after step {t}")

    out, S, z = stream(dq, dk, dv, dphi, T, HW, chunk, overlap, stab, absorb_all_at_end=True,
                       on_step=on_step)
    ref = cref.forward(*parity.oracle_inputs(q, k, v, phi), T, HW, chunk, overlap=overlap, stab=stab)
    parity.compare(out, None, ref, stab=stab, label="streaming vs oracle")
    # the whole-sequence entry point computes the same thing with another summation split
    full = binding.forward(dq, dk, dv, dphi, T, HW, chunk, overlap=overlap, stab_mode=stab)
    torch.cuda.synchronize()
    assert (out.float() - full.float()).abs().max().item() <= parity.OUT_MAX_ABS
    if B == 1:
        check_state(k, v, phi, T * HW, S, z, "final state")


def test_streaming_is_deterministic_and_leaves_inputs_alone():
    B, H, T, HW, d = 1, 2, 5, 130, 128
    q, k, v = synth.make_qkv(B, H, T * HW, d, seed=31)
    phi = synth.make_phi(H, d, seed=32, gain=3.0)
    dq, dk, dv, dphi = parity.to_device(q, k, v, phi)
    keep = (dq.clone(), dk.clone(), dv.clone())
    a = stream(dq, dk, dv, dphi, T, HW, 1, 1)
    b = stream(dq, dk, dv, dphi, T, HW, 1, 1)
    for x, y in zip(a, b):
        assert torch.equal(x, y)
    for x, y in zip((dq, dk, dv), keep):
        assert torch.equal(x, y)


def test_streaming_full_size_wan480p():
    """21 steps at the 480p shape (T_c = 1, T_o = 1 so that every step has a two-frame
    window); sampled rows against the oracle, all rows against the whole-sequence call."""
    w = synth.WORKLOADS["wan480p"]
    print("[gpu-test] streaming full size wan480p overlap 1", flush=True)
    q, k, v, phi = synth.make_workload(w, gain=0.35)
    dq, dk, dv, dphi = parity.to_device(q, k, v, phi)
    out, S, z = stream(dq, dk, dv, dphi, w.T, w.HW, w.chunk, 1)
    assert torch.isfinite(out.float()).all() and torch.isfinite(S).all()
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([rng.integers(0, w.N, 24), [0, w.HW - 1, w.HW, w.N - 1]]))
    for h in (1, 10):
        ref = cref.forward(*parity.oracle_inputs(q, k, v, phi, heads=[h]), w.T, w.HW, w.chunk,
                           overlap=1, rows=rows)
        e = parity.compare(out[:, h:h + 1], None, ref, rows=rows, label=f"streaming wan480p h{h}")
        print(f"   h{h}: max-abs {e[0]:.2e} mean-abs {e[1]:.2e} linear share {parity.linear_share(ref):.2f}",
              flush=True)
    full = binding.forward(dq, dk, dv, dphi, w.T, w.HW, w.chunk, overlap=1)
    torch.cuda.synchronize()
    assert (out.float() - full.float()).abs().max().item() <= parity.OUT_MAX_ABS


def test_state_that_is_only_four_byte_aligned():
    """The caller's state may sit at any 4-byte boundary: same bits as with an aligned one."""
    B, H, T, HW, d = 1, 2, 5, 130, 128
    q, k, v = synth.make_qkv(B, H, T * HW, d, seed=33)
    phi = synth.make_phi(H, d, seed=34, gain=3.0)
    dq, dk, dv, dphi = parity.to_device(q, k, v, phi)
    a = stream(dq, dk, dv, dphi, T, HW, 1, 1)
    b = stream(dq, dk, dv, dphi, T, HW, 1, 1, state_offset=1)
    assert b[1].data_ptr() % 16 == 4
    for x, y in zip(a, b):
        assert torch.equal(x, y)
