"""The whole-sequence entry point under HIP graph capture: with the workspace in place
a call allocates nothing and enqueues only kernels, so it can be recorded once and
replayed.  Every replay is checked against the eager result, with eager calls and
synchronisations between replays."""
import pytest
import torch

from paper_2601_04342_amd import binding, synth
from tests import parity

pytestmark = pytest.mark.gpu


def test_forward_replays_from_a_graph():
    B, H, T, HW, d = 1, 3, 6, 333, 128
    q, k, v = synth.make_qkv(B, H, T * HW, d, seed=41)
    phi = synth.make_phi(H, d, seed=42, gain=3.0)
    dq, dk, dv, dphi = parity.to_device(q, k, v, phi)
    out = torch.empty_like(dq)
    step = lambda: binding.forward(dq, dk, dv, dphi, T, HW, 2, out=out, overlap=1)
    step()                                   # allocates the workspace outside the capture
    torch.cuda.synchronize()
    want = out.clone()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for i in range(4):
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want), f"replay {i}"
        # eager work of the same library between replays (it shares the workspace)
        other = binding.forward(dq, dk, dv, dphi, T, HW, 1)
        torch.cuda.synchronize()
        assert torch.isfinite(other.float()).all()


def test_gradient_step_replays_from_a_graph():
    """rehyat_phi_backward takes its workspace per call and enqueues kernels only: one
    distillation step's worth of gradients can be recorded once and replayed."""
    B, H, T, HW, d = 1, 2, 5, 200, 128
    q, k, v = synth.make_qkv(B, H, T * HW, d, seed=43)
    phi = synth.make_phi(H, d, seed=44, gain=3.0)
    dq, dk, dv, dphi = parity.to_device(q, k, v, phi)
    dG = synth.make_grad_out(B, H, T * HW, d, seed=45).to("cuda", torch.bfloat16)
    ws = torch.empty(binding.phi_backward_workspace_bytes(B, H, T, HW, d, 1), device="cuda",
                     dtype=torch.uint8)
    grads = {n: torch.empty(t.shape, device="cuda", dtype=torch.float32) for n, t in dphi.items()}
    out = torch.empty_like(dq)
    step = lambda: binding.phi_backward(dq, dk, dv, dphi, dG, T, HW, 1, workspace=ws, out=out,
                                        grads=grads)
    step()
    torch.cuda.synchronize()
    want = {n: g.clone() for n, g in grads.items()}
    want_out = out.clone()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for i in range(3):
        for g in grads.values():
            g.fill_(float("nan"))
        out.fill_(float("nan"))
        ws.fill_(0xFF)                       # nothing in the workspace is assumed to survive
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for n in synth.PHI_NAMES:
            assert torch.equal(grads[n], want[n]), (n, f"replay {i}")
        assert torch.equal(out, want_out), f"replay {i}"
        other = binding.forward(dq, dk, dv, dphi, T, HW, 1)   # eager work between replays
        torch.cuda.synchronize()
        assert torch.isfinite(other.float()).all()


def test_streaming_steps_replay_from_a_graph():
    """rehyat_step forks its state update onto the library's second stream and joins it before
    returning: recorded into a graph, the fork and join become graph edges.  Three consecutive
    steps are recorded and replayed from the same starting state."""
    B, H, T, HW, d = 1, 2, 4, 200, 128
    q, k, v = synth.make_qkv(B, H, T * HW, d, seed=46)
    phi = synth.make_phi(H, d, seed=47, gain=3.0)
    dq, dk, dv, dphi = parity.to_device(q, k, v, phi)
    plan = binding.chunk_plan(T, HW, 1, 1).tolist()
    pieces = []
    for t, (q_lo, q_hi, s_lo, s_hi, _) in enumerate(plan[:3]):
        n_absorb = plan[t + 1][2] - s_lo
        pieces.append((dq[:, :, q_lo:q_hi].contiguous(), dk[:, :, s_lo:s_hi].contiguous(),
                       dv[:, :, s_lo:s_hi].contiguous(), torch.empty_like(dq[:, :, q_lo:q_hi]), n_absorb))
    S = torch.zeros(B, H, 2 * d, d, device="cuda")
    z = torch.zeros(B, H, 2 * d, device="cuda")

    def steps():
        for q_t, k_w, v_w, o_t, n_absorb in pieces:
            binding.step(q_t, k_w, v_w, dphi, S, z, n_absorb, out=o_t)

    steps()                                  # workspace and second stream exist before the capture
    torch.cuda.synchronize()
    want = [p[3].clone() for p in pieces]
    want_S, want_z = S.clone(), z.clone()
    assert float(want_S.abs().max()) > 0

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        S.zero_()
        z.zero_()
        steps()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    S.zero_()
    z.zero_()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        steps()
    for i in range(3):
        S.zero_()
        z.zero_()
        for p in pieces:
            p[3].fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, w in zip((p[3] for p in pieces), want):
            assert torch.equal(got, w), f"replay {i}"
        assert torch.equal(S, want_S) and torch.equal(z, want_z), f"replay {i}"
        # eager steps of the same library between replays
        S.zero_()
        z.zero_()
        steps()
        torch.cuda.synchronize()
        assert torch.equal(S, want_S)
