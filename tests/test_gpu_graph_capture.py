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
