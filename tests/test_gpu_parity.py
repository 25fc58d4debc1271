"""GPU parity: the HIP library against the fp64 CPU oracle, element by element,
on the same seeded bf16-rounded inputs, through the C ABI.  Small shapes span
several 64-key tiles, several 128-query workgroups and ragged tails."""
import numpy as np
import pytest
import torch

from oracle import cref
from paper_2601_04342_amd import binding, synth
from tests import parity

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _announce(request):
    print(f"[gpu-test] {request.node.nodeid}", flush=True)
    yield
    torch.cuda.synchronize()


def test_tiny_baseline_config_with_components():
    """The tiny benchmark configuration: B=1, H=2, d=64, T=4 x 8x8 tokens, chunk 1; q, k, v
    seed 0, phi seed 1."""
    w = synth.WORKLOADS["tiny"]
    q, k, v, phi = synth.make_workload(w)
    dq, dk, dv, dphi = parity.to_device(q, k, v, phi)
    out, comps = binding.forward(dq, dk, dv, dphi, w.T, w.HW, w.chunk, debug=True)
    ref = cref.forward(*parity.oracle_inputs(q, k, v, phi), w.T, w.HW, w.chunk)
    parity.compare(out, comps, ref, label="tiny")
    plain = binding.forward(dq, dk, dv, dphi, w.T, w.HW, w.chunk, plain=True)
    assert torch.equal(plain, out)   # rehyat_forward == rehyat_forward_ex defaults


CASES = [
    # B, H, T, HW, d, chunk, overlap, stab, gain
    (1, 2, 4, 64, 64, 1, 0, 0, 8.0),
    (2, 3, 5, 77, 128, 2, 0, 0, 4.0),      # T % chunk != 0, ragged key and query tiles
    (1, 2, 5, 77, 128, 2, 1, 0, 4.0),      # overlapping windows (Eq. 12)
    (1, 2, 7, 50, 64, 3, 2, 0, 6.0),
    (1, 2, 4, 30, 64, 1, 3, 0, 6.0),       # overlap reaches the first frame
    (1, 2, 5, 77, 64, 1, 0, 1, 4.0),       # stabiliser off
    (1, 1, 3, 300, 128, 1, 1, 1, 4.0),
    (1, 2, 6, 700, 128, 1, 0, 0, 2.0),     # 3 query tiles, 11 key tiles per chunk
    (1, 1, 3, 100, 128, 3, 0, 0, 1.0),     # one chunk: plain softmax attention
    (1, 1, 1, 1, 64, 1, 0, 0, 1.0),        # a single token
    (1, 1, 2, 1, 128, 1, 0, 0, 8.0),       # two tokens
    (1, 1, 4, 2000, 128, 1, 0, 0, 2.0),    # few (b,h,segment): segments are split
    (1, 2, 70, 20, 64, 1, 0, 0, 3.0),      # 70 chunks: three windows of chunk states
    (1, 1, 75, 12, 128, 2, 1, 0, 3.0),     # windows + overlap + short last chunk
]


@pytest.mark.parametrize("case", CASES)
def test_small_shapes_match_oracle(case):
    B, H, T, HW, d, chunk, overlap, stab, gain = case
    (emax, emean), ref = parity.run_case(B, H, T, HW, d, chunk, overlap, stab, gain,
                                         seed=sum(case[:6]))
    print(f"   max-abs {emax:.2e} mean-abs {emean:.2e} linear share "
          f"{parity.linear_share(ref, stab):.2f}", flush=True)


BIDIR_CASES = [
    # B, H, T, HW, d, chunk, overlap, stab, gain
    (1, 2, 4, 64, 64, 1, 0, 0, 8.0),
    (2, 3, 5, 77, 128, 2, 0, 0, 4.0),      # short last chunk
    (1, 2, 5, 77, 128, 2, 1, 0, 4.0),      # overlapping windows
    (1, 2, 7, 50, 64, 3, 2, 0, 6.0),
    (1, 2, 4, 30, 64, 1, 3, 0, 6.0),       # the last window is the whole sequence: empty linear set
    (1, 2, 5, 77, 64, 1, 0, 1, 4.0),       # stabiliser off
    (1, 1, 3, 100, 128, 3, 0, 0, 1.0),     # one chunk: plain softmax attention
    (1, 1, 4, 2000, 128, 1, 0, 0, 2.0),    # frames are split into pieces
    (1, 2, 70, 20, 64, 1, 0, 0, 3.0),      # more frames than partial slots: two passes
    (1, 1, 75, 12, 128, 2, 1, 0, 3.0),     # two passes + overlap + short last chunk
    (1, 1, 2, 40, 128, 1, 0, 0, 5.0),      # two chunks: each one's linear set is the other
]


@pytest.mark.parametrize("case", BIDIR_CASES)
def test_bidirectional_small_shapes_match_oracle(case):
    """Non-causal sets of Eq. 11-12: the linear part covers the tokens on both
    sides of the softmax window."""
    B, H, T, HW, d, chunk, overlap, stab, gain = case
    (emax, emean), ref = parity.run_case(B, H, T, HW, d, chunk, overlap, stab, gain,
                                         seed=sum(case[:6]) + 1, causal=False)
    print(f"   max-abs {emax:.2e} mean-abs {emean:.2e} linear share "
          f"{parity.linear_share(ref, stab):.2f}", flush=True)


@pytest.mark.parametrize("scale,stab", [(6.0, 0), (6.0, 1), (0.05, 0)])
def test_wide_and_narrow_score_ranges(scale, stab):
    """Scores far apart (row maxima keep growing from tile to tile by more and by less
    than the kernel's rescale threshold) and nearly equal scores."""
    B, H, T, HW, d = 1, 2, 3, 450, 128
    q, k, v = synth.make_qkv(B, H, T * HW, d, seed=17)
    q = synth.round_bf16(q * scale)
    if stab == 1:   # keep exp(score) itself inside fp32 when nothing is subtracted
        q = synth.round_bf16(q * 0.5)
    phi = synth.make_phi(H, d, seed=18, gain=3.0)
    dq, dk, dv, dphi = parity.to_device(q, k, v, phi)
    out, comps = binding.forward(dq, dk, dv, dphi, T, HW, 1, overlap=1, stab_mode=stab, debug=True,
                                 out=parity.nan_like(dq))
    torch.cuda.synchronize()
    ref = cref.forward(*parity.oracle_inputs(q, k, v, phi), T, HW, 1, overlap=1, stab=stab)
    spread = float(ref.m.max() - ref.m.min())
    # peaked rows return nearly a single v row, |y| up to about 4: the bars on the bf16
    # output get the per-element bf16 storage term, the fp32 components keep theirs
    mag = float(np.abs(ref.out).max())
    print(f"   row maxima span {spread:.1f} nats, largest |y| {mag:.2f}", flush=True)
    parity.compare(out, comps, ref, stab=stab, label=f"score scale {scale} stab {stab}",
                   bf16_output_allowance=True)


def test_zero_phi_is_block_diagonal_softmax():
    """phi = 0 isolates the softmax kernel: chunk-local softmax attention."""
    B, H, T, HW, d = 1, 2, 3, 200, 128
    q, k, v = synth.make_qkv(B, H, T * HW, d, seed=3)
    phi = {n: torch.zeros_like(p) for n, p in synth.make_phi(H, d).items()}
    dq, dk, dv, dphi = parity.to_device(q, k, v, phi)
    out = binding.forward(dq, dk, dv, dphi, T, HW, 1).float().cpu()
    for t in range(T):
        s = slice(t * HW, (t + 1) * HW)
        want = torch.softmax(q[:, :, s].double() @ k[:, :, s].double().transpose(-1, -2)
                             / np.sqrt(d), dim=-1) @ v[:, :, s].double()
        assert (out[:, :, s].double() - want).abs().max() <= parity.OUT_MAX_ABS


def test_constant_value_rows_return_the_constant():
    """Weights are jointly normalised (Eq. 5): constant v gives that constant,
    up to the bf16 rounding of the weights and of the output."""
    B, H, T, HW, d = 1, 2, 4, 150, 64
    q, k, _ = synth.make_qkv(B, H, T * HW, d, seed=5)
    v = synth.round_bf16(torch.linspace(-2, 2, d)).expand(B, H, T * HW, d).contiguous()
    phi = synth.make_phi(H, d, gain=4.0)
    dq, dk, dv, dphi = parity.to_device(q, k, v, phi)
    out = binding.forward(dq, dk, dv, dphi, T, HW, 1).float().cpu()
    assert (out - v).abs().max() <= 2e-2 * v.abs().max()


def test_repeat_calls_are_bit_identical_and_workspace_contents_do_not_matter():
    B, H, T, HW, d = 1, 2, 6, 300, 128
    q, k, v = synth.make_qkv(B, H, T * HW, d, seed=7)
    phi = synth.make_phi(H, d, gain=3.0)
    dq, dk, dv, dphi = parity.to_device(q, k, v, phi)
    a = binding.forward(dq, dk, dv, dphi, T, HW, 1).clone()
    b = binding.forward(dq, dk, dv, dphi, T, HW, 1).clone()
    assert torch.equal(a, b)
    # caller-owned workspace pre-filled with NaN bit patterns, with guard bands
    need = binding.workspace_bytes(B, H, d)
    guard = 4096
    buf = torch.full((need + 2 * guard,), 0xFF, dtype=torch.uint8, device="cuda")
    assert buf.data_ptr() % 256 == 0
    try:
        binding.set_workspace(buf[guard:guard + need])
        c = binding.forward(dq, dk, dv, dphi, T, HW, 1).clone()
        torch.cuda.synchronize()
    finally:
        binding.set_workspace(None)
    assert torch.equal(a, c)
    assert (buf[:guard] == 0xFF).all() and (buf[guard + need:] == 0xFF).all()


def test_state_hook_matches_oracle_state():
    """Chunk-state and prefix kernels alone (Eq. 14-15, 17-18)."""
    B, H, T, HW, d = 1, 2, 40, 37, 64
    _, k, v = synth.make_qkv(B, H, T * HW, d, seed=11)
    phi = synth.make_phi(H, d, gain=4.0)
    _, dk, dv, dphi = parity.to_device(k, k, v, phi)
    for upto in (0, 1, 33, 40):
        S, z = binding.state(dk, dv, dphi, T, HW, upto)
        torch.cuda.synchronize()
        for h in range(H):
            Sr, zr = cref.state(k[0, h].double().numpy(), v[0, h].double().numpy(), upto * HW,
                                *(phi[n][h].double().numpy() for n in ("w1_k", "b1_k", "w2_k", "b2_k")))
            tolS = 6e-3 * max(np.abs(Sr).max(), 1e-30)
            assert np.abs(S[0, h].cpu().numpy() - Sr).max() <= tolS + 1e-30, (upto, h)
            assert np.abs(z[0, h].cpu().numpy() - zr).max() <= 3e-3 * max(np.abs(zr).max(), 1e-30) + 1e-30


def test_causal_prefix_consistency_on_gpu():
    """Appending frames does not change earlier outputs (Eq. 13)."""
    B, H, T, HW, d = 1, 2, 6, 100, 128
    q, k, v = synth.make_qkv(B, H, T * HW, d, seed=13)
    phi = synth.make_phi(H, d, gain=3.0)
    dq, dk, dv, dphi = parity.to_device(q, k, v, phi)
    full = binding.forward(dq, dk, dv, dphi, T, HW, 2, overlap=1)
    n4 = 4 * HW
    part = binding.forward(dq[:, :, :n4].contiguous(), dk[:, :, :n4].contiguous(),
                           dv[:, :, :n4].contiguous(), dphi, 4, HW, 2, overlap=1)
    assert torch.equal(full[:, :, :n4], part)


def test_per_call_workspaces_on_two_streams():
    """rehyat_forward_ws: two calls in flight at once on two streams, each with its own
    workspace, give exactly what the library-held workspace path gives, and a
    workspace one byte short is refused."""
    B, H, T, HW, d = 1, 3, 9, 333, 128
    qa, ka, va = synth.make_qkv(B, H, T * HW, d, seed=21)
    qb, kb, vb = synth.make_qkv(B, H, T * HW, d, seed=22)
    phi = synth.make_phi(H, d, gain=3.0)
    da = parity.to_device(qa, ka, va, phi)
    db = parity.to_device(qb, kb, vb, phi)
    want_a = binding.forward(*da, T, HW, 2, overlap=1).clone()
    want_b = binding.forward(*db, T, HW, 1, causal=False).clone()
    need = binding.workspace_bytes(B, H, d)
    ws_a = torch.empty(need, dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(need, dtype=torch.uint8, device="cuda")
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    out_a, out_b = parity.nan_like(da[0]), parity.nan_like(db[0])
    torch.cuda.synchronize()
    for _ in range(3):   # several rounds so that the two streams really overlap
        binding.forward(*da, T, HW, 2, overlap=1, out=out_a, workspace=ws_a, stream=sa)
        binding.forward(*db, T, HW, 1, causal=False, out=out_b, workspace=ws_b, stream=sb)
    torch.cuda.synchronize()
    assert torch.equal(out_a, want_a) and torch.equal(out_b, want_b)
    with pytest.raises(binding.RehyatError) as e:
        binding.forward(*da, T, HW, 2, out=out_a, workspace=ws_a[:need - 256])
    assert e.value.code == binding.E_WORKSPACE


def test_state_hook_before_the_first_frame_is_zero():
    B, H, T, HW, d = 1, 2, 3, 20, 64
    _, k, v = synth.make_qkv(B, H, T * HW, d, seed=2)
    _, dk, dv, dphi = parity.to_device(k, k, v, synth.make_phi(H, d))
    S, z = binding.state(dk, dv, dphi, T, HW, 0)
    torch.cuda.synchronize()
    assert (S == 0).all() and (z == 0).all()


def test_xcd_mask_hook_skips_whole_workgroups_and_resets():
    """The measurement hook: with some XCDs masked, every output row is either untouched or
    bit-identical to the unmasked result (whole workgroups exit, nothing else changes), and
    the full mask restores normal operation."""
    B, H, T, HW, d = 1, 3, 5, 300, 128
    q, k, v = synth.make_qkv(B, H, T * HW, d, seed=71)
    phi = synth.make_phi(H, d, seed=72, gain=3.0)
    dq, dk, dv, dphi = parity.to_device(q, k, v, phi)
    want = binding.forward(dq, dk, dv, dphi, T, HW, 1)
    torch.cuda.synchronize()
    out = torch.full_like(want, float("nan"))
    try:
        binding.debug_set_xcd_mask(0x05)
        binding.forward(dq, dk, dv, dphi, T, HW, 1, out=out)
        torch.cuda.synchronize()
    finally:
        binding.debug_set_xcd_mask(0xFF)
    written = ~torch.isnan(out.float()).any(dim=-1)
    assert 0 < int(written.sum()) < written.numel()
    assert torch.equal(out[written], want[written])
    assert torch.isnan(out[~written].float()).all()
    again = binding.forward(dq, dk, dv, dphi, T, HW, 1)
    torch.cuda.synchronize()
    assert torch.equal(again, want)
