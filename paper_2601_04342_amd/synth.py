"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Holds no arithmetic of the attention method: only random draws, the per-token
RMS normalisation that Wan2.1-style blocks apply to q and k before attention,
and rounding to bf16 so that the CPU oracle and the GPU library consume the
same values.  Shapes follow the paper's workloads: an 81x480x832 video is a
21x30x52 latent (section 4.1 and section 5.2), 161 frames give 41 latent
frames (section 5.2, on-device results), and sampling uses a classifier-free
guidance pair, i.e. batch 2 (appendix, "Sampling").
"""
from dataclasses import dataclass

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    d: int
    T: int        # latent frames
    HW: int       # tokens per latent frame
    chunk: int    # T_c, latent frames per chunk
    rms_norm: bool = True

    @property
    def N(self):
        return self.T * self.HW


WORKLOADS = {
    # tiny case the oracle evaluates by brute force in seconds
    "tiny": Workload("tiny", B=1, H=2, d=64, T=4, HW=8 * 8, chunk=1, rms_norm=False),
    # Wan2.1-1.3B, 480p, one attention layer
    "wan480p": Workload("wan480p", B=1, H=12, d=128, T=21, HW=30 * 52, chunk=1),
    "wan480p_cfg_c1": Workload("wan480p_cfg_c1", B=2, H=12, d=128, T=21, HW=30 * 52, chunk=1),
    "wan480p_cfg_c2": Workload("wan480p_cfg_c2", B=2, H=12, d=128, T=21, HW=30 * 52, chunk=2),
    "wan480p_cfg_c3": Workload("wan480p_cfg_c3", B=2, H=12, d=128, T=21, HW=30 * 52, chunk=3),
    "wan480p_long": Workload("wan480p_long", B=1, H=12, d=128, T=41, HW=30 * 52, chunk=1),
    "wan720p": Workload("wan720p", B=1, H=12, d=128, T=21, HW=45 * 80, chunk=1, rms_norm=False),
    # the other supported head width at full length (not a shape of the paper: same bytes
    # per token as wan480p, twice the heads)
    "wide480p_d64": Workload("wide480p_d64", B=1, H=24, d=64, T=21, HW=30 * 52, chunk=1),
    # 320x480 generation (20 x 30 latent tokens per frame), the shape of the paper's
    # on-device tables (section 4.2): 21 to 41 latent frames, T_c = 3, and the larger
    # chunk sizes of the T_c ablation
    "p320_t21_c3": Workload("p320_t21_c3", B=1, H=12, d=128, T=21, HW=20 * 30, chunk=3),
    "p320_t41_c3": Workload("p320_t41_c3", B=1, H=12, d=128, T=41, HW=20 * 30, chunk=3),
    # a long generation: 34 chunks, more than one window of chunk-state slots
    "p320_t101_c3": Workload("p320_t101_c3", B=1, H=12, d=128, T=101, HW=20 * 30, chunk=3),
    "p320_t21_c5": Workload("p320_t21_c5", B=1, H=12, d=128, T=21, HW=20 * 30, chunk=5),
    "p320_t21_c7": Workload("p320_t21_c7", B=1, H=12, d=128, T=21, HW=20 * 30, chunk=7),
    # two chunks; with T_o = 8 the second chunk's window leaves 3 of the 21 frames outside
    # (bidirectional sets with a small complement)
    "p320_t21_c11": Workload("p320_t21_c11", B=1, H=12, d=128, T=21, HW=20 * 30, chunk=11),
}


def round_bf16(x):
    """fp32 tensor -> fp32 tensor holding the nearest-even bf16 values."""
    return x.to(torch.bfloat16).to(torch.float32)


def make_qkv(B, H, N, d, seed=0, rms_norm=True):
    """q, k, v ~ N(0,1), drawn in that order from one CPU generator.

    With ``rms_norm`` each q and k token is divided by sqrt(mean_d(x^2)).
    Returns fp32 CPU tensors [B, H, N, d] already rounded to bf16 values.
    """
    g = torch.Generator(device="cpu").manual_seed(seed)
    out = []
    for name in ("q", "k", "v"):
        x = torch.randn(B, H, N, d, generator=g, dtype=torch.float32)
        if rms_norm and name != "v":
            x = x / x.pow(2).mean(dim=-1, keepdim=True).sqrt()
        out.append(round_bf16(x))
    return tuple(out)


def make_grad_out(B, H, N, d, seed=2):
    """A stand-in for dL/dy_hat: N(0,1) draws rounded to bf16 values, fp32 CPU [B, H, N, d]."""
    g = torch.Generator(device="cpu").manual_seed(seed)
    return round_bf16(torch.randn(B, H, N, d, generator=g, dtype=torch.float32))


PHI_NAMES = ("w1_q", "b1_q", "w2_q", "b2_q", "w1_k", "b1_k", "w2_k", "b2_k")


def make_phi(H, d, hidden=None, dprime=None, seed=1, std=0.02, gain=1.0):
    """phi_q / phi_k parameters ~ N(0, std) (std = standard deviation), drawn
    in the order of ``PHI_NAMES``; weights rounded to bf16 values, biases kept
    fp32.  ``gain`` multiplies every draw before rounding (used to move the
    share of the linear part in the normaliser)."""
    hidden = 2 * d if hidden is None else hidden
    dprime = 2 * d if dprime is None else dprime
    g = torch.Generator(device="cpu").manual_seed(seed)
    shapes = {"w1": (H, hidden, d), "b1": (H, hidden), "w2": (H, dprime, hidden),
              "b2": (H, dprime)}
    p = {}
    for name in PHI_NAMES:
        x = torch.randn(*shapes[name[:2]], generator=g, dtype=torch.float32) * (std * gain)
        p[name] = round_bf16(x) if name.startswith("w") else x
    return p


def phi_param_count(H, d, hidden=None, dprime=None):
    hidden = 2 * d if hidden is None else hidden
    dprime = 2 * d if dprime is None else dprime
    return 2 * H * (hidden * d + hidden + dprime * hidden + dprime)


def make_workload(w, seed_qkv=0, seed_phi=1, gain=1.0):
    """(q, k, v, phi) for a ``Workload``."""
    q, k, v = make_qkv(w.B, w.H, w.N, w.d, seed=seed_qkv, rms_norm=w.rms_norm)
    return q, k, v, make_phi(w.H, w.d, seed=seed_phi, gain=gain)
