#!/usr/bin/env python3
"""Benchmark of the hybrid-attention hot path on one MI355X.

One step = one call of rehyat_forward (chunk-state kernel, prefix pass, fused
softmax / read-out / merge kernel) on the Wan2.1-1.3B 480p single-layer shape
(B=1, H=12, d=128, 21 latent frames x 30x52 tokens = 32,760 tokens, chunk = 1
frame), inputs resident in HBM.  Prints ONE JSON line.

Two passes of --steps steps each: the first, with the library's per-kernel events
off, gives the step time (median of per-step HIP event intervals on the launch
stream; the wall-clock mean over the same region is reported beside it); the second,
with them on, gives each kernel's average launch duration, from which the roofline
figure of the dominant kernel is computed.
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published
# HBM bytes per launch of the fused attention kernel, from two rocprofv3 --pmc runs per
# workload (FETCH_SIZE, then WRITE_SIZE; scaled by what a plain 1 GiB device copy reads on
# the same counters in the same runs: FETCH_SIZE x 2.0, WRITE_SIZE x 1.0), keyed by workload
# and valid for the library version they were measured on (profiles/*_hbm_traffic_pmc.md).
# Anything else reports null.
ATTN_TRAFFIC = {
    # 2.0 x 178,013 KiB + 1.0 x 98,280 KiB (profiles/wan480p_hbm_traffic_pmc.md)
    ("wan480p", "forward", 304): 465_200_000,   # 303 and 304 share the forward kernels
}


def algorithmic_flops(w, chunk, overlap=0, causal=True):
    """Work the method itself requires (no padding, no unused last-chunk state,
    no phi_q / read-out for chunks whose linear set is empty)."""
    from paper_2601_04342_amd import binding
    plan = binding.chunk_plan(w.T, w.HW, chunk, overlap).tolist()
    BH, d, h, Dp = w.B * w.H, w.d, 2 * w.d, 2 * w.d
    softmax = 4 * d * BH * sum((r[1] - r[0]) * (r[3] - r[2]) for r in plan)
    phi_tok = 2 * (d * h + h * Dp)                      # one map, one token
    if causal:
        n_lin_q = sum(r[1] - r[0] for r in plan if r[4] > 0)  # queries with a linear set
        n_state = plan[-1][4]                               # tokens ever absorbed
    else:   # every token outside the window: empty only when the window is everything
        n_lin_q = sum(r[1] - r[0] for r in plan if r[3] - r[2] < w.N)
        n_state = w.N if n_lin_q else 0
    phi_q = BH * n_lin_q * phi_tok
    phi_k = BH * n_state * phi_tok
    state = 2 * BH * n_state * Dp * (d + 1)
    readout = 2 * BH * n_lin_q * Dp * (d + 1)
    return dict(softmax=softmax, phi_q=phi_q, phi_k=phi_k, state=state, readout=readout,
                total=softmax + phi_q + phi_k + state + readout,
                attn_kernel=softmax + phi_q + readout, state_kernel=phi_k + state)


def backward_flops(w, chunk, fwd):
    """Algorithmic work of the feature-map gradient (Eq. 19) on top of the forward pass:
    per query with a linear set and per key in some linear set, dPhi (one read-out-sized
    product), the chunk-state gradient on the query side, and the two layers' input and
    weight gradients; phi itself is counted once (in the forward pass)."""
    from paper_2601_04342_amd import binding
    plan = binding.chunk_plan(w.T, w.HW, chunk, 0).tolist()
    BH, d, h, Dp = w.B * w.H, w.d, 2 * w.d, 2 * w.d
    n_q = sum(r[1] - r[0] for r in plan if r[4] > 0)
    n_k = plan[-1][4]
    per_tok = 2 * Dp * (d + 1) + 2 * h * Dp + 2 * Dp * h + 2 * h * d   # dPhi, dU, dW2, dW1
    grad = BH * (n_q + n_k) * per_tok + BH * n_q * 2 * Dp * (d + 1)     # + dS_t, dz_t
    return dict(forward=fwd["total"], gradient=grad, total=fwd["total"] + grad)


def cpu_baseline_backward(w, chunk, q, k, v, phi, G, heads, gpu_grads):
    """The fp64 gradient oracle on the first `heads` heads of the same workload, timed, then
    compared entry by entry with what the GPU produced in the timed configuration."""
    import numpy as np
    from oracle import grad as ograd
    qs, ks, vs, gs = (x[:, :heads].double().numpy() for x in (q, k, v, G))
    ps = {n: p[:heads].double().numpy() for n, p in phi.items()}
    t0 = time.perf_counter()
    ref, _ = ograd.phi_backward(qs, ks, vs, ps, gs, w.T, w.HW, chunk, hidden_round="bf16")
    dt = time.perf_counter() - t0
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    base = {"value": w.B * w.N * (heads / w.H) / dt, "unit": "tokens/s", "cores": threads,
            "kind": "oracle", "seconds": round(dt, 3),
            "sample": f"{heads} of {w.H} heads, all {w.N} tokens, fp64 numpy gradient oracle "
                      "(forward + gradient); value = layer-equivalent tokens/s"}
    worst_max, worst_fro = 0.0, 0.0
    for n, r in ref.items():
        g = gpu_grads[n][:heads].cpu().double().numpy()
        worst_max = max(worst_max, float(np.abs(g - r).max() / np.abs(r).max()))
        worst_fro = max(worst_fro, float(np.linalg.norm(g - r) / np.linalg.norm(r)))
    parity = {"max_abs_over_max_ref": worst_max, "relative_frobenius": worst_fro,
              "against": "gradient oracle, every entry of the eight tensors of the sampled heads "
                         "(worst tensor)"}
    return base, parity


def cpu_baseline(w, chunk, q, k, v, phi, heads, gpu_out):
    """The fp64 oracle, as it stands, on `heads` heads of the same workload, timed; its
    output is then compared with what the GPU produced in the timed configuration."""
    import numpy as np
    from oracle import cref
    qs, ks, vs = (x[:, :heads].double().numpy() for x in (q, k, v))
    ps = {n: p[:heads].double().numpy() for n, p in phi.items()}
    t0 = time.perf_counter()
    ref = cref.forward(qs, ks, vs, ps, w.T, w.HW, chunk)
    dt = time.perf_counter() - t0
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    base = {"value": w.B * w.N * (heads / w.H) / dt, "unit": "tokens/s", "cores": threads,
            "kind": "oracle", "seconds": round(dt, 3),
            "sample": f"{heads} of {w.H} heads, all {w.N} tokens, fp64 C oracle (OpenMP); "
                      "value = layer-equivalent tokens/s"}
    err = np.abs(gpu_out[:, :heads].float().cpu().double().numpy() - ref.out)
    parity = {"max_abs": float(err.max()), "mean_abs": float(err.mean()),
              "linear_share": float((ref.nL / (ref.nS + ref.nL)).mean()),
              "elements": int(err.size), "against": "oracle, every element of the sampled heads"}
    return base, parity


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="wan480p")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-heads", type=int, default=12)
    ap.add_argument("--cpu-heads-backward", type=int, default=4,
                    help="heads the gradient oracle evaluates in --mode backward (about 1 - 3 s each)")
    ap.add_argument("--mode", choices=("forward", "bidirectional", "stream", "fullsoftmax", "backward"),
                    default="forward",
                    help="forward: rehyat_forward (the headline path); bidirectional: "
                         "rehyat_forward_ex(causal=0); stream: one rehyat_step per chunk with "
                         "caller-owned state and window; fullsoftmax: rehyat_forward with one "
                         "chunk covering all frames (plain softmax attention, Eq. 2) on the same inputs; "
                         "backward: rehyat_phi_backward (forward recomputation + gradients of the "
                         "feature-map parameters, one distillation step of Eq. 19)")
    ap.add_argument("--overlap", type=int, default=0, help="T_o (bidirectional and stream modes)")
    ap.add_argument("--pmc-copy-mib", type=int, default=0,
                    help="after the timed steps also run one plain device-to-device copy of this "
                         "many MiB (a kernel of known HBM traffic that calibrates the FETCH_SIZE / "
                         "WRITE_SIZE counters of a rocprofv3 --pmc run)")
    ap.add_argument("--graph-steps", type=int, default=0,
                    help="forward modes: also record this many consecutive calls into one HIP graph and "
                         "report the time of a step when the graph is replayed (`ms_per_step_graph_replay`); "
                         "`value` stays the eager figure")
    ap.add_argument("--xcd-mask", type=lambda x: int(x, 0), default=0xFF,
                    help="measurement hook, timing only (forward modes): attention workgroups on the "
                         "XCDs whose bit is clear exit at once, the others do their usual share; the "
                         "output is then incomplete and is not checked")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (no sharding, no collectives); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2601_04342_amd import binding, synth
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    binding.library()   # fails loudly if the HIP library is not built
    probe = (args.xcd_mask & 0xFF) != 0xFF
    if probe:
        if args.mode not in ("forward", "fullsoftmax", "bidirectional"):
            print("bench.py: --xcd-mask applies to the whole-sequence forward modes", file=sys.stderr)
            sys.exit(2)
        binding.debug_set_xcd_mask(args.xcd_mask)
    w = synth.WORKLOADS[args.workload]
    chunk = w.T if args.mode == "fullsoftmax" else w.chunk
    q, k, v, phi = synth.make_workload(w)
    dq, dk, dv = (x.to("cuda", torch.bfloat16).contiguous() for x in (q, k, v))
    dphi = binding.phi_to_device(phi)
    out = torch.full_like(dq, float("nan"))
    causal = args.mode != "bidirectional"
    overlap = args.overlap if args.mode in ("bidirectional", "stream") else 0
    if args.mode in ("forward", "fullsoftmax"):
        step = lambda: binding.forward(dq, dk, dv, dphi, w.T, w.HW, chunk, out=out, plain=True)
    elif args.mode == "bidirectional":
        step = lambda: binding.forward(dq, dk, dv, dphi, w.T, w.HW, chunk, out=out,
                                       overlap=overlap, causal=False)
    elif args.mode == "backward":
        G = synth.make_grad_out(w.B, w.H, w.N, w.d)
        dG = G.to("cuda", torch.bfloat16)
        bws = torch.empty(binding.phi_backward_workspace_bytes(w.B, w.H, w.T, w.HW, w.d, chunk),
                          device="cuda", dtype=torch.uint8)
        grads = {n: torch.empty(t.shape, device="cuda", dtype=torch.float32) for n, t in dphi.items()}
        step = lambda: binding.phi_backward(dq, dk, dv, dphi, dG, w.T, w.HW, chunk, workspace=bws,
                                            out=out, grads=grads)
    else:
        # the caller's side of chunk-by-chunk generation: per chunk its queries, its K/V
        # window and the number of tokens that leave the window, prepared outside the timing
        plan = binding.chunk_plan(w.T, w.HW, chunk, overlap).tolist()
        pieces = []
        for t, (q_lo, q_hi, s_lo, s_hi, _) in enumerate(plan):
            n_absorb = plan[t + 1][2] - s_lo if t + 1 < len(plan) else 0
            pieces.append((dq[:, :, q_lo:q_hi].contiguous(), dk[:, :, s_lo:s_hi].contiguous(),
                           dv[:, :, s_lo:s_hi].contiguous(), torch.empty_like(dq[:, :, q_lo:q_hi]),
                           n_absorb))
        S = torch.zeros(w.B, w.H, 2 * w.d, w.d, device="cuda")
        z = torch.zeros(w.B, w.H, 2 * w.d, device="cuda")

        def step():
            S.zero_()
            z.zero_()
            for q_t, k_w, v_w, o_t, n_absorb in pieces:
                binding.step(q_t, k_w, v_w, dphi, S, z, n_absorb, out=o_t)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # ---- pass 1: step time, per-kernel events off --------------------------------
    binding.profile_enable(False)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(args.steps):
        step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    per_step = [marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps)]
    ms = statistics.median(per_step)

    # ---- pass 2: kernel durations, per-kernel events on ----------------------------
    binding.profile_enable(True)
    torch.cuda.synchronize()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    prof = binding.profile_read()
    binding.profile_enable(False)

    graph_ms = None
    if args.graph_steps > 0 and args.mode in ("forward", "fullsoftmax", "bidirectional"):
        # the workspace is in place after the passes above: a call only enqueues kernels
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for _ in range(args.graph_steps):
                step()
        n_rep = max(3, args.steps // args.graph_steps)
        for _ in range(2):
            graph.replay()
        g = [torch.cuda.Event(enable_timing=True) for _ in range(n_rep + 1)]
        torch.cuda.synchronize()
        g[0].record()
        for i in range(n_rep):
            graph.replay()
            g[i + 1].record()
        torch.cuda.synchronize()
        graph_ms = statistics.median(g[i].elapsed_time(g[i + 1]) for i in range(n_rep)) / args.graph_steps

    if args.mode == "stream":
        out = torch.cat([p[3] for p in pieces], dim=2)
    assert probe or torch.isfinite(out.float()).all()
    copy_gbps = None
    if args.pmc_copy_mib > 0:
        src = torch.full((args.pmc_copy_mib << 20,), 7, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)   # warm-up (also the copy a --pmc run calibrates on: the first of the three)
        torch.cuda.synchronize()
        c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        c0.record()
        dst.copy_(src)
        dst.copy_(src)
        c1.record()
        torch.cuda.synchronize()
        # bytes read + bytes written per second: what an HBM-bound pass can reach on this machine
        copy_gbps = 2 * 2 * src.numel() / (c0.elapsed_time(c1) * 1e-3) / 1e9
        del src, dst

    fl = algorithmic_flops(w, chunk, overlap, causal)
    if args.mode == "backward":
        # the library's per-kernel events cover forward calls only; rocprofv3 --kernel-trace
        # gives this mode's kernel breakdown
        bf = backward_flops(w, chunk, fl)
        extra = {}
        # the same step when the caller hands over the forward pass it has already run
        # (out, n^S, n^L of rehyat_forward_ex): the attention kernel is not run again
        fwd_out, comps = binding.forward(dq, dk, dv, dphi, w.T, w.HW, chunk, debug=True)
        saved = (fwd_out, comps["nS"], comps["nL"])
        del comps
        sstep = lambda: binding.phi_backward(dq, dk, dv, dphi, dG, w.T, w.HW, chunk, workspace=bws,
                                             grads=grads, saved=saved)
        for _ in range(args.warmup):
            sstep()
        sm = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
        torch.cuda.synchronize()
        sm[0].record()
        for i in range(args.steps):
            sstep()
            sm[i + 1].record()
        torch.cuda.synchronize()
        extra["ms_per_step_with_saved_forward"] = statistics.median(
            sm[i].elapsed_time(sm[i + 1]) for i in range(args.steps))
        step()   # grads of the full step again, for the parity check below
        torch.cuda.synchronize()
        if not args.no_cpu_baseline:
            extra["cpu_baseline"], extra["parity"] = cpu_baseline_backward(
                w, chunk, q, k, v, phi, G, min(args.cpu_heads_backward, w.H), grads)
        print(json.dumps({
            "metric": "feature-map gradient step (forward recomputation + backward), tokens/s per layer",
            "value": w.B * w.N / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": ms, "ms_per_step_wall_mean": wall_ms,
            "ms_per_step_min_max": [min(per_step), max(per_step)], "higher_is_better": True,
            "dtype": "bf16", "data": "synthetic",
            "config": {"workload": f"{w.name}: B={w.B} H={w.H} d={w.d} T={w.T} HW={w.HW} N={w.N} "
                                   f"chunk={chunk} causal row-max, rehyat_phi_backward"},
            "algorithmic_tflop": {kk: vv / 1e12 for kk, vv in bf.items()},
            "tflops": bf["total"] / (ms * 1e-3) / 1e12,
            "pct_mfma_peak": 100.0 * bf["total"] / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
            "workspace_bytes": int(bws.numel()), "library_version": binding.version(), **extra}))
        return
    kern_ms = {kk: (tot / n if n else None) for kk, (tot, n) in prof.items()}
    # all launches of the attention kernel in one step share the step's algorithmic work
    attn_ms = prof["attn"][0] / args.steps
    achieved = fl["attn_kernel"] / (attn_ms * 1e-3) / 1e12
    traffic = ATTN_TRAFFIC.get((w.name, args.mode, binding.version()))
    res = {
        "metric": "hybrid-attn tokens/s per layer @Wan2.1-480p shape; TFLOP/s and % MFMA peak",
        "value": w.B * w.N / (ms * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "ms_per_step_wall_mean": wall_ms,
        "ms_per_step_min_max": [min(per_step), max(per_step)],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}: B={w.B} H={w.H} d={w.d} T={w.T} HW={w.HW} "
                               f"N={w.N} chunk={chunk} overlap={overlap} "
                               f"{'causal' if causal else 'bidirectional'} row-max"
                               + (", one rehyat_step per chunk" if args.mode == "stream" else "")
                               + (", one chunk = plain softmax attention" if args.mode == "fullsoftmax" else ""),
                   "phi": "hidden=D'=2d, degree 2, ReLU, N(0,0.02) seed 1",
                   "qkv": "N(0,1) seed 0, bf16" + (", q,k RMS-normalised" if w.rms_norm else "")},
        "tflops": fl["total"] / (ms * 1e-3) / 1e12,
        "pct_mfma_peak": 100.0 * fl["total"] / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "algorithmic_tflop": {kk: vv / 1e12 for kk, vv in fl.items()},
        "kernel_ms": kern_ms,
        "kernel_launches_per_step": {kk: n / args.steps for kk, (_, n) in prof.items()},
        "workspace_bytes": binding.workspace_bytes(w.B, w.H, w.d),
        "library_version": binding.version(),
        "roofline": {"bound": "mfma", "kernel": binding.attn_kernel_name(w.d), "achieved": achieved,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS, "traffic": traffic},
        "copy_GBps": copy_gbps,
        "state_kernel_tflops": (fl["state_kernel"] / (prof["state"][0] / args.steps * 1e-3) / 1e12
                                if prof["state"][1] else None),
    }
    if graph_ms is not None:
        res["ms_per_step_graph_replay"] = graph_ms
        res["graph_steps"] = args.graph_steps
    if probe:
        res["probe"] = (f"xcd_mask={args.xcd_mask & 0xFF:#04x}: attention workgroups on the other XCDs exit at once; "
                        "timing only, `value`, `tflops` and `roofline` do not describe a complete call")
    if not args.no_cpu_baseline and args.mode == "forward" and not probe:
        res["cpu_baseline"], res["parity"] = cpu_baseline(w, chunk, q, k, v, phi, args.cpu_heads, out)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
