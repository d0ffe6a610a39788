#!/usr/bin/env python3
"""Benchmark of the FLARE mixer on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--cfg 4] [--no-cpu-baseline]

A step is one pass of the whole hot path -- flare_forward (encode partials, merge, decode)
followed by flare_backward -- over one batch of the synthetic million-token mesh workload
(B=1, H=8, d=16, N=1,000,000, M=256, bf16 storage, fp32 accumulation).  Inputs are resident in
HBM before the timed region.  One JSON line is printed:
  value        tokens/s of forward+backward (B*N tokens per step)
  fwd          the same for the forward alone (its own timed loop of K steps)
  roofline     the dominant kernel (most time per step) against the roofline that binds it: HBM
               (algorithmic bytes per launch / mean duration) or, where the softmax's exponentials
               need longer than the bytes, the vector ALUs' v_exp_f32 rate ("alu"); durations are
               measured with HIP events on the launch stream
  kernels      mean duration, algorithmic GB/s and exponentials/s of every kernel of the step
  cpu_baseline the fp64 CPU oracle timed on a bounded sample of the same workload
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16, published

# Rates of the softmax's exponentials on the vector ALUs (one v_exp_f32 per score and half):
# 256 CUs x 4 SIMDs x 64 lanes / 8 cycles per wave instruction x 2.4 GHz.
EXP_PEAK_GOPS = 256 * 4 * 64 / 8 * 2.4


def algorithmic_bytes(kernel, B, H, N, M, d, elem):
    """HBM bytes one launch of `kernel` must move: streamed token rows plus per-token statistics."""
    row = d * elem
    bhn = B * H * N
    per_token = {
        "encode_partial": 2 * row,              # k, v
        "decode": 2 * row,                      # k in, y out
        "bwd_token_stats": 2 * row + 8,         # k, dy in; lse_dec, delta out
        "bwd_prep": 2 * row + 12,               # y, dy, lse_dec in; lse_dec2, delta out
        "bwd_dz_partial": 3 * row + 8,          # k, dy, y, lse_dec in; delta out (saved-statistics path)
        "bwd_dq_partial": 3 * row + 8,          # k, v, dy, lse_dec, delta in
        "bwd_dkdv": 5 * row + 8,                # k, v, dy in; dk, dv out
        "bwd_dq_partial_2exp": 3 * row + 8,
        "bwd_dkdv_2exp": 5 * row + 8,
        "bwd_pass_a": 2 * row + 8,
        "bwd_pass_b": 5 * row + 8,
    }
    if kernel in per_token:
        return bhn * per_token[kernel]
    return None


def exponentials(kernel, B, H, N, M):
    """v_exp_f32 lane-operations one launch of `kernel` cannot avoid: one per score.  (The last two
    backward kernels need both softmax weights of a score, but the second follows from the first by
    a multiplication, R = P * 2^(lse_enc2[m] - lse_dec2[n]); their two-exponential fall-backs are
    priced at two.)"""
    per_pair = {"encode_partial": 1, "decode": 1, "bwd_token_stats": 1, "bwd_dz_partial": 1,
                "bwd_dq_partial": 1, "bwd_dkdv": 1, "bwd_dq_partial_2exp": 2, "bwd_dkdv_2exp": 2}
    return per_pair.get(kernel, 0) * B * H * N * M


# HBM bytes per launch (fetch, write) of the default workload, from two `rocprofv3 --pmc` runs
# (FETCH_SIZE, then WRITE_SIZE, KiB per dispatch), each scaled by what the same counter read for a
# plain 256 MB device copy in the same run (FETCH_SIZE x 2.00, WRITE_SIZE x 1.00); see
# profiles/forward_backward_cfg4_hbm_traffic.md.
MEASURED_TRAFFIC_CFG4 = {
    "encode_partial": (250642 * 2.0 * 1024, 18432 * 1024),
    "decode": (125963 * 2.0 * 1024, 281250 * 1024),
    "bwd_dz_partial": (441142 * 2.0 * 1024, 47911 * 1024),
    "bwd_dkdv": (408256 * 2.0 * 1024, 505120 * 1024),
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # Defaults: the GPU needs some tens of milliseconds of load to settle at its sustained clock (a step right
    # after an idle phase runs about 8 % slower than in the steady state), so 50 warm-up steps, then 200 timed.
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--cfg", type=int, default=4, help="synthetic workload id (4 = the headline)")
    ap.add_argument("--tokens", type=int, default=None, help="override N (for quick checks only)")
    ap.add_argument("--latents", type=int, default=None, help="override M (for quick checks only)")
    ap.add_argument("--head-dim", type=int, default=None, help="override d (for quick checks only)")
    ap.add_argument("--dtype", choices=["f32", "bf16", "f16"], default=None,
                    help="override the workload's storage type (for quick checks only)")
    ap.add_argument("--layout", choices=["bhnd", "bnhd"], default="bhnd",
                    help="memory order of k, v, y, dy, dk, dv: [B,H,N,d] (default) or [B,N,H,d]")
    ap.add_argument("--spectral", action="store_true",
                    help="also time flare_spectral (Algorithm 1 of the paper) on the workload; reported apart")
    ap.add_argument("--y-f32", action="store_true",
                    help="the forward writes y in fp32 and the backward takes delta from it (flare_shape.y_f32)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--machine-rates", action="store_true",
                    help="run the machine-rate micro-benchmarks of libflare_rates.so instead of the workload and "
                         "print their table (the rates the issue bound and the exponential ceiling are priced with)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run three plain device copies of k (known size) first, for scaling profiler counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding across GPUs); "
              "--gpus %d is not supported.  Run with --gpus 1." % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2508_12594_amd import binding, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    if args.machine_rates:
        from paper_2508_12594_amd import rates
        rows = rates.run_all()
        for r in rows:
            print("%-100s waves/SIMD %d param %2d: %9.4f ms  %7s clk/instr  %6.0f MHz %s" % (
                r["experiment"], r["waves_per_simd"], r["param"], r["ms"], r.get("clk_per_instr", "-"),
                r["shader_mhz"], ("%.0f GB/s" % r["GBps"]) if "GBps" in r else ""), file=sys.stderr, flush=True)
        print(json.dumps({"machine_rates": rows}), flush=True)
        return
    binding.load()

    over = {} if args.tokens is None else {"N": args.tokens}
    if args.latents is not None:
        over["M"] = args.latents
    if args.head_dim is not None:
        over["d"] = args.head_dim
    if args.dtype is not None:
        over["dtype"] = args.dtype
    inp = synth.make_inputs(args.cfg, with_dy=True, **over)
    B, H, N, M, d = (inp[x] for x in "BHNMd")
    dt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[inp["dtype"]]
    elem = 4 if inp["dtype"] == "f32" else 2
    dev = {n: torch.from_numpy(inp[n]).to("cuda", dt).contiguous() for n in ("q", "k", "v", "dy")}
    if args.layout == "bnhd":
        for n in ("k", "v", "dy"):
            dev[n] = dev[n].permute(0, 2, 1, 3).contiguous()
    lay = args.layout
    scale = inp["scale"]
    code = {"f32": binding.FLARE_F32, "bf16": binding.FLARE_BF16, "f16": binding.FLARE_F16}[inp["dtype"]]
    fwd_b, bwd_b = binding.workspace_bytes(B, H, N, M, d, code, args.y_f32)
    ws = torch.empty(max(fwd_b, bwd_b, 256), dtype=torch.uint8, device="cuda")
    y = torch.empty_like(dev["k"], dtype=torch.float32) if args.y_f32 else torch.empty_like(dev["k"])
    z = torch.empty((B, H, M, d), dtype=torch.float32, device="cuda")
    lse = torch.empty((B, H, M), dtype=torch.float32, device="cuda")
    lse_dec = torch.empty((B, H, N), dtype=torch.float32, device="cuda")
    dq = torch.empty((H, M, d), dtype=torch.float32, device="cuda")
    dk = torch.empty_like(dev["k"])
    dv = torch.empty_like(dev["k"])

    def fwd():
        binding.forward(dev["q"], dev["k"], dev["v"], scale, y=y, z=z, lse_enc=lse, lse_dec=lse_dec, workspace=ws,
                        layout=lay)

    def step():   # a training step: the forward saves z, lse_enc, lse_dec and y for the backward
        fwd()
        binding.backward(dev["q"], dev["k"], dev["v"], dev["dy"], z, lse, scale, y=y, lse_dec=lse_dec,
                         dq_lat=dq, dk=dk, dv=dv, workspace=ws, layout=lay)

    def timed(fn, steps):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    if args.copy_calibration:
        for _ in range(3):
            y.copy_(dev["k"])                 # reads and writes B*H*N*d*elem bytes each
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    t_step = timed(step, args.steps)          # the headline: forward + backward
    t_fwd = timed(fwd, args.steps)            # forward alone

    # per-kernel durations: HIP events recorded by the library on the launch stream, same K steps
    prof_steps = min(args.steps, 400)         # the library keeps at most 8192 event pairs
    binding.profile_enable(True)
    t_step_prof = timed(step, prof_steps)
    prof = binding.profile_read()
    binding.profile_enable(False)

    kernels = {}
    for name, (ms, cnt) in prof.items():
        mean_s = ms / cnt * 1e-3
        # beyond 256 latents a kernel is launched once per chunk of latents (or the backward launches it for the
        # statistics and again for dZ): bytes and exponentials are the whole operation's, so is the time
        per_step_s = mean_s * max(1, cnt // prof_steps)
        ab = algorithmic_bytes(name, B, H, N, M, d, elem)
        ex = exponentials(name, B, H, N, M)
        twin = name[:-5] if name.endswith("_2exp") else name + "_2exp"
        twin_ms = prof[twin][0] / prof[twin][1] if twin in prof else 0.0
        if ms / cnt < 0.05 * twin_ms or (ms / cnt < 0.010 and ms / cnt < 0.3 * twin_ms):
            ab, ex = None, 0     # launched, but every (b,h) slice went to the other variant: it left at once
        kernels[name] = {"mean_us": round(mean_s * 1e6, 2), "launches_per_step": cnt // prof_steps,
                         "algorithmic_GBps": (round(ab / per_step_s / 1e9, 1) if ab else None),
                         "hbm_frac": (round(ab / per_step_s / 1e9 / HBM_PEAK_GBS, 4) if ab else None),
                         "exp_Gops": (round(ex / per_step_s / 1e9, 1) if ex else None),
                         "exp_frac": (round(ex / per_step_s / 1e9 / EXP_PEAK_GOPS, 4) if ex else None)}
    streaming = {n: v for n, v in kernels.items() if v["algorithmic_GBps"] is not None}
    dom = max(streaming, key=lambda n: streaming[n]["mean_us"] * streaming[n]["launches_per_step"])
    dom_bytes = algorithmic_bytes(dom, B, H, N, M, d, elem)
    dom_exps = exponentials(dom, B, H, N, M)
    dom_s = kernels[dom]["mean_us"] * 1e-6 * max(1, kernels[dom]["launches_per_step"])
    default_workload = (args.cfg == 4 and args.tokens is None and args.latents is None and args.head_dim is None
                        and args.dtype is None and not args.y_f32)
    traffic = sum(MEASURED_TRAFFIC_CFG4[dom]) if default_workload and dom in MEASURED_TRAFFIC_CFG4 else None
    # the roofline that binds this kernel: whichever lower bound on its duration is larger
    if dom_exps / (EXP_PEAK_GOPS * 1e9) > dom_bytes / (HBM_PEAK_GBS * 1e9):
        roofline = {"kernel": dom, "bound": "alu", "achieved": round(dom_exps / dom_s / 1e9, 1),
                    "peak": EXP_PEAK_GOPS, "unit": "Gop/s (v_exp_f32 lane-ops)",
                    "frac": round(dom_exps / dom_s / 1e9 / EXP_PEAK_GOPS, 4), "traffic": traffic,
                    "ops_per_launch": dom_exps, "mean_us": kernels[dom]["mean_us"],
                    "hbm": {"achieved": round(dom_bytes / dom_s / 1e9, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                            "frac": round(dom_bytes / dom_s / 1e9 / HBM_PEAK_GBS, 4),
                            "bytes_per_launch": dom_bytes}}
    else:
        roofline = {"kernel": dom, "bound": "hbm", "achieved": round(dom_bytes / dom_s / 1e9, 1),
                    "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(dom_bytes / dom_s / 1e9 / HBM_PEAK_GBS, 4), "traffic": traffic,
                    "bytes_per_launch": dom_bytes, "mean_us": kernels[dom]["mean_us"]}

    tokens = B * N
    fwd_bytes = 4 * B * H * N * d * elem       # k twice, v once, y once
    fwd_flops = 8.0 * B * H * N * M * d
    out = {
        "metric": "FLARE fwd+bwd tokens/sec at N=%d, M=%d (one MI355X)" % (N, M),
        "value": round(tokens / t_step, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(t_step * 1e3, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": inp["dtype"], "data": "synthetic",
        "config": {"workload": synth.describe(args.cfg) + ("" if args.tokens is None else " [N overridden to %d]" % N)
                   + ("" if args.latents is None else " [M overridden to %d]" % M)
                   + ("" if args.head_dim is None else " [d overridden to %d]" % d)
                   + ("" if args.dtype is None else " [storage type overridden to %s]" % args.dtype)
                   + (" [y in fp32]" if args.y_f32 else ""),
                   "step": "flare_forward + flare_backward", "B": B, "H": H, "N": N, "M": M, "d": d,
                   "layout": "[B,H,N,d]" if lay == "bhnd" else "[B,N,H,d]"},
        "fwd": {"tokens_per_s": round(tokens / t_fwd, 1), "ms": round(t_fwd * 1e3, 4),
                "hbm_frac": round(fwd_bytes / t_fwd / 1e9 / HBM_PEAK_GBS, 4),
                "mfma_frac": round(fwd_flops / t_fwd / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                "exp_frac": round(2.0 * B * H * N * M / t_fwd / 1e9 / EXP_PEAK_GOPS, 4)},
        "ms_per_step_with_events": round(t_step_prof * 1e3, 4),
        "roofline": roofline, "kernels": kernels,
    }

    if args.spectral:     # not part of the step: the eigen-analysis of the same heads, from what the forward saved
        fwd()
        binding.spectral(dev["q"], dev["k"], lse, lse_dec, scale, layout=lay)      # warm-up
        binding.profile_enable(True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        binding.spectral(dev["q"], dev["k"], lse, lse_dec, scale, layout=lay)
        torch.cuda.synchronize()
        t_sp = time.perf_counter() - t0
        prof_sp = binding.profile_read()
        binding.profile_enable(False)
        out["spectral"] = {"ms": round(t_sp * 1e3, 3),
                           "kernels_us": {n: round(ms / cnt * 1e3, 1) for n, (ms, cnt) in prof_sp.items()
                                          if n.startswith("spectral")},
                           "gram_exp_frac": round(B * H * N * M / (prof_sp["spectral_gram"][0] * 1e-3)
                                                  / 1e9 / EXP_PEAK_GOPS, 4)}

    if not args.no_cpu_baseline:
        from oracle import flare_oracle
        n_s = min(N, 1 << 20)
        h_s = min(H, 4)    # about 10 s of work on 16 host threads at the headline workload
        sub = {n: inp[n][:1, :h_s, :n_s] for n in ("k", "v", "dy")}
        q1 = inp["q"][:h_s]
        t0 = time.perf_counter()
        flare_oracle.forward(q1, sub["k"], sub["v"], scale)
        flare_oracle.backward(q1, sub["k"], sub["v"], sub["dy"], scale)
        t_cpu = time.perf_counter() - t0
        out["cpu_baseline"] = {
            "value": round(n_s * h_s / (t_cpu * H), 1), "unit": "tokens/s", "cores": flare_oracle.threads(),
            "kind": "oracle",
            "sample": "fp64 oracle forward+backward on the first %d head(s), first %d tokens, M=%d, d=%d "
                      "(%.1f s); rate scaled to all H=%d heads" % (h_s, n_s, M, d, t_cpu, H)}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
