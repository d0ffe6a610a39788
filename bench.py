#!/usr/bin/env python3
"""Benchmark of the FLARE mixer on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--cfg 4] [--no-cpu-baseline] [--no-other-configs]
    python bench.py --machine-rates

A step is one pass of the whole hot path -- flare_forward (encode partials, merge, decode)
followed by flare_backward -- over one batch of the synthetic million-token mesh workload
(B=1, H=8, d=16, N=1,000,000, M=256, bf16 storage, fp32 accumulation).  Inputs are resident in
HBM before the timed region.  One JSON line is printed:
  value, ms_per_step   W untimed warm-up steps, then exactly K steps between two device synchronisations
  timing               the same step (and the forward alone) timed per call with a pair of events on the
                       launch stream: median and minimum, warm, and cold (1 GiB written between the calls
                       so that nothing of the token tensors is left in the L2s or the memory-side cache)
  the benchmark spec           encode + decode against the HBM and MFMA rooflines (the fraction the target of 0.60
                       is defined on), beside the instruction-issue bound of the same two kernels
  roofline             the dominant kernel (most time per step) against the roofline that binds it: HBM
                       (algorithmic bytes per launch / mean duration) or, where the softmax's exponentials
                       need longer than the bytes, the vector ALUs' v_exp_f32 rate ("alu"); durations are
                       measured with HIP events on the launch stream
  kernels              per kernel of the step: mean duration, algorithmic GB/s, exponentials/s, and issue_frac =
                       (time its minimal instruction mix needs on a SIMD at the measured issue clocks) / duration
  other_configs        the other reference workloads (1, 2, 3, 5), each with its step, forward and dominant kernel
  cpu_baseline         the fp64 CPU oracle timed on a bounded sample of the same workload
"""
import argparse
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16, published
SIMDS = 256 * 4                 # compute units x SIMDs
NOMINAL_GHZ = 2.4

# Issue clocks per wave64 instruction and SIMD, in 2.4 GHz clocks, as `bench.py --machine-rates` measures them
# (profiles/machine_rates.md): v_exp_f32 8.2; v_cvt_pk_bf16_f32 (and v_max3_f32, v_perm_b32, v_dot2c_f32_bf16)
# 4.25; v_fma_f32 / v_mul_f32 2.95; one v_mfma_f32_32x32x16_bf16 beside a saturated vector stream of the same
# SIMD costs that stream 13 clocks (its own pipe 32 clocks; measured 8.5 ... 17 from sparse to dense), a
# v_mfma_f32_16x16x32_bf16 half of that.
CLK = {"exp": 8.2, "pack": 4.25, "fma": 2.95, "mfma32_issue": 13.0, "mfma32_pipe": 32.0}

# The softmax's exponentials at the v_exp_f32 rate: 1024 SIMDs x 64 lanes / 8.15 clocks x 2.4 GHz.
EXP_PEAK_GOPS = SIMDS * 64 / CLK["exp"] * NOMINAL_GHZ


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
        "bwd_dkdv_2exp": 5 * row + 8,
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
                "bwd_dq_partial": 1, "bwd_dkdv": 1, "bwd_dkdv_2exp": 2}
    return per_pair.get(kernel, 0) * B * H * N * M


def issue_clocks_per_tile(kernel, d, fused_dq):
    """Issue clocks one SIMD needs for the minimal instruction mix of one 32 x 32 tile of scores (16 scores per
    lane): per score one exponential and half a pack of two weights, plus the matrix instructions that are
    algorithmic for the kernel at this head dimension (score products with the hi + lo pair of q', value
    products; at d <= 8 the pair rides in one product), each at what it costs the vector stream.  None: a kernel
    without a softmax tile."""
    ks = 2 if d == 32 else 1                     # k-steps of a score product; column groups of a value product
    score = ks * (1 if d <= 8 else 2)            # hi + lo
    value = 2 * ks                               # 32 contraction slots = two k-steps, per column group
    mix = {
        "encode_partial": (16, 8, 0, score + value),
        "decode": (16, 8, 0, score + value),
        "bwd_token_stats": (16, 8, 0, score + value),
        "bwd_dz_partial": (16, 8, 0, score + value),
        # dS = P (a + w u c): per score one exponential, two multiply-adds, a pack of P and a pack of dS
        "bwd_dq_partial": (16, 16, 32, score + 2 * ks + value),                       # scores, a, c, dS.K
        "bwd_dkdv": (16, 16, 32, score + 2 * ks + 2 * value + (1 if fused_dq else 0)),  # + dV, dK (, dQ: 16-row products)
    }
    mix["bwd_dkdv_2exp"] = (32,) + mix["bwd_dkdv"][1:]
    if kernel not in mix:
        return None
    n_exp, n_pack, n_fma, n_mfma = mix[kernel]
    vector = n_exp * CLK["exp"] + n_pack * CLK["pack"] + n_fma * CLK["fma"] + n_mfma * CLK["mfma32_issue"]
    return max(vector, n_mfma * CLK["mfma32_pipe"])


def measured_traffic(kernel):
    """HBM bytes per launch (fetch + write) of the default workload's kernels, as two `rocprofv3 --pmc` runs
    counted them (FETCH_SIZE, then WRITE_SIZE, scaled by a plain copy of known size): read from the json block of
    the tracked summary profiles/forward_backward_cfg4_hbm_traffic.md.  None when the file has no entry."""
    path = os.path.join(ROOT, "profiles", "forward_backward_cfg4_hbm_traffic.md")
    try:
        m = re.search(r"```json\s*(\{.*?\})\s*```", open(path).read(), re.S)
        table = json.loads(m.group(1))["bytes_per_launch"]
        return float(table[kernel]["fetch"]) + float(table[kernel]["write"])
    except (OSError, AttributeError, KeyError, ValueError):
        return None


def event_times(fn, iters, between=None):
    """Per-call durations in ms: a pair of events on the current stream around every call of fn."""
    import torch
    pairs = []
    for _ in range(iters):
        if between is not None:
            between()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        pairs.append((e0, e1))
    torch.cuda.synchronize()
    return [a.elapsed_time(b) for a, b in pairs]


def stats(ms):
    return {"median_ms": round(statistics.median(ms), 4), "min_ms": round(min(ms), 4), "calls": len(ms)}


def run_workload(cfg, args, steps, warmup, primary):
    """Times one reference workload; returns (summary dict, inputs on the host)."""
    import torch
    from paper_2508_12594_amd import binding, synth

    over = {}
    if primary:
        if args.tokens is not None:
            over["N"] = args.tokens
        if args.latents is not None:
            over["M"] = args.latents
        if args.head_dim is not None:
            over["d"] = args.head_dim
        if args.dtype is not None:
            over["dtype"] = args.dtype
    inp = synth.make_inputs(cfg, with_dy=True, **over)
    B, H, N, M, d = (inp[x] for x in "BHNMd")
    dt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[inp["dtype"]]
    elem = 4 if inp["dtype"] == "f32" else 2
    dev = {n: torch.from_numpy(inp[n]).to("cuda", dt).contiguous() for n in ("q", "k", "v", "dy")}
    lay = args.layout if primary else "bhnd"
    y_f32 = args.y_f32 and primary
    if lay == "bnhd":
        for n in ("k", "v", "dy"):
            dev[n] = dev[n].permute(0, 2, 1, 3).contiguous()
    scale = inp["scale"]
    code = {"f32": binding.FLARE_F32, "bf16": binding.FLARE_BF16, "f16": binding.FLARE_F16}[inp["dtype"]]
    fwd_b, bwd_b = binding.workspace_bytes(B, H, N, M, d, code, y_f32)
    ws = torch.empty(max(fwd_b, bwd_b, 256), dtype=torch.uint8, device="cuda")
    y = torch.empty_like(dev["k"], dtype=torch.float32) if y_f32 else torch.empty_like(dev["k"])
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

    def timed(fn, n):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n

    if primary and args.copy_calibration:
        for _ in range(3):
            y.copy_(dev["k"])                 # reads and writes B*H*N*d*elem bytes each
        torch.cuda.synchronize()
    for _ in range(warmup):
        step()
    t_step = timed(step, steps)               # the headline: forward + backward, K steps between two synchronisations
    t_fwd = timed(fn=fwd, n=steps)            # forward alone

    # per call, with events on the launch stream (the library enqueues on torch's current stream)
    n_ev = min(steps, 200)
    timing = {"step_warm": stats(event_times(step, n_ev)), "fwd_warm": stats(event_times(fwd, n_ev))}
    if primary:
        flush = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        count = [0]

        def dirty():          # 1 GiB of writes: more than the L2s (8 x 4 MiB) and the memory-side cache (256 MiB) hold
            count[0] += 1
            flush.fill_(count[0] & 0xFF)
        timing["step_cold"] = stats(event_times(step, 20, dirty))
        timing["fwd_cold"] = stats(event_times(fwd, 20, dirty))
        del flush

    # per-kernel durations: HIP events recorded by the library on the launch stream
    prof_steps = min(steps, 400)              # the library keeps at most 8192 event pairs
    binding.profile_enable(True)
    t_step_prof = timed(step, prof_steps)
    prof = binding.profile_read()
    binding.profile_enable(False)

    fused_dq = "bwd_dq_partial" not in prof
    tiles_per_simd = B * H * ((N + 31) // 32) * ((M + 31) // 32) / SIMDS
    kernels = {}
    for name, (ms, cnt) in prof.items():
        mean_s = ms / cnt * 1e-3
        # beyond 256 latents a kernel is launched once per chunk of latents (or the backward launches it for the
        # statistics and again for dZ): bytes and exponentials are the whole operation's, so is the time
        per_step_s = mean_s * max(1, cnt // prof_steps)
        ab = algorithmic_bytes(name, B, H, N, M, d, elem)
        ex = exponentials(name, B, H, N, M)
        ic = issue_clocks_per_tile(name, d, fused_dq) if inp["dtype"] != "f32" else None
        twin = name[:-5] if name.endswith("_2exp") else name + "_2exp"
        twin_ms = prof[twin][0] / prof[twin][1] if twin in prof else 0.0
        if ms / cnt < 0.05 * twin_ms or (ms / cnt < 0.010 and ms / cnt < 0.3 * twin_ms):
            ab, ex, ic = None, 0, None     # launched, but every (b,h) slice went to the other variant: it left at once
        kernels[name] = {"mean_us": round(mean_s * 1e6, 2), "launches_per_step": cnt // prof_steps,
                         "algorithmic_GBps": (round(ab / per_step_s / 1e9, 1) if ab else None),
                         "hbm_frac": (round(ab / per_step_s / 1e9 / HBM_PEAK_GBS, 4) if ab else None),
                         "exp_Gops": (round(ex / per_step_s / 1e9, 1) if ex else None),
                         "exp_frac": (round(ex / per_step_s / 1e9 / EXP_PEAK_GOPS, 4) if ex else None),
                         "issue_frac": (round(ic * tiles_per_simd / (NOMINAL_GHZ * 1e9) / per_step_s, 4)
                                        if ic else None)}
    streaming = {n: v for n, v in kernels.items() if v["algorithmic_GBps"] is not None}
    dom = max(streaming, key=lambda n: streaming[n]["mean_us"] * streaming[n]["launches_per_step"])
    dom_bytes = algorithmic_bytes(dom, B, H, N, M, d, elem)
    dom_exps = exponentials(dom, B, H, N, M)
    dom_s = kernels[dom]["mean_us"] * 1e-6 * max(1, kernels[dom]["launches_per_step"])
    default_workload = (primary and cfg == 4 and not over and not y_f32 and lay == "bhnd")
    traffic = measured_traffic(dom) if default_workload else None
    # the roofline that binds this kernel: whichever lower bound on its duration is larger
    hbm = {"achieved": round(dom_bytes / dom_s / 1e9, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
           "frac": round(dom_bytes / dom_s / 1e9 / HBM_PEAK_GBS, 4), "bytes_per_launch": dom_bytes}
    if dom_exps / (EXP_PEAK_GOPS * 1e9) > dom_bytes / (HBM_PEAK_GBS * 1e9):
        roofline = {"kernel": dom, "bound": "alu", "achieved": round(dom_exps / dom_s / 1e9, 1),
                    "peak": round(EXP_PEAK_GOPS, 1), "unit": "Gop/s (v_exp_f32 lane-ops)",
                    "frac": round(dom_exps / dom_s / 1e9 / EXP_PEAK_GOPS, 4), "traffic": traffic,
                    "ops_per_launch": dom_exps, "mean_us": kernels[dom]["mean_us"], "hbm": hbm}
    else:
        roofline = dict(hbm, kernel=dom, bound="hbm", traffic=traffic, mean_us=kernels[dom]["mean_us"])
    if traffic is not None:
        roofline["traffic_source"] = "profiles/forward_backward_cfg4_hbm_traffic.md (rocprofv3 --pmc, not this run)"
    roofline["issue_frac"] = kernels[dom]["issue_frac"]

    tokens = B * N
    fwd_bytes = 4 * B * H * N * d * elem       # k twice, v once, y once
    fwd_flops = 8.0 * B * H * N * M * d
    t_fwd_med = timing["fwd_warm"]["median_ms"] * 1e-3
    enc_dec_s = sum(kernels[n]["mean_us"] * kernels[n]["launches_per_step"] for n in ("encode_partial", "decode")
                    if n in kernels) * 1e-6
    ic_fwd = issue_clocks_per_tile("encode_partial", d, fused_dq) if inp["dtype"] != "f32" else None
    north = {"what": "encode + decode (flare_forward, median of per-call event times, warm)",
             "ms": round(t_fwd_med * 1e3, 4),
             "hbm_frac": round(fwd_bytes / t_fwd_med / 1e9 / HBM_PEAK_GBS, 4),
             "mfma_frac": round(fwd_flops / t_fwd_med / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
             "exp_frac": round(2.0 * B * H * N * M / t_fwd_med / 1e9 / EXP_PEAK_GOPS, 4),
             "issue_frac": (round(2 * ic_fwd * tiles_per_simd / (NOMINAL_GHZ * 1e9) / enc_dec_s, 4)
                            if ic_fwd and enc_dec_s else None),
             "target_hbm_frac": 0.60}
    if "fwd_cold" in timing:
        t_cold = timing["fwd_cold"]["median_ms"] * 1e-3
        north["cold_ms"] = round(t_cold * 1e3, 4)
        north["cold_hbm_frac"] = round(fwd_bytes / t_cold / 1e9 / HBM_PEAK_GBS, 4)
    out = {
        "workload": synth.describe(cfg) + ("" if "N" not in over else " [N overridden to %d]" % N)
        + ("" if "M" not in over else " [M overridden to %d]" % M)
        + ("" if "d" not in over else " [d overridden to %d]" % d)
        + ("" if "dtype" not in over else " [storage type overridden to %s]" % over["dtype"])
        + (" [y in fp32]" if y_f32 else ""),
        "shape": {"B": B, "H": H, "N": N, "M": M, "d": d, "dtype": inp["dtype"],
                  "layout": "[B,H,N,d]" if lay == "bhnd" else "[B,N,H,d]"},
        "tokens": tokens, "t_step": t_step, "t_fwd": t_fwd, "t_step_prof": t_step_prof, "timing": timing,
        "north_star": north, "roofline": roofline, "kernels": kernels,
    }
    return out, inp, dev, (lse, lse_dec, lay, scale)


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
    ap.add_argument("--projection", action="store_true",
                    help="also time the forward with the output projection fused into the decode "
                         "(flare_forward_project, [B,N,H,d] layout) against flare_forward followed by a library GEMM")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the short runs of the other reference workloads (1, 2, 3, 5)")
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
    from paper_2508_12594_amd import binding

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
        print(json.dumps({"machine_rates": rows, "derived": rates.derive(rows)}), flush=True)
        return
    binding.load()

    res, inp, dev, (lse, lse_dec, lay, scale) = run_workload(args.cfg, args, args.steps, args.warmup, True)
    B, H, N, M, d = (res["shape"][x] for x in "BHNMd")
    t_step, t_fwd = res["t_step"], res["t_fwd"]
    fwd_bytes = 4 * B * H * N * d * (4 if res["shape"]["dtype"] == "f32" else 2)
    out = {
        "metric": "FLARE fwd+bwd tokens/sec at N=%d, M=%d (one MI355X)" % (N, M),
        "value": round(res["tokens"] / t_step, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(t_step * 1e3, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": res["shape"]["dtype"], "data": "synthetic",
        "config": dict(res["shape"], workload=res["workload"], step="flare_forward + flare_backward"),
        "fwd": {"tokens_per_s": round(res["tokens"] / t_fwd, 1), "ms": round(t_fwd * 1e3, 4),
                "hbm_frac": round(fwd_bytes / t_fwd / 1e9 / HBM_PEAK_GBS, 4),
                "mfma_frac": round(8.0 * B * H * N * M * d / t_fwd / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                "exp_frac": round(2.0 * B * H * N * M / t_fwd / 1e9 / EXP_PEAK_GOPS, 4)},
        "timing": res["timing"], "north_star": res["north_star"],
        "ms_per_step_with_events": round(res["t_step_prof"] * 1e3, 4),
        "roofline": res["roofline"], "kernels": res["kernels"],
    }

    if args.spectral:     # not part of the step: the eigen-analysis of the same heads, from what the forward saved
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
    if args.projection:   # the block's output linear layer behind the mixer: fused into the decode, or a GEMM of its own
        C = H * d
        tdt = dev["k"].dtype
        kk, vv = (dev[n] if lay == "bnhd" else dev[n].permute(0, 2, 1, 3).contiguous() for n in ("k", "v"))
        gen = torch.Generator(device="cuda").manual_seed(1)
        w_out = (torch.randn((C, C), generator=gen, device="cuda") / C ** 0.5).to(tdt)
        y_p = torch.empty_like(kk)
        out_p = torch.empty((B, N, C), dtype=tdt, device="cuda")
        z_p = torch.empty((B, H, M, d), dtype=torch.float32, device="cuda")
        l_p = torch.empty((B, H, M), dtype=torch.float32, device="cuda")
        fb, _ = binding.workspace_bytes(B, H, N, M, d, binding.FLARE_BF16 if tdt == torch.bfloat16 else binding.FLARE_F16)
        ws_p = torch.empty(max(fb, 256), dtype=torch.uint8, device="cuda")

        def separate():
            binding.forward(dev["q"], kk, vv, scale, y=y_p, z=z_p, lse_enc=l_p, workspace=ws_p, layout="bnhd")
            torch.matmul(y_p.view(B * N, C), w_out, out=out_p.view(B * N, C))

        def fused():
            binding.forward_project(dev["q"], kk, vv, w_out, scale, out=out_p, z=z_p, lse_enc=l_p, workspace=ws_p)

        def fused_keep_y():
            binding.forward_project(dev["q"], kk, vv, w_out, scale, out=out_p, y=y_p, z=z_p, lse_enc=l_p, workspace=ws_p)

        proj = {}
        for name, fn in (("forward_then_gemm", separate), ("fused", fused), ("fused_storing_y", fused_keep_y)):
            for _ in range(20):
                fn()
            proj[name] = stats(event_times(fn, 100))
        out["projection"] = proj
        del kk, vv, y_p, out_p, ws_p
    del dev, lse, lse_dec
    torch.cuda.empty_cache()

    if not args.no_other_configs and args.cfg == 4:
        others = {}
        for cfg in (1, 2, 3, 5):
            r, _, _, _ = run_workload(cfg, args, 50, 20, False)
            dom = r["roofline"]
            others["cfg%d" % cfg] = {
                "shape": r["shape"], "ms_per_step": round(r["t_step"] * 1e3, 4),
                "tokens_per_s": round(r["tokens"] / r["t_step"], 1),
                "step_median_ms": r["timing"]["step_warm"]["median_ms"], "step_min_ms": r["timing"]["step_warm"]["min_ms"],
                "fwd_median_ms": r["timing"]["fwd_warm"]["median_ms"], "fwd_hbm_frac": r["north_star"]["hbm_frac"],
                "fwd_mfma_frac": r["north_star"]["mfma_frac"], "fwd_issue_frac": r["north_star"]["issue_frac"],
                "dominant_kernel": dom["kernel"], "dominant_bound": dom["bound"], "dominant_frac": dom["frac"],
                "dominant_hbm_frac": dom["hbm"]["frac"] if "hbm" in dom else dom["frac"],
                "dominant_issue_frac": dom["issue_frac"], "dominant_us": dom["mean_us"]}
            torch.cuda.empty_cache()
        out["other_configs"] = others

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
