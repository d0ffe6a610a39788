"""GPU parity of the fp32-y option (flare_shape.y_f32): the forward writes y in fp32 and the backward takes
delta_n = <dY_n, Y_n> from that unrounded Y instead of recomputing the token statistics (d < 16) or using a
bf16 y (d >= 16).  Forward and gradients against the fp64 oracle, element by element."""
import sys

import numpy as np
import pytest

from paper_2508_12594_amd import binding, synth
from tests._util import TOL, slice_relerr, to_device, to_host

pytestmark = pytest.mark.gpu

CASES = [
    # cfg, overrides, layout
    (4, dict(N=3001), "bhnd"),                       # d = 16, M = 256, mesh-like
    (4, dict(N=2500, d=8), "bhnd"),                  # the head dimensions that otherwise recompute
    (4, dict(N=2500, d=4, M=100), "bnhd"),
    (2, dict(B=2, N=1500, d=8), "bnhd"),
    (5, dict(N=2048), "bhnd"),                       # d = 32: separate dQ kernel
    (3, dict(B=2, N=700, dtype="f16"), "bhnd"),
    (2, dict(B=1, N=20, M=7, d=8), "bhnd"),          # a single token tile, few latents
    (2, dict(B=2, H=3, N=365, M=200, d=4, seed=777 + 1375), "bhnd"),   # a latent that dominates many tokens
    (2, dict(B=1, N=1500, M=512, d=8), "bhnd"),      # more than 256 latents: fp32 partial rows per chunk of latents
    (4, dict(N=900, M=300, d=16), "bnhd"),
    (2, dict(B=1, H=2, N=700, M=1000, d=4, dtype="f16"), "bhnd"),
    # fp16 storage at d = 16: delta comes from a pass of its own, which must round dY to bf16 as the kernels do
    (2, dict(B=1, H=1, N=12, M=234, d=16, dtype="f16", seed=777 + 542), "bhnd"),
    (3, dict(B=1, N=333, M=234, d=16, dtype="f16"), "bnhd"),
    # fewer than 16 tokens: the fp32 kernels write the fp32 y, the backward recomputes the statistics
    (2, dict(B=1, H=1, N=2, M=234, d=16, dtype="f16", seed=777 + 542), "bhnd"),
    (2, dict(B=2, H=3, N=5, M=96, d=8), "bnhd"),
    (1, dict(B=1, H=2, N=7, M=300, d=32, dtype="f16"), "bhnd"),
]


@pytest.mark.parametrize("cfg,over,layout", CASES)
def test_forward_backward_with_fp32_y(oracle, cfg, over, layout):
    import torch
    print("[case] fp32 y: cfg%d %s %s" % (cfg, over, layout), flush=True)
    sys.stdout.flush()
    inp = synth.make_inputs(cfg, with_dy=True, **over)
    scale, tol = inp["scale"], TOL["bf16"]
    dev = to_device(inp)
    conv = (lambda t: t.permute(0, 2, 1, 3).contiguous()) if layout == "bnhd" else (lambda t: t)
    back = (lambda t: t.permute(0, 2, 1, 3)) if layout == "bnhd" else (lambda t: t)
    k, v, dy = conv(dev["k"]), conv(dev["v"]), conv(dev["dy"])
    lse_dec = torch.empty(dev["k"].shape[:3], dtype=torch.float32, device="cuda")
    y, z, lse = binding.forward(dev["q"], k, v, scale, lse_dec=lse_dec, layout=layout, y_f32=True)
    assert y.dtype == torch.float32 and y.shape == k.shape
    dq, dk, dv = binding.backward(dev["q"], k, v, dy, z, lse, scale, y=y, lse_dec=lse_dec, layout=layout)
    # the ordinary path on the same inputs, for comparison
    y16, _, _ = binding.forward(dev["q"], k, v, scale, layout=layout)
    dq0, dk0, dv0 = binding.backward(dev["q"], k, v, dy, z, lse, scale, layout=layout)
    torch.cuda.synchronize()
    y_ref, z_ref, _ = oracle.forward(inp["q"], inp["k"], inp["v"], scale)
    dq_ref, dk_ref, dv_ref = oracle.backward(inp["q"], inp["k"], inp["v"], inp["dy"], scale)
    errs = dict(y=slice_relerr(to_host(back(y)), y_ref), dq=slice_relerr(to_host(dq), dq_ref),
                dk=slice_relerr(to_host(back(dk)), dk_ref), dv=slice_relerr(to_host(back(dv)), dv_ref))
    base = dict(y=slice_relerr(to_host(back(y16)), y_ref), dq=slice_relerr(to_host(dq0), dq_ref),
                dk=slice_relerr(to_host(back(dk0)), dk_ref))
    print("[case]    " + "  ".join("%s %.2e" % kv for kv in errs.items()) + "   (recomputed statistics: "
          + "  ".join("%s %.2e" % kv for kv in base.items()) + ")", flush=True)
    assert max(errs.values()) <= tol
    assert errs["y"] <= base["y"] * 1.05 + 1e-6          # an unrounded y is at least as close as the rounded one
    # dV does not depend on y (only on lse_dec, saved here and recomputed there: equal up to rounding)
    assert slice_relerr(to_host(dv), to_host(dv0)) <= 1e-2


def test_fp32_y_is_refused_where_it_is_not_built():
    import torch
    inp = synth.make_inputs(2, B=1, H=1, N=100, M=2100, with_dy=False)
    dev = to_device(inp)
    with pytest.raises(binding.FlareError):
        binding.forward(dev["q"], dev["k"], dev["v"], inp["scale"], y_f32=True)      # beyond the matrix-core kernels
    inp = synth.make_inputs(1, N=300, with_dy=False)
    dev = to_device(inp)
    shp = binding._shape_of(dev["q"], dev["k"], "bhnd", True)                        # fp32 storage: y is fp32 anyway
    import ctypes
    assert binding.load().flare_workspace_bytes(ctypes.byref(shp), None, None) == -2
    torch.cuda.synchronize()


def test_decode_alone_writes_the_same_fp32_y():
    import torch
    inp = synth.make_inputs(2, B=2, N=1111, d=8, with_dy=False)
    dev = to_device(inp)
    y, z, _ = binding.forward(dev["q"], dev["k"], dev["v"], inp["scale"], y_f32=True)
    y2 = binding.decode(dev["q"], dev["k"], z, inp["scale"], y_f32=True)
    y16 = binding.decode(dev["q"], dev["k"], z, inp["scale"])
    torch.cuda.synchronize()
    assert y2.dtype == torch.float32 and torch.equal(y, y2)
    # the 16-bit y of the ordinary path is this one rounded, up to the lo part of Z that only the fp32 rows carry
    assert float((y16.float() - y).abs().max()) <= 2.0 ** -7 * float(y.abs().max())


def test_million_tokens_fp32_y_agrees_with_recomputed_statistics():
    """Full size (N = 1,000,000, M = 256, H = 8, d = 8, the launch configuration of bench.py --head-dim 8 --y-f32):
    the gradients from the fp32 y against those from the recomputed statistics, which the full-size tests
    check against the oracle."""
    import torch
    inp = synth.make_inputs(4, with_dy=True, d=8)
    dev = to_device(inp)
    scale = inp["scale"]
    lse_dec = torch.empty(dev["k"].shape[:3], dtype=torch.float32, device="cuda")
    y, z, lse = binding.forward(dev["q"], dev["k"], dev["v"], scale, lse_dec=lse_dec, y_f32=True)
    dq, dk, dv = binding.backward(dev["q"], dev["k"], dev["v"], dev["dy"], z, lse, scale, y=y, lse_dec=lse_dec)
    dq0, dk0, dv0 = binding.backward(dev["q"], dev["k"], dev["v"], dev["dy"], z, lse, scale)
    torch.cuda.synchronize()
    rel = lambda a, b: float((a.double() - b.double()).norm() / b.double().norm())
    errs = (rel(dq, dq0), rel(dk, dk0), rel(dv, dv0))
    print("[case]    fp32 y against recomputed statistics at N = 10^6: dq %.2e dk %.2e dv %.2e" % errs, flush=True)
    assert max(errs) <= 5e-3
