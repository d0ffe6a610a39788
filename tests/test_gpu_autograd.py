"""The autograd wrapper returns the library's forward and routes gradients through flare_backward:
checked against the fp64 oracle's forward and backward on the same seeded inputs."""
import numpy as np
import pytest

from paper_2508_12594_amd import synth
from paper_2508_12594_amd.autograd import flare_mixer
from tests._util import slice_relerr, to_device, to_host, tol_for

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cfg,over,layout,y_f32", [(1, dict(N=600), "bhnd", False), (2, dict(B=2, N=1500), "bhnd", False),
                                                   (4, dict(N=1200, dtype="f16"), "bnhd", False),
                                                   (2, dict(B=2, N=1500, d=8), "bnhd", True)])
def test_autograd_matches_oracle(oracle, cfg, over, layout, y_f32):
    import torch
    print("[case] autograd cfg%d %s %s" % (cfg, over, layout), flush=True)
    inp = synth.make_inputs(cfg, with_dy=True, **over)
    scale, tol = inp["scale"], tol_for(inp)
    dev = to_device(inp)
    conv = (lambda t: t.permute(0, 2, 1, 3).contiguous()) if layout == "bnhd" else (lambda t: t)
    back = (lambda t: t.permute(0, 2, 1, 3)) if layout == "bnhd" else (lambda t: t)
    q = dev["q"].clone().requires_grad_(True)
    k = conv(dev["k"]).clone().requires_grad_(True)
    v = conv(dev["v"]).clone().requires_grad_(True)
    y = flare_mixer(q, k, v, scale, layout=layout, y_f32=y_f32)
    assert y.dtype == (torch.float32 if y_f32 else k.dtype)
    y.backward(conv(dev["dy"]).to(y.dtype))
    torch.cuda.synchronize()
    y_ref, _, _ = oracle.forward(inp["q"], inp["k"], inp["v"], scale)
    dq_ref, dk_ref, dv_ref = oracle.backward(inp["q"], inp["k"], inp["v"], inp["dy"], scale)
    assert q.grad.dtype == q.dtype and k.grad.shape == k.shape
    errs = dict(y=slice_relerr(to_host(back(y)), y_ref), dq=slice_relerr(to_host(q.grad), dq_ref),
                dk=slice_relerr(to_host(back(k.grad)), dk_ref), dv=slice_relerr(to_host(back(v.grad)), dv_ref))
    print("[case]    " + "  ".join("%s %.2e" % kv for kv in errs.items()), flush=True)
    # dq_lat is cast to q's dtype for autograd: one more rounding of a 16-bit type
    assert max(errs.values()) <= tol
