"""GPU parity of the shared-latent variant (flare_shape.shared_latents = 1): all heads use one latent
sequence q_lat[M,d] (the ablation of the paper's Appendix G, "Effect of head dimension and parallel
low-rank projections" / shared latents), i.e. a head stride of zero on q_lat, and dq_lat[M,d] is
summed over the heads as well as over the batch.

The oracle takes per-head queries; the test hands it the same rows for every head and adds its dq over
the heads (data movement and one sum, no method arithmetic).  A second check runs the library itself
with the queries repeated per head: y, z, dk, dv must be bit-identical, dq equal up to summation order.
"""
import sys

import numpy as np
import pytest

from paper_2508_12594_amd import binding, synth
from tests._util import slice_relerr, to_device, to_host, tol_for

pytestmark = pytest.mark.gpu

CASES = [
    # dtype, B, H, N, M, d, layout
    ("f32", 2, 3, 500, 40, 8, "bhnd"),
    ("bf16", 2, 4, 1500, 64, 16, "bhnd"),
    ("bf16", 1, 2, 700, 256, 32, "bnhd"),
    ("f16", 1, 3, 900, 128, 8, "bhnd"),
    ("bf16", 1, 2, 600, 512, 16, "bhnd"),      # two latent chunks
    ("bf16", 3, 2, 333, 192, 4, "bnhd"),       # dK/dV on the vector kernels
    ("bf16", 2, 3, 5, 96, 16, "bnhd"),         # fewer than 16 tokens: 16-bit storage on the fp32 kernels
    ("f16", 3, 2, 3, 40, 8, "bhnd"),
]


@pytest.mark.parametrize("saved", [False, True])
@pytest.mark.parametrize("dtype,B,H,N,M,d,layout", CASES)
def test_shared_latents(oracle, dtype, B, H, N, M, d, layout, saved):
    import torch
    print("[case] shared latents %s B=%d H=%d N=%d M=%d d=%d %s saved=%s" % (dtype, B, H, N, M, d, layout, saved),
          flush=True)
    sys.stdout.flush()
    inp = synth.make_inputs(2, B=B, H=H, N=N, M=M, d=d, dtype=dtype, with_dy=True, seed=4242 + N + M + d)
    q_shared = np.ascontiguousarray(inp["q"][0])                    # [M, d]
    inp["q"] = np.ascontiguousarray(np.broadcast_to(q_shared, (H, M, d)))
    scale, tol = inp["scale"], tol_for(inp)
    dev = to_device(inp)
    conv = (lambda t: t.permute(0, 2, 1, 3).contiguous()) if layout == "bnhd" else (lambda t: t)
    back = (lambda t: t.permute(0, 2, 1, 3)) if layout == "bnhd" else (lambda t: t)
    k, v, dy = conv(dev["k"]), conv(dev["v"]), conv(dev["dy"])

    def run(q):
        lse_dec = torch.empty((B, H, N), dtype=torch.float32, device="cuda") if saved else None
        y, z, lse = binding.forward(q, k, v, scale, lse_dec=lse_dec, layout=layout)
        dq, dk, dv = binding.backward(q, k, v, dy, z, lse, scale, y=y if saved else None, lse_dec=lse_dec,
                                      layout=layout)
        torch.cuda.synchronize()
        return y, z, lse, dq, dk, dv

    y, z, lse, dq, dk, dv = run(dev["q"][0].contiguous())           # one latent sequence
    assert tuple(dq.shape) == (M, d)
    y2, z2, lse2, dq2, dk2, dv2 = run(dev["q"])                     # the same rows, repeated per head
    for a, b, name in ((y, y2, "y"), (z, z2, "z"), (lse, lse2, "lse_enc"), (dk, dk2, "dk"), (dv, dv2, "dv")):
        assert torch.equal(a, b), "%s differs from the per-head run" % name
    assert slice_relerr(to_host(dq)[None], to_host(dq2).sum(axis=0)[None]) <= 1e-5

    y_ref, z_ref, lse_ref = oracle.forward(inp["q"], inp["k"], inp["v"], scale)
    dq_ref, dk_ref, dv_ref = oracle.backward(inp["q"], inp["k"], inp["v"], inp["dy"], scale)
    errs = dict(y=slice_relerr(to_host(back(y)), y_ref), z=slice_relerr(to_host(z), z_ref),
                dq=slice_relerr(to_host(dq)[None], dq_ref.sum(axis=0)[None]),
                dk=slice_relerr(to_host(back(dk)), dk_ref), dv=slice_relerr(to_host(back(dv)), dv_ref))
    print("[case]    " + "  ".join("%s %.2e" % kv for kv in errs.items()) + "  (tol %.0e)" % tol, flush=True)
    assert max(errs.values()) <= tol
    assert float(np.max(np.abs(to_host(lse) - lse_ref))) <= 1e-2


def test_shared_latents_flag_is_validated():
    import ctypes
    lib = binding.load()
    shp = binding.FlareShape(1, 1, 8, 32, 16, binding.FLARE_F32, 0, 2)
    assert lib.flare_workspace_bytes(ctypes.byref(shp), None, None) == -1
