"""GPU parity on seeded random shapes: every storage type, both layouts of the token tensors, with and
without the forward's saved statistics, scales other than 1/sqrt(d).

Each case draws (B, H, N, M, d) from ranges that cross the tile sizes of every kernel (32-token tiles,
32/64/256-latent groups, chunk boundaries of the token split) and compares forward and backward with the
fp64 oracle element by element.  The outputs live inside larger buffers whose margins are filled with a
sentinel and checked afterwards, so a store outside an output tensor fails the case.
"""
import sys

import numpy as np
import pytest

from paper_2508_12594_amd import binding, synth
from tests._util import slice_relerr, to_device, to_host, tol_for

pytestmark = pytest.mark.gpu

MATRIX_M = [32, 64, 128, 192, 256, 512]
HEAD_DIMS = [4, 8, 16, 32]


def _draw_case(i):
    rng = np.random.Generator(np.random.PCG64(90210 + i))
    dtype = ["f32", "bf16", "f16"][i % 3]
    d = int(HEAD_DIMS[rng.integers(0, 4)])
    if dtype != "f32" and rng.random() < 0.7:
        M = int(MATRIX_M[rng.integers(0, len(MATRIX_M))])         # matrix-core shapes
    else:
        M = int(rng.integers(1, 300))                             # anything: vector kernels
    B = int(rng.integers(1, 4))
    H = int(rng.integers(1, 4))
    top = 2600 if M <= 256 else 900
    N = int(rng.integers(1, top)) if rng.random() < 0.85 else int(rng.integers(1, 70))
    layout = "bnhd" if rng.random() < 0.4 else "bhnd"
    saved = bool(rng.random() < 0.5)
    gain = float(rng.choice([0.5, 1.0, 1.0, 2.0]))               # scale = gain / sqrt(d)
    kind = 2 if rng.random() < 0.5 else 1                        # mesh-like or normal inputs
    return dict(i=i, dtype=dtype, B=B, H=H, N=N, M=M, d=d, layout=layout, saved=saved, gain=gain, kind=kind)


CASES = [_draw_case(i) for i in range(128)]
SENTINEL = 12288.0   # exactly representable in fp32, bf16 and fp16


def _guarded(shape, dtype, device):
    """A tensor of `shape` carved out of the middle of a sentinel-filled buffer (16-byte aligned)."""
    import torch
    n = int(np.prod(shape))
    pad = 64
    buf = torch.full((n + 2 * pad,), SENTINEL, dtype=dtype, device=device)
    return buf, buf[pad:pad + n].view(*shape)


def _margins_intact(buf, n):
    pad = 64
    return bool((buf[:pad] == SENTINEL).all().item()) and bool((buf[pad + n:] == SENTINEL).all().item())


@pytest.mark.parametrize("case", CASES, ids=lambda c: "%(i)d-%(dtype)s-B%(B)dH%(H)dN%(N)dM%(M)dd%(d)d-%(layout)s" % c)
def test_random_shape(oracle, case):
    import torch
    print("[case] random shape %s" % (case,), flush=True)
    sys.stdout.flush()
    c = case
    inp = synth.make_inputs(c["kind"], B=c["B"], H=c["H"], N=c["N"], M=c["M"], d=c["d"], dtype=c["dtype"],
                            with_dy=True, seed=777 + c["i"])
    scale = c["gain"] / np.sqrt(c["d"])
    tol = tol_for(inp)
    dev = to_device(inp)
    conv = (lambda t: t.permute(0, 2, 1, 3).contiguous()) if c["layout"] == "bnhd" else (lambda t: t)
    back = (lambda t: t.permute(0, 2, 1, 3)) if c["layout"] == "bnhd" else (lambda t: t)
    k, v, dy = conv(dev["k"]), conv(dev["v"]), conv(dev["dy"])
    B, H, N, M, d = c["B"], c["H"], c["N"], c["M"], c["d"]
    f32 = torch.float32
    ybuf, y = _guarded(k.shape, k.dtype, "cuda")
    zbuf, z = _guarded((B, H, M, d), f32, "cuda")
    lbuf, lse = _guarded((B, H, M), f32, "cuda")
    ldbuf, lse_dec = _guarded((B, H, N), f32, "cuda")
    dqbuf, dq = _guarded((H, M, d), f32, "cuda")
    dkbuf, dk = _guarded(k.shape, k.dtype, "cuda")
    dvbuf, dv = _guarded(k.shape, k.dtype, "cuda")
    binding.forward(dev["q"], k, v, scale, y=y, z=z, lse_enc=lse, lse_dec=lse_dec if c["saved"] else None,
                    layout=c["layout"])
    binding.backward(dev["q"], k, v, dy, z, lse, scale, y=y if c["saved"] else None,
                     lse_dec=lse_dec if c["saved"] else None, dq_lat=dq, dk=dk, dv=dv, layout=c["layout"])
    torch.cuda.synchronize()
    for name, buf, t in (("y", ybuf, y), ("z", zbuf, z), ("lse_enc", lbuf, lse), ("dq", dqbuf, dq),
                         ("dk", dkbuf, dk), ("dv", dvbuf, dv)):
        assert _margins_intact(buf, t.numel()), "store outside %s" % name
    if c["saved"]:
        assert _margins_intact(ldbuf, lse_dec.numel()), "store outside lse_dec"
    else:
        assert bool((ldbuf == SENTINEL).all().item()), "lse_dec written although not asked for"

    y_ref, z_ref, lse_ref = oracle.forward(inp["q"], inp["k"], inp["v"], scale)
    dq_ref, dk_ref, dv_ref = oracle.backward(inp["q"], inp["k"], inp["v"], inp["dy"], scale)
    errs = dict(y=slice_relerr(to_host(back(y)), y_ref), z=slice_relerr(to_host(z), z_ref),
                dv=slice_relerr(to_host(back(dv)), dv_ref))
    if N > 1:   # with one token both softmaxes are constant in q and k: dq = dk = 0 exactly
        errs["dq"] = slice_relerr(to_host(dq), dq_ref)
        errs["dk"] = slice_relerr(to_host(back(dk)), dk_ref)
    else:
        ref = float(np.linalg.norm(dv_ref))
        errs["dq"] = float(np.linalg.norm(to_host(dq))) / ref
        errs["dk"] = float(np.linalg.norm(to_host(dk))) / ref
    e_l = float(np.max(np.abs(to_host(lse) - lse_ref)))
    print("[case]    " + "  ".join("%s %.2e" % kv for kv in errs.items()) + "  lse %.2e  (tol %.0e)" % (e_l, tol),
          flush=True)
    # Forward outputs and dV: the bar of the workloads.  dQ and dK at twice the usual score scale: the
    # softmaxes are sharp, so where a latent attends to few tokens a - eps = <dZ_m, V_n - Z_m> (and
    # c - delta likewise) is a small difference of large terms, and the error that z, lse_enc and y
    # already carry from the forward (bf16 weights; within their own bar) is amplified in the
    # gradients: measured up to 2.1e-2 (bf16, N = 11 and N = 60 tokens) and 1.9e-5 (fp32; a plain
    # fp32 numpy evaluation of the same formulas gives 1.4e-5 on that case).  2.5 x the bar there.
    grad_tol = tol * (2.5 if c["gain"] > 1.0 else 1.0)
    assert max(errs["y"], errs["z"], errs["dv"]) <= tol
    assert max(errs["dq"], errs["dk"]) <= grad_tol
    assert e_l <= (5e-3 if tol >= 1e-2 else 1e-5) + 1e-5 * float(np.max(np.abs(lse_ref)))
