"""GPU parity at the full sizes of the five workloads, in the launch configuration bench.py
times (same entry points, same shapes).

Where the oracle finishes the whole workload in seconds (configs 1-3) every element is
compared.  For the million-token forward (config 4) and the 262k-token forward+backward
(config 5) the oracle computes, for EVERY head, the full latent sequence Z, lse_enc and
dq_lat (these need every token) and Y, dK, dV on sampled tokens (first and last tiles, the
ragged tail, and random tokens); properties that hold at any size cover the other tokens.
Next to every normwise error stands the worst row (tests._util.row_relerr).
"""
import sys

import numpy as np
import pytest

from paper_2508_12594_amd import binding, synth
from tests._util import ROW_FACTOR, TOL, row_relerr, slice_relerr, to_device, to_host, tol_for

pytestmark = pytest.mark.gpu


def _say(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


def _sample_tokens(N, n_random, seed):
    rng = np.random.default_rng(seed)
    edge = np.concatenate([np.arange(0, min(N, 96)), np.arange(max(0, N - 96), N)])
    return np.unique(np.concatenate([edge, rng.integers(0, N, n_random)]))


@pytest.mark.parametrize("cfg", [1, 2, 3])
def test_forward_full_every_element(oracle, cfg):
    import torch
    _say("full forward cfg%d: %s" % (cfg, synth.describe(cfg)))
    inp = synth.make_inputs(cfg, with_dy=False)
    dev = to_device(inp)
    y, z, lse = binding.forward(dev["q"], dev["k"], dev["v"], inp["scale"])
    torch.cuda.synchronize()
    y_ref, z_ref, lse_ref = oracle.forward(inp["q"], inp["k"], inp["v"], inp["scale"])
    tol = TOL[inp["dtype"]]
    e_y, e_z = slice_relerr(to_host(y), y_ref), slice_relerr(to_host(z), z_ref)
    e_l = float(np.max(np.abs(to_host(lse) - lse_ref)))
    r_y, r_z = row_relerr(to_host(y), y_ref), row_relerr(to_host(z), z_ref)
    _say("   err y %.3e  z %.3e  lse(abs) %.3e  (tol %.0e); worst row y %.3e  z %.3e" % (e_y, e_z, e_l, tol, r_y, r_z))
    assert e_y <= tol and e_z <= tol and e_l <= 1e-2
    assert max(r_y, r_z) <= ROW_FACTOR * tol


def test_forward_million_tokens(oracle):
    """Config 4: B=1, H=8, d=16, N=1,000,000, M=256, bf16."""
    import torch
    _say("full forward cfg4: " + synth.describe(4))
    inp = synth.make_inputs(4, with_dy=False)
    N, scale, tol = inp["N"], inp["scale"], TOL["bf16"]
    dev = to_device(inp)
    y, z, lse = binding.forward(dev["q"], dev["k"], dev["v"], scale)
    torch.cuda.synchronize()
    y_h, z_h, lse_h = to_host(y), to_host(z), to_host(lse)
    assert np.isfinite(y_h).all() and np.isfinite(z_h).all() and np.isfinite(lse_h).all()
    tok = _sample_tokens(N, 4096, 4)
    for h in range(inp["H"]):
        _say("   oracle on head %d (all tokens for Z, %d sampled tokens for Y)" % (h, tok.size))
        y_ref, z_ref, lse_ref = oracle.forward(inp["q"][h:h + 1], inp["k"][:, h:h + 1], inp["v"][:, h:h + 1],
                                               scale, tok=tok)
        e_z = slice_relerr(z_h[:, h:h + 1], z_ref)
        e_y = slice_relerr(y_h[:, h:h + 1, tok], y_ref)
        e_l = float(np.max(np.abs(lse_h[:, h:h + 1] - lse_ref)))
        r_y, r_z = row_relerr(y_h[:, h:h + 1, tok], y_ref), row_relerr(z_h[:, h:h + 1], z_ref)
        _say("   head %d: err y %.3e  z %.3e  lse(abs) %.3e  (tol %.0e); worst row y %.3e  z %.3e"
             % (h, e_y, e_z, e_l, tol, r_y, r_z))
        assert e_y <= tol and e_z <= tol and e_l <= 1e-2
        assert max(r_y, r_z) <= ROW_FACTOR * tol
    # a property that holds at any size: every output row is a convex combination of the rows of Z
    zmin = torch.from_numpy(z_h.min(axis=2, keepdims=True)).cuda()
    zmax = torch.from_numpy(z_h.max(axis=2, keepdims=True)).cuda()
    slack = 2.0 ** -7 * torch.maximum(zmin.abs(), zmax.abs()) + 1e-6
    yf = y.float()
    assert bool(((yf >= zmin - slack) & (yf <= zmax + slack)).all())


def test_forward_backward_262k(oracle):
    """Config 5: B=1, H=8, d=32, N=262,144, M=256, bf16, gradients dq_lat, dK, dV."""
    import torch
    _say("full forward+backward cfg5: " + synth.describe(5))
    inp = synth.make_inputs(5, with_dy=True)
    N, scale, tol = inp["N"], inp["scale"], TOL["bf16"]
    dev = to_device(inp)
    lse_dec = torch.empty(dev["k"].shape[:3], dtype=torch.float32, device="cuda")
    y, z, lse = binding.forward(dev["q"], dev["k"], dev["v"], scale, lse_dec=lse_dec)
    dq, dk, dv = binding.backward(dev["q"], dev["k"], dev["v"], dev["dy"], z, lse, scale, y=y, lse_dec=lse_dec)
    torch.cuda.synchronize()
    y_h, z_h, dq_h, dk_h, dv_h = (to_host(t) for t in (y, z, dq, dk, dv))
    for t in (y_h, z_h, dq_h, dk_h, dv_h):
        assert np.isfinite(t).all()
    # dV = W^T dY with W row-stochastic: summed over tokens it equals the sum of dY (any size)
    s_dv = dv_h.astype(np.float64).sum(axis=2)
    s_dy = inp["dy"].astype(np.float64).sum(axis=2)
    assert np.abs(s_dv - s_dy).max() <= 2e-2 * np.sqrt(N)
    tok = _sample_tokens(N, 2048, 5)
    for h in range(inp["H"]):
        _say("   oracle on head %d (all tokens for Z and dq, %d sampled tokens for Y, dK, dV)" % (h, tok.size))
        sl = (slice(None), slice(h, h + 1))
        y_ref, z_ref, _ = oracle.forward(inp["q"][h:h + 1], inp["k"][sl], inp["v"][sl], scale, tok=tok)
        dq_ref, dk_ref, dv_ref = oracle.backward(inp["q"][h:h + 1], inp["k"][sl], inp["v"][sl], inp["dy"][sl],
                                                 scale, tok=tok)
        errs = dict(y=slice_relerr(y_h[:, h:h + 1, tok], y_ref), z=slice_relerr(z_h[sl], z_ref),
                    dq=slice_relerr(dq_h[h:h + 1], dq_ref), dk=slice_relerr(dk_h[:, h:h + 1, tok], dk_ref),
                    dv=slice_relerr(dv_h[:, h:h + 1, tok], dv_ref))
        rows = dict(y=row_relerr(y_h[:, h:h + 1, tok], y_ref), dq=row_relerr(dq_h[h:h + 1], dq_ref),
                    dk=row_relerr(dk_h[:, h:h + 1, tok], dk_ref), dv=row_relerr(dv_h[:, h:h + 1, tok], dv_ref))
        _say("   head %d: " % h + "  ".join("%s %.3e" % kv for kv in errs.items()) + "  (tol %.0e); worst rows " % tol
             + "  ".join("%s %.3e" % kv for kv in rows.items()))
        assert max(errs.values()) <= tol
        assert max(rows.values()) <= ROW_FACTOR * tol


MILLION_VARIANTS = [
    # overrides of config 4, saved statistics, bnhd layout
    (dict(), True, False),
    (dict(), False, False),
    (dict(dtype="f16"), True, False),             # the paper's autocast type on the matrix cores
    (dict(M=200), True, False),                   # 56 padding latents in the last tiles
    (dict(d=8), False, True),                     # the paper's head dimension for PDE meshes, token-major layout
    (dict(M=512, H=2, d=8), True, False),         # two latent chunks
    (dict(dtype="f32", M=64), True, False),       # the fp32 vector kernels: sums of 10^6 terms within 1e-5
]


@pytest.mark.parametrize("over,saved,bnhd", MILLION_VARIANTS)
def test_forward_backward_million_tokens(oracle, over, saved, bnhd):
    """The step bench.py times: config 4 (N = 1,000,000, M = 256, d = 16) forward + backward, with the
    forward's y and lse_dec handed to the backward (saved) or recomputed; and variants of it (storage
    type, number of latents, head dimension, layout) at the same million tokens."""
    import torch
    _say("full forward+backward cfg4 %s saved=%s bnhd=%s" % (over, saved, bnhd))
    inp = synth.make_inputs(4, with_dy=True, **over)
    N, scale, tol = inp["N"], inp["scale"], tol_for(inp)
    dev = to_device(inp)
    layout = "bnhd" if bnhd else "bhnd"
    conv = (lambda t: t.permute(0, 2, 1, 3).contiguous()) if bnhd else (lambda t: t)
    back = (lambda t: t.permute(0, 2, 1, 3)) if bnhd else (lambda t: t)
    k, v, dy = conv(dev["k"]), conv(dev["v"]), conv(dev["dy"])
    lse_dec = torch.empty(dev["k"].shape[:3], dtype=torch.float32, device="cuda") if saved else None
    y, z, lse = binding.forward(dev["q"], k, v, scale, lse_dec=lse_dec, layout=layout)
    dq, dk, dv = binding.backward(dev["q"], k, v, dy, z, lse, scale, y=y if saved else None, lse_dec=lse_dec,
                                  layout=layout)
    torch.cuda.synchronize()
    dq_h, dk_h, dv_h = to_host(dq), to_host(back(dk)), to_host(back(dv))
    for t in (dq_h, dk_h, dv_h):
        assert np.isfinite(t).all()
    tok = _sample_tokens(N, 2048, 6)
    # the step bench.py times (no override): the oracle on every head; the variants: on their last head
    for h in (range(inp["H"]) if not over else (inp["H"] - 1,)):
        sl = (slice(None), slice(h, h + 1))
        dq_ref, dk_ref, dv_ref = oracle.backward(inp["q"][h:h + 1], inp["k"][sl], inp["v"][sl], inp["dy"][sl], scale,
                                                 tok=tok)
        errs = dict(dq=slice_relerr(dq_h[h:h + 1], dq_ref), dk=slice_relerr(dk_h[:, h:h + 1, tok], dk_ref),
                    dv=slice_relerr(dv_h[:, h:h + 1, tok], dv_ref))
        rows = dict(dq=row_relerr(dq_h[h:h + 1], dq_ref), dk=row_relerr(dk_h[:, h:h + 1, tok], dk_ref),
                    dv=row_relerr(dv_h[:, h:h + 1, tok], dv_ref))
        _say("   head %d: " % h + "  ".join("%s %.3e" % kv for kv in errs.items()) + "  (tol %.0e); worst rows " % tol
             + "  ".join("%s %.3e" % kv for kv in rows.items()))
        assert max(errs.values()) <= tol
        assert max(rows.values()) <= ROW_FACTOR * tol


def test_backward_full_small_workloads(oracle):
    """Gradients of configs 1 and 2 at their full sizes, every element."""
    import torch
    for cfg in (1, 2):
        _say("full backward cfg%d" % cfg)
        inp = synth.make_inputs(cfg, with_dy=True)
        dev = to_device(inp)
        y, z, lse = binding.forward(dev["q"], dev["k"], dev["v"], inp["scale"])
        dq, dk, dv = binding.backward(dev["q"], dev["k"], dev["v"], dev["dy"], z, lse, inp["scale"])
        torch.cuda.synchronize()
        dq_ref, dk_ref, dv_ref = oracle.backward(inp["q"], inp["k"], inp["v"], inp["dy"], inp["scale"])
        tol = TOL[inp["dtype"]]
        errs = (slice_relerr(to_host(dq), dq_ref), slice_relerr(to_host(dk), dk_ref),
                slice_relerr(to_host(dv), dv_ref))
        rows = (row_relerr(to_host(dq), dq_ref), row_relerr(to_host(dk), dk_ref), row_relerr(to_host(dv), dv_ref))
        _say("   err dq %.3e  dk %.3e  dv %.3e  (tol %.0e); worst rows %.3e  %.3e  %.3e" % (errs + (tol,) + rows))
        assert max(errs) <= tol
        assert max(rows) <= ROW_FACTOR * tol


@pytest.mark.parametrize("dtype,layout", [("bf16", "bhnd"), ("bf16", "bnhd"), ("f32", "bhnd")])
def test_token_tensors_beyond_two_to_the_31_elements(dtype, layout):
    """Maximum sizes: 17 copies of the million-token item in one call, so that the element offsets
    into k, v, y, dy, dk, dv pass 2^31 (and the byte offsets 2^32, fp32: 2^33).  The
    batch items are independent and go through the same kernels in the same configuration, so every
    item must equal item 0 bit for bit (y, z, lse_enc, dk, dv); item 0 must agree with a one-item call
    (whose token axis is split differently, so only up to rounding), and dq_lat, the sum over the
    batch, must be B times the one-item result."""
    import torch
    B = 17
    over = dict(dtype=dtype) if dtype != "bf16" else dict()
    if dtype == "f32":
        over.update(M=64)       # the fp32 kernels run on the vector ALUs: fewer latents keep the case short
    _say("offsets beyond 2^31 elements: %d copies of cfg4 %s %s" % (B, over, layout))
    inp = synth.make_inputs(4, with_dy=True, **over)
    scale = inp["scale"]
    dev = to_device(inp)
    conv = (lambda t: t.permute(0, 2, 1, 3).contiguous()) if layout == "bnhd" else (lambda t: t)
    one = {n: conv(dev[n]) for n in ("k", "v", "dy")}
    assert B * one["k"].numel() > 2 ** 31
    y1, z1, lse1 = binding.forward(dev["q"], one["k"], one["v"], scale, layout=layout)
    dq1, dk1, dv1 = binding.backward(dev["q"], one["k"], one["v"], one["dy"], z1, lse1, scale, layout=layout)
    many = {n: t.expand(B, *t.shape[1:]).contiguous() for n, t in one.items()}
    y, z, lse = binding.forward(dev["q"], many["k"], many["v"], scale, layout=layout)
    dq, dk, dv = binding.backward(dev["q"], many["k"], many["v"], many["dy"], z, lse, scale, layout=layout)
    torch.cuda.synchronize()
    # two runs of the library with different splits of the 10^6 tokens: each carries its own rounding
    # (fp32 sums of 10^6 terms; bf16 weights), so their distance is up to twice that of one run from the truth
    loose = 1e-5 if dtype == "f32" else 4e-3
    for name, got, want in (("y", y, y1), ("z", z, z1), ("lse_enc", lse, lse1), ("dk", dk, dk1), ("dv", dv, dv1)):
        for b in range(1, B):
            assert torch.equal(got[b], got[0]), "%s of batch item %d differs from item 0" % (name, b)
        err = float((got[0].double() - want[0].double()).norm() / want[0].double().norm())
        _say("   %s of item 0 against the one-item call: %.2e" % (name, err))
        assert err <= loose
    e_q = float((dq.double() - B * dq1.double()).norm() / (B * dq1.double()).norm())
    _say("   dq against B x one item: %.2e" % e_q)
    assert e_q <= loose
