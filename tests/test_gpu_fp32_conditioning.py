"""fp32 storage, mesh-like inputs: the shapes on which random sweeps read a gradient above the 1e-5 bar of
the fp32 path (dq_lat 1.2e-5, 1.5e-5, 2.2e-5 at d = 4; dk 1.4e-4 on a two-token input), pinned here with the cause.

In every one of them the error sits in ONE latent row whose gradient is large and ill-conditioned:
    dQ_m = scale * [ sum_n P_mn a_mn k_n  -  eps_m * sum_n P_mn k_n ]  +  (decode half, likewise with delta_n),
a_mn = <dZ_m, V_n>, eps_m = <dZ_m, Z_m> = sum_n P_mn a_mn.  The two terms of the bracket are each K_m times
larger than their difference (K_m ~ 200 for the worst row of these inputs: keys of a 4-channel mesh lift lie
almost on a line, so the P-weighted mean key is long), and eps_m, Z_m, the log-sum-exp normalisers and the
scores reach the backward rounded to fp32 (2^-24 relative each).  A plain numpy evaluation of the same
formulas in fp32 -- and even in fp64 from fp32-rounded normalisers -- is off by 4e-5 ... 5e-5 on the third case
(the kernels: 2.2e-5): the bar of 1e-5 is not reachable in fp32 arithmetic on such rows, whatever the order
of operations (forming a - eps as <dZ_m, V_n - Z_m> first, or replacing eps by the kernel's own P-weighted mean
of a, moves the error by less than a factor of 2.5).

So the test states the bound the arithmetic does meet: forward outputs and dV at the fp32 bar, and
    err(dq_lat) <= 1e-5 + 8 * 2^-24 * K,    K = scale * (||eps_m kbar_m||_F + ||sum_n R_nm delta_n k_n||_F) / ||dQ||_F
over the latents of a head (K: the cancellation factor of the two halves, from fp64 quantities; the mean-zero
part of each half needs no such allowance).  Well-conditioned inputs have K of order 1-10, where the bound is
the plain bar (checked below on the first reference workload's shape).

The token gradients have the mirror image of it,
    dK_n = scale * [ sum_m P_mn a_mn q_m - sum_m P_mn eps_m q_m ] + scale * [ sum_m R_nm c_mn q_m - delta_n qbar_n ],
and the same bound with K_dK = scale * (||sum_m P_mn eps_m q_m||_F + ||delta_n qbar_n||_F) / ||dK||_F per (b, h)
slice.  It stays near 10 on the shapes above; the fourth case (two tokens, 252 latents, scores doubled, found
by a random sweep at dk = 1.4e-4) has K_dK = 384: with two tokens every latent's encode weights are almost
one-hot, dK is a small remainder of terms 384 times its size, and 1e-5 + 8 * 2^-24 * 384 = 1.9e-4.

The last test of the file pins the three 16-bit cases of the same kind that the sweeps found (many more latents than
tokens), with the rounding of the bf16 weights in place of the fp32 one.
"""
import sys

import numpy as np
import pytest

from paper_2508_12594_amd import binding, synth
from tests._util import slice_relerr, to_device, to_host

pytestmark = pytest.mark.gpu

LOG2E = 1.4426950408889634

CASES = [
    # kind, B, H, N, M, d, seed, layout, saved, shared;   measured dq_lat: 1.2e-5, 1.5e-5, 2.2e-5
    dict(kind=2, B=1, H=2, N=150000, M=237, d=4, seed=777 + 123, layout="bhnd", saved=False, shared=False),
    dict(kind=2, B=2, H=2, N=211, M=264, d=4, seed=777 + 5001, layout="bhnd", saved=True, shared=False),
    dict(kind=2, B=1, H=1, N=2243, M=248, d=4, seed=4242 + 2243 + 248 + 4, layout="bnhd", saved=False, shared=True),
    # two tokens, 252 latents, scores doubled: here it is dK that cancels (measured 1.4e-4)
    dict(kind=2, B=2, H=3, N=2, M=252, d=32, seed=777 + 4497, layout="bhnd", saved=False, shared=False, gain=2.0),
    # two more of the same two families from a later sweep (dq_lat 1.02e-5; two tokens: dq_lat 1.1e-5, dk 1.8e-5)
    dict(kind=2, B=2, H=1, N=683, M=189, d=4, seed=777 + 15120, layout="bnhd", saved=False, shared=False),
    dict(kind=2, B=2, H=3, N=2, M=191, d=32, seed=777 + 16236, layout="bhnd", saved=False, shared=False),
    # and two from a third sweep (fewer tokens than latents at d = 4)
    dict(kind=2, B=3, H=1, N=217, M=296, d=4, seed=777 + 21402, layout="bhnd", saved=True, shared=False),
    dict(kind=2, B=1, H=2, N=59, M=176, d=4, seed=777 + 22884, layout="bnhd", saved=False, shared=False),
    dict(kind=2, B=2, H=3, N=436, M=257, d=4, seed=777 + 25080, layout="bhnd", saved=False, shared=False),
    # a well-conditioned shape for comparison (first reference workload: normal inputs): plain bar
    dict(kind=1, B=1, H=4, N=1024, M=64, d=32, seed=250812595, layout="bhnd", saved=False, shared=False),
]


def _cancellation_factor(q, k, v, dy, scale, dq_ref, dk_ref=None):
    """K per head (max over heads): how much larger than dQ the cancelling terms of its two halves are.  With
    dk_ref also the same for dK_n = scale * [sum_m P_mn a_mn q_m - sum_m P_mn eps_m q_m] + (decode half, with
    delta_n sum_m R_nm q_m), per (b,h) slice: returns (K_dq, K_dk)."""
    worst = 0.0
    worst_k = 0.0
    B, H = k.shape[0], k.shape[1]
    for h in range(H):
        num_e = np.zeros(q.shape[1:], np.float64)
        num_d = np.zeros(q.shape[1:], np.float64)
        for b in range(B):
            kk, vv, gg = (x[b, h].astype(np.float64) for x in (k, v, dy))
            s2 = (q[h].astype(np.float64) * (scale * LOG2E)) @ kk.T                 # [M, N]
            p = np.exp2(s2 - s2.max(axis=1, keepdims=True))
            p /= p.sum(axis=1, keepdims=True)
            r = np.exp2(s2 - s2.max(axis=0, keepdims=True))
            r /= r.sum(axis=0, keepdims=True)
            z = p @ vv
            dz = r @ gg
            delta = np.einsum("nj,nj->n", gg, r.T @ z)
            eps = np.einsum("mj,mj->m", dz, z)
            num_e += eps[:, None] * (p @ kk)                                         # eps_m * kbar_m, summed over b
            num_d += (r * delta[None, :]) @ kk                                       # sum_n R_nm delta_n k_n
            if dk_ref is not None:
                qq = q[h].astype(np.float64)
                t_e = (p * eps[:, None]).T @ qq                                      # sum_m P_mn eps_m q_m   [N, d]
                t_d = delta[:, None] * (r.T @ qq)                                    # delta_n sum_m R_nm q_m [N, d]
                worst_k = max(worst_k, scale * (np.linalg.norm(t_e) + np.linalg.norm(t_d)) /
                              np.linalg.norm(dk_ref[b, h]))
        worst = max(worst, scale * (np.linalg.norm(num_e) + np.linalg.norm(num_d)) / np.linalg.norm(dq_ref[h]))
    return worst if dk_ref is None else (worst, worst_k)


@pytest.mark.parametrize("case", CASES, ids=lambda c: "N%(N)d-M%(M)d-d%(d)d-%(layout)s" % c)
def test_fp32_gradients_meet_the_bar_up_to_their_conditioning(oracle, case):
    import torch
    c = case
    print("[case] fp32 conditioning %s" % (c,), flush=True)
    sys.stdout.flush()
    B, H, N, M, d = c["B"], c["H"], c["N"], c["M"], c["d"]
    inp = synth.make_inputs(c["kind"], B=B, H=H, N=N, M=M, d=d, dtype="f32", with_dy=True, seed=c["seed"])
    if c["shared"]:
        inp["q"] = np.ascontiguousarray(np.broadcast_to(inp["q"][0], (H, M, d)))
    scale = c.get("gain", 1.0) / np.sqrt(d)
    dev = to_device(inp)
    conv = (lambda t: t.permute(0, 2, 1, 3).contiguous()) if c["layout"] == "bnhd" else (lambda t: t)
    back = (lambda t: t.permute(0, 2, 1, 3)) if c["layout"] == "bnhd" else (lambda t: t)
    k, v, dy = conv(dev["k"]), conv(dev["v"]), conv(dev["dy"])
    q = dev["q"][0].contiguous() if c["shared"] else dev["q"]
    lse_dec = torch.empty((B, H, N), dtype=torch.float32, device="cuda") if c["saved"] else None
    y, z, lse = binding.forward(q, k, v, scale, lse_dec=lse_dec, layout=c["layout"])
    dq, dk, dv = binding.backward(q, k, v, dy, z, lse, scale, y=y if c["saved"] else None, lse_dec=lse_dec,
                                  layout=c["layout"])
    torch.cuda.synchronize()
    y_ref, z_ref, _ = oracle.forward(inp["q"], inp["k"], inp["v"], scale)
    dq_ref, dk_ref, dv_ref = oracle.backward(inp["q"], inp["k"], inp["v"], inp["dy"], scale)
    dq_h = to_host(dq)
    if c["shared"]:
        dq_h, dq_cmp = dq_h[None], dq_ref.sum(axis=0)[None]
    else:
        dq_cmp = dq_ref
    errs = dict(y=slice_relerr(to_host(back(y)), y_ref), z=slice_relerr(to_host(z), z_ref),
                dk=slice_relerr(to_host(back(dk)), dk_ref), dv=slice_relerr(to_host(back(dv)), dv_ref),
                dq=slice_relerr(dq_h, dq_cmp))
    K, K_dk = _cancellation_factor(inp["q"], inp["k"], inp["v"], inp["dy"], scale, dq_cmp if not c["shared"] else
                                   np.broadcast_to(dq_cmp, (H, M, d)), dk_ref)
    bound = 1e-5 + 8.0 * 2.0 ** -24 * K
    bound_dk = 1e-5 + 8.0 * 2.0 ** -24 * K_dk
    print("[case]    " + "  ".join("%s %.2e" % kv for kv in errs.items()) +
          "  cancellation factors K %.1f (dQ) %.1f (dK) -> bounds %.2e, %.2e" % (K, K_dk, bound, bound_dk), flush=True)
    assert max(errs["y"], errs["z"], errs["dv"]) <= 1e-5
    assert errs["dq"] <= bound
    assert errs["dk"] <= bound_dk
    if c["kind"] == 1:
        assert max(K, K_dk) <= 20.0 and max(errs["dq"], errs["dk"]) <= 1e-5      # well-conditioned: the plain bar


SIXTEEN_BIT_CASES = [
    # over the bar in the sweep: measured dq_lat 2.16e-2
    dict(dtype="bf16", B=2, H=2, N=185, M=1536, d=16, seed=777 + 7074, layout="bhnd"),
    # 2.11e-2 and 2.91e-2 on the matrix cores; shapes of fewer than 16 tokens run on the fp32 kernels since: 5e-6, 6e-6
    dict(dtype="bf16", B=2, H=1, N=12, M=1489, d=16, seed=777 + 2880, layout="bhnd"),
    dict(dtype="f16", B=1, H=1, N=9, M=1157, d=16, seed=777 + 15775, layout="bhnd"),
    # 2.39e-2 and 2.49e-2 while the fused kernel carried Z as one bf16 term; with the lo term: 1.14e-2, 6.96e-3
    dict(dtype="bf16", B=1, H=1, N=242, M=692, d=16, seed=777 + 7966, layout="bhnd"),
    dict(dtype="bf16", B=1, H=1, N=427, M=1539, d=16, seed=777 + 17910, layout="bnhd"),
    # delta from the forward's saved bf16 y (1990 tokens, 192 latents; one case in 30 000 of the general sweep): 2.40e-2,
    # five rows hold 91 % of the squared error; 3.9e-3 with the statistics recomputed (or with the fp32 y)
    dict(dtype="bf16", B=1, H=1, N=1990, M=192, d=16, seed=777 + 50548, layout="bhnd", saved=True),
]


@pytest.mark.parametrize("case", SIXTEEN_BIT_CASES, ids=lambda c: "%(dtype)s-N%(N)d-M%(M)d" % c)
def test_16bit_gradient_of_dominating_latents_within_its_conditioning(oracle, case):
    """The same conditioning on the matrix cores (16-bit storage, mesh-like inputs, many more latents than tokens: the
    cases over the bar of 2e-2 in 21 000 shapes of a random sweep over 257 ... 2048 latents, before and after the fused
    backward kernel got the lo term of Z for such shapes and shapes of 8 ... 15 tokens went to the fp32 kernels):
    dq_lat read up to 2.9e-2, now 2.2e-2 on one of them, most of the squared error in a handful of latent rows --
    rows whose two halves are each K times their difference.  The weights P and dS enter
    the matrix products rounded to bf16 (2^-9 relative) whatever the storage type, so the bound the arithmetic meets
    is 2e-2 + 2^-9 K; every other output is at the plain bar."""
    import torch
    c = case
    print("[case] 16-bit conditioning %s" % (c,), flush=True)
    inp = synth.make_inputs(2, B=c["B"], H=c["H"], N=c["N"], M=c["M"], d=c["d"], dtype=c["dtype"], with_dy=True,
                            seed=c["seed"])
    scale = 1.0 / np.sqrt(c["d"])
    dev = to_device(inp)
    conv = (lambda t: t.permute(0, 2, 1, 3).contiguous()) if c["layout"] == "bnhd" else (lambda t: t)
    back = (lambda t: t.permute(0, 2, 1, 3)) if c["layout"] == "bnhd" else (lambda t: t)
    k, v, dy = conv(dev["k"]), conv(dev["v"]), conv(dev["dy"])
    saved = c.get("saved", False)
    lse_dec = torch.empty((c["B"], c["H"], c["N"]), dtype=torch.float32, device="cuda") if saved else None
    y, z, lse = binding.forward(dev["q"], k, v, scale, lse_dec=lse_dec, layout=c["layout"])
    dq, dk, dv = binding.backward(dev["q"], k, v, dy, z, lse, scale, y=y if saved else None, lse_dec=lse_dec,
                                  layout=c["layout"])
    torch.cuda.synchronize()
    y_ref, z_ref, _ = oracle.forward(inp["q"], inp["k"], inp["v"], scale)
    dq_ref, dk_ref, dv_ref = oracle.backward(inp["q"], inp["k"], inp["v"], inp["dy"], scale)
    errs = dict(y=slice_relerr(to_host(back(y)), y_ref), z=slice_relerr(to_host(z), z_ref),
                dk=slice_relerr(to_host(back(dk)), dk_ref), dv=slice_relerr(to_host(back(dv)), dv_ref),
                dq=slice_relerr(to_host(dq), dq_ref))
    K, K_dk = _cancellation_factor(inp["q"], inp["k"], inp["v"], inp["dy"], scale, dq_ref, dk_ref)
    # in the head with the largest error: the part of the squared error that 2 % of the latent rows hold
    diff = to_host(dq).astype(np.float64) - dq_ref
    h = int(np.argmax([np.linalg.norm(diff[i]) / np.linalg.norm(dq_ref[i]) for i in range(c["H"])]))
    rows = np.sort(np.sum(diff[h] ** 2, axis=1))[::-1]
    share = float(rows[:max(5, c["M"] // 50)].sum() / rows.sum())
    bound = 2e-2 + 2.0 ** -9 * K
    print("[case]    " + "  ".join("%s %.2e" % kv for kv in errs.items()) +
          "  K %.1f (dQ) %.1f (dK) -> bound %.2e; 2 %% of the rows hold %.0f %% of the squared error" % (K, K_dk, bound, 100 * share),
          flush=True)
    assert max(errs["y"], errs["z"], errs["dv"], errs["dk"]) <= 2e-2
    assert errs["dq"] <= bound
    assert share >= 0.5      # the error is a few ill-conditioned rows, not a level over all of them
