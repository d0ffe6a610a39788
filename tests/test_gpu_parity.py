"""GPU parity: libflare.so (through its C ABI) against the fp64 CPU oracle, element by element,
on the same seeded inputs.  Sizes here finish in seconds on the oracle yet span several
tiles, several token chunks and ragged tails.  The full sizes of the reference workloads are in
test_gpu_fullsize.py.

Metric: max over (b,h) slices of ||T_gpu - T_ref||_F / ||T_ref||_F.  Bar: 1e-5 for the
fp32 path, 2e-2 for bf16 inputs with fp32 accumulation.
"""
import sys

import numpy as np
import pytest

from paper_2508_12594_amd import binding, synth
from tests._util import ROW_FACTOR, TOL, on_matrix_cores, row_relerr, slice_relerr, to_device, to_host

pytestmark = pytest.mark.gpu


def _say(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


def _forward_case(oracle, inp, scale=None, tol=None):
    import torch
    scale = inp["scale"] if scale is None else scale
    tol = TOL[inp["dtype"]] if tol is None else tol
    dev = to_device(inp)
    y, z, lse = binding.forward(dev["q"], dev["k"], dev["v"], scale)
    torch.cuda.synchronize()
    y_ref, z_ref, lse_ref = oracle.forward(inp["q"], inp["k"], inp["v"], scale)
    e_y = slice_relerr(to_host(y), y_ref)
    e_z = slice_relerr(to_host(z), z_ref)
    e_l = float(np.max(np.abs(to_host(lse) - lse_ref)))
    _say("   err y %.3e  z %.3e  lse(abs) %.3e  (tol %.0e)" % (e_y, e_z, e_l, tol))
    assert e_y <= tol and e_z <= tol
    if y_ref.shape[2] >= 10000:     # many tokens: a few wrong rows would vanish in the norm; look at the worst one
        r_y, r_z = row_relerr(to_host(y), y_ref), row_relerr(to_host(z), z_ref)
        _say("   worst row y %.3e  z %.3e" % (r_y, r_z))
        assert max(r_y, r_z) <= ROW_FACTOR * tol
    # absolute error of the log-sum-exp: rounding of the scores (relative to |S|) plus, on the bf16
    # path, the bf16 rounding of the weights that are summed
    coarse = inp["dtype"] == "bf16" or (inp["dtype"] == "f16" and tol >= TOL["bf16"])
    assert e_l <= (5e-3 if coarse else 1e-5) + 1e-5 * float(np.max(np.abs(lse_ref)))
    return y, z, lse


def _backward_case(oracle, inp, scale=None, tol=None, zero_dq_dk=False, saved=False, variant=0):
    """saved=True hands the forward's y and lse_dec to the backward (no recomputation); variant: flare_variant
    bits that force a kernel variant of the backward."""
    import torch
    scale = inp["scale"] if scale is None else scale
    tol = TOL[inp["dtype"]] if tol is None else tol
    dev = to_device(inp)
    lse_dec = torch.empty(dev["k"].shape[:3], dtype=torch.float32, device="cuda") if saved else None
    y, z, lse = binding.forward(dev["q"], dev["k"], dev["v"], scale, lse_dec=lse_dec)
    dq, dk, dv = binding.backward(dev["q"], dev["k"], dev["v"], dev["dy"], z, lse, scale,
                                  y=y if saved else None, lse_dec=lse_dec, variant=variant)
    torch.cuda.synchronize()
    dq_ref, dk_ref, dv_ref = oracle.backward(inp["q"], inp["k"], inp["v"], inp["dy"], scale)
    e_v = slice_relerr(to_host(dv), dv_ref)
    if zero_dq_dk:
        # the exact gradients vanish (e.g. N = 1: both softmaxes are constant in q and k), so
        # measure dq and dk against the size of dv instead of against themselves
        ref = float(np.linalg.norm(dv_ref))
        assert float(np.linalg.norm(dq_ref)) <= 1e-12 * ref and float(np.linalg.norm(dk_ref)) <= 1e-12 * ref
        e_q = float(np.linalg.norm(to_host(dq))) / ref
        e_k = float(np.linalg.norm(to_host(dk))) / ref
    else:
        e_q = slice_relerr(to_host(dq), dq_ref)
        e_k = slice_relerr(to_host(dk), dk_ref)
    _say("   err dq %.3e  dk %.3e  dv %.3e  (tol %.0e)" % (e_q, e_k, e_v, tol))
    assert e_q <= tol and e_k <= tol and e_v <= tol
    if dk_ref.shape[2] >= 10000 and not zero_dq_dk:
        rows = (row_relerr(to_host(dq), dq_ref), row_relerr(to_host(dk), dk_ref), row_relerr(to_host(dv), dv_ref))
        _say("   worst row dq %.3e  dk %.3e  dv %.3e" % rows)
        assert max(rows) <= ROW_FACTOR * tol
    return dq, dk, dv


# ---- the five workloads, at sizes the oracle finishes in seconds -----------------------------
FWD_CASES = [
    # (cfg, overrides)
    (1, dict()),                                # the fp32 workload at its full size
    (1, dict(N=1000)),                          # ragged
    (2, dict(B=2, N=3001)),                     # mesh, bf16, d=16, M=64
    (3, dict(B=2, N=4096)),                     # bf16, d=32, M=128
    (3, dict(B=1, N=777)),
    (4, dict(N=10007)),                         # mesh, bf16, d=16, M=256, ragged
    (5, dict(N=4099)),                          # bf16, d=32, M=256
]


@pytest.mark.parametrize("cfg,over", FWD_CASES)
def test_forward_workloads(oracle, cfg, over):
    _say("forward cfg%d %s" % (cfg, over))
    inp = synth.make_inputs(cfg, with_dy=False, **over)
    _forward_case(oracle, inp)


def test_forward_scale_one(oracle):
    """The paper's own setting: scale = 1 in both attention calls."""
    for cfg, over in [(1, dict(N=515)), (2, dict(B=1, N=1030))]:
        _say("forward scale=1 cfg%d %s" % (cfg, over))
        inp = synth.make_inputs(cfg, with_dy=False, **over)
        _forward_case(oracle, inp, scale=1.0)


BWD_CASES = [
    (1, dict()),
    (1, dict(N=999, B=2)),
    (2, dict(B=2, N=2050)),
    (3, dict(B=3, N=1024)),
    (4, dict(N=5003)),
    (5, dict(N=3001)),
]


@pytest.mark.parametrize("saved", [False, True])
@pytest.mark.parametrize("cfg,over", BWD_CASES)
def test_backward_workloads(oracle, cfg, over, saved):
    _say("backward cfg%d %s saved=%s" % (cfg, over, saved))
    inp = synth.make_inputs(cfg, with_dy=True, **over)
    _backward_case(oracle, inp, saved=saved)


@pytest.mark.parametrize("cfg,over", [(1, dict(N=700)), (4, dict(N=3000)), (3, dict(B=2, N=900))])
def test_saved_lse_dec_matches_oracle(oracle, cfg, over):
    """lse_dec[n] = log sum_m exp(S[m][n]) as written by the forward."""
    import torch
    inp = synth.make_inputs(cfg, with_dy=False, **over)
    dev = to_device(inp)
    lse_dec = torch.empty(dev["k"].shape[:3], dtype=torch.float32, device="cuda")
    binding.forward(dev["q"], dev["k"], dev["v"], inp["scale"], lse_dec=lse_dec)
    torch.cuda.synchronize()
    s = inp["scale"] * np.einsum("hmd,bhnd->bhmn", inp["q"].astype(np.float64), inp["k"].astype(np.float64))
    mx = s.max(axis=2, keepdims=True)
    ref = (mx + np.log(np.exp(s - mx).sum(axis=2, keepdims=True)))[:, :, 0]
    err = float(np.max(np.abs(to_host(lse_dec) - ref)))
    _say("   lse_dec abs err %.3e" % err)
    assert err <= (1e-5 if inp["dtype"] == "f32" else 1e-2)


# ---- edge cases ---------------------------------------------------------------------------------
EDGE_SHAPES = [
    # B, H, N, M, d
    (1, 1, 1, 32, 16),        # a single token: Y = v
    (1, 2, 7, 32, 32),        # fewer tokens than one group
    (2, 1, 63, 64, 16),
    (1, 1, 65, 96, 16),       # M a multiple of 32 but not of 64
    (1, 3, 257, 1, 16),       # one latent: Y_n = Z_1
    (1, 1, 300, 33, 8),       # odd M, small d
    (1, 2, 129, 300, 4),      # M above one latent block, d = 4
    (1, 1, 40, 513, 32),      # three latent blocks
    (1, 2, 1000, 192, 16),    # three latent groups per workgroup on the matrix-core path
    (2, 1, 100, 128, 32),
    (1, 1, 33, 256, 32),      # one token past a 32-token tile
    (1, 1, 31, 256, 16),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", EDGE_SHAPES)
def test_edge_shapes_forward_backward(oracle, shape, dtype):
    B, H, N, M, d = shape
    _say("edge %s %s" % (shape, dtype))
    inp = synth.make_inputs(1, B=B, H=H, N=N, M=M, d=d, dtype=dtype, with_dy=True, seed=1234 + N + M)
    y, _, _ = _forward_case(oracle, inp)
    _backward_case(oracle, inp, zero_dq_dk=(N == 1))
    _backward_case(oracle, inp, zero_dq_dk=(N == 1), saved=True)
    if N == 1:
        assert slice_relerr(to_host(y), inp["v"]) <= (1e-6 if dtype == "f32" else 4e-3)


# Two to seven tokens with 16-bit storage: every Z_m lies in the span of those few value rows, so both
# softmax-gradient differences cancel almost completely; such shapes run on the fp32 kernels (bf16 operands
# gave dq_lat and dK errors up to 1.6e-1 on these very inputs).
FEW_TOKEN_SHAPES = [
    # seed offset, kind, B, H, N, M, d, dtype
    (98, 1, 1, 3, 2, 192, 16, "f16"),
    (560, 2, 2, 2, 2, 512, 16, "f16"),
    (308, 2, 1, 1, 2, 64, 16, "f16"),
    (1247, 2, 1, 3, 3, 512, 16, "f16"),
    (542, 2, 1, 1, 2, 234, 16, "bf16"),
    (7, 1, 1, 2, 7, 256, 32, "bf16"),
    (8, 2, 2, 1, 4, 100, 8, "bf16"),
    (9, 2, 1, 2, 5, 33, 4, "f16"),
]


@pytest.mark.parametrize("saved", [False, True])
@pytest.mark.parametrize("shape", FEW_TOKEN_SHAPES)
def test_few_tokens_sixteen_bit_storage(oracle, shape, saved):
    i, kind, B, H, N, M, d, dtype = shape
    _say("few tokens %s saved=%s" % (shape, saved))
    inp = synth.make_inputs(kind, B=B, H=H, N=N, M=M, d=d, dtype=dtype, with_dy=True, seed=777 + i)
    _forward_case(oracle, inp)
    _backward_case(oracle, inp, saved=saved)


# Head dimensions below 16 on the matrix-core path (contraction padded to 16): the regime of the paper's
# PDE models (C = 64, H = 8, so D = 8; Section 5 and Appendix D settings) and of its D = 4 ablation.
SMALL_D_SHAPES = [
    # B, H, N, M, d
    (1, 2, 1000, 64, 8),
    (2, 1, 777, 256, 8),
    (1, 3, 515, 128, 8),
    (1, 2, 2049, 32, 8),
    (1, 1, 999, 192, 8),      # three latent groups; dK/dV with two padding tiles
    (1, 2, 1000, 64, 4),
    (1, 2, 333, 256, 4),
    (2, 2, 65, 128, 4),
]


@pytest.mark.parametrize("shape", SMALL_D_SHAPES)
def test_small_head_dims_matrix_core_path(oracle, shape):
    B, H, N, M, d = shape
    _say("small d %s bf16" % (shape,))
    inp = synth.make_inputs(2, B=B, H=H, N=N, M=M, d=d, dtype="bf16", with_dy=True, seed=4321 + N + M + d)
    _forward_case(oracle, inp)
    _backward_case(oracle, inp, saved=False)
    _backward_case(oracle, inp, saved=True)


# More than 256 latents per head on the matrix-core path (chunks of 256 latents): the paper's
# million-point model uses up to M = 2048 (Section 5.2; Appendix E).
LARGE_M_SHAPES = [
    # B, H, N, M, d
    (1, 2, 1500, 512, 16),
    (2, 1, 700, 768, 16),
    (1, 1, 1031, 1024, 8),
    (1, 1, 300, 2048, 8),
    (1, 2, 900, 512, 32),
    (1, 1, 333, 1024, 4),
]


@pytest.mark.parametrize("shape", LARGE_M_SHAPES)
def test_many_latents_matrix_core_path(oracle, shape):
    B, H, N, M, d = shape
    _say("large M %s bf16" % (shape,))
    inp = synth.make_inputs(2, B=B, H=H, N=N, M=M, d=d, dtype="bf16", with_dy=True, seed=999 + N + M + d)
    _forward_case(oracle, inp)
    _backward_case(oracle, inp, saved=False)
    _backward_case(oracle, inp, saved=True)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("shape", [(1, 1, 200, 2100, 8), (1, 2, 70, 2049, 16)])
def test_sixteen_bit_storage_on_vector_kernels(oracle, shape, dtype):
    """More than 2048 latents per head: the fp32 vector kernels with 16-bit storage (fp32 arithmetic, so
    only the rounding of the outputs separates the result from the fp32 path's)."""
    B, H, N, M, d = shape
    assert not on_matrix_cores(dtype, M)
    _say("16-bit storage on the vector kernels %s %s" % (dtype, shape))
    inp = synth.make_inputs(1, B=B, H=H, N=N, M=M, d=d, dtype=dtype, with_dy=True, seed=606 + N + M)
    tol = TOL["f16"] if dtype == "f16" else 8e-3       # outputs rounded to 2^-11 / 2^-8 relative
    _forward_case(oracle, inp, tol=tol)
    _backward_case(oracle, inp, tol=tol, saved=False)
    _backward_case(oracle, inp, tol=tol, saved=True)


# Numbers of latents that are not a multiple of the tile sizes: padding latents inside the last tile, whole
# padding tiles (M = 40 runs on the 64-latent geometry, M = 300 on two chunks of 256), M = 1.
ODD_M_SHAPES = [
    # B, H, N, M, d
    (1, 2, 1000, 1, 16),
    (2, 1, 700, 16, 16),
    (1, 2, 900, 40, 32),
    (1, 3, 600, 96, 8),
    (1, 1, 1500, 100, 16),
    (1, 2, 800, 160, 32),
    (1, 1, 999, 200, 4),
    (1, 2, 500, 255, 16),
    (1, 1, 600, 300, 16),
    (1, 1, 400, 513, 8),
    (1, 1, 300, 1000, 32),
]


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("shape", ODD_M_SHAPES)
def test_any_number_of_latents_matrix_core_path(oracle, shape, dtype):
    B, H, N, M, d = shape
    _say("odd M %s %s" % (shape, dtype))
    inp = synth.make_inputs(2, B=B, H=H, N=N, M=M, d=d, dtype=dtype, with_dy=True, seed=515 + N + M + d)
    tol = TOL["bf16"]
    _forward_case(oracle, inp, tol=tol)
    _backward_case(oracle, inp, tol=tol, saved=False)
    _backward_case(oracle, inp, tol=tol, saved=True)


def test_padding_latents_do_not_depend_on_what_lies_beyond_q(oracle):
    """The last tile's loads are clamped to the last real latent: the result must not change when the
    memory after q_lat changes (q_lat placed at the end of one buffer, then followed by other data)."""
    import torch
    inp = synth.make_inputs(2, B=1, H=2, N=700, M=40, d=16, dtype="bf16", with_dy=True, seed=99)
    dev = to_device(inp)
    outs = []
    for fill in (0.0, 1e30):
        buf = torch.full((dev["q"].numel() + 4096,), fill, dtype=torch.bfloat16, device="cuda")
        q = buf[:dev["q"].numel()].view_as(dev["q"])
        q.copy_(dev["q"])
        y, z, lse = binding.forward(q, dev["k"], dev["v"], inp["scale"])
        dq, dk, dv = binding.backward(q, dev["k"], dev["v"], dev["dy"], z, lse, inp["scale"])
        torch.cuda.synchronize()
        outs.append((y, z, lse, dq, dk, dv))
    for a, b in zip(*outs):
        assert torch.equal(a, b)


# fp16 storage on the matrix-core path: scores from fp16 products (exact as with bf16 storage), softmax
# weights and dS in bf16, V / dY rounded to bf16 on load, fp32 accumulation: the bf16 path's tolerance.
F16_MATRIX_CASES = [
    # cfg, overrides
    (2, dict(B=2, N=3001)),                       # d=16, M=64
    (3, dict(B=2, N=1500)),                       # d=32, M=128
    (4, dict(N=5003)),                            # d=16, M=256
    (5, dict(N=3001)),                            # d=32, M=256 (decode with Z in LDS)
    (2, dict(B=1, N=1000, M=32)),
    (2, dict(B=1, N=1200, M=192)),                # dK/dV with two padding tiles
    (2, dict(B=1, H=2, N=1000, M=64, d=8)),
    (2, dict(B=1, H=2, N=333, M=256, d=4)),
    (2, dict(B=1, H=2, N=900, M=512)),            # two latent chunks
    (2, dict(B=1, H=1, N=400, M=1024, d=8)),
    (4, dict(N=1, H=2)),                          # a single token
    (4, dict(N=33, H=3)),
]


@pytest.mark.parametrize("cfg,over", F16_MATRIX_CASES)
def test_fp16_storage_matrix_core_path(oracle, cfg, over):
    _say("fp16 on matrix cores cfg%d %s" % (cfg, over))
    inp = synth.make_inputs(cfg, with_dy=True, dtype="f16", **over)
    assert on_matrix_cores("f16", inp["q"].shape[1])
    tol = TOL["bf16"]
    single = inp["k"].shape[2] == 1
    y, _, _ = _forward_case(oracle, inp, tol=tol)
    _backward_case(oracle, inp, tol=tol, saved=False, zero_dq_dk=single)
    _backward_case(oracle, inp, tol=tol, saved=True, zero_dq_dk=single)
    if single:
        assert slice_relerr(to_host(y), inp["v"]) <= 4e-3   # Y = v, through one rounding to bf16


def test_fp16_matrix_core_two_exponential_kernels(oracle):
    _say("fp16 on matrix cores, two-exponential backward")
    for cfg, over in [(4, dict(N=2100)), (5, dict(N=1100))]:
        inp = synth.make_inputs(cfg, with_dy=True, dtype="f16", **over)
        _backward_case(oracle, inp, tol=TOL["bf16"], saved=True, variant=binding.VARIANT_TWO_EXP)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_sharp_softmax_stress(oracle, dtype):
    """Scores eight times larger: nearly one-hot softmaxes, the running max moves a lot."""
    _say("stress gain 8 %s" % dtype)
    inp = synth.make_inputs(1, B=1, H=2, N=2500, M=64, d=16, dtype=dtype, with_dy=True, score_gain=8.0)
    _forward_case(oracle, inp)
    _backward_case(oracle, inp, tol=TOL[dtype] * (3 if dtype == "f32" else 1))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_large_score_offsets(oracle, dtype):
    """Scores far from zero (|S| ~ 100 and a per-latent spread of hundreds): nothing may overflow."""
    _say("large offsets %s" % dtype)
    inp = synth.make_inputs(1, B=1, H=1, N=1500, M=64, d=16, dtype=dtype, with_dy=False)
    q, k = inp["q"].copy(), inp["k"].copy()
    k[..., 0] = 4.0                                   # S[m][n] gets + scale * 4 * q[m][0]
    q[..., 0] = np.linspace(-150.0, 150.0, q.shape[1], dtype=np.float32)[None, :]
    if dtype == "bf16":
        q, k = synth.bf16_round(q), synth.bf16_round(k)
    inp["q"], inp["k"] = q, k
    # a score of magnitude |S| carries about |S| * 2^-23 of fp32 rounding before the exponential
    _forward_case(oracle, inp, tol=1e-4 if dtype == "f32" else None)


@pytest.mark.parametrize("dtype,M,d", [("bf16", 256, 16), ("bf16", 64, 8), ("f16", 128, 32), ("bf16", 256, 32),
                                       ("f32", 64, 16)])
def test_decode_with_every_token_shifted_differently(dtype, M, d):
    """The decode's softmax runs over the latents of one token, so adding the same amount to all scores of a token
    leaves y unchanged and moves lse_dec by that amount.  Here token n's scores are shifted by a ramp from -138 to
    +138 log2 units, so the tokens of one 32-token tile differ by about 2 units and the tiles span the whole range
    of fp32 exponents that a stabiliser has to absorb, per token.  Reference: the definition, in fp64
    (Eq. flare_decode)."""
    import torch
    _say("decode, per-token score shifts, %s M=%d d=%d" % (dtype, M, d))
    N = 4000
    inp = synth.make_inputs(1, B=1, H=2, N=N, M=M, d=d, dtype=dtype, with_dy=False)
    scale = 1.0 / np.sqrt(d)
    q, k = inp["q"].copy(), inp["k"].copy()
    q[..., 0] = 16.0                                   # token n's scores get + scale * 16 * k[n][0]
    ramp = np.linspace(-1.0, 1.0, N, dtype=np.float32) * np.float32(138.0 / (scale * 16.0 * 1.4426950408889634))
    k[..., 0] = ramp[None, None, :]
    if dtype == "bf16":
        q, k = synth.bf16_round(q), synth.bf16_round(k)
    elif dtype == "f16":
        q, k = q.astype(np.float16).astype(np.float32), k.astype(np.float16).astype(np.float32)
    rng = np.random.Generator(np.random.PCG64(20250812))
    z = rng.standard_normal((1, 2, M, d)).astype(np.float32)
    dev = to_device(dict(inp, q=q, k=k))
    zt = torch.from_numpy(z).cuda()
    lse_dec = torch.empty((1, 2, N), dtype=torch.float32, device="cuda")
    y = binding.decode(dev["q"], dev["k"], zt, scale, lse_dec=lse_dec)
    torch.cuda.synchronize()
    s = scale * np.einsum("hmj,bhnj->bhnm", q.astype(np.float64), k.astype(np.float64))      # [B, H, N, M]
    top = s.max(axis=-1, keepdims=True)
    w = np.exp(s - top)
    den = w.sum(axis=-1, keepdims=True)
    y_ref = (w / den) @ z.astype(np.float64)
    lse_ref = (top + np.log(den))[..., 0]
    shift = lse_ref / np.log(2.0)
    assert shift.min() < -100.0 and shift.max() > 100.0   # the ramp does cross both limits
    tol = TOL["bf16"] if dtype == "f16" else TOL[dtype]   # 16-bit storage: the matrix-core kernels (bf16 weights)
    e_y = slice_relerr(to_host(y), y_ref)
    r_y = row_relerr(to_host(y), y_ref)
    e_l = float(np.max(np.abs(to_host(lse_dec) - lse_ref)))
    _say("   err y %.3e (worst row %.3e)  lse_dec(abs) %.3e  (tol %.0e)" % (e_y, r_y, e_l, tol))
    assert e_y <= tol and r_y <= ROW_FACTOR * tol
    # a score of magnitude |S| carries |S| * 2^-23 of fp32 rounding (2^-9 of it through bf16 keys: exact here,
    # the ramp is rounded before both sides see it)
    assert e_l <= (5e-3 if dtype != "f32" else 2e-5) + 1e-5 * float(np.max(np.abs(lse_ref)))


@pytest.mark.parametrize("cfg,over", [(2, dict(B=2, N=2050)), (4, dict(N=3001)), (5, dict(N=1999)), (3, dict(B=1, N=700))])
def test_backward_two_exponential_kernels(oracle, cfg, over):
    """The matrix-core backward has a one-exponential and a two-exponential variant of its last
    two kernels; the library picks per (b,h).  Force the second and check it to the same bar."""
    _say("backward, two-exponential kernels forced, cfg%d %s" % (cfg, over))
    inp = synth.make_inputs(cfg, with_dy=True, **over)
    dq1, dk1, dv1 = _backward_case(oracle, inp, saved=True)
    dq2, dk2, dv2 = _backward_case(oracle, inp, saved=True, variant=binding.VARIANT_TWO_EXP)
    # dV does not depend on the variant's arithmetic beyond P: identical; dq, dk agree closely
    assert slice_relerr(to_host(dq2), to_host(dq1)) <= TOL["bf16"]
    assert slice_relerr(to_host(dk2), to_host(dk1)) <= TOL["bf16"]


@pytest.mark.parametrize("cfg,over", [(4, dict(N=3001)), (2, dict(B=1, N=1500, d=8)), (2, dict(B=1, N=1500, d=4)),
                                      (4, dict(N=900, M=100, dtype="f16"))])
def test_backward_separate_dq_kernel(oracle, cfg, over):
    """At d <= 16 the dK/dV kernel also forms dQ; FLARE_VARIANT_SEPARATE_DQ runs the separate dQ kernel
    (the one d = 32 uses) on the same shapes.  Both must meet the bar and agree closely."""
    _say("backward with the separate dQ kernel, cfg%d %s" % (cfg, over))
    inp = synth.make_inputs(cfg, with_dy=True, **over)
    tol = TOL["bf16"]
    dq1, dk1, dv1 = _backward_case(oracle, inp, tol=tol, saved=True)
    dq2, dk2, dv2 = _backward_case(oracle, inp, tol=tol, saved=True, variant=binding.VARIANT_SEPARATE_DQ)
    import torch
    assert torch.equal(dv1, dv2)
    assert slice_relerr(to_host(dq2), to_host(dq1)) <= tol and slice_relerr(to_host(dk2), to_host(dk1)) <= tol


@pytest.mark.parametrize("M,d", [(64, 16), (128, 32), (256, 32)])
def test_backward_wide_score_range_picks_variant_per_head(oracle, M, d):
    """Head 0 has ordinary scores; head 1 has per-latent score offsets hundreds of log2 units apart,
    where one exponential per score would underflow: the library must take the two-exponential
    kernels for that head alone and stay within tolerance on both.  (d = 16: dQ, dK and dV from one kernel that
    holds both variants; d = 32: a dQ kernel of that kind and, at 256 latents, one dK/dV launch per variant.)"""
    _say("backward wide score range, mixed heads, M = %d, d = %d" % (M, d))
    inp = synth.make_inputs(2, B=1, H=2, N=1500, M=M, d=d, with_dy=True)
    q, k = inp["q"].copy(), inp["k"].copy()
    k[:, 1, :, 0] = 4.0
    q[1, :, 0] = np.linspace(-120.0, 120.0, q.shape[1], dtype=np.float32)
    inp["q"], inp["k"] = synth.bf16_round(q), synth.bf16_round(k)
    _, _, lse = oracle.forward(inp["q"], inp["k"], inp["v"], inp["scale"])
    spread = (lse.max(axis=2) - lse.min(axis=2))[0] * np.log2(np.e)
    _say("   lse_enc spread (log2 units) per head: %s" % np.round(spread, 1))
    assert spread[0] < 40 and spread[1] > 60      # the scenario is what the docstring says
    import torch
    dev = to_device(inp)
    dq_ref, dk_ref, dv_ref = oracle.backward(inp["q"], inp["k"], inp["v"], inp["dy"], inp["scale"])
    for saved in (True, False):
        lse_dec = torch.empty(dev["k"].shape[:3], dtype=torch.float32, device="cuda") if saved else None
        y, z, lse_g = binding.forward(dev["q"], dev["k"], dev["v"], inp["scale"], lse_dec=lse_dec)
        dq, dk, dv = binding.backward(dev["q"], dev["k"], dev["v"], dev["dy"], z, lse_g, inp["scale"],
                                      y=y if saved else None, lse_dec=lse_dec)
        torch.cuda.synchronize()
        assert float(np.max(np.abs(to_host(lse_g) - lse))) <= 5e-3 + 1e-5 * float(np.max(np.abs(lse)))
        for h in range(2):
            e = dict(dq=slice_relerr(to_host(dq)[h], dq_ref[h]), dk=slice_relerr(to_host(dk)[:, h], dk_ref[:, h]),
                     dv=slice_relerr(to_host(dv)[:, h], dv_ref[:, h]))
            _say("   saved=%s head %d: " % (saved, h) + "  ".join("%s %.3e" % kv for kv in e.items()))
            assert e["dq"] <= TOL["bf16"] and e["dv"] <= TOL["bf16"]
            # head 1: dK_n = scale * sum_m dS[m][n] q_m with |q_m[0]| up to 120 and sum_m dS ~ 0: the bf16
            # rounding of dS (2^-9 per entry) is amplified by that cancellation, whatever the kernel
            assert e["dk"] <= (TOL["bf16"] if h == 0 else 1e-1)


@pytest.mark.parametrize("key0", [15.0, 21.0])
def test_backward_with_every_score_shifted(oracle, key0):
    """All scores of head 1 are shifted by one large constant (first query coordinate 8, first key coordinate
    key0): both log-sum-exps sit at about 55 (key0 = 15) or 72 (key0 = 21) log2 units, either side of the limit
    up to which the one-exponential kernels work with weights 2^S that carry no normaliser.  Head 0 is ordinary.
    Gradients within tolerance on both sides of the limit, with saved and with recomputed statistics."""
    _say("backward, scores of one head shifted: first key coordinate %g" % key0)
    inp = synth.make_inputs(2, B=1, H=2, N=1500, M=64, d=16, with_dy=True)
    q, k = inp["q"].copy(), inp["k"].copy()
    q[1, :, 0] = 8.0
    k[:, 1, :, 0] = key0
    inp["q"], inp["k"] = synth.bf16_round(q), synth.bf16_round(k)
    _, _, lse = oracle.forward(inp["q"], inp["k"], inp["v"], inp["scale"])
    level = lse[0].mean(axis=1) * np.log2(np.e)
    _say("   lse_enc (log2 units) per head: %s" % np.round(level, 1))
    assert abs(level[0]) < 30 and ((50 < level[1] < 60) if key0 == 15.0 else (65 < level[1] < 80))
    _backward_case(oracle, inp, saved=True)
    _backward_case(oracle, inp, saved=False)


@pytest.mark.parametrize("M,d", [(64, 16), (256, 16), (128, 32), (256, 32), (64, 8)])
def test_keys_huge_where_every_latent_is_zero(oracle, M, d):
    """Every other token has a key that is huge in the dimensions where all latent queries are zero: the
    norms |q_m| |k_n| are hundreds of log2 units above the scores themselves, so any stabiliser derived
    from norms rather than from the scores would underflow every weight of those tokens."""
    _say("huge orthogonal keys M=%d d=%d" % (M, d))
    inp = synth.make_inputs(1, B=1, H=2, N=1111, M=M, d=d, dtype="bf16", with_dy=True, seed=77 + M + d)
    q, k = inp["q"].copy(), inp["k"].copy()
    q[..., d // 2:] = 0.0
    q[..., :d // 2] *= 6.0
    k[:, :, ::2, d // 2:] = 300.0
    k[:, :, 5::64, d // 2:] = -250.0          # and a few lone tokens elsewhere in a tile
    inp["q"], inp["k"] = synth.bf16_round(q), synth.bf16_round(k)
    _forward_case(oracle, inp)
    _backward_case(oracle, inp, saved=False)
    _backward_case(oracle, inp, saved=True)


def test_constant_v_gives_constant_y():
    import torch
    inp = synth.make_inputs(2, B=1, N=2000, with_dy=False)
    dev = to_device(inp)
    v = torch.full_like(dev["v"], 1.5)
    y, z, _ = binding.forward(dev["q"], dev["k"], v, inp["scale"])
    torch.cuda.synchronize()
    assert float((y.float() - 1.5).abs().max()) <= 1.5 * 2 ** -7
    assert float((z - 1.5).abs().max()) <= 1e-5


@pytest.mark.parametrize("M,d,dtype", [(282, 4, "bf16"), (512, 4, "bf16"), (282, 4, "f16"), (2, 8, "bf16"), (512, 16, "bf16")])
def test_latent_that_dominates_many_tokens(oracle, M, d, dtype):
    """Mesh-like inputs on which one latent of head 1 decodes 66 tokens almost alone (R ~ 1, Y_n ~ Z_m): there
    c - delta = <dY_n, Z_m - Y_n> cancels, and it only does so if both sides see the same Z_m.  With delta
    from a decode that rounded Z to bf16 and c from Z as a hi + lo pair that latent's row of dq_lat was wrong
    by half (dq_lat 2.9e-2 at M = 282, 6.9e-2 at M = 512).  At d <= 8 half the bar now, and no row far off;
    d = 16 (delta from the saved bf16 y, rounded independently per token) for comparison, at the bar."""
    _say("dominant latent M=%d d=%d %s" % (M, d, dtype))
    inp = synth.make_inputs(2, B=2, H=3, N=365, M=M, d=d, dtype=dtype, with_dy=True, seed=777 + 1375)
    for saved in (False, True):
        dq, _, _ = _backward_case(oracle, inp, scale=1.0 / np.sqrt(d), tol=1e-2 if d <= 8 else TOL["bf16"], saved=saved)
        dq_ref = oracle.backward(inp["q"], inp["k"], inp["v"], inp["dy"], 1.0 / np.sqrt(d))[0]
        rows = np.linalg.norm(to_host(dq) - dq_ref, axis=2) / np.linalg.norm(dq_ref, axis=2).mean(axis=1, keepdims=True)
        _say("   worst row of dq: %.2f of the mean row norm" % rows.max())
        # it was 1.5 (M = 512, d = 4).  d = 16 with the saved bf16 y: that row's error is the per-token rounding of
        # y in delta, 0.55 ... 0.61 of the mean row norm depending on where the decode's stabiliser puts the
        # rounding points of the weights (0.19 with the recomputed fp32 y); the normwise bar above is what binds
        assert rows.max() <= (0.25 if d <= 8 else 0.7)


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_zero_scale_gives_plain_means(dtype):
    """scale = 0: every score is zero, both softmaxes are uniform, so each latent holds the mean of the
    values, every token receives it back, and the scores do not depend on q or k: dq = dk = 0 and
    dv_n = mean of dy for every token (closed forms, no oracle needed)."""
    import torch
    _say("zero scale %s" % dtype)
    inp = synth.make_inputs(1, B=2, H=2, N=777, M=96, d=16, dtype=dtype, with_dy=True, seed=4242)
    dev = to_device(inp)
    y, z, lse = binding.forward(dev["q"], dev["k"], dev["v"], 0.0)
    dq, dk, dv = binding.backward(dev["q"], dev["k"], dev["v"], dev["dy"], z, lse, 0.0)
    torch.cuda.synchronize()
    tol = 1e-5 if dtype == "f32" else 2e-2
    v_mean = dev["v"].double().mean(dim=2, keepdim=True)                     # [B,H,1,d]
    g_mean = dev["dy"].double().mean(dim=2, keepdim=True)
    rel = lambda a, b: float((a.double() - b).norm() / b.norm())
    assert rel(z, v_mean.expand(-1, -1, 96, -1)) <= (1e-5 if dtype == "f32" else 2e-3)
    assert rel(y, v_mean.expand(-1, -1, 777, -1)) <= tol
    assert rel(dv, g_mean.expand(-1, -1, 777, -1)) <= tol
    assert float((lse - float(np.log(777))).abs().max()) <= 1e-5
    assert float(dq.abs().max()) == 0.0 and float(dk.float().abs().max()) == 0.0


@pytest.mark.parametrize("cfg,over", [(1, dict()), (2, dict(B=1, N=5000)), (5, dict(N=2048))])
def test_bit_reproducible(cfg, over):
    """Same inputs, same shape: identical bits on every run (fixed-order reductions)."""
    import torch
    inp = synth.make_inputs(cfg, with_dy=True, **over)
    dev = to_device(inp)
    outs = []
    for _ in range(2):
        y, z, lse = binding.forward(dev["q"], dev["k"], dev["v"], inp["scale"])
        dq, dk, dv = binding.backward(dev["q"], dev["k"], dev["v"], dev["dy"], z, lse, inp["scale"])
        torch.cuda.synchronize()
        outs.append([t.clone() for t in (y, z, lse, dq, dk, dv)])
    for a, b in zip(*outs):
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))


def test_encode_decode_equal_forward():
    import torch
    inp = synth.make_inputs(3, B=1, N=1111, with_dy=False)
    dev = to_device(inp)
    y, z, lse = binding.forward(dev["q"], dev["k"], dev["v"], inp["scale"])
    z2, lse2 = binding.encode(dev["q"], dev["k"], dev["v"], inp["scale"])
    y2 = binding.decode(dev["q"], dev["k"], z2, inp["scale"])
    torch.cuda.synchronize()
    assert torch.equal(z, z2) and torch.equal(lse, lse2) and torch.equal(y.view(torch.uint8), y2.view(torch.uint8))


def test_side_stream_and_caller_buffers():
    """Runs on a caller-chosen stream with caller-owned outputs and workspace."""
    import torch
    inp = synth.make_inputs(1, with_dy=False)
    dev = to_device(inp)
    y0, z0, l0 = binding.forward(dev["q"], dev["k"], dev["v"], inp["scale"])
    torch.cuda.synchronize()
    f, _ = binding.workspace_bytes(inp["B"], inp["H"], inp["N"], inp["M"], inp["d"], binding.FLARE_F32)
    ws = torch.empty(f, dtype=torch.uint8, device="cuda")
    y, z, l = torch.empty_like(y0), torch.empty_like(z0), torch.empty_like(l0)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        binding.forward(dev["q"], dev["k"], dev["v"], inp["scale"], y=y, z=z, lse_enc=l, workspace=ws, stream=s)
    s.synchronize()
    assert torch.equal(y, y0) and torch.equal(z, z0) and torch.equal(l, l0)
    with pytest.raises(binding.FlareError):
        binding.forward(dev["q"], dev["k"], dev["v"], inp["scale"], workspace=ws[:64])
