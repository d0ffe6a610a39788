"""Helpers shared by the GPU parity tests (no method arithmetic here)."""
import numpy as np

# Tolerances on the max normwise relative error (per (b,h) slice, Frobenius norm):
# fp32 path 1e-5; bf16 inputs with fp32 accumulation 2e-2.
# fp16 storage on the fp32 vector kernels: only the outputs are rounded (2^-11 relative) -> 1e-3; on
# the matrix-core path the softmax weights are bf16 as with bf16 storage -> the bf16 bar (tol_for).
TOL = {"f32": 1e-5, "bf16": 2e-2, "f16": 1e-3}


def on_matrix_cores(dtype, M, N=None):
    """The library's documented rule: 16-bit storage with at most 2048 latents per head and at least 16
    tokens runs on the matrix-core kernels (tiles of 32 latents, the last ones padded)."""
    return dtype != "f32" and M <= 2048 and (N is None or N >= 16)


def tol_for(inp):
    if inp["dtype"] == "f16" and on_matrix_cores("f16", inp["q"].shape[1], inp["k"].shape[2]):
        return TOL["bf16"]
    return TOL[inp["dtype"]]


def slice_relerr(got, ref):
    """max over leading-index slices [..., :, :] of ||got-ref||_F / ||ref||_F, in fp64."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    g = got.reshape(-1, got.shape[-2] * got.shape[-1])
    r = ref.reshape(-1, ref.shape[-2] * ref.shape[-1])
    num = np.linalg.norm(g - r, axis=1)
    den = np.linalg.norm(r, axis=1)
    return float(np.max(num / np.maximum(den, 1e-300)))


def row_relerr(got, ref):
    """Worst row: max over rows (last axis = one token's or latent's vector) of ||got_n - ref_n|| divided by the
    root-mean-square row norm of ref, per leading-index slice [..., :, :]; the maximum over slices.  A few wrong
    rows among 10^5 vanish in a Frobenius norm; they do not vanish here."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    g = got.reshape(-1, got.shape[-2], got.shape[-1])
    r = ref.reshape(-1, ref.shape[-2], ref.shape[-1])
    num = np.linalg.norm(g - r, axis=2).max(axis=1)
    rms = np.sqrt((np.linalg.norm(r, axis=2) ** 2).mean(axis=1))
    return float(np.max(num / np.maximum(rms, 1e-300)))


# Bound on row_relerr as a multiple of the normwise bar.  The rounding of the softmax weights to bf16 is
# independent from row to row, so among 10^5 ... 10^6 rows the worst one lies a few standard deviations above
# the typical one, and a row whose reference is far longer than the rms row carries proportionally more; measured
# worst rows: 0.6 ... 3 x the normwise error of the same tensor.  A row that is simply wrong (a lost tile, a
# wrong head, an unmasked tail) is off by 1 or more of the rms row norm, 50 x the bf16 bar and 10^5 x the fp32 bar.
ROW_FACTOR = 8.0


def to_device(inp, names=("q", "k", "v", "dy")):
    """numpy float32 arrays (already representable in the workload dtype) -> device tensors."""
    import torch
    dt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[inp["dtype"]]
    out = {}
    for n in names:
        if n in inp:
            out[n] = torch.from_numpy(inp[n]).to(device="cuda", dtype=dt).contiguous()
    return out


def to_host(t):
    import torch
    return t.detach().to(torch.float32).cpu().numpy()
