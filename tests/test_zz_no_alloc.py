"""flare_forward_static (the entry point that allocates nothing) against flare_forward, through the C ABI.

Two calls in a row on the same GPU, the second with a smaller input: the static scratch keeps the first
call's contents, and nothing of them may leak into the second result.  Same kernels, same partial-slot
geometry, so the outputs must agree bit for bit (which is within the operator's tolerance a fortiori).
"""
import ctypes

import numpy as np
import pytest

from paper_2508_12594_amd import binding, synth

pytestmark = pytest.mark.gpu


def _call(lib, fn, shp, t, scale, ws=None):
    import torch
    B, H, N, M, d = shp.B, shp.H, shp.N, shp.M, shp.d
    y = torch.full_like(t["k"], float("nan"))
    z = torch.full((B, H, M, d), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((B, H, M), float("nan"), dtype=torch.float32, device="cuda")
    lse_dec = torch.full((B, H, N), float("nan"), dtype=torch.float32, device="cuda")
    p = lambda x: ctypes.c_void_p(x.data_ptr())
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if fn == "static":
        rc = lib.flare_forward_static(ctypes.byref(shp), p(t["q"]), p(t["k"]), p(t["v"]), p(y), p(z), p(lse),
                                      p(lse_dec), ctypes.c_float(scale), stream)
    else:
        rc = lib.flare_forward(ctypes.byref(shp), p(t["q"]), p(t["k"]), p(t["v"]), p(y), p(z), p(lse), p(lse_dec),
                               ctypes.c_float(scale), p(ws), ctypes.c_size_t(ws.numel()), stream)
    assert rc == 0, binding.strerror(rc)
    torch.cuda.synchronize()
    return y, z, lse, lse_dec


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_static_scratch_forward_matches_workspace_forward(dtype):
    import torch
    lib = binding.load()
    tdt = {"bf16": torch.bfloat16, "f32": torch.float32}[dtype]
    code = {"bf16": binding.FLARE_BF16, "f32": binding.FLARE_F32}[dtype]
    # the second call is smaller in every respect: fewer tokens (ragged against the 32-token tiles), fewer
    # latents, fewer heads -- its partial slots cover only the beginning of what the first call left behind
    for B, H, N, M, d, seed in [(2, 4, 9001, 256, 16, 11), (1, 2, 1237, 96, 16, 12)]:
        inp = synth.make_inputs(2, B=B, H=H, N=N, M=M, d=d, dtype=dtype, with_dy=False, seed=seed)
        t = {n: torch.from_numpy(inp[n]).to("cuda", tdt).contiguous() for n in ("q", "k", "v")}
        shp = binding.FlareShape(B, H, N, M, d, code, binding.FLARE_BHND, 0, 0)
        fwd_b, _ = binding.workspace_bytes(B, H, N, M, d, code)
        assert fwd_b <= binding.STATIC_SCRATCH_BYTES
        # the reference call gets a workspace full of NaN bit patterns: whatever it reads, it wrote before
        ws = torch.full((max(fwd_b, 256),), 0xFF, dtype=torch.uint8, device="cuda")
        want = _call(lib, "workspace", shp, t, inp["scale"], ws)
        got = _call(lib, "static", shp, t, inp["scale"])
        for name, a, b in zip(("y", "z", "lse_enc", "lse_dec"), got, want):
            a, b = a.float().cpu().numpy(), b.float().cpu().numpy()
            assert np.isfinite(a).all(), name
            assert np.array_equal(a, b), "%s differs (N=%d, M=%d): max |diff| %.3e" % (name, N, M, np.abs(a - b).max())


def test_static_scratch_refuses_shapes_beyond_its_size():
    import torch
    lib = binding.load()
    B, H, N, M, d = 1, 8, 1 << 20, 2048, 8          # 1.2 GiB of per-chunk decode rows
    fwd_b, _ = binding.workspace_bytes(B, H, N, M, d, binding.FLARE_BF16)
    assert fwd_b > binding.STATIC_SCRATCH_BYTES
    shp = binding.FlareShape(B, H, N, M, d, binding.FLARE_BF16, binding.FLARE_BHND, 0, 0)
    x = torch.zeros(4096, dtype=torch.uint8, device="cuda")     # never touched: the size check comes first
    p = ctypes.c_void_p(x.data_ptr())
    rc = lib.flare_forward_static(ctypes.byref(shp), p, p, p, p, p, p, None, ctypes.c_float(1.0), None)
    assert rc == -6 and "static" in binding.strerror(rc)
