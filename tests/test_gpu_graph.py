"""The library only enqueues kernels on the caller's stream (no allocation, no memset, no synchronisation),
so a training step can be captured in a HIP graph.  Capture flare_forward + flare_backward with caller-owned
buffers, replay it several times with other GPU work and synchronisations in between, and require every replay
to reproduce the eager result bit for bit."""
import pytest

from paper_2508_12594_amd import binding, synth
from tests._util import to_device

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cfg,over", [(2, dict(B=2, N=3000)), (5, dict(N=2000)), (1, dict(N=700)),
                                      (4, dict(N=2500, M=300))])
def test_step_in_a_hip_graph(cfg, over):
    import torch
    print("[case] graph capture cfg%d %s" % (cfg, over), flush=True)
    inp = synth.make_inputs(cfg, with_dy=True, **over)
    scale = inp["scale"]
    dev = to_device(inp)
    q, k, v, dy = dev["q"], dev["k"], dev["v"], dev["dy"]
    B, H, N, d = k.shape
    M = q.shape[1]
    f32 = dict(dtype=torch.float32, device="cuda")
    code = binding._dtype_code(k)
    fwd_b, bwd_b = binding.workspace_bytes(B, H, N, M, d, code)
    ws_f = torch.empty(max(fwd_b, 256), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(max(bwd_b, 256), dtype=torch.uint8, device="cuda")

    def buffers():
        return dict(y=torch.empty_like(k), z=torch.empty((B, H, M, d), **f32), lse=torch.empty((B, H, M), **f32),
                    lse_dec=torch.empty((B, H, N), **f32), dq=torch.empty((H, M, d), **f32),
                    dk=torch.empty_like(k), dv=torch.empty_like(k))

    def step(o):
        binding.forward(q, k, v, scale, y=o["y"], z=o["z"], lse_enc=o["lse"], lse_dec=o["lse_dec"], workspace=ws_f)
        binding.backward(q, k, v, dy, o["z"], o["lse"], scale, y=o["y"], lse_dec=o["lse_dec"], dq_lat=o["dq"],
                         dk=o["dk"], dv=o["dv"], workspace=ws_b)

    eager = buffers()
    step(eager)
    torch.cuda.synchronize()

    out = buffers()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):       # warm-up on the capture stream, as torch asks for
        step(out)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(out)
    for rep in range(3):
        for t in out.values():
            t.fill_(float("nan"))        # eager work between the replays (a fill kernel, not a memset node)
        torch.cuda.synchronize()
        graph.replay()
        scratch = (k.float() * 2).sum()  # unrelated eager work queued behind the replay
        torch.cuda.synchronize()
        for name in out:
            assert torch.equal(out[name], eager[name]), "replay %d: %s differs from the eager run" % (rep, name)
        assert torch.isfinite(scratch)


def _capture_and_replay(run, make_out, what):
    """run(out) enqueues library calls that fill the dict of tensors `out`; eager result against three replays."""
    import torch
    eager = make_out()
    run(eager)
    torch.cuda.synchronize()
    out = make_out()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(out)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run(out)
    for rep in range(3):
        for t in out.values():
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name in out:
            assert torch.equal(out[name], eager[name]), "%s, replay %d: %s differs from the eager run" % (what, rep, name)


def test_other_entry_points_in_a_hip_graph():
    """The fused projection, the forward on the library's static scratch and the spectral analysis: each captured
    with caller-owned buffers and replayed, bit for bit the eager result."""
    import torch
    import ctypes
    inp = synth.make_inputs(4, with_dy=False, N=3001)
    scale = inp["scale"]
    dev = to_device(inp)
    q, k, v = dev["q"], dev["k"], dev["v"]
    B, H, N, d = k.shape
    M = q.shape[1]
    C = H * d
    f32 = dict(dtype=torch.float32, device="cuda")
    code = binding._dtype_code(k)
    fwd_b, _ = binding.workspace_bytes(B, H, N, M, d, code)
    ws = torch.empty(max(fwd_b, 256), dtype=torch.uint8, device="cuda")

    print("[case] graph capture: forward on the static scratch", flush=True)
    _capture_and_replay(
        lambda o: binding.forward_static(q, k, v, scale, o["y"], o["z"], o["lse"], lse_dec=o["lse_dec"]),
        lambda: dict(y=torch.empty_like(k), z=torch.empty((B, H, M, d), **f32), lse=torch.empty((B, H, M), **f32),
                     lse_dec=torch.empty((B, H, N), **f32)), "flare_forward_static")

    print("[case] graph capture: forward with the fused output projection", flush=True)
    kn, vn = k.permute(0, 2, 1, 3).contiguous(), v.permute(0, 2, 1, 3).contiguous()
    gen = torch.Generator(device="cpu").manual_seed(3)
    w_out = (torch.randn((C, C), generator=gen) / C ** 0.5).to(device="cuda", dtype=k.dtype)
    bias = torch.randn((C,), generator=gen).to(device="cuda", dtype=torch.float32)
    _capture_and_replay(
        lambda o: binding.forward_project(q, kn, vn, w_out, scale, bias=bias, out=o["out"], y=o["y"], z=o["z"],
                                          lse_enc=o["lse"], lse_dec=o["lse_dec"], workspace=ws),
        lambda: dict(out=torch.empty((B, N, C), dtype=k.dtype, device="cuda"), y=torch.empty_like(kn),
                     z=torch.empty((B, H, M, d), **f32), lse=torch.empty((B, H, M), **f32),
                     lse_dec=torch.empty((B, H, N), **f32)), "flare_forward_project")

    print("[case] graph capture: spectral analysis", flush=True)
    lse_dec = torch.empty((B, H, N), **f32)
    _, _, lse_enc = binding.forward(q, k, v, scale, lse_dec=lse_dec, workspace=ws)
    shp = binding._shape_of(q, k, "bhnd")
    need = ctypes.c_size_t(0)
    binding._check(binding.load().flare_spectral_workspace_bytes(ctypes.byref(shp), ctypes.byref(need)), "bytes")
    ws_s = torch.empty(max(int(need.value), 256), dtype=torch.uint8, device="cuda")

    def spectral(o):
        binding._check(binding.load().flare_spectral(
            ctypes.byref(shp), ctypes.c_void_p(q.data_ptr()), ctypes.c_void_p(k.data_ptr()),
            ctypes.c_void_p(lse_enc.data_ptr()), ctypes.c_void_p(lse_dec.data_ptr()), ctypes.c_float(scale),
            ctypes.c_int(0), ctypes.c_void_p(o["ev"].data_ptr()), ctypes.c_void_p(o["zv"].data_ptr()),
            ctypes.c_void_p(o["gram"].data_ptr()), ctypes.c_void_p(ws_s.data_ptr()), ctypes.c_size_t(ws_s.numel()),
            ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)), "flare_spectral")
    _capture_and_replay(spectral, lambda: dict(ev=torch.empty((B, H, M), **f32), zv=torch.empty((B, H, M, d), **f32),
                                               gram=torch.empty((B, H, M, M), **f32)), "flare_spectral")
