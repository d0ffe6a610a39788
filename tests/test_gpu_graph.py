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
