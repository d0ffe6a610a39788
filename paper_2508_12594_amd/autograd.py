"""torch.autograd wrapper around the binding: `flare_mixer(q_lat, k, v, scale)` is differentiable.

Nothing is computed here: the forward calls flare_forward (keeping z, lse_enc, lse_dec and y for the
backward), the backward calls flare_backward; the only torch arithmetic is the cast of dq_lat (fp32 out
of the library) to q_lat's dtype, which autograd requires of a gradient.  This is how the paper's layer
would use the operator in place of its two attention calls (listing in Section 3.1).
"""
from . import binding


def _function():
    import torch

    class FlareMixer(torch.autograd.Function):
        @staticmethod
        def forward(ctx, q_lat, k, v, scale, layout, y_f32):
            q_lat, k, v = q_lat.contiguous(), k.contiguous(), v.contiguous()
            B, N = (k.shape[0], k.shape[2]) if layout == "bhnd" else (k.shape[0], k.shape[1])
            H = k.shape[1] if layout == "bhnd" else k.shape[2]
            lse_dec = torch.empty((B, H, N), dtype=torch.float32, device=k.device)
            y, z, lse_enc = binding.forward(q_lat, k, v, scale, lse_dec=lse_dec, layout=layout, y_f32=y_f32)
            ctx.save_for_backward(q_lat, k, v, y, z, lse_enc, lse_dec)
            ctx.scale, ctx.layout = scale, layout
            return y

        @staticmethod
        def backward(ctx, dy):
            q_lat, k, v, y, z, lse_enc, lse_dec = ctx.saved_tensors
            # (with an fp32 y autograd hands over an fp32 dY: the library takes it in the storage type)
            dq, dk, dv = binding.backward(q_lat, k, v, dy.to(k.dtype).contiguous(), z, lse_enc, ctx.scale, y=y,
                                          lse_dec=lse_dec, layout=ctx.layout)
            return dq.to(q_lat.dtype), dk, dv, None, None, None

    return FlareMixer


_FN = None


def flare_mixer(q_lat, k, v, scale, layout="bhnd", y_f32=False):
    """y = FLARE(q_lat, k, v): q_lat [H,M,d] (or [M,d]: shared latents), k, v [B,H,N,d] ('bhnd') or
    [B,N,H,d] ('bnhd'); returns y in k's shape and dtype.  Differentiable in q_lat, k and v.

    y_f32 (16-bit inputs, at most 2048 latents): y comes back in fp32 and the backward reads it instead of
    recomputing the token statistics, which pays at d < 16 (flare_shape.y_f32)."""
    global _FN
    if _FN is None:
        _FN = _function()
    return _FN.apply(q_lat, k, v, float(scale), layout, bool(y_f32))
