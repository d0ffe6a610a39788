"""Seeded synthetic inputs for the FLARE token mixer.

This module only draws numbers and shapes them; it contains none of the method's
arithmetic (no scores, no softmax).  It is the one piece shared by the HIP path's
callers and by the CPU oracle's callers, so that both consume identical values.

The five workloads mirror the shapes the paper times or trains on (Fig. 2 and
Appendix G "Time and memory complexity": C=128, H=8, up to one million tokens;
Section 5.2 / Appendix E: million-point meshes; Table 2: 4k-token sequences).
The paper's datasets are not available, so smooth mesh-like fields stand in for them:
points drawn uniformly in the unit square / cube, three smooth sine fields of the
coordinates, lifted to C channels and projected to keys and values.

Every array is returned as float32 holding values exactly representable in the
workload's dtype (bf16 inputs are rounded once here, round-to-nearest-even), so the
oracle (after an exact upcast to fp64) and the GPU see the same numbers.
"""
import math

import numpy as np

SEED_BASE = 250812594

# id -> shape and recipe.  `kind`: "normal" (i.i.d. N(0,1)) or "mesh" (smooth fields on points).
CONFIGS = {
    1: dict(B=1, H=4, d=32, N=1024, M=64, dtype="f32", kind="normal", backward=False),
    2: dict(B=4, H=8, d=16, N=16384, M=64, dtype="bf16", kind="mesh", mesh_dim=2, backward=False),
    3: dict(B=32, H=8, d=32, N=4096, M=128, dtype="bf16", kind="normal", backward=False),
    4: dict(B=1, H=8, d=16, N=1000000, M=256, dtype="bf16", kind="mesh", mesh_dim=3, backward=False),
    5: dict(B=1, H=8, d=32, N=262144, M=256, dtype="bf16", kind="normal", backward=True),
}


def bf16_round(x):
    """Round float32 values to the nearest bf16 (ties to even); result is float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(x.shape)


def bf16_bits(x):
    """uint16 bit patterns of float32 values that are already bf16-representable."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    if np.any(u & 0xFFFF):
        raise ValueError("values are not bf16-representable; call bf16_round first")
    return (u >> 16).astype(np.uint16).reshape(x.shape)


def bf16_from_bits(b):
    """float32 values of uint16 bf16 bit patterns."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).reshape(b.shape)


def _mesh_item(rng, N, C, H, d, mesh_dim):
    """One batch item: keys/values [H,N,d] from smooth fields on N random mesh points."""
    p = rng.random((N, mesh_dim), dtype=np.float32)
    a = rng.integers(1, 4, size=(3, mesh_dim)).astype(np.float32)
    phi = (rng.random(3, dtype=np.float32) * (2.0 * math.pi)).astype(np.float32)
    fields = np.sin(2.0 * math.pi * (p @ a.T) + phi).astype(np.float32)        # [N,3]
    feat = np.concatenate([p, fields], axis=1)                                  # [N,mesh_dim+3]
    lift = rng.standard_normal((feat.shape[1], C), dtype=np.float32)
    x = feat @ lift + 0.1 * rng.standard_normal((N, C), dtype=np.float32)       # [N,C]
    w_k = rng.standard_normal((C, C), dtype=np.float32) / np.float32(math.sqrt(C))
    w_v = rng.standard_normal((C, C), dtype=np.float32) / np.float32(math.sqrt(C))
    k = (x @ w_k).reshape(N, H, d).transpose(1, 0, 2)
    v = (x @ w_v).reshape(N, H, d).transpose(1, 0, 2)
    return np.ascontiguousarray(k), np.ascontiguousarray(v)


def make_inputs(cfg, *, B=None, H=None, N=None, M=None, d=None, dtype=None, with_dy=None,
                score_gain=1.0, seed=None):
    """Draw the inputs of workload `cfg` (1..5), optionally at an overridden size.

    Returns a dict: q[H,M,d], k,v[B,H,N,d] (and dy[B,H,N,d] when asked) as float32 arrays
    representable in `dtype`; `scale` (= 1/sqrt(d), a multiplier on q.k); the shape fields.
    `score_gain` multiplies q before rounding (a sharper-softmax stress case).
    """
    c = dict(CONFIGS[cfg])
    B = c["B"] if B is None else B
    H = c["H"] if H is None else H
    N = c["N"] if N is None else N
    M = c["M"] if M is None else M
    d = c["d"] if d is None else d
    dtype = c["dtype"] if dtype is None else dtype
    with_dy = c["backward"] if with_dy is None else with_dy
    seed = SEED_BASE + cfg if seed is None else seed
    rng = np.random.Generator(np.random.PCG64(seed))

    q = rng.standard_normal((H, M, d), dtype=np.float32) * np.float32(score_gain)
    if c["kind"] == "normal":
        k = rng.standard_normal((B, H, N, d), dtype=np.float32)
        v = rng.standard_normal((B, H, N, d), dtype=np.float32)
    else:
        k = np.empty((B, H, N, d), np.float32)
        v = np.empty((B, H, N, d), np.float32)
        for b in range(B):
            item = np.random.Generator(np.random.PCG64(seed * 1000 + b))
            k[b], v[b] = _mesh_item(item, N, H * d, H, d, c["mesh_dim"])
    out = dict(cfg=cfg, B=B, H=H, N=N, M=M, d=d, dtype=dtype, scale=1.0 / math.sqrt(d))
    dy = rng.standard_normal((B, H, N, d), dtype=np.float32) if with_dy else None
    if dtype == "bf16":
        q, k, v = bf16_round(q), bf16_round(k), bf16_round(v)
        if dy is not None:
            dy = bf16_round(dy)
    elif dtype == "f16":
        q, k, v = (x.astype(np.float16).astype(np.float32) for x in (q, k, v))
        if dy is not None:
            dy = dy.astype(np.float16).astype(np.float32)
    elif dtype != "f32":
        raise ValueError("dtype must be 'f32', 'bf16' or 'f16'")
    out.update(q=q, k=k, v=v)
    if dy is not None:
        out["dy"] = dy
    return out


def describe(cfg):
    c = CONFIGS[cfg]
    if c["kind"] == "normal":
        data = "q,k,v~N(0,1)"
    else:
        data = "%d-D uniform mesh points + 3 smooth sine fields, lifted to C=%d, random K/V projections" % (
            c["mesh_dim"], c["H"] * c["d"])
    return "cfg%d B=%d H=%d d=%d N=%d M=%d %s; %s; seed %d" % (
        cfg, c["B"], c["H"], c["d"], c["N"], c["M"], c["dtype"], data, SEED_BASE + cfg)
