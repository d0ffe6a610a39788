"""Thin Python binding of libflare.so (see include/flare.h).

Argument marshalling only: every step of the operator runs in the library's HIP kernels.
torch is used for device memory and for the current stream, nothing else.  There is no
fallback: if the library is missing or a call fails, an exception is raised.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libflare.so")

FLARE_F32 = 0
FLARE_BF16 = 1
FLARE_F16 = 2
FLARE_BHND = 0   # token tensors [B,H,N,d]
FLARE_BNHD = 1   # token tensors [B,N,H,d] (= [B,N,C], C = H*d)
LAYOUTS = {"bhnd": FLARE_BHND, "bnhd": FLARE_BNHD}
VARIANT_TWO_EXP = 1       # flare_variant bits of include/flare.h (tests and A/B measurements of the backward)
VARIANT_SEPARATE_DQ = 2

EXPORTS = [
    "flare_version", "flare_strerror", "flare_workspace_bytes", "flare_encode", "flare_decode",
    "flare_forward", "flare_forward_static", "flare_decode_project", "flare_forward_project", "flare_backward", "flare_profile_enable", "flare_profile_kernels",
    "flare_profile_name", "flare_profile_read", "flare_spectral_workspace_bytes", "flare_spectral",
]


class FlareShape(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int), ("H", ctypes.c_int), ("N", ctypes.c_int), ("M", ctypes.c_int),
                ("d", ctypes.c_int), ("dtype", ctypes.c_int), ("layout", ctypes.c_int),
                ("shared_latents", ctypes.c_int), ("y_f32", ctypes.c_int), ("variant", ctypes.c_int)]


class FlareError(RuntimeError):
    pass


_lib = None


def load():
    """dlopen libflare.so (built by paper_2508_12594_amd.build); raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    path = LIB_PATH    # (to time another build, point LIB_PATH at it before the first call)
    if not os.path.exists(path):
        raise FlareError("libflare.so not found at %s: run `python -m paper_2508_12594_amd.build`" % path)
    lib = ctypes.CDLL(path)
    vp, fp, sp = ctypes.c_void_p, ctypes.c_void_p, ctypes.POINTER(FlareShape)
    lib.flare_version.restype = ctypes.c_int
    lib.flare_strerror.restype = ctypes.c_char_p
    lib.flare_strerror.argtypes = [ctypes.c_int]
    lib.flare_workspace_bytes.argtypes = [sp, ctypes.POINTER(ctypes.c_size_t), ctypes.POINTER(ctypes.c_size_t)]
    lib.flare_encode.argtypes = [sp, vp, vp, vp, fp, fp, ctypes.c_float, vp, ctypes.c_size_t, vp]
    lib.flare_decode.argtypes = [sp, vp, vp, fp, vp, fp, ctypes.c_float, vp, ctypes.c_size_t, vp]
    lib.flare_forward.argtypes = [sp, vp, vp, vp, vp, fp, fp, fp, ctypes.c_float, vp, ctypes.c_size_t, vp]
    lib.flare_forward_static.argtypes = [sp, vp, vp, vp, vp, fp, fp, fp, ctypes.c_float, vp]
    lib.flare_forward_static.restype = ctypes.c_int
    lib.flare_decode_project.argtypes = [sp, vp, vp, fp, vp, fp, vp, vp, fp, ctypes.c_float, vp]
    lib.flare_decode_project.restype = ctypes.c_int
    lib.flare_forward_project.argtypes = [sp, vp, vp, vp, vp, fp, vp, vp, fp, fp, fp, ctypes.c_float, vp,
                                          ctypes.c_size_t, vp]
    lib.flare_forward_project.restype = ctypes.c_int
    lib.flare_backward.argtypes = [sp, vp, vp, vp, vp, fp, vp, fp, fp, fp, vp, vp, ctypes.c_float, vp,
                                   ctypes.c_size_t, vp]
    lib.flare_spectral_workspace_bytes.argtypes = [sp, ctypes.POINTER(ctypes.c_size_t)]
    lib.flare_spectral.argtypes = [sp, vp, vp, fp, fp, ctypes.c_float, ctypes.c_int, fp, fp, fp, vp, ctypes.c_size_t, vp]
    lib.flare_profile_enable.argtypes = [ctypes.c_int]
    lib.flare_profile_name.restype = ctypes.c_char_p
    lib.flare_profile_name.argtypes = [ctypes.c_int]
    lib.flare_profile_read.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int)]
    for name in ("flare_spectral_workspace_bytes", "flare_spectral", "flare_workspace_bytes", "flare_encode", "flare_decode", "flare_forward", "flare_backward",
                 "flare_profile_enable", "flare_profile_kernels", "flare_profile_read"):
        getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def strerror(code):
    return load().flare_strerror(int(code)).decode()


def _check(code, what):
    if code != 0:
        raise FlareError("%s failed: %d (%s)" % (what, code, strerror(code)))


def version():
    return int(load().flare_version())


def _torch():
    import torch
    return torch


def _dtype_code(t):
    torch = _torch()
    if t.dtype == torch.float32:
        return FLARE_F32
    if t.dtype == torch.bfloat16:
        return FLARE_BF16
    if t.dtype == torch.float16:
        return FLARE_F16
    raise FlareError("dtype must be float32, bfloat16 or float16, got %s" % t.dtype)


def _shape_of(q, k, layout="bhnd", y_f32=False):
    if layout not in LAYOUTS:
        raise FlareError("layout must be 'bhnd' or 'bnhd'")
    if q.dim() not in (2, 3) or k.dim() != 4:
        raise FlareError("expected q_lat[H,M,d] (or [M,d]: one latent sequence shared by all heads) and "
                         "k[B,H,N,d] (layout 'bhnd') or k[B,N,H,d] (layout 'bnhd')")
    if layout == "bhnd":
        B, Hk, N, dk = k.shape
    else:
        B, N, Hk, dk = k.shape
    shared = q.dim() == 2
    H, M, d = (Hk,) + tuple(q.shape) if shared else tuple(q.shape)
    if Hk != H or dk != d or q.dtype != k.dtype:
        raise FlareError("q_lat and k disagree on H, d or dtype")
    return FlareShape(B, H, N, M, d, _dtype_code(k), LAYOUTS[layout], 1 if shared else 0, 1 if y_f32 else 0)


def _wants_f32_y(y, k, y_f32):
    """flare_shape.y_f32: asked for, or implied by an fp32 y next to 16-bit token tensors."""
    torch = _torch()
    return bool(y_f32) or (y is not None and y.dtype == torch.float32 and k.dtype != torch.float32)


def _dev(t, name, dtype=None, shape=None):
    if not t.is_cuda or not t.is_contiguous():
        raise FlareError("%s must be a contiguous device tensor" % name)
    if dtype is not None and t.dtype != dtype:
        raise FlareError("%s must have dtype %s" % (name, dtype))
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise FlareError("%s must have shape %s, got %s" % (name, tuple(shape), tuple(t.shape)))
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    torch = _torch()
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def workspace_bytes(B, H, N, M, d, dtype_code, y_f32=False):
    """(forward bytes, backward bytes) of scratch for this shape (the same for both layouts)."""
    return _shape_workspace_bytes(FlareShape(B, H, N, M, d, dtype_code, FLARE_BHND, 0, 1 if y_f32 else 0))


def _shape_workspace_bytes(shp):
    f, b = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(load().flare_workspace_bytes(ctypes.byref(shp), ctypes.byref(f), ctypes.byref(b)),
           "flare_workspace_bytes")
    return int(f.value), int(b.value)


def _workspace(shp, which, workspace, device, stream=None):
    torch = _torch()
    f, b = _shape_workspace_bytes(shp)
    need = f if which == "fwd" else b
    if workspace is None:
        # A temporary block: the kernels are only enqueued when the call returns, so the caching allocator must
        # learn on which stream they run, or it could hand the block to other work on the allocating stream
        # while kernels on `stream` still use it.
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=device)
        if stream is not None and stream != torch.cuda.current_stream():
            workspace.record_stream(stream)
    if workspace.dtype != torch.uint8:
        raise FlareError("workspace must be a uint8 tensor")
    return workspace, ctypes.c_void_p(workspace.data_ptr()), ctypes.c_size_t(workspace.numel())


def encode(q_lat, k, v, scale, z=None, lse_enc=None, workspace=None, stream=None, layout="bhnd"):
    """flare_encode: returns (z[B,H,M,d] fp32, lse_enc[B,H,M] fp32)."""
    torch = _torch()
    shp = _shape_of(q_lat, k, layout)
    if z is None:
        z = torch.empty((shp.B, shp.H, shp.M, shp.d), dtype=torch.float32, device=k.device)
    if lse_enc is None:
        lse_enc = torch.empty((shp.B, shp.H, shp.M), dtype=torch.float32, device=k.device)
    ws, ws_p, ws_n = _workspace(shp, "fwd", workspace, k.device, stream)
    _check(load().flare_encode(ctypes.byref(shp), _dev(q_lat, "q_lat"), _dev(k, "k"),
                               _dev(v, "v", k.dtype, k.shape),
                               _dev(z, "z", torch.float32, (shp.B, shp.H, shp.M, shp.d)),
                               _dev(lse_enc, "lse_enc", torch.float32, (shp.B, shp.H, shp.M)),
                               ctypes.c_float(scale), ws_p, ws_n, _stream(stream)), "flare_encode")
    return z, lse_enc


def _opt_lse_dec(lse_dec, shp):
    torch = _torch()
    if lse_dec is None:
        return None
    return _dev(lse_dec, "lse_dec", torch.float32, (shp.B, shp.H, shp.N))


def decode(q_lat, k, z, scale, y=None, lse_dec=None, workspace=None, stream=None, layout="bhnd", y_f32=False):
    """flare_decode: returns y (k's shape; k's dtype, or fp32 with y_f32 / when an fp32 y is passed);
    fills lse_dec[B,H,N] (fp32) when given."""
    torch = _torch()
    f32y = _wants_f32_y(y, k, y_f32)
    shp = _shape_of(q_lat, k, layout, f32y)
    ydt = torch.float32 if f32y else k.dtype
    if y is None:
        y = torch.empty(k.shape, dtype=ydt, device=k.device)
    ws, ws_p, ws_n = _workspace(shp, "fwd", workspace, k.device, stream)
    _check(load().flare_decode(ctypes.byref(shp), _dev(q_lat, "q_lat"), _dev(k, "k"),
                               _dev(z, "z", torch.float32, (shp.B, shp.H, shp.M, shp.d)),
                               _dev(y, "y", ydt, k.shape), _opt_lse_dec(lse_dec, shp),
                               ctypes.c_float(scale), ws_p, ws_n, _stream(stream)),
           "flare_decode")
    return y


def forward(q_lat, k, v, scale, y=None, z=None, lse_enc=None, lse_dec=None, workspace=None, stream=None,
            layout="bhnd", y_f32=False):
    """flare_forward: returns (y, z, lse_enc); fills lse_dec[B,H,N] (fp32) when given.

    layout 'bhnd': k, v, y are [B,H,N,d]; 'bnhd': they are [B,N,H,d].  y_f32 (or an fp32 y next to 16-bit
    inputs): y is written in fp32, for a backward that takes delta from it (flare_shape.y_f32)."""
    torch = _torch()
    f32y = _wants_f32_y(y, k, y_f32)
    shp = _shape_of(q_lat, k, layout, f32y)
    ydt = torch.float32 if f32y else k.dtype
    if y is None:
        y = torch.empty(k.shape, dtype=ydt, device=k.device)
    if z is None:
        z = torch.empty((shp.B, shp.H, shp.M, shp.d), dtype=torch.float32, device=k.device)
    if lse_enc is None:
        lse_enc = torch.empty((shp.B, shp.H, shp.M), dtype=torch.float32, device=k.device)
    ws, ws_p, ws_n = _workspace(shp, "fwd", workspace, k.device, stream)
    _check(load().flare_forward(ctypes.byref(shp), _dev(q_lat, "q_lat"), _dev(k, "k"),
                                _dev(v, "v", k.dtype, k.shape), _dev(y, "y", ydt, k.shape),
                                _dev(z, "z", torch.float32, (shp.B, shp.H, shp.M, shp.d)),
                                _dev(lse_enc, "lse_enc", torch.float32, (shp.B, shp.H, shp.M)),
                                _opt_lse_dec(lse_dec, shp),
                                ctypes.c_float(scale), ws_p, ws_n, _stream(stream)), "flare_forward")
    return y, z, lse_enc


def forward_project(q_lat, k, v, w_out, scale, bias=None, out=None, y=None, z=None, lse_enc=None, lse_dec=None,
                    workspace=None, stream=None, keep_y=False):
    """flare_forward_project: the forward with the output projection fused into the decode.  Token tensors are
    [B,N,H,d] (layout 'bnhd'), w_out [C,C] in their dtype, bias [C] fp32 or None.  Returns (out[B,N,C], z, lse_enc);
    y (the mixer's own output, for a backward) is written only when given or when keep_y is set."""
    torch = _torch()
    shp = _shape_of(q_lat, k, "bnhd", False)
    C = shp.H * shp.d
    if out is None:
        out = torch.empty((shp.B, shp.N, C), dtype=k.dtype, device=k.device)
    if y is None and keep_y:
        y = torch.empty_like(k)
    if z is None:
        z = torch.empty((shp.B, shp.H, shp.M, shp.d), dtype=torch.float32, device=k.device)
    if lse_enc is None:
        lse_enc = torch.empty((shp.B, shp.H, shp.M), dtype=torch.float32, device=k.device)
    ws, ws_p, ws_n = _workspace(shp, "fwd", workspace, k.device, stream)
    _check(load().flare_forward_project(ctypes.byref(shp), _dev(q_lat, "q_lat"), _dev(k, "k"),
                                        _dev(v, "v", k.dtype, k.shape), _dev(w_out, "w_out", k.dtype, (C, C)),
                                        None if bias is None else _dev(bias, "bias", torch.float32, (C,)),
                                        _dev(out, "out", k.dtype, (shp.B, shp.N, C)),
                                        None if y is None else _dev(y, "y", k.dtype, k.shape),
                                        _dev(z, "z", torch.float32, (shp.B, shp.H, shp.M, shp.d)),
                                        _dev(lse_enc, "lse_enc", torch.float32, (shp.B, shp.H, shp.M)),
                                        _opt_lse_dec(lse_dec, shp), ctypes.c_float(scale), ws_p, ws_n,
                                        _stream(stream)), "flare_forward_project")
    return out, z, lse_enc


STATIC_SCRATCH_BYTES = 32 << 20   # FLARE_STATIC_SCRATCH_BYTES of include/flare.h


def forward_static(q_lat, k, v, scale, y, z, lse_enc, lse_dec=None, stream=None, layout="bhnd"):
    """flare_forward_static: the forward with the library's own static scratch; every output is the caller's."""
    torch = _torch()
    f32y = _wants_f32_y(y, k, False)
    shp = _shape_of(q_lat, k, layout, f32y)
    ydt = torch.float32 if f32y else k.dtype
    _check(load().flare_forward_static(ctypes.byref(shp), _dev(q_lat, "q_lat"), _dev(k, "k"),
                                       _dev(v, "v", k.dtype, k.shape), _dev(y, "y", ydt, k.shape),
                                       _dev(z, "z", torch.float32, (shp.B, shp.H, shp.M, shp.d)),
                                       _dev(lse_enc, "lse_enc", torch.float32, (shp.B, shp.H, shp.M)),
                                       _opt_lse_dec(lse_dec, shp), ctypes.c_float(scale), _stream(stream)),
           "flare_forward_static")
    return y, z, lse_enc


def backward(q_lat, k, v, dy, z, lse_enc, scale, y=None, lse_dec=None, dq_lat=None, dk=None, dv=None,
             workspace=None, stream=None, layout="bhnd", variant=0):
    """flare_backward: returns (dq_lat[H,M,d] fp32, dk, dv in k's dtype).

    Pass the forward's y and lse_dec to reuse them; without both, they are recomputed from z.  An fp32 y next
    to 16-bit inputs is the forward's y_f32 output."""
    torch = _torch()
    f32y = _wants_f32_y(y, k, False)
    shp = _shape_of(q_lat, k, layout, f32y)
    shp.variant = int(variant)     # flare_variant bits: force a kernel variant (tests, measurements)
    if dq_lat is None:
        dq_lat = torch.empty(tuple(q_lat.shape), dtype=torch.float32, device=k.device)
    if dk is None:
        dk = torch.empty_like(k)
    if dv is None:
        dv = torch.empty_like(k)
    ws, ws_p, ws_n = _workspace(shp, "bwd", workspace, k.device, stream)
    _check(load().flare_backward(ctypes.byref(shp), _dev(q_lat, "q_lat"), _dev(k, "k"),
                                 _dev(v, "v", k.dtype, k.shape),
                                 None if y is None else _dev(y, "y", torch.float32 if f32y else k.dtype, k.shape),
                                 _opt_lse_dec(lse_dec, shp), _dev(dy, "dy", k.dtype, k.shape),
                                 _dev(z, "z", torch.float32, (shp.B, shp.H, shp.M, shp.d)),
                                 _dev(lse_enc, "lse_enc", torch.float32, (shp.B, shp.H, shp.M)),
                                 _dev(dq_lat, "dq_lat", torch.float32, tuple(q_lat.shape)),
                                 _dev(dk, "dk", k.dtype, k.shape), _dev(dv, "dv", k.dtype, k.shape),
                                 ctypes.c_float(scale), ws_p, ws_n, _stream(stream)), "flare_backward")
    return dq_lat, dk, dv


def spectral(q_lat, k, lse_enc, lse_dec, scale, first=0, want_gram=False, stream=None, layout="bhnd"):
    """flare_spectral: returns (eigenvalues[B,H,M] descending, z_vec[B,H,M,d], gram[B,H,M,M] or None).

    decode(q_lat, k, z_vec, scale) then gives the eigenvectors number first .. first+d-1 of W."""
    torch = _torch()
    shp = _shape_of(q_lat, k, layout)
    need = ctypes.c_size_t(0)
    _check(load().flare_spectral_workspace_bytes(ctypes.byref(shp), ctypes.byref(need)), "flare_spectral_workspace_bytes")
    ws = torch.empty(max(int(need.value), 256), dtype=torch.uint8, device=k.device)
    if stream is not None and stream != torch.cuda.current_stream():
        ws.record_stream(stream)          # a temporary block used by kernels on another stream (see _workspace)
    ev = torch.empty((shp.B, shp.H, shp.M), dtype=torch.float32, device=k.device)
    zv = torch.empty((shp.B, shp.H, shp.M, shp.d), dtype=torch.float32, device=k.device)
    gram = torch.empty((shp.B, shp.H, shp.M, shp.M), dtype=torch.float32, device=k.device) if want_gram else None
    _check(load().flare_spectral(ctypes.byref(shp), _dev(q_lat, "q_lat"), _dev(k, "k"),
                                 _dev(lse_enc, "lse_enc", torch.float32, (shp.B, shp.H, shp.M)),
                                 _dev(lse_dec, "lse_dec", torch.float32, (shp.B, shp.H, shp.N)),
                                 ctypes.c_float(scale), ctypes.c_int(first), _dev(ev, "eigenvalues"),
                                 _dev(zv, "z_vec"), None if gram is None else _dev(gram, "gram"),
                                 ctypes.c_void_p(ws.data_ptr()), ctypes.c_size_t(ws.numel()), _stream(stream)),
           "flare_spectral")
    return ev, zv, gram


def profile_enable(on):
    _check(load().flare_profile_enable(1 if on else 0), "flare_profile_enable")


def profile_read():
    """{kernel name: (total ms, launches)} for kernels launched since profile_enable(True)."""
    lib = load()
    out = {}
    for kid in range(lib.flare_profile_kernels()):
        ms, cnt = ctypes.c_double(0), ctypes.c_int(0)
        _check(lib.flare_profile_read(kid, ctypes.byref(ms), ctypes.byref(cnt)), "flare_profile_read")
        if cnt.value:
            out[lib.flare_profile_name(kid).decode()] = (float(ms.value), int(cnt.value))
    return out
