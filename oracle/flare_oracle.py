"""ctypes loader for the fp64 CPU oracle (oracle/flare_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg.  The product package never imports this module, and this module never
imports the product package.

All arrays are numpy float64 on the host; shapes follow the paper's listing in
Section 3.1 (Q:[H M D], K,V:[B H N D] -> Y:[B H N D]).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "flare_oracle.c")
_LIB = os.path.join(_HERE, "libflare_oracle.so")
_lib = None

_dp = ctypes.POINTER(ctypes.c_double)
_lp = ctypes.POINTER(ctypes.c_longlong)


def build(force=False):
    """Compile the oracle with gcc (plain C99 + OpenMP, no fast-math)."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    tmp = _LIB + ".tmp.%d" % os.getpid()
    cmd = ["gcc", "-std=c99", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", tmp, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.flare_oracle_threads.restype = ctypes.c_int
        lib.flare_oracle_forward.restype = ctypes.c_int
        lib.flare_oracle_forward.argtypes = [ctypes.c_int] * 5 + [_dp, _dp, _dp, ctypes.c_double,
                                                                  _lp, ctypes.c_int, _dp, _dp, _dp]
        lib.flare_oracle_backward.restype = ctypes.c_int
        lib.flare_oracle_backward.argtypes = [ctypes.c_int] * 5 + [_dp, _dp, _dp, _dp, ctypes.c_double,
                                                                   _lp, ctypes.c_int, _dp, _dp, _dp]
        lib.flare_oracle_explicit_w.restype = ctypes.c_int
        lib.flare_oracle_explicit_w.argtypes = [ctypes.c_int] * 3 + [_dp, _dp, ctypes.c_double, _dp, _dp, _dp]
        _lib = lib
    return _lib


def threads():
    return int(_load().flare_oracle_threads())


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _ptr(a):
    return a.ctypes.data_as(_dp) if a is not None else None


def _dims(q, k, v):
    if q.ndim != 3 or k.ndim != 4 or v.shape != k.shape:
        raise ValueError("expected q[H,M,d], k/v[B,H,N,d]")
    H, M, d = q.shape
    B, Hk, N, dk = k.shape
    if Hk != H or dk != d:
        raise ValueError("q and k disagree on H or d")
    return B, H, N, M, d


def _tokens(tok, N):
    if tok is None:
        return None, 0, N
    t = np.ascontiguousarray(tok, dtype=np.int64)
    if t.ndim != 1 or t.size == 0:
        raise ValueError("tok must be a non-empty 1-D index array")
    return t, int(t.size), int(t.size)


def forward(q, k, v, scale, tok=None):
    """Returns (y, z, lse_enc).  y is [B,H,N,d], or [B,H,len(tok),d] when tok is given."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    B, H, N, M, d = _dims(q, k, v)
    t, n_tok, n_out = _tokens(tok, N)
    y = np.empty((B, H, n_out, d), np.float64)
    z = np.empty((B, H, M, d), np.float64)
    lse = np.empty((B, H, M), np.float64)
    rc = _load().flare_oracle_forward(B, H, N, M, d, _ptr(q), _ptr(k), _ptr(v), float(scale),
                                      t.ctypes.data_as(_lp) if t is not None else None, n_tok,
                                      _ptr(y), _ptr(z), _ptr(lse))
    if rc != 0:
        raise RuntimeError("flare_oracle_forward failed: %d" % rc)
    return y, z, lse


def backward(q, k, v, dy, scale, tok=None, want_dkdv=True):
    """Returns (dq[H,M,d], dk, dv); dk/dv are [B,H,N,d] or [B,H,len(tok),d]; None if not wanted."""
    q, k, v, dy = _f64(q), _f64(k), _f64(v), _f64(dy)
    B, H, N, M, d = _dims(q, k, v)
    if dy.shape != k.shape:
        raise ValueError("dy must have k's shape")
    t, n_tok, n_out = _tokens(tok, N)
    dq = np.empty((H, M, d), np.float64)
    dk = np.empty((B, H, n_out, d), np.float64) if want_dkdv else None
    dv = np.empty((B, H, n_out, d), np.float64) if want_dkdv else None
    rc = _load().flare_oracle_backward(B, H, N, M, d, _ptr(q), _ptr(k), _ptr(v), _ptr(dy), float(scale),
                                       t.ctypes.data_as(_lp) if t is not None else None, n_tok,
                                       _ptr(dq), _ptr(dk), _ptr(dv))
    if rc != 0:
        raise RuntimeError("flare_oracle_backward failed: %d" % rc)
    return dq, dk, dv


def explicit_w(q_h, k_h, scale):
    """One head: q_h[M,d], k_h[N,d] -> (w_enc[M,N], w_dec[N,M], w[N,N])."""
    q_h, k_h = _f64(q_h), _f64(k_h)
    M, d = q_h.shape
    N = k_h.shape[0]
    if k_h.shape[1] != d:
        raise ValueError("q_h and k_h disagree on d")
    we = np.empty((M, N), np.float64)
    wd = np.empty((N, M), np.float64)
    w = np.empty((N, N), np.float64)
    rc = _load().flare_oracle_explicit_w(N, M, d, _ptr(q_h), _ptr(k_h), float(scale), _ptr(we), _ptr(wd), _ptr(w))
    if rc != 0:
        raise RuntimeError("flare_oracle_explicit_w failed: %d" % rc)
    return we, wd, w


def spectral(q_h, k_h, scale):
    """Eigenpairs of one head's mixing matrix W = W_dec W_enc from its M x M companion
    (Appendix C.1, Algorithm 1), in the algorithm's own steps and notation, fp64 numpy:

        A = exp(scale * Q K^T)                       (step 1; the stabiliser below cancels in J)
        L_N = 1 / column sums of A,  L_M = 1 / row sums of A          (steps 2, 3)
        J = L_M^(1/2) A L_N^(1/2)                                      (step 4)
        U Sigma^2 U^T = J J^T                                          (step 5, numpy.linalg.eigh)
        eigenvalues = Sigma^2, eigenvectors = L_N^(1/2) J^T U Sigma^(-1)  (steps 6, 7)

    q_h[M,d], k_h[N,d] -> (eigenvalues[M] in descending order, gram = J J^T [M,M],
    eigenvectors[N,M] with column j belonging to eigenvalue j).  Columns whose eigenvalue is below
    1e-300 are returned as zeros (Sigma^(-1) does not exist there)."""
    q_h, k_h = _f64(q_h), _f64(k_h)
    s = float(scale) * (q_h @ k_h.T)
    smax = s.max()
    a = np.exp(s - smax)                    # A / exp(smax): the common factor cancels in J ...
    l_n = 1.0 / a.sum(axis=0)
    l_m = 1.0 / a.sum(axis=1)
    j = np.sqrt(l_m)[:, None] * a * np.sqrt(l_n)[None, :]
    l_n = l_n * np.exp(-smax)               # ... and is put back into L_N, which step 7 uses on its own
    gram = j @ j.T
    lam, u = np.linalg.eigh(gram)
    order = np.argsort(lam)[::-1]
    lam, u = lam[order], u[:, order]
    ok = lam > 1e-300
    inv_sigma = np.where(ok, 1.0 / np.sqrt(np.where(ok, lam, 1.0)), 0.0)
    vec = np.sqrt(l_n)[:, None] * (j.T @ u) * inv_sigma[None, :]
    return lam, gram, vec


def output_projection(y, w_out, bias=None):
    """The linear layer that follows the mixer (Section 3.1: the head outputs are concatenated along the
    feature dimension and passed through a final linear projection; Appendix B.2 "FLARE": a single linear layer):

        out[b][n][:] = concat_h(y[b][h][n][:]) @ w_out + bias,      w_out[C][C_out], C = H * d, bias[C_out] or None

    y[B,H,N,d] -> out[B,N,C_out], fp64, written as the definition (head concatenation, then one matrix product)."""
    y = _f64(y)
    w_out = _f64(w_out)
    B, H, N, d = y.shape
    if w_out.ndim != 2 or w_out.shape[0] != H * d:
        raise ValueError("w_out must be [H*d, C_out]")
    cat = np.ascontiguousarray(np.transpose(y, (0, 2, 1, 3))).reshape(B, N, H * d)     # [B, N, C]: head h in columns h*d ...
    out = cat @ w_out
    if bias is not None:
        out = out + _f64(bias)[None, None, :]
    return out
