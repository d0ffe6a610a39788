"""Pins for the oracle's forward (CPU only).

Each test checks the oracle against something the paper or the mathematics fixes, not
against itself: explicit W.V (Section 3.1, Eq. attn_W; Appendix C listing), the structure of
W (rank <= M, row-stochastic), the spectral identity of Appendix C.1 / Algorithm 1,
permutation equivariance (Section 5.3), closed forms that follow from the per-latent and
per-token equations of Appendix F, and a library second opinion (the paper's own listing
run with torch's fp64 scaled_dot_product_attention).
"""
import os
from fractions import Fraction

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def _rand(seed, B, H, N, M, d, gain=1.0):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((H, M, d)) * gain
    k = rng.standard_normal((B, H, N, d))
    v = rng.standard_normal((B, H, N, d))
    return q, k, v


def _relerr(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


def test_golden_cluster_example(oracle):
    """Hand-computed rationals (tests/golden/cluster_example.txt)."""
    vals = {}
    with open(os.path.join(HERE, "golden", "cluster_example.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, *nums = line.split()
            vals[name] = np.array([float(Fraction(x)) for x in nums])
    beta = np.log(2.0)
    q = (beta * np.eye(2))[None]                       # [H=1, M=2, d=2]
    k = np.array([[1.0, 0], [1, 0], [0, 1]])[None, None]
    v = np.array([[1.0, 0], [3, 0], [0, 6]])[None, None]
    y, z, lse = oracle.forward(q, k, v, 1.0)
    np.testing.assert_allclose(z.ravel(), vals["Z"], rtol=1e-14, atol=1e-15)
    np.testing.assert_allclose(y.ravel(), vals["Y"], rtol=1e-14, atol=1e-15)
    np.testing.assert_allclose(np.exp(lse).ravel(), vals["exp_lse_enc"], rtol=1e-14)
    we, wd, _ = oracle.explicit_w(q[0], k[0, 0], 1.0)
    np.testing.assert_allclose(we.ravel(), vals["W_enc"], rtol=1e-14)
    np.testing.assert_allclose(wd.ravel(), vals["W_dec"], rtol=1e-14)


@pytest.mark.parametrize("N,M,d,scale", [(37, 8, 4, 1.0), (64, 16, 16, 0.25), (5, 12, 3, 0.7)])
def test_fused_equals_explicit_w(oracle, N, M, d, scale):
    """Y from encode-then-decode == (W_dec W_enc) V formed explicitly (Eq. attn_W)."""
    q, k, v = _rand(1, 2, 3, N, M, d)
    y, z, _ = oracle.forward(q, k, v, scale)
    for b in range(2):
        for h in range(3):
            we, wd, w = oracle.explicit_w(q[h], k[b, h], scale)
            assert _relerr(y[b, h], w @ v[b, h]) < 1e-13
            assert _relerr(z[b, h], we @ v[b, h]) < 1e-13
            assert _relerr(w, wd @ we) < 1e-14


@pytest.mark.parametrize("N,M", [(48, 8), (40, 40), (24, 32)])
def test_w_invariants(oracle, N, M):
    """W has non-negative entries, unit row sums and rank <= min(M, N)."""
    q, k, _ = _rand(2, 1, 1, N, M, 6, gain=1.5)
    we, wd, w = oracle.explicit_w(q[0], k[0, 0], 1.0)
    for mat in (we, wd, w):
        assert mat.min() >= 0.0
        np.testing.assert_allclose(mat.sum(axis=1), 1.0, rtol=0, atol=1e-14)
    sv = np.linalg.svd(w, compute_uv=False)
    r = min(M, N)
    if r < N:
        assert sv[r:].max() < 1e-12 * sv[0]


def test_spectral_identity(oracle):
    """Appendix C.1 / Algorithm 1: the nonzero eigenvalues of W are those of J J^T with
    J = L_M^{1/2} A L_N^{1/2}, A = exp(Q K^T); they are real, lie in [0,1], the largest is 1."""
    N, M, d = 50, 7, 5
    q, k, _ = _rand(3, 1, 1, N, M, d)
    _, _, w = oracle.explicit_w(q[0], k[0, 0], 1.0)
    a = np.exp(q[0] @ k[0, 0].T)
    l_m = 1.0 / a.sum(axis=1)
    l_n = 1.0 / a.sum(axis=0)
    j = np.sqrt(l_m)[:, None] * a * np.sqrt(l_n)[None, :]
    ev_small = np.sort(np.linalg.eigvalsh(j @ j.T))[::-1]
    ev = np.linalg.eigvals(w)
    assert np.abs(ev.imag).max() < 1e-10
    ev = np.sort(ev.real)[::-1]
    np.testing.assert_allclose(ev[:M], ev_small, rtol=1e-9, atol=1e-12)
    assert np.abs(ev[M:]).max() < 1e-10
    assert abs(ev[0] - 1.0) < 1e-12 and ev_small.min() > -1e-14 and ev_small.max() < 1 + 1e-12
    # eigenvectors: L_N^{1/2} J^T U Sigma^{-1} satisfy W x = lambda x
    lam, u = np.linalg.eigh(j @ j.T)
    vec = np.sqrt(l_n)[:, None] * (j.T @ u) / np.sqrt(lam)[None, :]
    assert _relerr(w @ vec, vec * lam[None, :]) < 1e-10


def test_spectral_function_against_brute_force(oracle):
    """oracle.spectral (Algorithm 1) against the dense N x N eigenproblem it avoids, with a scale that
    is not 1, and against what a row-stochastic W fixes: eigenvalue 1 with a constant eigenvector."""
    N, M, d = 41, 6, 4
    q, k, _ = _rand(11, 1, 1, N, M, d)
    scale = 0.7
    lam, gram, vec = oracle.spectral(q[0], k[0, 0], scale)
    _, _, w = oracle.explicit_w(q[0], k[0, 0], scale)
    ev = np.linalg.eigvals(w)
    assert np.abs(ev.imag).max() < 1e-10
    ev = np.sort(ev.real)[::-1]
    np.testing.assert_allclose(lam, ev[:M], rtol=1e-9, atol=1e-13)
    assert np.all(np.diff(lam) <= 1e-15) and abs(lam[0] - 1.0) < 1e-12
    assert np.allclose(gram, gram.T, atol=1e-15) and abs(np.trace(gram) - lam.sum()) < 1e-12
    # W x = lambda x for every returned column, and the first column is constant
    assert _relerr(w @ vec, vec * lam[None, :]) < 1e-9
    assert np.ptp(vec[:, 0]) < 1e-10 * abs(vec[0, 0])
    # the columns are the right singular vectors of J scaled by L_N^(1/2): V^T V = I
    a = np.exp(scale * q[0] @ k[0, 0].T)
    l_n = 1.0 / a.sum(axis=0)
    v = vec / np.sqrt(l_n)[:, None]
    assert np.abs(v.T @ v - np.eye(M)).max() < 1e-9


def test_permutation_equivariance(oracle):
    q, k, v = _rand(4, 2, 2, 33, 8, 4)
    perm = np.random.default_rng(0).permutation(33)
    y, z, lse = oracle.forward(q, k, v, 0.5)
    y2, z2, lse2 = oracle.forward(q, k[:, :, perm], v[:, :, perm], 0.5)
    assert _relerr(y2, y[:, :, perm]) < 1e-13
    assert _relerr(z2, z) < 1e-13 and _relerr(lse2, lse) < 1e-13


def test_constant_v_and_linearity(oracle):
    q, k, v = _rand(5, 1, 2, 29, 6, 4)
    c = np.array([1.5, -2.0, 0.25, 7.0])
    y, z, _ = oracle.forward(q, k, np.broadcast_to(c, v.shape).copy(), 1.0)
    np.testing.assert_allclose(y, np.broadcast_to(c, y.shape), rtol=1e-14)
    np.testing.assert_allclose(z, np.broadcast_to(c, z.shape), rtol=1e-14)
    v2 = np.random.default_rng(9).standard_normal(v.shape)
    ya, _, _ = oracle.forward(q, k, v, 1.0)
    yb, _, _ = oracle.forward(q, k, v2, 1.0)
    yc, _, _ = oracle.forward(q, k, 2.0 * v - 3.0 * v2, 1.0)
    assert _relerr(yc, 2.0 * ya - 3.0 * yb) < 1e-13


def test_closed_forms(oracle):
    q, k, v = _rand(6, 2, 2, 21, 5, 4)
    mean_v = v.mean(axis=2, keepdims=True)
    # Q = 0: every softmax is uniform, Z_m = Y_n = mean of V
    y, z, lse = oracle.forward(np.zeros_like(q), k, v, 1.0)
    assert _relerr(y, np.broadcast_to(mean_v, y.shape)) < 1e-14
    assert _relerr(z, np.broadcast_to(mean_v, z.shape)) < 1e-14
    np.testing.assert_allclose(lse, np.log(21.0), rtol=1e-14)
    # K = 0 likewise
    y, _, _ = oracle.forward(q, np.zeros_like(k), v, 1.0)
    assert _relerr(y, np.broadcast_to(mean_v, y.shape)) < 1e-14
    # M = 1: the decode softmax is trivial, Y_n = Z_1 = softmax-pooled mean of V
    y, z, _ = oracle.forward(q[:, :1], k, v, 0.3)
    s = 0.3 * np.einsum("hd,bhnd->bhn", q[:, 0], k)
    w = np.exp(s - s.max(-1, keepdims=True))
    w /= w.sum(-1, keepdims=True)
    pooled = np.einsum("bhn,bhnd->bhd", w, v)
    assert _relerr(z[:, :, 0], pooled) < 1e-14
    assert _relerr(y, np.broadcast_to(pooled[:, :, None], y.shape)) < 1e-14
    # N = 1: W is the 1x1 matrix [1], Y_1 = v_1
    y, z, _ = oracle.forward(q, k[:, :, :1], v[:, :, :1], 1.0)
    assert _relerr(y, v[:, :, :1]) < 1e-15
    # duplicating every token leaves Z and the per-token outputs unchanged
    y1, z1, l1 = oracle.forward(q, k, v, 1.0)
    y2, z2, l2 = oracle.forward(q, np.concatenate([k, k], 2), np.concatenate([v, v], 2), 1.0)
    assert _relerr(z2, z1) < 1e-14 and _relerr(y2[:, :, :21], y1) < 1e-14 and _relerr(y2[:, :, 21:], y1) < 1e-14
    np.testing.assert_allclose(l2, l1 + np.log(2.0), rtol=1e-13)


def test_cluster_closed_form(oracle):
    """d = M, Q = beta I, one-hot keys: S[m][n] = beta [m = c(n)], closed forms for Z and Y."""
    M, N, beta = 4, 23, 1.7
    rng = np.random.default_rng(7)
    c = rng.integers(0, M, N)
    c[:M] = np.arange(M)
    v = rng.standard_normal((N, 3))
    vpad = np.concatenate([v, np.zeros((N, 1))], 1)       # the oracle needs v's width == d
    k = np.eye(M)[c]
    y, z, _ = oracle.forward(beta * np.eye(M)[None], k[None, None], vpad[None, None], 1.0)
    eb = np.exp(beta)
    z_ref = np.empty((M, 3))
    for m in range(M):
        inside = c == m
        z_ref[m] = (eb * v[inside].sum(0) + v[~inside].sum(0)) / (eb * inside.sum() + N - inside.sum())
    y_ref = np.stack([(eb * z_ref[c[n]] + z_ref.sum(0) - z_ref[c[n]]) / (eb + M - 1) for n in range(N)])
    assert _relerr(z[0, 0, :, :3], z_ref) < 1e-14
    assert _relerr(y[0, 0, :, :3], y_ref) < 1e-14


def test_shift_invariance(oracle):
    """A per-latent offset on row m of S leaves Z; a per-token offset on column n leaves W_dec."""
    q, k, v = _rand(8, 1, 1, 19, 6, 4)
    off_m = np.random.default_rng(1).standard_normal(6) * 3
    off_n = np.random.default_rng(2).standard_normal(19) * 3
    _, z0, _ = oracle.forward(q, k, v, 1.0)
    qa = np.concatenate([q, off_m[None, :, None]], 2)                 # extra feature: S += off_m
    ka = np.concatenate([k, np.ones((1, 1, 19, 1))], 3)
    va = np.concatenate([v, np.zeros((1, 1, 19, 1))], 3)
    _, z1, _ = oracle.forward(qa, ka, va, 1.0)
    assert _relerr(z1[..., :4], z0) < 1e-13
    _, wd0, _ = oracle.explicit_w(q[0], k[0, 0], 1.0)
    qb = np.concatenate([q[0], np.ones((6, 1))], 1)                   # S += off_n
    kb = np.concatenate([k[0, 0], off_n[:, None]], 1)
    _, wd1, _ = oracle.explicit_w(qb, kb, 1.0)
    assert _relerr(wd1, wd0) < 1e-13


def test_token_subset_matches_full(oracle):
    q, k, v = _rand(10, 2, 2, 41, 8, 4)
    tok = np.array([40, 0, 7, 7, 13])
    y, z, _ = oracle.forward(q, k, v, 0.5)
    ys, zs, _ = oracle.forward(q, k, v, 0.5, tok=tok)
    assert np.array_equal(ys, y[:, :, tok]) and np.array_equal(zs, z)


def test_large_scores_are_stable(oracle):
    """Scores of magnitude ~1e3 must not overflow (two-pass softmax)."""
    q, k, v = _rand(11, 1, 1, 17, 4, 4, gain=300.0)
    y, z, lse = oracle.forward(q, k, v, 1.0)
    assert np.isfinite(y).all() and np.isfinite(z).all() and np.isfinite(lse).all()
    _, _, w = oracle.explicit_w(q[0], k[0, 0], 1.0)
    assert _relerr(y[0, 0], w @ v[0, 0]) < 1e-13


def test_torch_sdpa_second_opinion(oracle):
    """The paper's listing (two attention calls, same scale) in torch fp64."""
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    q, k, v = _rand(12, 2, 3, 45, 8, 16)
    for scale in (1.0, 0.25):
        tq, tk, tv = (torch.from_numpy(a) for a in (q, k, v))
        tz = F.scaled_dot_product_attention(tq.expand(2, -1, -1, -1), tk, tv, scale=scale)
        ty = F.scaled_dot_product_attention(tk, tq.expand(2, -1, -1, -1), tz, scale=scale)
        y, z, _ = oracle.forward(q, k, v, scale)
        assert _relerr(z, tz.numpy()) < 1e-12 and _relerr(y, ty.numpy()) < 1e-12


# ---- the output projection behind the mixer (Section 3.1, Appendix B.2) ----------------------------------------
def test_output_projection_against_loops_and_special_weights(oracle):
    rng = np.random.default_rng(31)
    B, H, N, d, Co = 2, 3, 5, 4, 7
    y = rng.standard_normal((B, H, N, d))
    w = rng.standard_normal((H * d, Co))
    bias = rng.standard_normal(Co)
    out = oracle.output_projection(y, w, bias)
    assert out.shape == (B, N, Co)
    # brute force: every output element from its definition, loops only
    for b in range(B):
        for n in range(N):
            for c in range(Co):
                s = bias[c]
                for h in range(H):
                    for j in range(d):
                        s += y[b, h, n, j] * w[h * d + j, c]
                assert abs(out[b, n, c] - s) <= 1e-12
    # identity weights: the projection is the concatenation of the heads, head h in columns h*d .. h*d+d-1
    cat = oracle.output_projection(y, np.eye(H * d))
    for h in range(H):
        assert np.array_equal(cat[:, :, h * d:(h + 1) * d], y[:, h])
    # a one-hot column picks one channel of one head; a transposed weight matrix would pick another
    e = np.zeros((H * d, 1))
    e[1 * d + 2, 0] = 1.0
    assert np.array_equal(oracle.output_projection(y, e)[..., 0], y[:, 1, :, 2])
    # linear in y and in w_out, affine in the bias
    y2 = rng.standard_normal(y.shape)
    lhs = oracle.output_projection(2.0 * y - 3.0 * y2, w)
    rhs = 2.0 * oracle.output_projection(y, w) - 3.0 * oracle.output_projection(y2, w)
    assert np.abs(lhs - rhs).max() <= 1e-12
    assert np.abs(oracle.output_projection(y, w, bias) - oracle.output_projection(y, w) - bias).max() <= 1e-13
    # the heads do not mix before the projection: zeroing head 0's rows of w_out removes exactly head 0's part
    w0 = w.copy()
    w0[:d] = 0.0
    y0 = y.copy()
    y0[:, 0] = 0.0
    assert np.abs(oracle.output_projection(y, w0) - oracle.output_projection(y0, w)).max() <= 1e-13
