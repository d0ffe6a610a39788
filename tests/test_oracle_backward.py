"""Pins for the oracle's backward (CPU only).

The paper derives no gradient (it relies on automatic differentiation through its two
attention calls, Appendix G "Time and memory complexity"), so the oracle's formulas are
pinned by central finite differences of the oracle-independent explicit form W.V, by
identities that follow from W being row-stochastic, and by torch autograd through the
paper's listing in fp64.
"""
import numpy as np
import pytest


def _rand(seed, B, H, N, M, d):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((H, M, d)), rng.standard_normal((B, H, N, d)),
            rng.standard_normal((B, H, N, d)), rng.standard_normal((B, H, N, d)))


def _relerr(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


def _loss_numpy(q, k, v, dy, scale):
    """sum(dY * Y) with Y formed from explicit softmax matrices in numpy (no oracle code)."""
    total = 0.0
    B, H = k.shape[:2]
    for b in range(B):
        for h in range(H):
            s = scale * q[h] @ k[b, h].T
            we = np.exp(s - s.max(1, keepdims=True))
            we /= we.sum(1, keepdims=True)
            wd = np.exp(s.T - s.T.max(1, keepdims=True))
            wd /= wd.sum(1, keepdims=True)
            total += np.sum(dy[b, h] * (wd @ (we @ v[b, h])))
    return total


def _fd(fun, x, idx, h=1e-6):
    xp, xm = x.copy(), x.copy()
    xp[idx] += h
    xm[idx] -= h
    return (fun(xp) - fun(xm)) / (2 * h)


@pytest.mark.parametrize("B,H,N,M,d,scale", [(2, 2, 11, 5, 3, 1.0), (3, 1, 7, 9, 4, 0.5)])
def test_finite_differences(oracle, B, H, N, M, d, scale):
    q, k, v, dy = _rand(21, B, H, N, M, d)
    dq, dk, dv = oracle.backward(q, k, v, dy, scale)
    rng = np.random.default_rng(0)
    for _ in range(12):
        i = tuple(rng.integers(0, s) for s in q.shape)
        g = _fd(lambda x: _loss_numpy(x, k, v, dy, scale), q, i)
        assert abs(g - dq[i]) < 1e-7 * max(1.0, abs(g)), ("dq", i)
        i = tuple(rng.integers(0, s) for s in k.shape)
        g = _fd(lambda x: _loss_numpy(q, x, v, dy, scale), k, i)
        assert abs(g - dk[i]) < 1e-7 * max(1.0, abs(g)), ("dk", i)
        g = _fd(lambda x: _loss_numpy(q, k, x, dy, scale), v, i)
        assert abs(g - dv[i]) < 1e-7 * max(1.0, abs(g)), ("dv", i)


def test_gradient_identities(oracle):
    """dV = W^T dY with W 1 = 1  =>  sum_n dV_n = sum_n dY_n; dV does not depend on V;
    dV equals W^T dY with W formed explicitly."""
    q, k, v, dy = _rand(22, 2, 2, 26, 6, 4)
    dq, dk, dv = oracle.backward(q, k, v, dy, 0.7)
    np.testing.assert_allclose(dv.sum(2), dy.sum(2), rtol=1e-12, atol=1e-12)
    v2 = np.random.default_rng(5).standard_normal(v.shape)
    _, _, dv2 = oracle.backward(q, k, v2, dy, 0.7)
    assert _relerr(dv2, dv) < 1e-13
    for b in range(2):
        for h in range(2):
            _, _, w = oracle.explicit_w(q[h], k[b, h], 0.7)
            assert _relerr(dv[b, h], w.T @ dy[b, h]) < 1e-13
    # the loss is invariant to adding a constant vector to all scores of one token through K
    # only via decode; a uniform shift of all keys along q-orthogonal directions is not
    # generic, so check instead the scale derivative: d/dscale = <dq,q>/scale = <dk,k>/scale
    lhs = np.sum(dq * q)
    rhs = np.sum(dk * k)
    assert abs(lhs - rhs) < 1e-10 * max(1.0, abs(lhs))
    g = (_loss_numpy(q, k, v, dy, 0.7 + 1e-6) - _loss_numpy(q, k, v, dy, 0.7 - 1e-6)) / 2e-6
    assert abs(g - lhs / 0.7) < 1e-6 * max(1.0, abs(g))


def test_batch_sum_of_dq(oracle):
    """dq_lat is the sum over batch items of the per-item gradients (Q is shared over B)."""
    q, k, v, dy = _rand(23, 3, 2, 13, 4, 4)
    dq, _, _ = oracle.backward(q, k, v, dy, 1.0)
    parts = [oracle.backward(q, k[b:b + 1], v[b:b + 1], dy[b:b + 1], 1.0)[0] for b in range(3)]
    assert _relerr(dq, sum(parts)) < 1e-13


def test_token_subset_matches_full(oracle):
    q, k, v, dy = _rand(24, 2, 2, 31, 6, 4)
    tok = np.array([30, 2, 2, 17])
    dq, dk, dv = oracle.backward(q, k, v, dy, 0.5)
    dq2, dk2, dv2 = oracle.backward(q, k, v, dy, 0.5, tok=tok)
    assert np.array_equal(dq, dq2)
    assert np.array_equal(dk2, dk[:, :, tok]) and np.array_equal(dv2, dv[:, :, tok])
    dq3, none_k, none_v = oracle.backward(q, k, v, dy, 0.5, want_dkdv=False)
    assert np.array_equal(dq, dq3) and none_k is None and none_v is None


def test_torch_autograd_second_opinion(oracle):
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    q, k, v, dy = _rand(25, 2, 3, 40, 8, 16)
    for scale in (1.0, 0.25):
        tq, tk, tv = (torch.from_numpy(a).clone().requires_grad_(True) for a in (q, k, v))
        tz = F.scaled_dot_product_attention(tq.expand(2, -1, -1, -1), tk, tv, scale=scale)
        ty = F.scaled_dot_product_attention(tk, tq.expand(2, -1, -1, -1), tz, scale=scale)
        ty.backward(torch.from_numpy(dy))
        dq, dk, dv = oracle.backward(q, k, v, dy, scale)
        assert _relerr(dq, tq.grad.numpy()) < 1e-11
        assert _relerr(dk, tk.grad.numpy()) < 1e-11
        assert _relerr(dv, tv.grad.numpy()) < 1e-11
