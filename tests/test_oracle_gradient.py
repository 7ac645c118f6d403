"""Pins of the oracle's full-precision pass (margins, gradient, loss) against
library routines and finite differences (no GPU)."""
import numpy as np
import pytest
from scipy.special import log_expit, logsumexp

import halp_inputs as inp
from oracle import ref


def test_squared_loss_gradient_matches_blas_and_normal_equations():
    X, y, _ = inp.linreg(200, 17, seed=1)
    w = np.random.default_rng(0).standard_normal(17).astype(np.float32)
    prob = ref.make_problem(200, 17, lam=0.0)
    phi, g, loss = ref.full_gradient(prob, X, y, w)
    Xd, yd, wd = X.astype(np.float64), y.astype(np.float64), w.astype(np.float64)
    assert np.allclose(phi[:, 0], Xd @ wd, rtol=1e-13, atol=1e-13)
    assert np.allclose(g[0], Xd.T @ (Xd @ wd - yd) / 200, rtol=1e-12, atol=1e-13)
    assert np.isclose(loss, 0.5 * np.mean((Xd @ wd - yd) ** 2), rtol=1e-13)
    # at the least-squares solution (LAPACK) the gradient vanishes
    w_ls = np.linalg.lstsq(Xd, yd, rcond=None)[0]
    _, g_ls, _ = ref.full_gradient(prob, X, y, w_ls.astype(np.float32))
    assert np.linalg.norm(g_ls) < 1e-5 * np.linalg.norm(g)


def test_l2_term():
    X, y, _ = inp.linreg(50, 5, seed=2)
    w = np.arange(5, dtype=np.float32) - 2
    g0 = ref.full_gradient(ref.make_problem(50, 5, lam=0.0), X, y, w)
    g1 = ref.full_gradient(ref.make_problem(50, 5, lam=0.3), X, y, w)
    assert np.allclose(g1[1] - g0[1], 0.3 * w, atol=1e-12)
    assert np.isclose(g1[2] - g0[2], 0.15 * np.sum(w.astype(np.float64) ** 2))


def _fd_grad(f, w, eps=1e-3):
    g = np.zeros_like(w, dtype=np.float64)
    for k in range(w.size):
        e = np.zeros_like(w)
        e.flat[k] = eps
        g.flat[k] = (f(w + e) - f(w - e)) / (2 * eps)
    return g


def test_logistic_loss_and_gradient():
    X, y, _ = inp.logistic(120, 9, seed=3)
    rng = np.random.default_rng(1)
    w = (3 * rng.standard_normal(9)).astype(np.float32)
    prob = ref.make_problem(120, 9, loss=ref.LOGISTIC, lam=1e-2)
    phi, g, loss = ref.full_gradient(prob, X, y, w)
    Xd, yd, wd = X.astype(np.float64), y.astype(np.float64), w.astype(np.float64)
    # loss against scipy's log-sigmoid
    want = -np.mean(log_expit(yd * (Xd @ wd))) + 0.5e-2 * np.sum(wd ** 2)
    assert np.isclose(loss, want, rtol=1e-12)
    # gradient against central differences of the oracle's own loss (fp32 steps are exact here)
    f = lambda v: ref.full_gradient(prob, X, y, v.astype(np.float32))[2]
    w_grid = np.round(w * 256) / 256  # representable offsets
    _, g2, _ = ref.full_gradient(prob, X, y, w_grid.astype(np.float32))
    fd = _fd_grad(f, w_grid.astype(np.float64), eps=2.0 ** -8)
    assert np.allclose(g2[0], fd, rtol=2e-4, atol=1e-6)
    # extreme margins neither overflow nor lose the sign
    big = ref.make_problem(2, 1, loss=ref.LOGISTIC)
    phi, gb, lb = ref.full_gradient(big, np.array([[1000.0], [-1000.0]], np.float32),
                                    np.array([1.0, 1.0], np.float32), np.array([1.0], np.float32))
    assert np.isfinite(lb) and np.isclose(lb, 500.0)
    assert np.allclose(gb, [[(0.0 * 1000 + -1.0 * -1000) / 2]])


def test_softmax_loss_and_gradient():
    X, y, _ = inp.softmax_sparse(90, 11, 4, seed=4)
    rng = np.random.default_rng(2)
    W = rng.standard_normal((4, 11)).astype(np.float32)
    prob = ref.make_problem(90, 11, K=4, loss=ref.SOFTMAX, lam=1e-3)
    phi, g, loss = ref.full_gradient(prob, X, y, W)
    Xd, Wd = X.astype(np.float64), W.astype(np.float64)
    A = Xd @ Wd.T
    assert np.allclose(phi, A, rtol=1e-13, atol=1e-13)
    want = np.mean(logsumexp(A, axis=1) - A[np.arange(90), y]) + 0.5e-3 * np.sum(Wd ** 2)
    assert np.isclose(loss, want, rtol=1e-12)
    P = np.exp(A - logsumexp(A, axis=1, keepdims=True))
    P[np.arange(90), y] -= 1
    assert np.allclose(g, P.T @ Xd / 90 + 1e-3 * Wd, rtol=1e-11, atol=1e-13)
    # and against finite differences of the loss
    Wg = np.round(W * 256) / 256
    f = lambda v: ref.full_gradient(prob, X, y, v.astype(np.float32))[2]
    _, g2, _ = ref.full_gradient(prob, X, y, Wg.astype(np.float32))
    fd = _fd_grad(f, Wg.astype(np.float64), eps=2.0 ** -8)
    assert np.allclose(g2, fd, rtol=2e-4, atol=1e-6)


def test_binary_softmax_equals_logistic():
    """K = 2 softmax with W = (0, w) has the logistic margins, loss and gradient."""
    X, y, _ = inp.logistic(80, 6, seed=5)
    w = np.random.default_rng(3).standard_normal(6).astype(np.float32)
    pl = ref.make_problem(80, 6, loss=ref.LOGISTIC)
    ps = ref.make_problem(80, 6, K=2, loss=ref.SOFTMAX)
    _, gl, ll = ref.full_gradient(pl, X, y, w)
    W = np.stack([np.zeros(6, np.float32), w])
    ys = ((y + 1) / 2).astype(np.int32)
    _, gs, ls = ref.full_gradient(ps, X, ys, W)
    assert np.isclose(ll, ls, rtol=1e-12)
    assert np.allclose(gs[1], gl[0], rtol=1e-10, atol=1e-14)
    assert np.allclose(gs[0], -gl[0], rtol=1e-10, atol=1e-14)


def test_bad_label_is_an_error():
    prob = ref.make_problem(3, 2, K=3, loss=ref.SOFTMAX)
    with pytest.raises(ValueError):
        ref.full_gradient(prob, np.zeros((3, 2), np.float32), np.array([0, 3, 1], np.int32),
                          np.zeros((3, 2), np.float32))
