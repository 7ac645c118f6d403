"""Pins of the oracle's SVRG inner loop (Algorithm 1 for linear models, C, fp64; no GPU):
against the generic numpy form of Algorithm 1 on the same index stream, and against the
closed-form least-squares optimum."""
import numpy as np
import pytest

import halp_inputs as inp
from oracle import alg_generic as gen
from oracle import ref


def _callables(X, y, loss, lam):
    Xd, yd = X.astype(np.float64), y.astype(np.float64)
    N = len(yd)
    if loss == ref.SQUARED:
        r = lambda A: A - yd
    else:
        r = lambda A: -yd / (1 + np.exp(yd * A))
    grad_i = lambda i, w: r(Xd @ w)[i] * Xd[i] + lam * w
    full = lambda w: Xd.T @ r(Xd @ w) / N + lam * w
    return grad_i, full


@pytest.mark.parametrize("loss,lam", [(ref.SQUARED, 0.0), (ref.SQUARED, 0.05), (ref.LOGISTIC, 0.01)])
def test_matches_the_generic_algorithm_1(loss, lam):
    N, d, T = 80, 9, 300
    X, y, _ = (inp.logistic if loss == ref.LOGISTIC else inp.linreg)(N, d, seed=3)
    grad_i, full = _callables(X, y, loss, lam)
    prob = ref.make_problem(N, d, loss=loss, alpha=0.03, lam=lam, seed=17, algorithm=ref.ALG_SVRG)
    w0 = (0.2 * np.random.default_rng(1).standard_normal(d))
    # exact margins and gradient (fp64) so that both sides see the same inputs
    Xd = X.astype(np.float64)
    phi = Xd @ w0
    g = full(w0)
    # the C loop takes fp32 phi and g: make them exactly representable
    phi32, g32 = phi.astype(np.float32), g.astype(np.float32)
    idx = lambda k, t: ref.sample_index(17, 5, t, 1, 0, N)
    # generic form with the same (rounded) anchors: grad_i(i, w~) + g~ replaced accordingly
    w = w0.copy()
    yd = y.astype(np.float64)
    for t in range(T):
        i = idx(0, t)
        a1 = Xd[i] @ w
        if loss == ref.SQUARED:
            diff = a1 - float(phi32[i])
        else:
            dl = lambda a: -yd[i] / (1 + np.exp(yd[i] * a))
            diff = dl(a1) - dl(float(phi32[i]))
        w = w - 0.03 * (diff * Xd[i] + lam * (w - w0) + g32.astype(np.float64))
    out = ref.svrg_inner(prob, X, y, phi32, g32, w0, 5, T)
    assert np.linalg.norm(out - w0) > 1e-3
    assert np.allclose(out, w, rtol=1e-11, atol=1e-13)
    # and the library form of Algorithm 1 itself (exact anchors) stays within their rounding
    sv = gen.svrg(grad_i, full, w0, 0.03, T, 1, idx)[1]
    assert np.linalg.norm(out - sv) < 1e-5 * max(1.0, np.linalg.norm(sv))


def test_minibatch_averages_the_rows():
    N, d, T, B = 60, 5, 40, 4
    X, y, _ = inp.linreg(N, d, seed=4)
    Xd, yd = X.astype(np.float64), y.astype(np.float64)
    prob = ref.make_problem(N, d, B=B, alpha=0.05, seed=2, algorithm=ref.ALG_SVRG)
    w0 = np.zeros(d)
    phi32 = (Xd @ w0).astype(np.float32)
    g32 = (Xd.T @ (Xd @ w0 - yd) / N).astype(np.float32)
    w = w0.copy()
    for t in range(T):
        rows = [ref.sample_index(2, 0, t, B, m, N) for m in range(B)]
        step = g32.astype(np.float64).copy()
        for i in rows:
            step += (Xd[i] @ w - float(phi32[i])) / B * Xd[i]
        w = w - 0.05 * step
    out = ref.svrg_inner(prob, X, y, phi32, g32, w0, 0, T)
    assert np.allclose(out, w, rtol=1e-11, atol=1e-13)


def test_epochs_reach_the_least_squares_solution():
    N, d = 200, 8
    X, y, _ = inp.linreg(N, d, seed=6)
    w_star = np.linalg.lstsq(X.astype(np.float64), y.astype(np.float64), rcond=None)[0]
    prob = ref.make_problem(N, d, alpha=0.02, seed=1, algorithm=ref.ALG_SVRG)
    w = np.zeros((1, d), np.float32)
    errs = []
    for k in range(12):
        w = ref.svrg_epoch(prob, X, y, w, k, 2 * N)["w"]
        errs.append(np.linalg.norm(w[0] - w_star))
    assert errs[-1] < 1e-5 * np.linalg.norm(w_star)
    assert errs[5] < 0.1 * errs[0]
