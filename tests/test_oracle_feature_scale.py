"""Pins of the per-feature data scales (diagonal preconditioning, the remark after Theorem 2),
no GPU: the scaled forms are the plain algorithm on column-rescaled data, the scaled gradient
is the derivative with respect to the scaled model, and the scales rescue columns that one
scalar data scale rounds away."""
import numpy as np
import pytest

import halp_inputs as inp
from oracle import ref


def _columns_over_decades(N, d, seed, decades=3.0):
    X0, _, ws = inp.linreg(N, d, seed=seed, x_var="inv_d", noise=0.0)
    col = np.logspace(0, -decades, d).astype(np.float32)
    X = (X0 * col).astype(np.float32)
    y = (X.astype(np.float64) @ (ws / col)).astype(np.float32)
    return X, y


@pytest.mark.parametrize("loss,b", [(ref.SQUARED, 8), (ref.LOGISTIC, 16), (ref.SOFTMAX, 8)])
def test_power_of_two_scales_are_plain_halp_on_rescaled_data(loss, b):
    """With s_j = 2^e every division by s_j is exact, so two epochs of the scaled forms on X must
    equal, bit for bit, two plain epochs on X' = X / s."""
    N, d, K = 300, 24, (3 if loss == ref.SOFTMAX else 1)
    rng = np.random.default_rng(3)
    if loss == ref.SOFTMAX:
        X, y, _ = inp.softmax_sparse(N, d, K, seed=2)
    elif loss == ref.LOGISTIC:
        X, y, _ = inp.logistic(N, d, seed=2)
    else:
        X, y, _ = inp.linreg(N, d, seed=2, x_var="inv_d", noise=0.1)
    s = (2.0 ** rng.integers(-6, 3, size=d)).astype(np.float32)
    Xp = (X / s).astype(np.float32)
    assert np.array_equal(Xp.astype(np.float64) * s, X.astype(np.float64))
    dd = inp.default_delta_d(Xp, b)
    Xq_plain = ref.quantize_data(Xp, dd, b)
    Xq_scaled = ref.quantize_data_scaled(X, dd, s, b)
    assert np.array_equal(Xq_plain, Xq_scaled)
    prob = ref.make_problem(N, d, K=K, loss=loss, b=b, alpha=0.05, mu=0.3, delta_d=dd, seed=8)
    va = np.zeros((K, d), np.float32)
    vb = va.copy()
    for k in range(2):
        a = ref.epoch(prob, Xp, Xq_plain, y, va, k, 2 * N)
        c = ref.epoch_scaled(prob, X, Xq_scaled, y, vb, s, k, 2 * N)
        for name in ("phi", "g", "h", "z", "w"):
            assert np.array_equal(a[name], c[name]), (k, name)
        assert np.array_equal(a["scales"][:6], c["scales"][:6])
        va, vb = a["w"], c["w"]
    assert np.any(va != 0)


def test_scaled_gradient_is_the_derivative_in_v():
    N, d = 120, 9
    X, y, _ = inp.logistic(N, d, seed=6)
    rng = np.random.default_rng(0)
    s = rng.uniform(0.05, 3.0, size=d).astype(np.float32)
    v = rng.standard_normal(d).astype(np.float32)
    prob = ref.make_problem(N, d, loss=ref.LOGISTIC)
    phi, g, loss = ref.full_gradient_scaled(prob, X, y, v, s)
    Xd, yd = X.astype(np.float64), y.astype(np.float64)
    f = lambda vv: np.mean(np.log1p(np.exp(-yd * (Xd @ (vv / s.astype(np.float64))))))
    assert abs(loss - f(v.astype(np.float64))) < 1e-6
    assert np.allclose(phi[:, 0], Xd @ (v.astype(np.float64) / s), rtol=0, atol=1e-5)
    for j in range(d):
        e = np.zeros(d); e[j] = 1e-5
        num = (f(v + e) - f(v - e)) / 2e-5
        assert abs(g[0, j] - num) < 1e-6 * max(1.0, abs(num)), j
    # unit scales: the plain pass
    phi1, g1, loss1 = ref.full_gradient_scaled(prob, X, y, v, np.ones(d, np.float32))
    phi0, g0, loss0 = ref.full_gradient(prob, X, y, v.reshape(1, d))
    assert np.array_equal(phi1, phi0) and np.array_equal(g1, g0) and loss1 == loss0
    with pytest.raises(ValueError):   # an L2 term on w is not an L2 term on v
        ref.full_gradient_scaled(ref.make_problem(N, d, loss=ref.LOGISTIC, lam=0.1), X, y, v, s)


def test_feature_scales_keep_the_columns_a_scalar_scale_rounds_away():
    N, d, T, K, b = 800, 32, 1600, 20, 8
    X, y = _columns_over_decades(N, d, seed=5)
    best = {}
    for mode in ("scalar", "feature"):
        if mode == "scalar":
            s, dd = np.ones(d, np.float32), inp.default_delta_d(X, b)
        else:
            s, dd = np.abs(X).max(axis=0).astype(np.float32), 1.0 / 127
        Xq = ref.quantize_data_scaled(X, dd, s, b)
        lost = int((Xq == 0).all(axis=0).sum())
        losses = []
        for alpha, mu in [(0.1, 0.1), (0.03, 0.1), (0.3, 0.01)]:
            prob = ref.make_problem(N, d, b=b, alpha=alpha, mu=mu, delta_d=dd, seed=1)
            v = np.zeros((1, d), np.float32)
            for k in range(K):
                out = ref.epoch_scaled(prob, X, Xq, y, v, s, k, T)
                v = out["w"]
            losses.append(out["loss"])
        best[mode] = (min(losses), lost)
    assert best["scalar"][1] >= 5 and best["feature"][1] == 0   # whole columns quantize to zero
    assert best["scalar"][0] > 0.1                               # ... and their share of the loss stays
    assert best["feature"][0] < 1e-8
