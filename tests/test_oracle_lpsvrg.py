"""Pins of the oracle's integer form of LP-SVRG (Algorithm 2; no GPU): unbiased for the
update Algorithm 2 writes in reals, full-precision SVRG in the limit of a fine lattice, the
accuracy floor of Theorem 1 scaling with delta^2, and the fixed box around 0."""
import numpy as np
import pytest

import halp_inputs as inp
from oracle import alg_generic as gen
from oracle import ref
from test_oracle_halp import exact_lowprec_data, lsq_callables


def _lp(N, d, **kw):
    return ref.make_problem(N, d, algorithm=ref.ALG_LPSVRG, **kw)


@pytest.mark.parametrize("loss,b", [(ref.SQUARED, 8), (ref.LOGISTIC, 8), (ref.SQUARED, 16)])
def test_integer_step_is_unbiased_for_algorithm_2(loss, b):
    """E over the rounding and the sampled i of the integer step from a state w != w~ equals
    u = w - alpha (grad f_i(w) - grad f_i(w~) + g~) averaged over i, in units of delta."""
    N, d = 7, 8
    X, Xq, delta_d = exact_lowprec_data(N, d, b, seed=11, scale_pow=-6 if b == 8 else -14)
    if b == 16:
        Xq = (Xq.astype(np.int32) * 150).astype(np.int16)
        X = (Xq.astype(np.float64) * delta_d).astype(np.float32)
    rng = np.random.default_rng(5)
    y = (rng.choice([-1.0, 1.0], size=N) if loss == ref.LOGISTIC else rng.standard_normal(N)).astype(np.float32)
    qmax = 2 ** (b - 1) - 1
    delta = 2.0 ** -7 if b == 8 else 2.0 ** -15
    Wt = rng.integers(-qmax // 4, qmax // 4, size=(1, d)).astype(np.int32)     # w~ / delta
    W0 = Wt + rng.integers(-qmax // 8, qmax // 8, size=(1, d)).astype(np.int32)  # w / delta
    w_tilde = (Wt * delta).astype(np.float32)
    assert np.array_equal(w_tilde.astype(np.float64), Wt * delta)
    alpha = 0.05
    base = dict(loss=loss, b=b, alpha=alpha, delta_d=delta_d, delta=delta)
    prob = _lp(N, d, seed=0, **base)
    phi, g, _ = ref.full_gradient(prob, X, y, w_tilde)
    phi32, g32 = phi.astype(np.float32), g.astype(np.float32)
    sc, _, z_begin = ref.lp_begin(prob, g32, w_tilde, 0)
    assert np.array_equal(z_begin, Wt) and sc[0] == delta   # the epoch starts from w~ itself

    Xd = X.astype(np.float64)
    def resid(w):
        a = Xd @ w
        if loss == ref.SQUARED:
            return a - y.astype(np.float64)
        yy = y.astype(np.float64)
        return -yy / (1 + np.exp(yy * a))
    w_real, wt_real = W0[0] * delta, phi32.astype(np.float64)  # margins of w~ as the pass hands them on
    diff = (resid(w_real) - (wt_real[:, 0] - y if loss == ref.SQUARED else
                             -y.astype(np.float64) / (1 + np.exp(y.astype(np.float64) * wt_real[:, 0])))) @ Xd / N
    want = (w_real - alpha * (diff + g32[0].astype(np.float64))) / delta

    n = 12000
    acc, acc2 = np.zeros(d), np.zeros(d)
    for s in range(n):
        ps = _lp(N, d, seed=1000 + s, **base)
        scs, h, _ = ref.lp_begin(ps, g32, w_tilde, 0)
        out = ref.inner_loop(ps, Xq, phi32, y, h, scs, 0, 1, z0=W0)
        assert out["counters"][0] == 0 and out["counters"][1] == 0
        acc += out["z"][0]
        acc2 += out["z"][0].astype(np.float64) ** 2
    mean = acc / n
    std = np.sqrt(np.maximum(acc2 / n - mean ** 2, 1e-12))
    assert np.all(np.abs(mean - want) < 5 * std / np.sqrt(n) + 1e-6), (mean - want, std)
    assert np.max(np.abs(want - W0[0])) > 50 * np.max(std) / np.sqrt(n)


def test_fine_lattice_tracks_svrg():
    """b = 24 and a tiny delta: the integer LP-SVRG epoch follows full-precision SVRG on the
    same index stream."""
    N, d, b = 50, 6, 24
    rng = np.random.default_rng(30)
    Xq = rng.integers(-(2 ** 22), 2 ** 22, size=(N, d)).astype(np.int32)
    delta_d = 2.0 ** -22
    X = (Xq * delta_d).astype(np.float32)
    y = (X @ rng.standard_normal(d) + 0.05 * rng.standard_normal(N)).astype(np.float32)
    grad_i, full, _ = lsq_callables((Xq * delta_d), y)
    prob = _lp(N, d, b=b, alpha=0.05, delta_d=delta_d, delta=2.0 ** -21, seed=31)
    T = 150
    out = ref.epoch(prob, X, Xq, y, np.zeros((1, d), np.float32), 0, T)
    idx = lambda k, t: ref.sample_index(31, k, t, 1, 0, N)
    sv = gen.svrg(grad_i, full, np.zeros(d), 0.05, T, 1, idx)
    move = np.linalg.norm(sv[1])
    assert move > 0.1
    assert np.linalg.norm(out["w"][0] - sv[1]) < 2e-5 * move + 3e-7 * np.linalg.norm(sv[1])


def _floor(delta, b, seed):
    """mean objective gap of the last epochs of an integer LP-SVRG run on a small regression"""
    X, y, _ = inp.linreg(200, 6, seed=40)
    dd = inp.default_delta_d(X, 16)
    Xq = ref.quantize_data(X, dd, 16)
    Xe = (Xq.astype(np.float64) * dd)               # the data the inner loop sees
    Xf = Xe.astype(np.float32)
    w_star = np.linalg.lstsq(Xe, y.astype(np.float64), rcond=None)[0]
    f = lambda w: 0.5 * np.mean((Xe @ w - y) ** 2)
    prob = _lp(200, 6, b=b, alpha=0.02, delta_d=dd, delta=delta, seed=seed)
    w = np.zeros((1, 6), np.float32)
    gaps = []
    for k in range(30):
        w = ref.epoch(prob, Xf, Xq, y, w, k, 400)["w"]
        gaps.append(f(w[0].astype(np.float64)) - f(w_star))
    return float(np.mean(gaps[15:])), float(np.max(np.abs(w_star)))


def test_accuracy_floor_scales_with_delta_squared():
    """Theorem 1: the limit is O(delta^2).  Halving delta twice lowers the floor ~16x, and the
    floor stays under the theorem's 2 d delta^2 L / (gamma (1 - gamma)) at gamma = 1/2."""
    _, wmax = _floor(1e-2, 16, 0)
    d1 = 4 * wmax / 32767 * 64            # coarse enough for the floor to dominate quickly
    f1 = np.mean([_floor(d1, 16, s)[0] for s in range(3)])
    f4 = np.mean([_floor(d1 / 4, 16, s)[0] for s in range(3)])
    assert 6 < f1 / f4 < 40, (f1, f4)
    X, _, _ = inp.linreg(200, 6, seed=40)
    L = np.max(np.sum(X.astype(np.float64) ** 2, axis=1))
    assert f1 < 2 * 6 * d1 ** 2 * L / 0.25


def test_iterates_stay_in_the_fixed_box():
    """The box is [-2^(b-1) delta, (2^(b-1)-1) delta] around 0 (the theorem's condition on w*):
    with an optimum outside it the iterates saturate at the boundary and the clamp counter says so."""
    X, y, w_true = inp.linreg(100, 4, seed=50)
    dd = inp.default_delta_d(X, 8)
    Xq = ref.quantize_data(X, dd, 8)
    delta = 0.25 * np.max(np.abs(w_true)) / 127
    prob = _lp(100, 4, b=8, alpha=0.02, delta_d=dd, delta=delta, seed=3)
    w = np.zeros((1, 4), np.float32)
    hits = 0
    for k in range(6):
        out = ref.epoch(prob, X, Xq, y, w, k, 300)
        w, hits = out["w"], hits + int(out["counters"][0])
        assert out["z"].max() <= 127 and out["z"].min() >= -128
        assert np.array_equal(w[0].astype(np.float64), (delta * out["z"][0]).astype(np.float32).astype(np.float64))
    assert hits > 0
    assert np.max(np.abs(w)) <= 128 * delta * (1 + 1e-6)


def test_l2_is_refused_in_this_mode():
    prob = _lp(10, 3, b=8, alpha=0.02, delta_d=1.0, delta=0.1, lam=1e-3)
    with pytest.raises(ValueError):
        ref.lp_begin(prob, np.ones((1, 3), np.float32), np.zeros((1, 3), np.float32), 0)
