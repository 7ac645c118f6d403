"""Pins of the oracle's algorithms (no GPU): the generic forms against each
other, the integer linear-model form against the generic update in
expectation, the closed-form least-squares optimum, the linear rate of
Theorem 2, the bit-centering box, and bookkeeping identities of the scales."""
import numpy as np
import pytest

import halp_inputs as inp
from oracle import alg_generic as gen
from oracle import ref


# ----------------------------------------------------------------- helpers

def lsq_callables(X, y, lam=0.0):
    X = X.astype(np.float64)
    y = y.astype(np.float64)
    N = X.shape[0]
    grad_i = lambda i, w: (X[i] @ w - y[i]) * X[i] + lam * w
    full = lambda w: X.T @ (X @ w - y) / N + lam * w
    f = lambda w: 0.5 * np.mean((X @ w - y) ** 2) + 0.5 * lam * w @ w
    return grad_i, full, f


def exact_lowprec_data(N, d, b, seed, scale_pow=-6):
    """Integer data and the fp32 matrix that equals delta_d * Xq exactly."""
    rng = np.random.default_rng(seed)
    qmax = 2 ** (b - 1) - 1
    lim = min(qmax, 100)
    Xq = rng.integers(-lim, lim + 1, size=(N, d)).astype(ref.xq_dtype(b))
    delta_d = 2.0 ** scale_pow
    X = (Xq.astype(np.float64) * delta_d).astype(np.float32)
    assert np.array_equal(X.astype(np.float64), Xq.astype(np.float64) * delta_d)
    return X, Xq, delta_d


# ------------------------------------------- Algorithm 3 with Q = id is Algorithm 1

def test_identity_q_halp_is_svrg():
    X, y, _ = inp.linreg(60, 7, seed=0)
    grad_i, full, _ = lsq_callables(X, y)
    rng = np.random.default_rng(0)
    stream = {}
    idx = lambda k, t: stream.setdefault((k, t), int(rng.integers(0, 60)))
    w0 = np.zeros(7)
    a = gen.svrg(grad_i, full, w0, 0.02, 150, 4, idx)
    b_, _ = gen.halp(grad_i, full, w0, 0.02, 150, 4, idx, mu=1.0, b=8, rng=None, Q=gen.identity_q)
    for wa, wb in zip(a, b_):
        assert np.allclose(wa, wb, rtol=1e-10, atol=1e-12)
    assert np.linalg.norm(full(a[-1])) < 1e-2 * np.linalg.norm(full(w0))


# --------------------------- Algorithm 4 (integers) is Algorithm 3 in expectation

def _expected_step(prob, X, y, w, z0_real, g):
    """E_i of u = z - alpha (grad f_i(w~ + z) - grad f_i(w~) + g~), in reals (Algorithm 3)."""
    Xd = X.astype(np.float64)
    K, d = prob.K, prob.d
    W0 = w.astype(np.float64).reshape(K, d)
    W1 = W0 + z0_real
    def resid(W):
        A = Xd @ W.T
        if prob.loss == ref.SQUARED:
            return A - y.astype(np.float64)[:, None]
        if prob.loss == ref.LOGISTIC:
            yy = y.astype(np.float64)[:, None]
            return -yy / (1 + np.exp(yy * A))
        P = np.exp(A - A.max(axis=1, keepdims=True))
        P /= P.sum(axis=1, keepdims=True)
        P[np.arange(len(y)), y] -= 1
        return P
    diff = (resid(W1) - resid(W0)).T @ Xd / X.shape[0] + prob.lam * z0_real
    return z0_real - prob.alpha * (diff + g)


@pytest.mark.parametrize("loss,K,B,lam,b", [
    (ref.SQUARED, 1, 1, 0.0, 8),
    (ref.LOGISTIC, 1, 1, 0.0, 8),
    (ref.SQUARED, 1, 3, 0.05, 8),
    (ref.SOFTMAX, 3, 2, 0.02, 8),
    (ref.LOGISTIC, 1, 2, 0.0, 16),
])
def test_integer_step_is_unbiased_for_the_generic_update(loss, K, B, lam, b):
    N, d = 7, 8
    X, Xq, delta_d = exact_lowprec_data(N, d, b, seed=11, scale_pow=-6 if b == 8 else -14)
    if b == 16:  # use the width
        Xq = (Xq.astype(np.int32) * 150).astype(np.int16)
        X = (Xq.astype(np.float64) * delta_d).astype(np.float32)
    rng = np.random.default_rng(5)
    if loss == ref.SOFTMAX:
        y = rng.integers(0, K, size=N).astype(np.int32)
    elif loss == ref.LOGISTIC:
        y = rng.choice([-1.0, 1.0], size=N).astype(np.float32)
    else:
        y = rng.standard_normal(N).astype(np.float32)
    w = (0.5 * rng.standard_normal((K, d))).astype(np.float32)
    alpha, mu = 0.05, 0.5
    base = dict(N=N, d=d, K=K, loss=loss, b=b, B=B, alpha=alpha, mu=mu, lam=lam, delta_d=delta_d)
    prob = ref.make_problem(seed=0, **base)
    phi, g, _ = ref.full_gradient(prob, X, y, w)
    phi32, g32 = phi.astype(np.float32), g.astype(np.float32)
    scales, _, _ = ref.recenter(prob, g32, 0)
    qmax = 2 ** (b - 1) - 1
    z0 = rng.integers(-qmax // 4, qmax // 4, size=(K, d)).astype(np.int32)
    want = _expected_step(prob, X, y, w, scales[0] * z0, g32.astype(np.float64)) / scales[0]
    n = 12000
    acc = np.zeros((K, d))
    acc2 = np.zeros((K, d))
    for s in range(n):
        ps = ref.make_problem(seed=1000 + s, **base)
        sc, h, _ = ref.recenter(ps, g32, 0)
        out = ref.inner_loop(ps, Xq, phi32, y, h, sc, 0, 1, z0=z0)
        assert out["counters"][0] == 0 and out["counters"][1] == 0  # nothing clamped
        acc += out["z"]
        acc2 += out["z"].astype(np.float64) ** 2
    mean = acc / n
    std = np.sqrt(np.maximum(acc2 / n - mean ** 2, 1e-12))
    assert np.all(np.abs(mean - want) < 5 * std / np.sqrt(n) + 1e-6), (mean - want, std)
    # the step is not a no-op: it moved away from z0 by much more than the tolerance
    assert np.max(np.abs(want - z0)) > 50 * np.max(std) / np.sqrt(n)


# ------------------------------------------------ closed-form least squares

def test_halp_reaches_the_least_squares_solution():
    """Integer HALP epochs contract ||w~ - w*|| geometrically towards the LAPACK
    solution, far below one 8-bit grid step of the first epoch (bit centering)."""
    N, d, b = 300, 16, 8
    X, Xq, delta_d = exact_lowprec_data(N, d, b, seed=3, scale_pow=-6)
    rng = np.random.default_rng(4)
    w_true = rng.standard_normal(d)
    y = (X.astype(np.float64) @ w_true + 0.01 * rng.standard_normal(N)).astype(np.float32)
    w_star = np.linalg.lstsq(X.astype(np.float64), y.astype(np.float64), rcond=None)[0]
    H = X.astype(np.float64).T @ X.astype(np.float64) / N
    lam_min, L = np.linalg.eigvalsh(H)[0], np.max(np.sum(X.astype(np.float64) ** 2, axis=1))
    prob = ref.make_problem(N, d, b=b, alpha=0.2 / L, mu=0.9 * lam_min, delta_d=delta_d, seed=7)
    w = np.zeros((1, d), np.float32)
    dist, deltas = [np.linalg.norm(w[0] - w_star)], []
    for k in range(14):
        out = ref.epoch(prob, X, Xq, y, w, k, 2 * N)
        w = out["w"]
        dist.append(np.linalg.norm(w[0] - w_star))
        deltas.append(out["scales"][0])
        assert out["counters"][0] == 0  # z* is inside the box, nothing saturates
    assert dist[-1] < 1e-4 * dist[0]
    assert dist[7] < 0.05 * dist[0]
    assert deltas[-1] < 1e-3 * deltas[0]            # the lattice shrinks with the gradient
    assert dist[-1] < 0.05 * deltas[0]              # far finer than the first epoch's grid


def test_box_contains_the_optimum_when_mu_is_a_lower_bound():
    """||z*|| <= ||grad f(w~)|| / mu, so z* lies in dom(delta_m, b) (Sec. 4, bit centering)."""
    X, y, _ = inp.linreg(200, 10, seed=8)
    Xd, yd = X.astype(np.float64), y.astype(np.float64)
    w_star = np.linalg.lstsq(Xd, yd, rcond=None)[0]
    lam_min = np.linalg.eigvalsh(Xd.T @ Xd / 200)[0]
    rng = np.random.default_rng(9)
    for b in (8, 16):
        prob = ref.make_problem(200, 10, b=b, mu=lam_min, delta_d=1.0)
        for _ in range(5):
            w = rng.standard_normal(10).astype(np.float32)
            _, g, _ = ref.full_gradient(prob, X, y, w)
            scales, _, _ = ref.recenter(prob, g.astype(np.float32), 0)
            qmax = 2 ** (b - 1) - 1
            assert np.max(np.abs(w_star - w)) <= scales[0] * qmax * (1 + 1e-6)
            assert np.linalg.norm(w_star - w) <= scales[0] * qmax * (1 + 1e-6)


# --------------------------------------------------------------- Theorem 2

def _theorem2_instance():
    # d = 2, rows sqrt(2) e_1 / sqrt(2) e_2: mu = 1, L = ||x_i||^2 = 2, kappa = 2
    N = 8
    X = np.zeros((N, 2))
    for i in range(N):
        X[i, i % 2] = np.sqrt(2.0) * (1 if (i // 2) % 2 == 0 else -1)
    rng = np.random.default_rng(12)
    y = X @ np.array([0.7, -1.1]) + 0.3 * rng.standard_normal(N)
    return X, y


def test_theorem2_linear_rate_generic():
    X, y = _theorem2_instance()
    grad_i, full, f = lsq_callables(X, y)
    w_star = np.linalg.lstsq(X, y, rcond=None)[0]
    kappa, L, d, gam, b = 2.0, 2.0, 2, 0.5, 8
    assert b > 1 + np.log2(1 + np.sqrt(2 * kappa ** 2 * d * (1 + gam) / gam ** 2))
    alpha = gam / (4 * L * (1 + gam))
    T = int(np.ceil(8 * kappa * (1 + gam) /
                    (gam ** 2 - 2 * kappa ** 2 * d * (1 + gam) / (2 ** (b - 1) - 1) ** 2)))
    K, seeds = 4, 150
    gaps = np.zeros(K + 1)
    for s in range(seeds):
        rng = np.random.default_rng(100 + s)
        idx = lambda k, t: int(rng.integers(0, len(y)))
        outs, _ = gen.halp(grad_i, full, np.zeros(2), alpha, T, K, idx, mu=1.0, b=b, rng=rng,
                           option="II", option_rng=rng)
        gaps += np.array([f(w) - f(w_star) for w in outs])
    gaps /= seeds
    for k in range(1, K + 1):
        assert gaps[k] <= gam ** k * gaps[0] * 1.05


def test_theorem2_linear_rate_integer_form():
    X, y = _theorem2_instance()
    _, _, f = lsq_callables(X, y)
    w_star = np.linalg.lstsq(X, y, rcond=None)[0]
    b = 8
    delta_d = np.sqrt(2.0) / 90
    Xq = np.rint(X / delta_d).astype(np.int8)
    X32, y32 = X.astype(np.float32), y.astype(np.float32)
    alpha, T, K, gam = 0.5 / (4 * 2 * 1.5), 97, 4, 0.5
    gaps = np.zeros(K + 1)
    seeds = 150
    for s in range(seeds):
        prob = ref.make_problem(8, 2, b=b, alpha=alpha, mu=1.0, delta_d=delta_d, seed=500 + s)
        w = np.zeros((1, 2), np.float32)
        gaps[0] += f(w[0].astype(np.float64)) - f(w_star)
        for k in range(K):
            w = ref.epoch(prob, X32, Xq, y32, w, k, T)["w"]
            gaps[k + 1] += f(w[0].astype(np.float64)) - f(w_star)
    gaps /= seeds
    for k in range(1, K + 1):
        assert gaps[k] <= gam ** k * gaps[0] * 1.05


def test_theorem2_linear_rate_integer_form_option2():
    """Theorem 2 as it is stated: option II ends every epoch at a uniformly drawn iterate."""
    X, y = _theorem2_instance()
    _, _, f = lsq_callables(X, y)
    w_star = np.linalg.lstsq(X, y, rcond=None)[0]
    b = 8
    delta_d = np.sqrt(2.0) / 90
    Xq = np.rint(X / delta_d).astype(np.int8)
    X32, y32 = X.astype(np.float32), y.astype(np.float32)
    alpha, T, K, gam = 0.5 / (4 * 2 * 1.5), 97, 4, 0.5
    gaps = np.zeros(K + 1)
    seeds = 300
    for s in range(seeds):
        prob = ref.make_problem(8, 2, b=b, alpha=alpha, mu=1.0, delta_d=delta_d, seed=900 + s)
        w = np.zeros((1, 2), np.float32)
        gaps[0] += f(w[0].astype(np.float64)) - f(w_star)
        for k in range(K):
            w = ref.epoch(prob, X32, Xq, y32, w, k, T, option2=True)["w"]
            gaps[k + 1] += f(w[0].astype(np.float64)) - f(w_star)
    gaps /= seeds
    for k in range(1, K + 1):
        assert gaps[k] <= gam ** k * gaps[0] * 1.05


def test_option2_draw_is_uniform_on_0_to_T_minus_1():
    T = 12
    draws = np.array([ref.option2_steps(seed, ep, T) for seed in range(300) for ep in range(80)])
    assert draws.min() == 0 and draws.max() == T - 1          # never T: w_{k,T} is not a candidate
    counts = np.bincount(draws, minlength=T)
    chi2 = np.sum((counts - len(draws) / T) ** 2 / (len(draws) / T))
    assert chi2 < 35.0                                        # 11 degrees of freedom, p ~ 2e-4
    assert all(ref.option2_steps(s, 0, 1) == 0 for s in range(50))
    assert ref.option2_steps(3, 0, 0) == 0
    # its own stream: independent of the index draws of the same epoch
    idx = np.array([ref.sample_index(seed, 0, 0, 1, 0, T) for seed in range(4000)])
    d2 = np.array([ref.option2_steps(seed, 0, T) for seed in range(4000)])
    assert abs(np.corrcoef(idx, d2)[0, 1]) < 0.06


def test_option2_epoch_ends_at_a_recorded_iterate():
    """the epoch's result is the iterate the full run passes through after t steps"""
    X, y, _ = inp.linreg(80, 12, seed=2)
    dd = inp.default_delta_d(X, 8)
    Xq = ref.quantize_data(X, dd, 8)
    T = 40
    seen = set()
    for seed in range(6):
        prob = ref.make_problem(80, 12, alpha=0.02, mu=0.7, delta_d=dd, seed=seed)
        w0 = np.zeros((1, 12), np.float32)
        full = ref.epoch(prob, X, Xq, y, w0, 1, T)
        tr = ref.inner_loop(prob, Xq, full["phi"], y, full["h"], full["scales"], 1, T, trace_steps=T)
        t = ref.option2_steps(seed, 1, T)
        seen.add(t)
        out = ref.epoch(prob, X, Xq, y, w0, 1, T, option2=True)
        want = tr["ztraj"][t - 1] if t > 0 else np.zeros_like(out["z"])
        assert np.array_equal(out["z"], want.reshape(out["z"].shape))
        assert np.array_equal(out["w"], ref.apply_offset(prob, full["scales"], want.reshape(1, 12), w0))
    assert len(seen) > 3


# -------------------------------------------- HALP beats the fixed lattice

def test_halp_goes_below_the_lp_svrg_floor():
    """LP-SVRG stalls at an error set by its fixed delta (Theorem 1); HALP with the
    same number of bits keeps contracting (Sec. 4)."""
    X, y, _ = inp.linreg(100, 5, seed=20)
    grad_i, full, f = lsq_callables(X, y)
    w_star = np.linalg.lstsq(X.astype(np.float64), y.astype(np.float64), rcond=None)[0]
    rng = np.random.default_rng(21)
    idx = lambda k, t: int(rng.integers(0, 100))
    delta = 1.2 * np.max(np.abs(w_star)) / 127
    lp = gen.lp_svrg(grad_i, full, np.zeros(5), 0.02, 200, 12, idx, delta, 8, rng)
    hp, _ = gen.halp(grad_i, full, np.zeros(5), 0.02, 200, 12, idx, mu=0.5, b=8, rng=rng)
    gap_lp = f(lp[-1]) - f(w_star)
    gap_hp = f(hp[-1]) - f(w_star)
    assert gap_hp < 1e-3 * gap_lp
    assert gap_lp < 2 * 5 * delta ** 2 * np.max(np.sum(X.astype(np.float64) ** 2, 1)) / (0.5 * 0.5) + 1e-3


def test_many_bits_track_svrg():
    """With b = 24 the integer form follows full-precision SVRG on the same index stream."""
    N, d, b = 50, 6, 24
    rng = np.random.default_rng(30)
    Xq = rng.integers(-(2 ** 22), 2 ** 22, size=(N, d)).astype(np.int32)
    delta_d = 2.0 ** -22
    X = (Xq * delta_d).astype(np.float32)
    y = (X @ rng.standard_normal(d) + 0.05 * rng.standard_normal(N)).astype(np.float32)
    grad_i, full, _ = lsq_callables((Xq * delta_d), y)
    prob = ref.make_problem(N, d, b=b, alpha=0.05, mu=0.3, delta_d=delta_d, seed=31)
    T = 150
    out = ref.epoch(prob, X, Xq, y, np.zeros((1, d), np.float32), 0, T)
    idx = lambda k, t: ref.sample_index(31, k, t, 1, 0, N)
    sv = gen.svrg(grad_i, full, np.zeros(d), 0.05, T, 1, idx)
    move = np.linalg.norm(sv[1])
    assert move > 0.1
    assert np.linalg.norm(out["w"][0] - sv[1]) < 2e-5 * move + 3e-7 * np.linalg.norm(sv[1])


# ------------------------------------------------------------- bookkeeping

@pytest.mark.parametrize("b", [8, 16])
def test_scales_are_compatible(b):
    """delta_m = 2^b delta_i exactly; delta_i = delta_s delta_d to rounding (text after Alg. 4)."""
    rng = np.random.default_rng(40)
    g = rng.standard_normal((3, 9)).astype(np.float32)
    prob = ref.make_problem(10, 9, K=3, loss=ref.SOFTMAX, b=b, alpha=0.03, mu=2.5, delta_d=0.0123)
    s, h, z = ref.recenter(prob, g, 4)
    nrm = np.sqrt(np.sum(g.astype(np.float64) ** 2))
    assert np.isclose(s[3], nrm, rtol=1e-14)
    assert np.isclose(s[0], nrm / (2.5 * (2 ** (b - 1) - 1)), rtol=1e-15)
    assert s[1] * 2.0 ** b == s[0]
    assert np.isclose(s[2] * 0.0123, s[1], rtol=4e-16)
    assert s[4] == 1.0 / s[1] and s[5] == 1.0 / s[2] and s[7] == 0
    assert not z.any()
    # h~ is alpha g~ on the (delta_i, 2b) lattice, within one step, and uses the wide range
    assert np.all(np.abs(h * s[1] - 0.03 * g.astype(np.float64)) <= s[1] * (1 + 1e-9))
    assert np.max(np.abs(h)) > 2 ** (b - 1)


def test_zero_and_nonfinite_gradients():
    prob = ref.make_problem(4, 3)
    s, h, z = ref.recenter(prob, np.zeros((1, 3), np.float32), 0)
    assert s[7] == 1.0 and not h.any() and not z.any()
    s, _, _ = ref.recenter(prob, np.array([[1.0, np.inf, 0.0]], np.float32), 0)
    assert s[7] == -1.0
    # a flagged epoch leaves w~ untouched
    X, Xq, dd = exact_lowprec_data(4, 3, 8, seed=1)
    y = (X @ np.ones(3)).astype(np.float32)
    out = ref.epoch(ref.make_problem(4, 3, delta_d=dd), X, Xq, y, np.ones((1, 3), np.float32), 0, 10)
    assert out["scales"][7] == 1.0 and np.array_equal(out["w"], np.ones((1, 3), np.float32))


def test_state_is_only_w_epoch_seed():
    """6 epochs in one go equal 3 + 3 restarted from the stored w~ (z is reset every epoch)."""
    X, Xq, dd = exact_lowprec_data(80, 8, 8, seed=50)
    y = (X @ np.arange(8) / 8).astype(np.float32)
    prob = ref.make_problem(80, 8, alpha=0.01, mu=0.05, delta_d=dd, seed=3)
    w = np.zeros((1, 8), np.float32)
    for k in range(6):
        w = ref.epoch(prob, X, Xq, y, w, k, 100)["w"]
    w2 = np.zeros((1, 8), np.float32)
    for k in range(3):
        w2 = ref.epoch(prob, X, Xq, y, w2, k, 100)["w"]
    saved = w2.copy()
    for k in range(3, 6):
        saved = ref.epoch(prob, X, Xq, y, saved, k, 100)["w"]
    assert np.array_equal(w, saved)
    # another seed or epoch number gives another trajectory
    other = ref.epoch(prob, X, Xq, y, np.zeros((1, 8), np.float32), 1, 100)["w"]
    first = ref.epoch(prob, X, Xq, y, np.zeros((1, 8), np.float32), 0, 100)["w"]
    assert not np.array_equal(other, first)


def test_saturation_bounds_the_epoch_move():
    """With mu far too large the box is tiny: z saturates and the move per epoch is
    bounded by the box (the clipping effect discussed in the paper's appendix)."""
    X, Xq, dd = exact_lowprec_data(100, 8, 8, seed=60)
    y = (X @ np.ones(8)).astype(np.float32)
    prob = ref.make_problem(100, 8, alpha=0.05, mu=500.0, delta_d=dd, seed=1)
    out = ref.epoch(prob, X, Xq, y, np.zeros((1, 8), np.float32), 0, 400)
    assert out["counters"][0] > 0
    assert out["z"].max() <= 127 and out["z"].min() >= -128
    assert np.max(np.abs(out["w"])) <= out["scales"][0] * 128 * (1 + 1e-6)


def test_trace_records_the_steps():
    X, Xq, dd = exact_lowprec_data(20, 8, 8, seed=70)
    y = (X @ np.ones(8)).astype(np.float32)
    prob = ref.make_problem(20, 8, alpha=0.05, mu=0.2, delta_d=dd, seed=9, B=2)
    phi, g, _ = ref.full_gradient(prob, X, y, np.zeros((1, 8), np.float32))
    s, h, _ = ref.recenter(prob, g.astype(np.float32), 0)
    out = ref.inner_loop(prob, Xq, phi.astype(np.float32), y, h, s, 0, 5, trace_steps=5)
    assert np.array_equal(out["ztraj"][-1], out["z"])
    z_prev = np.zeros((1, 8), np.int64)
    for t in range(5):
        for m in range(2):
            i = out["idx"][t, m]
            assert i == ref.sample_index(9, 0, t, 2, m, 20)
            assert out["D"][t, m, 0] == int(Xq[i].astype(np.int64) @ z_prev[0])
        z_prev = out["ztraj"][t].astype(np.int64)


# ---------------------------------------- scalar path of the inner loop (fp64)

@pytest.mark.parametrize("loss,K,B", [(ref.SOFTMAX, 5, 1), (ref.SOFTMAX, 10, 2), (ref.SOFTMAX, 16, 1),
                                      (ref.LOGISTIC, 1, 3)])
def test_beta_matches_the_plain_definition(loss, K, B):
    """beta = (alpha/B)(l'(phi_i + x_i^T z) - l'(phi_i)) recomputed with numpy's exp and plain
    sums from the traced indices and dot products: the inner loop's own exp and its pairwise
    normaliser agree with the definition to rounding error, class by class."""
    N, d, b = 40, 12, 8
    X, Xq, dd = exact_lowprec_data(N, d, b, seed=21)
    rng = np.random.default_rng(22)
    if loss == ref.SOFTMAX:
        y = rng.integers(0, K, size=N).astype(np.int32)
    else:
        y = rng.choice([-1.0, 1.0], size=N).astype(np.float32)
    w = (2.0 * rng.standard_normal((K, d))).astype(np.float32)  # margins of a few units
    alpha = 0.05
    prob = ref.make_problem(N, d, K=K, loss=loss, b=b, B=B, alpha=alpha, mu=0.05, delta_d=dd, seed=3)
    phi, g, _ = ref.full_gradient(prob, X, y, w)
    phi32 = phi.astype(np.float32)
    s, h, _ = ref.recenter(prob, g.astype(np.float32), 0)
    M = 60
    out = ref.inner_loop(prob, Xq, phi32, y, h, s, 0, M, trace_steps=M)
    assert np.abs(out["D"]).max() > 0
    dscale = dd * s[0]
    worst = 0.0
    for t in range(M):
        for m in range(B):
            i = out["idx"][t, m]
            a0 = phi32[i].astype(np.float64)
            a1 = a0 + dscale * out["D"][t, m].astype(np.float64)
            if loss == ref.SOFTMAX:
                sm = lambda a: np.exp(a - a.max()) / np.exp(a - a.max()).sum()
                want = (alpha / B) * (sm(a1) - sm(a0))
            else:
                dl = lambda a: -float(y[i]) / (1.0 + np.exp(float(y[i]) * a))
                want = (alpha / B) * (dl(a1) - dl(a0))
            worst = max(worst, np.abs(out["beta"][t, m] - want).max())
    assert worst < 1e-15 * alpha * 20, worst
    assert np.abs(out["beta"]).max() > 1e-6 * alpha  # the comparison is not between zeros
