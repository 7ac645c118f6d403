"""The conditioning study (paper, appendix "Conditioning Evaluation") on the oracle, no GPU:
the data recipe has the spectrum it claims, and the three algorithms behave as that section
reports -- all of them slow down as the condition number grows, and past a threshold HALP
falls behind SVRG, the 8-bit form first."""
import numpy as np
import pytest

import halp_inputs as inp
from oracle import ref

N, D, T, EPOCHS = 1000, 64, 1000, 50


@pytest.mark.parametrize("kappa", [1.0, 37.0, 1e4])
def test_conditioned_recipe_has_the_prescribed_spectrum(kappa):
    X, y, w_star, eig = inp.linreg_conditioned(200, 16, kappa, seed=4, noise=0.0)
    H = X.astype(np.float64).T @ X.astype(np.float64) / 200
    ev = np.linalg.eigvalsh(H)
    assert np.allclose(ev, np.sort(eig), rtol=2e-5)
    assert abs(ev[0] - 1.0) < 1e-4 and abs(ev[-1] / ev[0] - kappa) < 1e-4 * kappa   # mu = 1, L = kappa
    assert np.allclose(np.diff(np.log(eig)), np.log(kappa) / 15 if kappa > 1 else 0.0, atol=1e-12)
    assert np.allclose(X.astype(np.float64) @ w_star.astype(np.float64), y, rtol=1e-4, atol=1e-4)
    # a different seed is a different rotation of the same spectrum
    X2 = inp.linreg_conditioned(200, 16, kappa, seed=5, noise=0.0)[0]
    assert not np.allclose(X, X2)
    assert np.allclose(np.linalg.eigvalsh(X2.astype(np.float64).T @ X2.astype(np.float64) / 200), ev, rtol=2e-5)


def _final_gradient_norm(X, y, alg, b, alpha, mu):
    w = np.zeros((1, D), np.float32)
    if alg == "svrg":
        prob = ref.make_problem(N, D, alpha=alpha, seed=3, algorithm=ref.ALG_SVRG)
        for k in range(EPOCHS):
            w = ref.svrg_epoch(prob, X, y, w, k, T)["w"]
            if not np.all(np.isfinite(w)):
                return np.inf
    else:
        dd = inp.default_delta_d(X, b)
        Xq = ref.quantize_data(X, dd, b)
        prob = ref.make_problem(N, D, b=b, alpha=alpha, mu=mu, delta_d=dd, seed=3)
        for k in range(EPOCHS):
            w = ref.epoch(prob, X, Xq, y, w, k, T)["w"]
            if not np.all(np.isfinite(w)):
                return np.inf
    return float(np.linalg.norm(ref.full_gradient(prob, X, y, w)[1]))


def _best(X, y, alg, b, alphas, mus):
    return min(_final_gradient_norm(X, y, alg, b, a, m) for a in alphas for m in (mus if alg != "svrg" else [1.0]))


def test_threshold_in_the_condition_number():
    """T = 1000, 50 epochs, best of a small grid of step sizes and mu around each algorithm's
    optimum, as in that section."""
    res = {}
    for kappa, alphas, mus8, mus16 in [(1.0, [3e-3, 1e-3], [2.0, 8.0], [2.0, 8.0]),
                                       (1e4, [3e-5, 1e-5], [512.0, 2000.0], [8.0, 32.0])]:
        X, y, _, _ = inp.linreg_conditioned(N, D, kappa, seed=1)
        g0 = np.linalg.norm(ref.full_gradient(ref.make_problem(N, D), X, y, np.zeros((1, D), np.float32))[1])
        with np.errstate(over="ignore"):
            res[kappa] = dict(g0=g0, svrg=_best(X, y, "svrg", 0, alphas, None),
                              h16=_best(X, y, "halp", 16, alphas, mus16),
                              h8=_best(X, y, "halp", 8, alphas, mus8))
    lo, hi = res[1.0], res[1e4]
    # well conditioned: all three converge linearly down to what fp32 iterates resolve
    for k in ("svrg", "h16", "h8"):
        assert lo[k] < 1e-6 * lo["g0"], (k, lo)
        assert hi[k] / hi["g0"] > 1e3 * lo[k] / lo["g0"], (k, lo, hi)   # everyone is slower at kappa = 1e4
    # below the threshold the bit width does not matter; above it 8 bits fall behind SVRG
    # while 16 bits still keep up
    assert lo["h8"] < 2 * lo["svrg"] and lo["h16"] < 2 * lo["svrg"]
    assert hi["h8"] > 2 * hi["svrg"], hi
    assert hi["h16"] < 1.5 * hi["svrg"], hi
