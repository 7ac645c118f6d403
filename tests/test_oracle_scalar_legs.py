"""The two legs of the oracle's inner-loop scalar path against each other, and the
rounding-bit layout against what the method needs of it (no GPU).

Algorithm 4's beta line needs l', i.e. exp, and the paper does not say how exp is
rounded.  The oracle has the definition written out (libm exp, normaliser added from
left to right: SCALAR_PLAIN) and the reproducible reading that GPU parity is held to
(SCALAR_FIXED).  They differ by rounding only; a rounding difference moves the integer
gamma = floor(beta/delta_s + rho) exactly when rho falls between the two values of
beta/delta_s, i.e. with probability |q_fixed - q_plain| per draw.  The tests below
measure that step by step on the same state and the same draw.

The rounding bits of z (Sec. 3 "Quantization": independent, unbiased rounding of every
coordinate at every step) are pinned here by that property itself: uniform per
coordinate and step, and independent across coordinates, classes and steps, also when
d does not fill the last strip of the layout.
"""
import numpy as np
import pytest
from scipy import stats

import halp_inputs as inp
from oracle import ref


def _problem(loss, K, b, seed, scalar_path=ref.SCALAR_FIXED, alpha=0.05, mu=0.05):
    if loss == ref.LOGISTIC:
        N, d = 1500, 24
        X, y, _ = inp.logistic(N, d, seed=seed)
    else:
        N, d = 1500, 20
        X, y, _ = inp.softmax_sparse(N, d, K, seed=seed, zero_frac=0.5)
    dd = inp.default_delta_d(X, b)
    Xq = ref.quantize_data(X, dd, b)
    prob = ref.make_problem(N, d, K=K, loss=loss, b=b, alpha=alpha, mu=mu, lam=1e-4 if K > 1 else 0.0,
                            delta_d=dd, seed=seed, scalar_path=scalar_path)
    return prob, X, Xq, y


def _ulp_bound(loss, K):
    """|l'_fixed - l'_plain| per evaluated difference.  Every exp is within 1 ulp of the true
    value on both legs (2 ulp apart), 1 + e and the division round once each per leg; for the
    softmax the K-term normaliser adds one rounding per term per leg.  All values are below 1,
    where an ulp is at most 2^-53; the bracket of the beta line holds two such values."""
    per_value = (4 if loss == ref.LOGISTIC else 2 * K + 8) * 2.0 ** -53
    return 2 * per_value


@pytest.mark.parametrize("loss,K,b", [(ref.LOGISTIC, 1, 8), (ref.SOFTMAX, 10, 8), (ref.SOFTMAX, 7, 16)])
def test_the_fixed_reading_never_moved_a_gamma_over_1e5_steps(loss, K, b):
    """5 epochs of 20 000 steps each (1e5 steps; K gammas per step).  Per step the two legs'
    beta/delta_s differ by at most the ulp bound, the expected number of moved gammas is the
    sum of those differences (about 1e-8 here), and the observed number is 0; run as two
    separate trajectories the two legs therefore end every epoch with the same z."""
    prob, X, Xq, y = _problem(loss, K, b, seed=3)
    plain, _, _, _ = _problem(loss, K, b, seed=3, scalar_path=ref.SCALAR_PLAIN)
    T, epochs = 20000, 5
    w = np.zeros((K, prob.d), np.float32)
    expected, moved, n_gamma = 0.0, 0, 0
    for k in range(epochs):
        phi, g, _ = ref.full_gradient(prob, X, y, w)
        phi32, g32 = phi.astype(np.float32), g.astype(np.float32)
        scales, h, _ = ref.recenter(prob, g32, k)
        out = ref.inner_loop(prob, Xq, phi32, y, h, scales, k, T, trace_steps=T, trace_z=False,
                             trace_other=True)
        dq = np.abs(out["beta"] - out["beta_other"]) * scales[5]
        assert dq.max() <= _ulp_bound(loss, K) * prob.alpha * scales[5]
        expected += dq.sum()
        moved += int(np.count_nonzero(out["gamma"] != out["gamma_other"]))
        n_gamma += out["gamma"].size
        assert np.any(out["gamma"] != 0)  # the steps are not trivial
        other = ref.inner_loop(plain, Xq, phi32, y, h, scales, k, T)
        assert np.array_equal(other["z"], out["z"])
        assert np.array_equal(other["counters"], out["counters"])
        w = ref.apply_offset(prob, scales, out["z"], w)
    assert n_gamma == epochs * T * K
    print(f"loss={loss} K={K} b={b}: expected moved gammas over {epochs * T} steps = {expected:.3g}")
    assert expected < 1e-3  # what the 1-ulp bound predicts: none in 1e5 steps
    assert moved == 0


@pytest.mark.parametrize("loss,K", [(ref.LOGISTIC, 1), (ref.SOFTMAX, 10)])
def test_moved_gammas_follow_the_rounding_difference_when_the_lattice_is_very_fine(loss, K):
    """Stress: the gradient scaled down by 2e-12, so that delta_m ~ 1e-14 and one ulp of l' is
    about 1e-4 of a lattice step of gamma (the regime where fp64 itself stops resolving the
    margin's move).  Over 1e5 steps a handful of gammas then move, each by one; the count is
    the Poisson number the summed rounding differences predict; and the two legs, run as
    separate trajectories, agree bit for bit up to the first such step."""
    b = 8
    prob, X, Xq, y = _problem(loss, K, b, seed=5, alpha=0.5)
    plain, _, _, _ = _problem(loss, K, b, seed=5, scalar_path=ref.SCALAR_PLAIN, alpha=0.5)
    w = np.random.default_rng(9).standard_normal((K, prob.d)).astype(np.float32)  # margins of order 1
    phi, g, _ = ref.full_gradient(prob, X, y, w)
    phi32 = phi.astype(np.float32)
    scales, h, _ = ref.recenter(prob, (g * 2e-12).astype(np.float32), 0)
    T = 100000
    out = ref.inner_loop(prob, Xq, phi32, y, h, scales, 0, T, trace_steps=T, trace_z=False,
                         trace_other=True)
    dq = np.abs(out["beta"] - out["beta_other"]) * scales[5]
    expected = dq.sum()
    diff = out["gamma"].astype(np.int64) - out["gamma_other"]
    moved = int(np.count_nonzero(diff))
    print(f"loss={loss} K={K}: expected {expected:.2f}, moved {moved}")
    assert 1.0 < expected < 200.0, expected
    assert np.abs(diff).max() == 1
    assert stats.poisson.ppf(1e-6, expected) <= moved <= stats.poisson.isf(1e-6, expected), (moved, expected)
    # separate trajectories: identical until the first moved gamma, which differs by one
    first = int(np.flatnonzero(np.any(diff.reshape(T, -1) != 0, axis=1))[0])
    M = first + 1
    a = ref.inner_loop(prob, Xq, phi32, y, h, scales, 0, M, trace_steps=M)
    c = ref.inner_loop(plain, Xq, phi32, y, h, scales, 0, M, trace_steps=M)
    assert np.array_equal(a["ztraj"][:first], c["ztraj"][:first])
    assert np.array_equal(a["gamma"][:first], c["gamma"][:first])
    assert np.abs(a["gamma"][first].astype(np.int64) - c["gamma"][first]).max() == 1
    # what the trace called "the other leg" is what the plain leg computes on its own
    assert np.array_equal(c["beta"], out["beta_other"][:M])
    assert np.array_equal(c["gamma"], out["gamma_other"][:M])


def test_squared_loss_has_one_leg():
    """No transcendental in the squared loss: both legs are the same arithmetic."""
    X, y, _ = inp.linreg(400, 16, seed=2)
    dd = inp.default_delta_d(X, 8)
    Xq = ref.quantize_data(X, dd, 8)
    prob = ref.make_problem(400, 16, alpha=0.02, mu=0.5, delta_d=dd, seed=1)
    phi, g, _ = ref.full_gradient(prob, X, y, np.zeros((1, 16), np.float32))
    scales, h, _ = ref.recenter(prob, g.astype(np.float32), 0)
    out = ref.inner_loop(prob, Xq, phi.astype(np.float32), y, h, scales, 0, 3000, trace_steps=3000,
                         trace_z=False, trace_other=True)
    assert np.array_equal(out["beta"], out["beta_other"])
    assert np.array_equal(out["gamma"], out["gamma_other"])


# ------------------------------------------------- rounding bits of z: what the method needs

def _bits_table(b, d, K, windows, seed=17, epoch=2):
    """values[w, s, c, j]: the b rounding bits of coordinate (c, j) at step 8 w + s"""
    out = np.empty((windows, 8, K, d), dtype=np.int64)
    for w in range(windows):
        for s in range(8):
            for c in range(K):
                for j in range(d):
                    out[w, s, c, j] = ref.zround_bits(seed, epoch, 8 * w + s, d, b, c, j)
    return out


@pytest.mark.parametrize("b,d,K", [(8, 5, 2), (8, 3, 3), (16, 3, 2)])
def test_rounding_bits_are_uniform_and_independent_across_coordinates_and_steps(b, d, K):
    """d odd, so at 8 bits the last strip of every class is half used and the next class starts
    a new one.  Over many windows of 8 steps, the 8 K d draws of a window (every coordinate at
    every step of the window: all the draws that could share a generator block) are treated as
    8 K d random variables: each is uniform on {0 .. 2^b-1} (chi-square on its top byte or
    its value), no two are correlated, no two are equal more often than chance, and no two
    share a bit (the xor of any pair has balanced bits) -- so no coordinate-step reuses
    another's bits and a partly used strip neither repeats nor skews anything."""
    W = 6000 if b == 8 else 5000
    v = _bits_table(b, d, K, W).reshape(W, -1)
    n, m = v.shape
    # each draw uniform: chi-square over 256 cells of its top 8 bits, every bit balanced
    top = v >> (b - 8)
    for k in range(m):
        counts = np.bincount(top[:, k], minlength=256)
        chi2 = np.sum((counts - n / 256) ** 2 / (n / 256))
        assert chi2 < 255 + 6.5 * np.sqrt(2 * 255), (k, chi2)
    for bit in range(b):
        ones = ((v >> bit) & 1).sum(axis=0)
        assert np.all(np.abs(ones - n / 2) < 5.5 * np.sqrt(n / 4)), bit
    # pairwise: correlation, equality rate, bit sharing
    x = (v - v.mean(axis=0)) / v.std(axis=0)
    corr = (x.T @ x) / n
    off = corr[~np.eye(m, dtype=bool)]
    assert np.abs(off).max() < 5.5 / np.sqrt(n), np.abs(off).max()
    p_eq = 2.0 ** -b
    worst_eq, worst_bit = 0, 0.0
    for k in range(m):
        eq = (v[:, k:k + 1] == v[:, k + 1:]).sum(axis=0)
        if eq.size:
            worst_eq = max(worst_eq, int(eq.max()))
        for bit in range(b):  # same-position bits of two draws agree half of the time
            agree = (((v[:, k:k + 1] ^ v[:, k + 1:]) >> bit) & 1).sum(axis=0)
            if agree.size:
                worst_bit = max(worst_bit, float(np.abs(agree - n / 2).max()))
    assert worst_eq <= stats.binom.isf(1e-9 / (m * m), n, p_eq)
    assert worst_bit < 6.0 * np.sqrt(n / 4)


def test_rounding_bits_differ_between_seeds_epochs_and_windows():
    """The same coordinate-step under another seed, epoch or window of steps draws afresh."""
    d, K, b = 5, 2, 8
    base = _bits_table(b, d, K, 400, seed=17, epoch=2).ravel()
    for other in (_bits_table(b, d, K, 400, seed=18, epoch=2).ravel(),
                  _bits_table(b, d, K, 400, seed=17, epoch=3).ravel(),
                  np.roll(_bits_table(b, d, K, 401, seed=17, epoch=2), -1, axis=0)[:400].ravel()):
        eq = np.count_nonzero(base == other)
        n = base.size
        assert abs(eq - n / 256) < 6 * np.sqrt(n / 256)
