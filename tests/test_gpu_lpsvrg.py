"""GPU parity of the LP-SVRG mode (Algorithm 2 in integers) against the oracle, through the
C ABI: epoch start, inner loop on every kernel that takes the mode, whole epochs."""
import numpy as np
import pytest
import torch

import halp_inputs as inp
import paper_1803_03383_amd as hp
from gpu_util import GpuProblem
from oracle import ref

pytestmark = pytest.mark.gpu


def _data(loss, N, d, K, seed):
    if loss == hp.LOSS_SOFTMAX:
        X, y, _ = inp.softmax_sparse(N, d, K, seed=seed)
    elif loss == hp.LOSS_LOGISTIC:
        X, y, _ = inp.logistic(N, d, seed=seed)
    else:
        X, y, _ = inp.linreg(N, d, seed=seed)
    return X, y


def _lp_case(loss, N, d, K, B, b, R, seed, alpha, delta):
    """Oracle-made inputs of the inner loop in LP-SVRG mode, R chains."""
    rng = np.random.default_rng(seed)
    data = [_data(loss, N, d, K, seed + r) for r in range(R)]
    Xs, ys = [x for x, _ in data], [y for _, y in data]
    dd = inp.default_delta_d(np.stack(Xs), b)
    mk = lambda r: ref.make_problem(N, d, K=K, loss=loss, b=b, B=B, alpha=alpha, delta_d=dd,
                                    seed=500 + seed + r, algorithm=ref.ALG_LPSVRG, delta=delta)
    qmax = 2 ** (b - 1) - 1
    Xqs, phis, hs, scs, ws, zs = [], [], [], [], [], []
    for r in range(R):
        W = rng.integers(-qmax // 3, qmax // 3, size=(K, d))
        w = (W * delta + 0.3 * delta * rng.uniform(-1, 1, size=(K, d))).astype(np.float32)  # off the lattice
        prob = mk(r)
        phi, g, _ = ref.full_gradient(prob, Xs[r], ys[r], w)
        s, h, z = ref.lp_begin(prob, g.astype(np.float32), w, 3)
        Xqs.append(ref.quantize_data(Xs[r], dd, b)); phis.append(phi.astype(np.float32))
        hs.append(h); scs.append(s); ws.append(w); zs.append(z)
    return dict(X=np.stack(Xs), Xq=np.stack(Xqs), y=np.stack(ys), phi=np.stack(phis), h=np.stack(hs),
                scales=np.stack(scs), w=np.stack(ws), z=np.stack(zs), dd=dd, mk=mk,
                g=None)


def _problem(case, loss, K, B, b, R, T, seed, alpha, delta):
    return GpuProblem(case["X"], case["Xq"], case["y"], K=K, R=R, loss=loss, b=b, B=B, T=T,
                      alpha=alpha, delta_d=case["dd"], seed=500 + seed, w0=case["w"],
                      algorithm=hp.ALG_LPSVRG, delta=delta)


@pytest.mark.parametrize("b,K,d,R", [(8, 1, 100, 2), (16, 1, 64, 1), (8, 4, 50, 1)])
def test_epoch_start_bit_exact(b, K, d, R):
    loss = hp.LOSS_SOFTMAX if K > 1 else hp.LOSS_SQUARED
    N, seed, alpha = 200, 7 + d, 0.02
    delta = 2.0 ** -6 if b == 8 else 2.0 ** -13
    case = _lp_case(loss, N, d, K, 1, b, R, seed, alpha, delta)
    P = _problem(case, loss, K, 1, b, R, 10, seed, alpha, delta)
    # the gradient of the oracle, so that h~ is compared on identical inputs
    g = np.stack([ref.full_gradient(case["mk"](r), case["X"][r], case["y"][r], case["w"][r])[1]
                  for r in range(R)]).astype(np.float32)
    P.put("g", g)
    P.h.recenter(3)
    sc, h, z = P.get("scales"), P.get("h"), P.get("z")
    for r in range(R):
        assert np.array_equal(sc[r][[0, 1, 2, 3, 4, 5, 7]], case["scales"][r][[0, 1, 2, 3, 4, 5, 7]])
        assert sc[r][0] == delta
        assert np.array_equal(h[r].astype(np.int64), case["h"][r])
        assert np.array_equal(z[r].astype(np.int32), case["z"][r])
    assert np.abs(case["z"]).max() > 5  # the start is w~, not 0


LP_CASES = [
    # loss, N, d, K, B, b, R, T, variants
    (hp.LOSS_SQUARED, 600, 512, 1, 1, 8, 2, 700, (2, 1)),
    (hp.LOSS_SQUARED, 400, 100, 1, 1, 8, 1, 900, (2, 1)),
    (hp.LOSS_SQUARED, 300, 256, 1, 1, 16, 1, 500, (2, 1)),
    (hp.LOSS_LOGISTIC, 500, 256, 1, 1, 8, 2, 800, (2, 1)),
    (hp.LOSS_LOGISTIC, 300, 128, 1, 1, 16, 1, 400, (2, 1)),
    (hp.LOSS_SQUARED, 300, 64, 1, 8, 8, 1, 300, (1,)),     # minibatch: general kernel
    (hp.LOSS_SOFTMAX, 300, 100, 3, 1, 8, 1, 300, (2, 1)),  # softmax: class waves, and the general kernel
    (hp.LOSS_SOFTMAX, 200, 784, 10, 1, 8, 2, 203, (2, 1)),  # the 10-class shape, ragged epoch
    (hp.LOSS_SOFTMAX, 150, 256, 15, 1, 16, 1, 150, (2, 1)),  # 15 classes at 16 bits
    (hp.LOSS_SOFTMAX, 150, 300, 16, 1, 8, 1, 150, (2, 1)),   # 16 classes: two rows of z per class wave
    (hp.LOSS_SOFTMAX, 200, 200, 5, 6, 8, 1, 60, (2, 1)),     # softmax with a minibatch
    (hp.LOSS_SOFTMAX, 120, 600, 3, 16, 16, 1, 40, (2, 1)),   # ... 16 strips per lane at 16 bits
    (hp.LOSS_SQUARED, 300, 64, 1, 100, 8, 1, 30, (2, 1)),    # a scalar margin, more than 64 rows per step
    (hp.LOSS_LOGISTIC, 200, 300, 1, 70, 16, 1, 25, (2, 1)),
]


@pytest.mark.parametrize("loss,N,d,K,B,b,R,T,variants", LP_CASES)
def test_inner_loop_bit_exact(loss, N, d, K, B, b, R, T, variants):
    seed, alpha = 11 + d + T, 0.02
    delta = 2.0 ** -7 if b == 8 else 2.0 ** -14
    case = _lp_case(loss, N, d, K, B, b, R, seed, alpha, delta)
    outs = [ref.inner_loop(case["mk"](r), case["Xq"][r], case["phi"][r], case["y"][r], case["h"][r],
                           case["scales"][r], 3, T, z0=case["z"][r]) for r in range(R)]
    assert any(not np.array_equal(o["z"], case["z"][r]) for r, o in enumerate(outs))
    # the register kernel with the library's choice of helper waves and without them
    for variant, helpers in [(v, hw) for v in variants for hw in ((0, 2) if v == 2 else (0,))]:
        P = _problem(case, loss, K, B, b, R, T, seed, alpha, delta)
        P.put("phi", case["phi"]); P.put("h", case["h"]); P.put("scales", case["scales"])
        P.put("z", case["z"])
        P.h.set_option(hp.OPT_INNER_VARIANT, variant)
        P.h.set_option(hp.OPT_INNER_HELPERS, helpers)
        P.h.inner_loop(3)
        z, w, cnt = P.get("z"), P.get("w"), P.get("counters")
        assert P.h.get_stats(0).inner_variant == variant
        for r in range(R):
            assert np.array_equal(z[r].astype(np.int32), outs[r]["z"]), (variant, r)
            w_r = ref.apply_offset(case["mk"](r), case["scales"][r], outs[r]["z"], case["w"][r])
            assert np.array_equal(w[r], w_r)
            assert np.array_equal(w[r].astype(np.float64), (delta * outs[r]["z"]).astype(np.float32))
            assert np.array_equal(cnt[r].astype(np.uint64), outs[r]["counters"])


def test_auto_takes_the_register_kernel_where_it_can():
    loss, N, d, b, T = hp.LOSS_SQUARED, 300, 128, 8, 50
    case = _lp_case(loss, N, d, 1, 1, b, 1, 3, 0.02, 2.0 ** -7)
    P = _problem(case, loss, 1, 1, b, 1, T, 3, 0.02, 2.0 ** -7)
    P.put("phi", case["phi"]); P.put("h", case["h"]); P.put("scales", case["scales"]); P.put("z", case["z"])
    P.h.inner_loop(3)
    assert P.h.get_stats(0).inner_variant == 2


def test_epochs_bit_exact_when_fp32_sums_are_exact():
    """Small-integer data, a power-of-two delta and w~ = 0 make every fp32 sum of the first
    gradient pass exact: that whole epoch must match to the bit; later ones run from its w~."""
    rng = np.random.default_rng(5)
    N, d, R = 256, 64, 2
    Xq = rng.integers(-100, 101, size=(R, N, d)).astype(np.int8)
    dd, delta = 2.0 ** -6, 2.0 ** -8
    X = (Xq * dd).astype(np.float32)
    y = (rng.integers(-64, 65, size=(R, N)) / 16.0).astype(np.float32)
    P = GpuProblem(X, Xq, y, R=R, T=2 * N, alpha=0.01, delta_d=dd, seed=21,
                   algorithm=hp.ALG_LPSVRG, delta=delta)
    P.h.epoch(0)
    for r in range(R):
        prob = ref.make_problem(N, d, alpha=0.01, delta_d=dd, seed=21 + r, algorithm=ref.ALG_LPSVRG,
                                delta=delta)
        out = ref.epoch(prob, X[r], Xq[r], y[r], np.zeros((1, d), np.float32), 0, 2 * N)
        assert np.array_equal(P.get("g")[r], out["g"])
        assert np.array_equal(P.get("h")[r].astype(np.int64), out["h"])
        assert np.array_equal(P.get("z")[r].astype(np.int32), out["z"])
        assert np.array_equal(P.get("w")[r], out["w"])
        assert np.abs(out["z"]).max() > 0


def test_runs_reach_the_floor_like_the_oracle():
    """Ten epochs on the GPU and in the oracle from the same start: the objective gaps agree
    within a factor (different fp32 gradients give different random paths, same statistics)."""
    N, d = 400, 16
    X, y, _ = inp.linreg(N, d, seed=8)
    dd = inp.default_delta_d(X, 8)
    Xq = ref.quantize_data(X, dd, 8)
    Xe = Xq.astype(np.float64) * dd
    w_star = np.linalg.lstsq(Xe, y.astype(np.float64), rcond=None)[0]
    f = lambda w: 0.5 * np.mean((Xe @ w - y) ** 2)
    delta = 2.5 * np.max(np.abs(w_star)) / 127
    P = GpuProblem(Xe.astype(np.float32), Xq, y, T=2 * N, alpha=0.02, delta_d=dd, seed=4,
                   algorithm=hp.ALG_LPSVRG, delta=delta)
    prob = ref.make_problem(N, d, alpha=0.02, delta_d=dd, seed=4, algorithm=ref.ALG_LPSVRG, delta=delta)
    w = np.zeros((1, d), np.float32)
    gg, go = [], []
    for k in range(10):
        P.h.epoch(k)
        w = ref.epoch(prob, Xe.astype(np.float32), Xq, y, w, k, 2 * N)["w"]
        gg.append(f(P.get("w")[0, 0].astype(np.float64)) - f(w_star))
        go.append(f(w[0].astype(np.float64)) - f(w_star))
    f0 = f(np.zeros(d)) - f(w_star)
    assert np.mean(gg[5:]) < 0.05 * f0 and np.mean(go[5:]) < 0.05 * f0
    assert 0.2 < np.mean(gg[5:]) / np.mean(go[5:]) < 5.0


def test_bad_parameters_are_errors():
    with pytest.raises(hp.HalpError):
        hp.Halp(100, 8, algorithm=hp.ALG_LPSVRG, delta=0.0)
    with pytest.raises(hp.HalpError):
        hp.Halp(100, 8, algorithm=hp.ALG_LPSVRG, delta=0.1, lam=1e-3)
    with pytest.raises(hp.HalpError):
        hp.Halp(100, 8, algorithm=7, delta=0.1)
