"""Per-feature data scales on the GPU (halp_set_feature_scale) against the oracle's scaled forms:
the quantizer bit for bit, the gradient pass of every kernel family within the fp32 tolerance,
and a whole epoch bit for bit where the fp32 sums are exact."""
import numpy as np
import pytest
import torch

import halp_inputs as inp
import paper_1803_03383_amd as hp
from oracle import ref
from gpu_util import GpuProblem, rel_l2

pytestmark = pytest.mark.gpu
TOL = 1e-5


def _scales(d, seed):
    rng = np.random.default_rng(seed)
    return np.exp(rng.uniform(np.log(0.02), np.log(5.0), size=d)).astype(np.float32)


@pytest.mark.parametrize("b", [8, 16])
def test_quantize_with_feature_scales_bit_exact(b):
    N, d = 333, 101
    X, y, _ = inp.linreg(N, d, seed=1, x_var="inv_d")
    s = _scales(d, 2)
    X = (X * s).astype(np.float32)
    dd = 0.2 / (2 ** (b - 1) - 1)   # some entries clamp
    P = GpuProblem(X, None, y, b=b, delta_d=dd)
    P.h.set_feature_scale(torch.from_numpy(s).cuda())
    P.h.quantize_data()
    torch.cuda.synchronize()
    got = P.Xq.cpu().numpy()[0][:, :d]
    want = ref.quantize_data_scaled(X, dd, s, b)
    assert np.array_equal(got, want)
    assert np.abs(want).max() == 2 ** (b - 1) - 1
    assert np.all(P.Xq.cpu().numpy()[0][:, d:] == 0)


@pytest.mark.parametrize("loss,N,d,K,R", [
    (hp.LOSS_SQUARED, 1000, 64, 1, 2),      # narrow rows
    (hp.LOSS_LOGISTIC, 700, 1000, 1, 1),    # a row per wave, ragged
    (hp.LOSS_SQUARED, 300, 4096, 1, 1),
    (hp.LOSS_SOFTMAX, 500, 784, 10, 1),     # matrix-core pass
    (hp.LOSS_SOFTMAX, 333, 100, 3, 2),
])
def test_full_gradient_with_feature_scales(loss, N, d, K, R):
    from test_gpu_parity import _make_data
    rng = np.random.default_rng(9)
    s = _scales(d, 4)
    Xs, ys = zip(*[_make_data(loss, N, d, K, seed=20 + r) for r in range(R)])
    X, y = (np.stack(Xs) * s).astype(np.float32), np.stack(ys)
    v0 = (rng.standard_normal((R, K, d)) * (0.3 if loss == hp.LOSS_SOFTMAX else 1.0) * s).astype(np.float32)
    P = GpuProblem(X, None, y, K=K, R=R, loss=loss, w0=v0)
    P.h.set_feature_scale(torch.from_numpy(s).cuda())
    P.h.full_gradient()
    phi, g, sc = P.get("phi"), P.get("g"), P.get("scales")
    for r in range(R):
        prob = ref.make_problem(N, d, K=K, loss=loss)
        phi_r, g_r, loss_r = ref.full_gradient_scaled(prob, X[r], y[r], v0[r], s)
        assert rel_l2(phi[r], phi_r) <= TOL
        assert rel_l2(g[r], g_r) <= TOL
        assert abs(sc[r, 6] - loss_r) <= TOL * abs(loss_r)
    # switched off again: the plain pass on the same buffers
    P.h.set_feature_scale(None)
    P.h.full_gradient()
    prob = ref.make_problem(N, d, K=K, loss=loss)
    _, g_plain, _ = ref.full_gradient(prob, X[0], y[0], v0[0])
    assert rel_l2(P.get("g")[0], g_plain) <= TOL


def test_epoch_with_power_of_two_scales_bit_exact():
    """Small-integer data, power-of-two scales and v = 0 make every fp32 sum exact: the epoch
    (scaled quantizer and pass, centering, inner loop, update of v) matches to the bit."""
    rng = np.random.default_rng(6)
    N, d, R = 256, 64, 2
    s = (2.0 ** rng.integers(-5, 3, size=d)).astype(np.float32)
    dd = 2.0 ** -6
    Q = rng.integers(-100, 101, size=(R, N, d))
    X = (Q * dd * s).astype(np.float32)
    y = (rng.integers(-64, 65, size=(R, N)) / 16.0).astype(np.float32)
    P = GpuProblem(X, None, y, R=R, T=2 * N, alpha=0.01, mu=0.3, delta_d=dd, seed=21)
    P.h.set_feature_scale(torch.from_numpy(s).cuda())
    P.h.quantize_data()
    P.h.epoch(0)
    torch.cuda.synchronize()
    assert np.array_equal(P.Xq.cpu().numpy()[:, :, :d], Q.astype(np.int8))
    for r in range(R):
        prob = ref.make_problem(N, d, alpha=0.01, mu=0.3, delta_d=dd, seed=21 + r)
        out = ref.epoch_scaled(prob, X[r], Q[r].astype(np.int8), y[r], np.zeros((1, d), np.float32), s, 0, 2 * N)
        assert np.array_equal(P.get("phi")[r], out["phi"])
        assert np.array_equal(P.get("g")[r], out["g"])
        assert np.array_equal(P.get("h")[r].astype(np.int64), out["h"])
        assert np.array_equal(P.get("z")[r].astype(np.int32), out["z"])
        assert np.array_equal(P.get("w")[r], out["w"])


def test_feature_scale_is_refused_where_it_has_no_meaning():
    X, y, _ = inp.linreg(50, 8, seed=0)
    s = torch.ones(8, device="cuda")
    P = GpuProblem(X, None, y, T=10, lam=1e-3)
    with pytest.raises(hp.HalpError) as e:
        P.h.set_feature_scale(s)
    assert e.value.code == hp.ERR_UNSUPPORTED
    P = GpuProblem(X, None, y, T=10, algorithm=hp.ALG_SVRG)
    with pytest.raises(hp.HalpError):
        P.h.set_feature_scale(s)
    P.h.set_feature_scale(None)


def test_feature_scales_rescue_small_columns_end_to_end():
    """Columns spread over three decades: with one scalar data scale the small columns quantize
    to zero and the loss stalls; with per-feature scales 8-bit HALP drives it to zero -- on the
    GPU as on the oracle."""
    N, d, T, K, b = 800, 32, 1600, 20, 8
    X0, _, ws = inp.linreg(N, d, seed=5, x_var="inv_d", noise=0.0)
    col = np.logspace(0, -3, d).astype(np.float32)
    X = (X0 * col).astype(np.float32)
    y = (X.astype(np.float64) @ (ws / col)).astype(np.float32)
    final = {}
    for mode in ("scalar", "feature"):
        if mode == "scalar":
            s, dd = np.ones(d, np.float32), inp.default_delta_d(X, b)
        else:
            s, dd = np.abs(X).max(axis=0).astype(np.float32), 1.0 / 127
        P = GpuProblem(X, None, y, b=b, T=T, alpha=0.1, mu=0.1, delta_d=dd, seed=1)
        P.h.set_feature_scale(torch.from_numpy(s).cuda())
        P.h.quantize_data()
        for k in range(K):
            P.h.epoch(k)
        P.h.full_gradient()
        loss_gpu = float(P.get("scales")[0, 6])
        prob = ref.make_problem(N, d, b=b, alpha=0.1, mu=0.1, delta_d=dd, seed=1)
        Xq = ref.quantize_data_scaled(X, dd, s, b)
        v = np.zeros((1, d), np.float32)
        for k in range(K):
            v = ref.epoch_scaled(prob, X, Xq, y, v, s, k, T)["w"]
        loss_ref = ref.full_gradient_scaled(prob, X, y, v, s)[2]
        final[mode] = (loss_gpu, loss_ref)
    assert final["scalar"][0] > 0.1 and final["scalar"][1] > 0.1
    assert abs(final["scalar"][0] / final["scalar"][1] - 1) < 0.2
    assert final["feature"][0] < 1e-8 and final["feature"][1] < 1e-8
