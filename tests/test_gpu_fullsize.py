"""GPU parity at the full sizes of the benchmark configurations, in the launch
configuration bench.py times.  The oracle checks what it can compute in seconds:
whole sampled chains (config 4), the whole problem (configs 2 and 3), sampled rows
and a short run of the minibatch loop (config 5).  Inputs flow generator -> both
sides, or oracle -> GPU; never GPU -> oracle."""
import numpy as np
import pytest
import torch

import halp_inputs as inp
import paper_1803_03383_amd as hp
from oracle import ref
from gpu_util import rel_l2

pytestmark = pytest.mark.gpu
TOL = 1e-5


def test_config4_sampled_chains_full_size():
    """R=256, N=16384, d=512, b=8, T=N: data as bench.py makes it; three sampled chains are
    checked whole against the oracle (quantized data, gradient, then -- with the oracle's
    gradient handed to the GPU -- bit centering and all 16384 inner steps)."""
    R, N, d, T = 256, 16384, 512, 16384
    alpha, mu, seed = 0.1, 0.02, 0
    X, y, _ = inp.linreg_chains_device(R, N, d, seed=seed, noise=0.1)
    delta_d = float(X.abs().max().item()) / 127.0
    st = hp.alloc_state(N, d, R=R, b=8)
    Xq = torch.zeros((R, N, d), dtype=torch.int8, device="cuda")
    h = hp.Halp(N, d, R=R, b=8, T=T, alpha=alpha, mu=mu, delta_d=delta_d, seed=seed)
    h.bind(X=X, Xq=Xq, y=y, **st)
    h.quantize_data()
    rng = np.random.default_rng(1)
    w0 = (0.05 * rng.standard_normal((R, 1, d))).astype(np.float32)
    st["w"].copy_(torch.from_numpy(w0))
    h.full_gradient()
    torch.cuda.synchronize()
    sample = [0, 101, 255]
    host = {}
    for r in sample:
        Xr, yr = X[r].cpu().numpy(), y[r].cpu().numpy()
        prob = ref.make_problem(N, d, b=8, alpha=alpha, mu=mu, delta_d=delta_d, seed=seed + r)
        Xq_ref = ref.quantize_data(Xr, delta_d, 8)
        assert np.array_equal(Xq[r].cpu().numpy(), Xq_ref)
        phi_ref, g_ref, loss_ref = ref.full_gradient(prob, Xr, yr, w0[r])
        assert rel_l2(st["phi"][r].cpu().numpy(), phi_ref) <= TOL
        assert rel_l2(st["g"][r].cpu().numpy(), g_ref) <= TOL
        assert abs(st["scales"][r, 6].item() - loss_ref) <= TOL * abs(loss_ref)
        host[r] = (prob, Xq_ref, yr, phi_ref.astype(np.float32), g_ref.astype(np.float32))
        st["g"][r].copy_(torch.from_numpy(host[r][4]))  # oracle's gradient in, for exact parity
    h.recenter(5)
    h.inner_loop(5)
    torch.cuda.synchronize()
    assert h.get_stats(0).inner_variant == 2
    for r in sample:
        prob, Xq_ref, yr, phi32, g32 = host[r]
        sc, hh, _ = ref.recenter(prob, g32, 5)
        assert np.array_equal(st["scales"][r].cpu().numpy()[[0, 1, 2, 3, 4, 5, 7]], sc[[0, 1, 2, 3, 4, 5, 7]])
        assert np.array_equal(st["h"][r].cpu().numpy().astype(np.int64), hh)
        out = ref.inner_loop(prob, Xq_ref, phi32, yr, hh, sc, 5, T)
        assert np.array_equal(st["z"][r].cpu().numpy().astype(np.int32), out["z"])
        assert np.array_equal(st["w"][r].cpu().numpy(), ref.apply_offset(prob, sc, out["z"], w0[r]))
        assert np.array_equal(st["counters"][r].cpu().numpy().astype(np.uint64), out["counters"])


def test_config2_single_chain_full_size():
    """N=100000, d=1024, b=8, alpha=1e-3, T=N, one chain: the whole epoch phase by phase."""
    N, d, T = 100000, 1024, 100000
    alpha, mu, seed = 1e-3, 0.01, 3
    X, y, _ = inp.linreg_chains_device(1, N, d, seed=seed, noise=0.1)
    delta_d = float(X.abs().max().item()) / 127.0
    st = hp.alloc_state(N, d, b=8)
    Xq = torch.zeros((1, N, d), dtype=torch.int8, device="cuda")
    h = hp.Halp(N, d, b=8, T=T, alpha=alpha, mu=mu, delta_d=delta_d, seed=seed)
    h.bind(X=X, Xq=Xq, y=y, **st)
    h.quantize_data()
    h.full_gradient()
    torch.cuda.synchronize()
    Xh, yh = X[0].cpu().numpy(), y[0].cpu().numpy()
    prob = ref.make_problem(N, d, b=8, alpha=alpha, mu=mu, delta_d=delta_d, seed=seed)
    Xq_ref = ref.quantize_data(Xh, delta_d, 8)
    assert np.array_equal(Xq[0].cpu().numpy(), Xq_ref)
    phi_ref, g_ref, _ = ref.full_gradient(prob, Xh, yh, np.zeros((1, d), np.float32))
    assert rel_l2(st["phi"][0].cpu().numpy(), phi_ref) <= TOL
    assert rel_l2(st["g"][0].cpu().numpy(), g_ref) <= TOL
    st["g"][0].copy_(torch.from_numpy(g_ref.astype(np.float32)))
    h.recenter(0)
    h.inner_loop(0)
    torch.cuda.synchronize()
    sc, hh, _ = ref.recenter(prob, g_ref.astype(np.float32), 0)
    out = ref.inner_loop(prob, Xq_ref, phi_ref.astype(np.float32), yh, hh, sc, 0, T)
    assert np.array_equal(st["h"][0].cpu().numpy().astype(np.int64), hh)
    assert np.array_equal(st["z"][0].cpu().numpy().astype(np.int32), out["z"])
    assert np.array_equal(st["counters"][0].cpu().numpy().astype(np.uint64), out["counters"])


@pytest.mark.parametrize("b", [8, 16])
def test_config3_softmax_full_size(b):
    """N=60000, d=784, K=10, lambda=1e-4, alpha=1e-2: gradient pass on the whole set, then
    603 inner steps on the register-resident softmax kernel against the oracle: two refills of
    the 256-step batches of step-only draws and a ragged last window of 8 steps."""
    N, d, K, T = 60000, 784, 10, 603
    alpha, mu, lam, seed = 1e-2, 2.5, 1e-4, 4
    X, y, _ = inp.softmax_sparse(N, d, K, seed=seed)
    delta_d = inp.default_delta_d(X, b)
    Xq_ref = ref.quantize_data(X, delta_d, b)
    rng = np.random.default_rng(2)
    W0 = (0.01 * rng.standard_normal((1, K, d))).astype(np.float32)
    st = hp.alloc_state(N, d, K=K, b=b)
    st["w"].copy_(torch.from_numpy(W0))
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    Xq = torch.zeros((1, N, d), dtype=torch.int8 if b == 8 else torch.int16, device="cuda")
    h = hp.Halp(N, d, K=K, loss=hp.LOSS_SOFTMAX, b=b, T=T, alpha=alpha, mu=mu, lam=lam,
                delta_d=delta_d, seed=seed)
    h.bind(X=Xd, Xq=Xq, y=yd, **st)
    h.quantize_data()
    h.full_gradient()
    torch.cuda.synchronize()
    assert np.array_equal(Xq[0].cpu().numpy(), Xq_ref)
    prob = ref.make_problem(N, d, K=K, loss=ref.SOFTMAX, b=b, alpha=alpha, mu=mu, lam=lam,
                            delta_d=delta_d, seed=seed)
    phi_ref, g_ref, loss_ref = ref.full_gradient(prob, X, y, W0[0])
    assert rel_l2(st["phi"][0].cpu().numpy(), phi_ref) <= TOL
    assert rel_l2(st["g"][0].cpu().numpy(), g_ref) <= TOL
    assert abs(st["scales"][0, 6].item() - loss_ref) <= TOL * abs(loss_ref)
    st["g"][0].copy_(torch.from_numpy(g_ref.astype(np.float32)))
    st["phi"][0].copy_(torch.from_numpy(phi_ref.astype(np.float32)))
    h.recenter(1)
    h.inner_loop(1)
    torch.cuda.synchronize()
    assert h.get_stats(0).inner_variant == 2  # not the general kernel
    sc, hh, _ = ref.recenter(prob, g_ref.astype(np.float32), 1)
    out = ref.inner_loop(prob, Xq_ref, phi_ref.astype(np.float32), y, hh, sc, 1, T)
    assert np.array_equal(st["h"][0].cpu().numpy().astype(np.int64), hh)
    assert np.array_equal(st["z"][0].cpu().numpy().astype(np.int32), out["z"])
    assert np.array_equal(st["counters"][0].cpu().numpy().astype(np.uint64), out["counters"])


@pytest.mark.parametrize("b", [8, 16])
def test_config3_softmax_minibatch_full_size(b):
    """The data of configuration 3 with 64 rows per step (what `bench.py --workload c3batch` runs): 43
    steps of the class-wave kernel against the oracle, counters included."""
    N, d, K, B, T = 60000, 784, 10, 64, 43
    alpha, mu, lam, seed = 1e-2, 2.5, 1e-4, 4
    X, y, _ = inp.softmax_sparse(N, d, K, seed=seed)
    delta_d = inp.default_delta_d(X, b)
    Xq_ref = ref.quantize_data(X, delta_d, b)
    rng = np.random.default_rng(2)
    W0 = (0.01 * rng.standard_normal((1, K, d))).astype(np.float32)
    prob = ref.make_problem(N, d, K=K, loss=ref.SOFTMAX, b=b, B=B, alpha=alpha, mu=mu, lam=lam,
                            delta_d=delta_d, seed=seed)
    phi_ref, g_ref, _ = ref.full_gradient(prob, X, y, W0[0])
    st = hp.alloc_state(N, d, K=K, b=b)
    st["w"].copy_(torch.from_numpy(W0))
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    Xq = torch.from_numpy(Xq_ref.astype(np.int8 if b == 8 else np.int16))[None].cuda()
    h = hp.Halp(N, d, K=K, loss=hp.LOSS_SOFTMAX, b=b, B=B, T=T, alpha=alpha, mu=mu, lam=lam,
                delta_d=delta_d, seed=seed)
    h.bind(X=Xd, Xq=Xq, y=yd, **st)
    st["g"][0].copy_(torch.from_numpy(g_ref.astype(np.float32)))
    st["phi"][0].copy_(torch.from_numpy(phi_ref.astype(np.float32)))
    h.recenter(1)
    h.inner_loop(1)
    torch.cuda.synchronize()
    assert h.get_stats(0).inner_variant == 2  # not the general kernel
    sc, hh, _ = ref.recenter(prob, g_ref.astype(np.float32), 1)
    out = ref.inner_loop(prob, Xq_ref, phi_ref.astype(np.float32), y, hh, sc, 1, T)
    assert np.array_equal(st["z"][0].cpu().numpy().astype(np.int32), out["z"])
    assert np.array_equal(st["counters"][0].cpu().numpy().astype(np.uint64), out["counters"])
    h.close()


def test_config5_logistic_full_size():
    """N=1e6, d=4096 fp32 (16.4 GB), lambda=1e-5, b=16, B=64.  Gradient pass: every margin, the
    gradient and the loss against the oracle run once over the whole matrix on the host (the
    one slow test: a 16 GB download and some ten seconds of single-threaded fp64), so that row
    offsets beyond 4 GB are held to the oracle; beside it an fp64 recomputation with torch's
    matmul in row blocks as a library cross-check.  Inner loop: 48 minibatch steps against the
    oracle, counters included."""
    N, d, B, T = 1_000_000, 4096, 64, 48
    alpha, mu, lam, seed = 0.05, 0.01, 1e-5, 0
    X, y, _ = inp.logistic_device(N, d, seed=seed)
    st = hp.alloc_state(N, d, b=16)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(7)
    st["w"].normal_(0.0, 0.5, generator=gen)
    delta_d = float(X.abs().max().item()) / 32767.0
    Xq = torch.zeros((1, N, d), dtype=torch.int16, device="cuda")
    h = hp.Halp(N, d, loss=hp.LOSS_LOGISTIC, b=16, B=B, T=T, alpha=alpha, mu=mu, lam=lam,
                delta_d=delta_d, seed=seed)
    h.bind(X=X, Xq=Xq, y=y, **st)
    h.quantize_data()
    h.full_gradient()
    torch.cuda.synchronize()
    w = st["w"][0, 0]
    # sampled margins, fp64 definition on the host
    rows = np.random.default_rng(3).choice(N, size=2000, replace=False)
    rows.sort()
    Xs = X[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
    phi_s = Xs @ w.cpu().numpy().astype(np.float64)
    got = st["phi"][0, :, 0][torch.from_numpy(rows).cuda()].cpu().numpy()
    assert rel_l2(got, phi_s) <= TOL
    # gradient and loss, fp64 in row blocks
    w64 = w.double()
    g64 = torch.zeros(d, dtype=torch.float64, device="cuda")
    loss64 = torch.zeros((), dtype=torch.float64, device="cuda")
    for s in range(0, N, 50000):
        Xb = X[s:s + 50000].double()
        yb = y[s:s + 50000].double()
        a = Xb @ w64
        r = -yb / (1.0 + torch.exp(yb * a))
        g64 += Xb.T @ r
        loss64 += torch.nn.functional.softplus(-yb * a).sum()
    g64 = g64 / N + lam * w64
    loss64 = loss64 / N + 0.5 * lam * (w64 * w64).sum()
    assert rel_l2(st["g"][0, 0].cpu().numpy(), g64.cpu().numpy()) <= TOL
    assert abs(st["scales"][0, 6].item() - loss64.item()) <= TOL * abs(loss64.item())
    del Xb, yb, a, r
    # the oracle over all 1e6 rows
    X_h = X.cpu().numpy()
    y_h = y.cpu().numpy()
    prob_g = ref.make_problem(N, d, loss=ref.LOGISTIC, b=16, B=B, alpha=alpha, mu=mu, lam=lam,
                              delta_d=delta_d, seed=seed)
    phi_ref, g_ref, loss_ref = ref.full_gradient(prob_g, X_h, y_h, w.cpu().numpy().reshape(1, d))
    phi_gpu = st["phi"][0, :, 0].cpu().numpy()
    assert rel_l2(phi_gpu, phi_ref[:, 0]) <= TOL
    assert rel_l2(phi_gpu[-200000:], phi_ref[-200000:, 0]) <= TOL  # rows past the 4 GB offsets
    assert np.max(np.abs(phi_gpu - phi_ref[:, 0])) <= 1e-4 * np.max(np.abs(phi_ref))
    assert rel_l2(st["g"][0, 0].cpu().numpy(), g_ref[0]) <= TOL
    assert abs(st["scales"][0, 6].item() - loss_ref) <= TOL * abs(loss_ref)
    assert rel_l2(g64.cpu().numpy(), g_ref[0]) <= 1e-9  # the two references agree
    # minibatch inner loop: oracle on the host copy of the quantized data
    Xq_h = Xq[0].cpu().numpy()
    assert np.array_equal(Xq_h[:4096], ref.quantize_data(X_h[:4096], delta_d, 16))
    assert np.array_equal(Xq_h[-4096:], ref.quantize_data(X_h[-4096:], delta_d, 16))
    del X_h
    rng = np.random.default_rng(5)
    phi32 = rng.standard_normal(N).astype(np.float32)          # any margins will do for parity
    g32 = (1e-3 * rng.standard_normal((1, d))).astype(np.float32)
    st["phi"][0, :, 0].copy_(torch.from_numpy(phi32))
    st["g"][0].copy_(torch.from_numpy(g32))
    w_before = st["w"][0].cpu().numpy().copy()
    h.recenter(2)
    h.inner_loop(2)
    torch.cuda.synchronize()
    prob = ref.make_problem(N, d, loss=ref.LOGISTIC, b=16, B=B, alpha=alpha, mu=mu, lam=lam,
                            delta_d=delta_d, seed=seed)
    sc, hh, _ = ref.recenter(prob, g32, 2)
    out = ref.inner_loop(prob, Xq_h, phi32, y_h, hh, sc, 2, T)
    assert np.array_equal(st["h"][0].cpu().numpy().astype(np.int64), hh)
    assert np.array_equal(st["z"][0].cpu().numpy().astype(np.int32), out["z"])
    assert np.array_equal(st["w"][0].cpu().numpy(), ref.apply_offset(prob, sc, out["z"], w_before))
    assert np.array_equal(st["counters"][0].cpu().numpy().astype(np.uint64), out["counters"])
    assert h.get_stats(0).inner_variant == 2 and h.get_stats(0).n_exchange_timeouts == 0


def test_config2_shape_makes_progress_like_the_oracle():
    """Configuration 2's regime (d=1024, b=8, alpha=1e-3, T=1e5, kappa ~ 1e3: outside Theorem
    2's bit condition, so the box of bit centering clips every epoch) on a reduced N with the
    mu the benchmark uses: three whole epochs through halp_epoch.  The loss falls every epoch
    and follows the oracle's own run of the same epochs (the two differ in the last bits of
    the fp32 gradient, hence in a few roundings of h~, not in the trend)."""
    N, d, T, epochs = 20000, 1024, 100000, 3
    alpha, mu, seed = 1e-3, 0.3, 3
    X, y, _ = inp.linreg(N, d, seed=seed, x_var="inv_d", noise=0.1)
    delta_d = inp.default_delta_d(X, 8)
    Xq_ref = ref.quantize_data(X, delta_d, 8)
    st = hp.alloc_state(N, d, b=8)
    Xd, yd = torch.from_numpy(X).cuda()[None], torch.from_numpy(y).cuda()[None]
    Xq = torch.zeros((1, N, d), dtype=torch.int8, device="cuda")
    h = hp.Halp(N, d, b=8, T=T, alpha=alpha, mu=mu, delta_d=delta_d, seed=seed)
    h.bind(X=Xd, Xq=Xq, y=yd, **st)
    h.quantize_data()
    gpu_loss, gpu_clamped = [], []
    for k in range(epochs):
        h.epoch(k)
        s = h.get_stats(0)
        gpu_loss.append(s.loss); gpu_clamped.append(s.n_clamped_z)
    h.full_gradient()
    gpu_loss.append(h.get_stats(0).loss)
    assert np.array_equal(Xq[0].cpu().numpy(), Xq_ref)
    prob = ref.make_problem(N, d, b=8, alpha=alpha, mu=mu, delta_d=delta_d, seed=seed)
    w = np.zeros((1, d), np.float32)
    ref_loss, ref_clamped = [], []
    for k in range(epochs):
        out = ref.epoch(prob, X, Xq_ref, y, w, k, T)
        ref_loss.append(float(out["scales"][6])); ref_clamped.append(int(out["counters"][0]))
        w = out["w"]
    ref_loss.append(ref.full_gradient(prob, X, y, w)[2])
    assert all(b < a for a, b in zip(gpu_loss, gpu_loss[1:])), gpu_loss
    assert all(b < a for a, b in zip(ref_loss, ref_loss[1:])), ref_loss
    assert gpu_loss[-1] < 0.9 * gpu_loss[0]
    assert abs(gpu_loss[0] - ref_loss[0]) <= TOL * ref_loss[0]   # same start: the fp32 pass
    for a, b in zip(gpu_loss[1:], ref_loss[1:]):
        assert abs(a - b) <= 0.01 * b, (gpu_loss, ref_loss)
    for a, b in zip(gpu_clamped, ref_clamped):                      # the box binds on both sides
        assert a > 0 and abs(a - b) <= 0.2 * b, (gpu_clamped, ref_clamped)


def test_ten_class_ten_thousand_feature_epoch():
    """The shape of the paper's synthetic classification set (Sec. 5.2 and the appendix on
    clipping: 10 classes, 10 000 features, 7500 examples; the records themselves are not
    reproduced -- seeded stand-in data): halp_epoch runs it.  Gradient pass (the two-pass
    softmax form) against the oracle, then -- with the oracle's gradient and margins handed in
    -- bit centering and 150 inner steps on the general kernel, whose 100 000-coordinate model
    lives in device memory, bit for bit."""
    N, d, K, T, b = 7500, 10000, 10, 150, 8
    alpha, mu, lam, seed = 0.5, 0.1, 1e-4, 9
    X, y, _ = inp.softmax_sparse(N, d, K, seed=seed, zero_frac=0.5)
    delta_d = inp.default_delta_d(X, b)
    Xq_ref = ref.quantize_data(X, delta_d, b)
    rng = np.random.default_rng(4)
    W0 = (0.01 * rng.standard_normal((1, K, d))).astype(np.float32)
    st = hp.alloc_state(N, d, K=K, b=b)
    st["w"].copy_(torch.from_numpy(W0))
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    Xq = torch.zeros((1, N, d), dtype=torch.int8, device="cuda")
    h = hp.Halp(N, d, K=K, loss=hp.LOSS_SOFTMAX, b=b, T=T, alpha=alpha, mu=mu, lam=lam,
                delta_d=delta_d, seed=seed)
    h.bind(X=Xd, Xq=Xq, y=yd, **st)
    h.quantize_data()
    h.epoch(0)   # the whole outer iteration runs at this shape
    torch.cuda.synchronize()
    s0 = h.get_stats(0)
    assert s0.status == 0 and s0.inner_variant == 1 and np.isfinite(s0.loss)
    assert np.array_equal(Xq[0].cpu().numpy(), Xq_ref)
    # phase by phase against the oracle, from the same start
    st["w"].copy_(torch.from_numpy(W0))
    h.full_gradient()
    torch.cuda.synchronize()
    prob = ref.make_problem(N, d, K=K, loss=ref.SOFTMAX, b=b, alpha=alpha, mu=mu, lam=lam,
                            delta_d=delta_d, seed=seed)
    phi_ref, g_ref, loss_ref = ref.full_gradient(prob, X, y, W0[0])
    assert rel_l2(st["phi"][0].cpu().numpy(), phi_ref) <= TOL
    assert rel_l2(st["g"][0].cpu().numpy(), g_ref) <= TOL
    assert abs(st["scales"][0, 6].item() - loss_ref) <= TOL * abs(loss_ref)
    assert abs(s0.loss - loss_ref) <= TOL * abs(loss_ref)
    st["g"][0].copy_(torch.from_numpy(g_ref.astype(np.float32)))
    st["phi"][0].copy_(torch.from_numpy(phi_ref.astype(np.float32)))
    h.recenter(1)
    h.inner_loop(1)
    torch.cuda.synchronize()
    sc, hh, _ = ref.recenter(prob, g_ref.astype(np.float32), 1)
    out = ref.inner_loop(prob, Xq_ref, phi_ref.astype(np.float32), y, hh, sc, 1, T)
    assert np.array_equal(st["h"][0].cpu().numpy().astype(np.int64), hh)
    assert np.array_equal(st["z"][0].cpu().numpy().astype(np.int32), out["z"])
    assert np.array_equal(st["counters"][0].cpu().numpy().astype(np.uint64), out["counters"])
    assert np.any(out["z"] != 0)


@pytest.mark.timeout(600)
def test_softmax_gradient_pass_at_the_bench_row_count():
    """The softmax gradient pass at the row count `bench.py --workload c3grad` times (960000 rows of the
    configuration-3 recipe, 3 GB: past the last-level cache), in the launch shape of that run, against the
    oracle on every output: both forms of the products (pairs of halves, fp32)."""
    N, d, K, lam = 960000, 784, 10, 1e-4
    X, y, _ = inp.softmax_sparse(N, d, K, seed=6)
    rng = np.random.default_rng(3)
    W0 = (0.01 * rng.standard_normal((1, K, d))).astype(np.float32)
    prob = ref.make_problem(N, d, K=K, loss=ref.SOFTMAX, lam=lam)
    phi_ref, g_ref, loss_ref = ref.full_gradient(prob, X, y, W0[0])
    st = hp.alloc_state(N, d, K=K, b=8)
    st["w"].copy_(torch.from_numpy(W0))
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    h = hp.Halp(N, d, K=K, loss=hp.LOSS_SOFTMAX, b=8, T=8, alpha=1e-2, mu=2.5, lam=lam, delta_d=1.0 / 127.0,
                seed=0)
    h.bind(X=Xd, y=yd, **st)
    for fp32 in (0, 1):
        h.set_option(hp.OPT_GRADIENT_FP32, fp32)
        st["phi"].zero_(); st["g"].zero_()
        h.full_gradient()
        torch.cuda.synchronize()
        assert rel_l2(st["phi"][0].cpu().numpy(), phi_ref) <= TOL, fp32
        assert rel_l2(st["g"][0].cpu().numpy(), g_ref) <= TOL, fp32
        assert abs(st["scales"][0, 6].item() - loss_ref) <= TOL * abs(loss_ref), fp32
    h.close()

