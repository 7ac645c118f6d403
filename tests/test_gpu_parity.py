"""GPU parity: the HIP library through its C ABI against the CPU oracle, on the
same seeded inputs.  Integer work (random streams, quantized data, h~, dot
products, gamma, the z trajectory, counters) must match bit for bit; fp32
margins / gradients / losses within rel-L2 1e-5.  Inputs of every GPU call come
from the seeded generators or from the oracle -- never the other way round."""
import numpy as np
import pytest
import torch

import halp_inputs as inp
import paper_1803_03383_amd as hp
from oracle import ref
from gpu_util import DEV, GpuProblem, rel_l2, xq_ld, xq_torch_dtype

pytestmark = pytest.mark.gpu

TOL = 1e-5  # rel-L2 for fp32 outputs of the full-gradient pass


# ------------------------------------------------------------ random streams

def test_stream_words_match_oracle():
    seed = 0x9E3779B97F4A7C15
    for purpose, epoch, n0, cnt in [(0, 0, 0, 1000), (1, 7, 4093, 777), (3, 2 ** 32 - 1, 2 ** 34 + 1, 64),
                                    (4, 3, 5, 129)]:
        got = hp.debug_stream_words(seed, purpose, epoch, n0, cnt).cpu().numpy().view(np.uint32)
        want = np.array([ref.stream_word(seed, purpose, epoch, n0 + k) for k in range(cnt)], np.uint32)
        assert np.array_equal(got, want)


@pytest.mark.parametrize("b,d,K", [(8, 64, 1), (8, 100, 3), (16, 50, 2), (16, 4096, 1)])
def test_zround_bits_match_oracle(b, d, K):
    seed, epoch = 12345, 9
    for t in (0, 1, 2, 2 ** 20 + 1):
        got = hp.debug_zround_bits(seed, epoch, t, d, b, K).cpu().numpy()
        cols = range(d) if d <= 128 else list(range(0, d, 97)) + [d - 1]
        for c in range(K):
            for j in cols:
                assert got[c, j] == ref.zround_bits(seed, epoch, t, d, b, c, j)


# ------------------------------------------------------------ data quantization

@pytest.mark.parametrize("b", [8, 16])
def test_quantize_data_bit_exact(b):
    rng = np.random.default_rng(0)
    X = rng.standard_normal((2, 301, 100)).astype(np.float32)
    X[0, 0, :5] = [0.5, 1.5, 2.5, -0.5, 1e9]  # ties and clamping
    dd = 1.0 if b == 8 else float(np.abs(X[:, 1:]).max()) / (2 ** 15 - 1)
    y = np.zeros((2, 301), np.float32)
    P = GpuProblem(X, None, y, R=2, b=b, delta_d=dd)
    P.h.quantize_data()
    torch.cuda.synchronize()
    got = P.Xq.cpu().numpy()
    want = ref.quantize_data(X, dd, b)
    assert np.array_equal(got[..., :100], want)
    assert not got[..., 100:].any()  # padding columns are zero


@pytest.mark.parametrize("b,dd", [(8, 0.25), (8, 0.0371), (16, 2.0 ** -9), (16, 1.7e-4)])
@pytest.mark.parametrize("ldx_pad", [0, 8])
def test_quantize_data_ties(b, dd, ldx_pad):
    """Half-integers of x / delta_d (exact ones when delta_d is a power of two), their fp32
    neighbours and values around the clamp; rows of 203 columns with and without extra padding."""
    N, d = 257, 203
    rng = np.random.default_rng(b + ldx_pad)
    qmax = 2 ** (b - 1) - 1
    k = rng.integers(-qmax - 3, qmax + 3, size=(N, d)).astype(np.float64)
    X = ((k + 0.5) * dd).astype(np.float32)
    X[1::3] = np.nextafter(X[1::3], np.float32(np.inf))
    X[2::3] = np.nextafter(X[2::3], np.float32(-np.inf))
    X[:, ::7] = (rng.standard_normal((N, (d + 6) // 7)) * dd * 50).astype(np.float32)
    X[0, :4] = [np.float32(1e30), np.float32(-1e30), 0.0, np.float32(dd * 0.5)]
    ldx = (d + 3) // 4 * 4 + ldx_pad
    ldxq = xq_ld(d, b) + ldx_pad
    Xt = torch.zeros((1, N, ldx), dtype=torch.float32, device=DEV)
    Xt[0, :, :d] = torch.from_numpy(X).to(DEV)
    Xq = torch.full((1, N, ldxq), 77, dtype=xq_torch_dtype(b), device=DEV)
    yt = torch.zeros((1, N), dtype=torch.float32, device=DEV)
    st = hp.alloc_state(N, d, b=b, device=DEV)
    h = hp.Halp(N, d, b=b, T=1, alpha=0.1, mu=1.0, delta_d=dd, seed=0)
    h.bind(X=Xt, Xq=Xq, y=yt, ldx=ldx, ldxq=ldxq, **st)
    h.quantize_data()
    torch.cuda.synchronize()
    got = Xq.cpu().numpy()[0]
    want = ref.quantize_data(X, dd, b)
    assert np.array_equal(got[:, :d], want)
    assert not got[:, d:].any()
    assert (np.abs(want) == qmax).any() and (np.abs(want) < qmax).any()
    h.close()


def test_read_yardstick_reads_every_word_once():
    import torch
    rng = np.random.default_rng(0)
    for n16 in (1, 255, 2048 * 256 * 8 + 12345):
        a = rng.integers(0, 2 ** 32, size=(n16, 4), dtype=np.uint64).astype(np.uint32)
        t = torch.from_numpy(a.view(np.int32)).cuda()
        out = hp.debug_read_bandwidth(t).cpu().numpy().view(np.uint32)
        want = np.bitwise_xor.reduce(a, axis=1).astype(np.uint64).sum() % 2 ** 32
        assert int(out.astype(np.uint64).sum() % 2 ** 32) == int(want)
    with pytest.raises(hp.HalpError):
        hp.debug_read_bandwidth(torch.zeros(5, dtype=torch.int32, device="cuda"))


# ------------------------------------------------------------ full gradient

FG_CASES = [
    # loss, N, d, K, R, lam
    (hp.LOSS_SQUARED, 1000, 64, 1, 1, 0.0),
    (hp.LOSS_SQUARED, 3001, 512, 1, 2, 0.0),
    (hp.LOSS_SQUARED, 777, 1000, 1, 1, 1e-3),
    (hp.LOSS_SQUARED, 301, 4096, 1, 1, 0.0),
    (hp.LOSS_SQUARED, 129, 2048, 1, 3, 0.0),
    (hp.LOSS_LOGISTIC, 2500, 1024, 1, 1, 1e-5),
    (hp.LOSS_LOGISTIC, 403, 4096, 1, 2, 1e-5),
    (hp.LOSS_LOGISTIC, 5, 7 * 4, 1, 1, 0.0),
    # narrow rows (d <= 128): several rows per wave, 4 / 8 / 16 / 32 lanes each
    (hp.LOSS_SQUARED, 1000, 64, 1, 3, 0.0),
    (hp.LOSS_SQUARED, 77, 5, 1, 2, 1e-3),
    (hp.LOSS_SQUARED, 2049, 16, 1, 1, 0.0),
    (hp.LOSS_LOGISTIC, 130, 33, 1, 2, 1e-5),
    (hp.LOSS_SQUARED, 513, 100, 1, 2, 1e-3),
    (hp.LOSS_LOGISTIC, 999, 128, 1, 1, 0.0),
    (hp.LOSS_SQUARED, 1, 128, 1, 1, 0.0),
    (hp.LOSS_SQUARED, 1, 1, 1, 1, 0.0),       # the smallest problem there is
    (hp.LOSS_LOGISTIC, 3, 2, 1, 2, 1e-3),
    (hp.LOSS_SOFTMAX, 2, 1, 2, 1, 0.0),
    (hp.LOSS_SOFTMAX, 37, 3, 16, 1, 1e-4),
    (hp.LOSS_SOFTMAX, 1500, 784, 10, 1, 1e-4),
    (hp.LOSS_SOFTMAX, 333, 100, 3, 2, 1e-4),
    (hp.LOSS_SOFTMAX, 64, 257, 16, 1, 0.0),
    # the pipelined softmax pass (d <= 800): several periods per workgroup, ragged last tile,
    # a row that is not a whole number of 16-byte pieces, waves without columns, its widest row
    (hp.LOSS_SOFTMAX, 20011, 784, 10, 1, 1e-4),
    (hp.LOSS_SOFTMAX, 9000, 799, 7, 2, 0.0),
    (hp.LOSS_SOFTMAX, 5000, 800, 16, 1, 1e-4),
    (hp.LOSS_SOFTMAX, 4100, 33, 4, 3, 0.0),
    (hp.LOSS_SOFTMAX, 17, 96, 2, 1, 0.0),
    (hp.LOSS_SOFTMAX, 1, 4, 2, 1, 0.0),           # one row, one float4: a single tile, one column group
    (hp.LOSS_SOFTMAX, 16, 12, 3, 2, 0.0),         # exactly one tile
    (hp.LOSS_SOFTMAX, 33, 800, 10, 2, 1e-4),      # the widest rows of the pipelined form, three tiles
    (hp.LOSS_SOFTMAX, 4099, 36, 16, 1, 1e-3),     # more workgroups than tiles per workgroup, 16 classes
    # rows wider than a wave holds (K = 1: the row cut across the waves of a workgroup)
    (hp.LOSS_SQUARED, 403, 4097, 1, 1, 0.0),
    (hp.LOSS_LOGISTIC, 301, 5000, 1, 2, 1e-5),
    (hp.LOSS_SQUARED, 257, 10000, 1, 1, 1e-3),
    (hp.LOSS_LOGISTIC, 130, 16384, 1, 1, 0.0),
    # softmax on rows wider than a tile on chip: two passes
    (hp.LOSS_SOFTMAX, 333, 1025, 3, 2, 1e-4),
    (hp.LOSS_SOFTMAX, 260, 4097, 16, 1, 0.0),
    (hp.LOSS_SOFTMAX, 1001, 5000, 10, 1, 1e-4),
    (hp.LOSS_SOFTMAX, 515, 10000, 10, 1, 1e-4),
    # beyond it, the form with a quarter of the columns per wave
    (hp.LOSS_SOFTMAX, 700, 801, 10, 1, 1e-4),
    (hp.LOSS_SOFTMAX, 300, 1024, 16, 2, 0.0),
]


def _make_data(loss, N, d, K, seed):
    if loss == hp.LOSS_SQUARED:
        X, y, _ = inp.linreg(N, d, seed=seed, x_var="inv_d", noise=0.1)
    elif loss == hp.LOSS_LOGISTIC:
        X, y, _ = inp.logistic(N, d, seed=seed)
    else:
        X, y, _ = inp.softmax_sparse(N, d, K, seed=seed)
    return X, y


@pytest.mark.parametrize("loss,N,d,K,R,lam", FG_CASES)
def test_full_gradient_matches_oracle(loss, N, d, K, R, lam):
    rng = np.random.default_rng(7)
    Xs, ys = zip(*[_make_data(loss, N, d, K, seed=10 + r) for r in range(R)])
    X, y = np.stack(Xs), np.stack(ys)
    w0 = (rng.standard_normal((R, K, d)) * (1.0 if loss != hp.LOSS_SOFTMAX else 0.3)).astype(np.float32)
    P = GpuProblem(X, None, y, K=K, R=R, loss=loss, lam=lam, w0=w0)
    P.h.full_gradient()
    phi, g, sc = P.get("phi"), P.get("g"), P.get("scales")
    for r in range(R):
        prob = ref.make_problem(N, d, K=K, loss=loss, lam=lam)
        phi_r, g_r, loss_r = ref.full_gradient(prob, X[r], y[r], w0[r])
        assert rel_l2(phi[r], phi_r) <= TOL
        assert rel_l2(g[r], g_r) <= TOL
        assert abs(sc[r, 6] - loss_r) <= TOL * abs(loss_r)
    # a second run gives the same bits (fixed-order reduction, no atomics)
    P.h.full_gradient()
    assert np.array_equal(P.get("g"), g) and np.array_equal(P.get("phi"), phi)


# The softmax pass on rows of whole float4s up to 800 coordinates multiplies on the matrix cores'
# 16-bit path, every fp32 operand as the sum of two halves.  X is scaled into the halves' range
# where its largest magnitude lies outside [2^-3, 2^15): every branch of that choice, the fp32
# products it replaces, and what the pair of halves costs in accuracy.
@pytest.mark.parametrize("N,d,K,R", [(1500, 784, 10, 1), (700, 100, 3, 2), (333, 800, 16, 1)])
@pytest.mark.parametrize("xscale", [1.0, 2.0 ** -14, 3.0e-2, 4.1e4, 7.0e8])
def test_softmax_gradient_in_halves_over_data_ranges(N, d, K, R, xscale):
    rng = np.random.default_rng(5)
    Xs, ys = zip(*[_make_data(hp.LOSS_SOFTMAX, N, d, K, seed=30 + r) for r in range(R)])
    X, y = (np.stack(Xs) * np.float32(xscale)).astype(np.float32), np.stack(ys)
    w0 = (rng.standard_normal((R, K, d)) * 0.3 / xscale).astype(np.float32)
    P = GpuProblem(X, None, y, K=K, R=R, loss=hp.LOSS_SOFTMAX, lam=1e-4, w0=w0)
    err = {}
    for fp32 in (0, 1):
        P.h.set_option(hp.OPT_GRADIENT_FP32, fp32)
        P.h.full_gradient()
        phi, g, sc = P.get("phi"), P.get("g"), P.get("scales")
        e = []
        for r in range(R):
            prob = ref.make_problem(N, d, K=K, loss=hp.LOSS_SOFTMAX, lam=1e-4)
            phi_r, g_r, loss_r = ref.full_gradient(prob, X[r], y[r], w0[r])
            e.append((rel_l2(phi[r], phi_r), rel_l2(g[r], g_r)))
            assert e[-1][0] <= TOL and e[-1][1] <= TOL
            assert abs(sc[r, 6] - loss_r) <= TOL * abs(loss_r)
        err[fp32] = np.max(np.array(e), axis=0)
    # two halves carry 22 of the 24 bits: the pass keeps the accuracy of fp32 products
    assert np.all(err[0] <= 2.0 * err[1] + 1e-6), (err[0], err[1])


def test_softmax_gradient_in_halves_follows_a_new_bind():
    N, d, K = 900, 784, 10
    X, y = _make_data(hp.LOSS_SOFTMAX, N, d, K, seed=41)
    rng = np.random.default_rng(6)
    w0 = (rng.standard_normal((1, K, d)) * 0.3).astype(np.float32)
    P = GpuProblem(X, None, y, K=K, loss=hp.LOSS_SOFTMAX, w0=w0)
    P.h.full_gradient()
    g1 = P.get("g")
    # all-zero data, then data 2^20 times larger: each bound anew, each with its own largest |X|
    prob = ref.make_problem(N, d, K=K, loss=hp.LOSS_SOFTMAX)
    for factor in (0.0, 2.0 ** 20):
        P.X.copy_(torch.from_numpy(np.ascontiguousarray(X * np.float32(factor)))[None])
        P.st["w"].copy_(torch.from_numpy(w0 / (factor if factor else 1.0)).reshape(P.st["w"].shape))
        P.h.bind(X=P.X, Xq=P.Xq, y=P.y, ldx=d, ldxq=P.Xq.shape[-1], **P.st)
        P.h.full_gradient()
        phi_r, g_r, loss_r = ref.full_gradient(prob, (X * np.float32(factor)).astype(np.float32), y,
                                               (w0[0] / (factor if factor else 1.0)).astype(np.float32))
        assert np.all(np.isfinite(P.get("g")))
        assert rel_l2(P.get("phi")[0], phi_r) <= TOL and rel_l2(P.get("g")[0], g_r) <= TOL
    assert np.all(np.isfinite(g1))


def test_full_gradient_shared_data_and_block_counts():
    X, y = _make_data(hp.LOSS_SQUARED, 2000, 512, 1, seed=3)
    rng = np.random.default_rng(1)
    w0 = rng.standard_normal((3, 1, 512)).astype(np.float32)
    P = GpuProblem(X, None, y, R=3, share_data=True, w0=w0)
    outs = []
    for blocks in (0, 1, 7, 64):
        P.h.set_option(hp.OPT_FULLGRAD_BLOCKS, blocks)
        P.h.full_gradient()
        outs.append(P.get("g"))
    prob = ref.make_problem(2000, 512)
    for r in range(3):
        _, g_r, _ = ref.full_gradient(prob, X, y, w0[r])
        for g in outs:
            assert rel_l2(g[r], g_r) <= TOL


# ------------------------------------------------------------ bit centering

@pytest.mark.parametrize("b,K,d,R", [(8, 1, 64, 1), (8, 10, 784, 1), (16, 1, 4096, 2), (16, 3, 50, 2),
                                     (8, 1, 5000, 1)])
def test_recenter_bit_exact(b, K, d, R):
    rng = np.random.default_rng(b + d)
    g = (rng.standard_normal((R, K, d)) * 10.0 ** rng.uniform(-6, 1)).astype(np.float32)
    X = np.zeros((R, 4, d), np.float32)
    loss = hp.LOSS_SOFTMAX if K > 1 else hp.LOSS_SQUARED
    yz = np.zeros((R, 4), np.int32 if K > 1 else np.float32)
    P = GpuProblem(X, None, yz, K=K, R=R, loss=loss, b=b, alpha=0.037, mu=2.5, delta_d=0.0123, seed=77)
    P.put("g", g)
    P.st["z"].fill_(5)
    P.h.recenter(11)
    sc, h, z = P.get("scales"), P.get("h"), P.get("z")
    for r in range(R):
        prob = ref.make_problem(4, d, K=K, loss=loss, b=b, alpha=0.037, mu=2.5, delta_d=0.0123,
                                seed=77 + r)
        s_r, h_r, _ = ref.recenter(prob, g[r], 11)
        for k in (0, 1, 2, 3, 4, 5, 7):
            assert sc[r, k] == s_r[k], (k, sc[r, k], s_r[k])
        assert np.array_equal(h[r].astype(np.int64), h_r)
        assert not z[r].any()


def test_recenter_flags_zero_and_nonfinite_gradients():
    X = np.zeros((3, 4, 16), np.float32)
    P = GpuProblem(X, None, np.zeros((3, 4), np.float32), R=3, T=5)
    g = np.zeros((3, 1, 16), np.float32)
    g[1, 0, 3] = np.inf
    g[2, 0, 0] = 1.0
    P.put("g", g)
    P.h.recenter(0)
    sc = P.get("scales")
    assert sc[0, 7] == 1.0 and sc[1, 7] == -1.0 and sc[2, 7] == 0.0
    assert not P.get("h")[:2].any()
    # flagged chains are left alone by the inner loop
    w_before = P.get("w").copy()
    P.h.inner_loop(0)
    assert np.array_equal(P.get("w")[:2], w_before[:2])
    st = P.h.get_stats(0)
    assert st.status == 1
    assert P.h.get_stats(1).status == -1


# ------------------------------------------------------------ inner loop

def _inner_case(loss, N, d, K, B, b, lam, R, T, seed, alpha=0.02, mu=0.5):
    """Oracle-made inputs of the inner loop for R chains."""
    Xqs, phis, hs, scs, ws = [], [], [], [], []
    rng = np.random.default_rng(seed)
    data = [_make_data(loss, N, d, K, seed=seed + r) for r in range(R)]
    Xs, ys = [x for x, _ in data], [y for _, y in data]
    dd = inp.default_delta_d(np.stack(Xs), b)  # one data scale for all chains
    for r in range(R):
        X, y = Xs[r], ys[r]
        Xq = ref.quantize_data(X, dd, b)
        w = (0.1 * rng.standard_normal((K, d))).astype(np.float32)
        prob = ref.make_problem(N, d, K=K, loss=loss, b=b, B=B, alpha=alpha, mu=mu, lam=lam,
                                delta_d=dd, seed=1000 + seed + r)
        phi, g, _ = ref.full_gradient(prob, X, y, w)
        s, h, _ = ref.recenter(prob, g.astype(np.float32), 3)
        Xqs.append(Xq); phis.append(phi.astype(np.float32))
        hs.append(h); scs.append(s); ws.append(w)
    return dict(X=np.stack(Xs), Xq=np.stack(Xqs), y=np.stack(ys), phi=np.stack(phis),
                h=np.stack(hs), scales=np.stack(scs), w=np.stack(ws), dd=dd,
                mk=lambda r: ref.make_problem(N, d, K=K, loss=loss, b=b, B=B, alpha=alpha, mu=mu,
                                              lam=lam, delta_d=dd, seed=1000 + seed + r))


def _run_inner(case, loss, K, B, b, lam, R, T, seed, variant, alpha=0.02, mu=0.5, trace=0):
    N, d = case["X"].shape[1:]
    P = GpuProblem(case["X"], case["Xq"], case["y"], K=K, R=R, loss=loss, b=b, B=B, T=T, alpha=alpha,
                   mu=mu, lam=lam, delta_d=case["dd"], seed=1000 + seed, w0=case["w"])
    P.put("phi", case["phi"]); P.put("h", case["h"]); P.put("scales", case["scales"])
    P.st["z"].zero_()
    P.h.set_option(hp.OPT_INNER_VARIANT, variant)
    return P


INNER_REG_CASES = [
    # loss, N, d, b, lam, R, T, mu
    (hp.LOSS_SQUARED, 1000, 64, 8, 0.0, 1, 2000, 0.5),      # one partly filled wave
    (hp.LOSS_SQUARED, 700, 512, 8, 0.0, 3, 1003, 0.05),     # one full wave, T not a multiple of 8
    (hp.LOSS_SQUARED, 600, 1024, 8, 0.0, 2, 700, 0.02),     # two waves
    (hp.LOSS_SQUARED, 300, 100, 8, 1e-2, 1, 900, 0.5),      # ragged last group, L2 draws
    (hp.LOSS_SQUARED, 200, 4096, 8, 0.0, 1, 300, 0.01),     # four waves, two groups per lane
    (hp.LOSS_LOGISTIC, 900, 512, 8, 1e-3, 2, 1500, 0.05),
    (hp.LOSS_LOGISTIC, 500, 256, 16, 1e-4, 2, 800, 0.05),
    (hp.LOSS_SQUARED, 400, 50, 16, 0.0, 1, 1000, 0.5),      # ragged, 16 bits
    (hp.LOSS_SQUARED, 300, 2048, 16, 0.0, 1, 300, 0.02),
    (hp.LOSS_SQUARED, 50, 64, 8, 0.0, 1, 1, 0.5),           # a single step
    (hp.LOSS_SQUARED, 50, 64, 8, 0.0, 1, 0, 0.5),           # no step at all
    (hp.LOSS_SQUARED, 64, 64, 8, 0.0, 1, 600, 500.0),       # box far too small: z saturates
    (hp.LOSS_SQUARED, 1, 1, 8, 0.0, 1, 50, 0.5),            # one example, one feature
    (hp.LOSS_LOGISTIC, 3, 2, 16, 1e-3, 2, 77, 0.5),
    (hp.LOSS_LOGISTIC, 300, 128, 16, 1e-4, 2, 600, 500.0),  # the same at 16 bits ("Clip")
]


# (kernel variant, waves per chain): the register-resident kernel in every launch shape, then
# the generic kernel; the result must not depend on the choice
# With two or four waves per chain and at most two strips per lane the library puts a helper
# wave beside every chain wave (third entry 0: its choice, which is "yes" for these few chains);
# 2 switches the helpers off, so that the plain several-wave kernel stays covered.
KERNELS = [(2, 0, 0), (2, 1, 0), (2, 2, 0), (2, 4, 0), (2, 2, 2), (2, 4, 2), (2, 16, 0), (1, 0, 0)]


@pytest.mark.parametrize("variant,waves,helpers", KERNELS)
@pytest.mark.parametrize("loss,N,d,b,lam,R,T,mu", INNER_REG_CASES)
def test_inner_loop_bit_exact(loss, N, d, b, lam, R, T, mu, variant, waves, helpers):
    seed = 40 + d + T
    case = _inner_case(loss, N, d, 1, 1, b, lam, R, T, seed, mu=mu)
    P = _run_inner(case, loss, 1, 1, b, lam, R, T, seed, variant, mu=mu)
    P.h.set_option(hp.OPT_INNER_WAVES, waves)
    P.h.set_option(hp.OPT_INNER_HELPERS, helpers)
    P.h.inner_loop(3)
    z, w, cnt = P.get("z"), P.get("w"), P.get("counters")
    assert P.h.get_stats(0).inner_variant == variant
    for r in range(R):
        out = _oracle_inner(case, r, T)
        assert np.array_equal(z[r].astype(np.int32), out["z"]), f"chain {r}"
        w_r = ref.apply_offset(case["mk"](r), case["scales"][r], out["z"], case["w"][r])
        assert np.array_equal(w[r], w_r)
        assert np.array_equal(cnt[r].astype(np.uint64), out["counters"])
    if mu > 100:
        assert cnt[0, 0] > 0  # the saturating case really saturates


@pytest.mark.parametrize("T", [0, 1, 2, 7, 8, 15, 16, 17, 31, 33, 255, 256, 257, 513])
@pytest.mark.parametrize("loss,d,b,lam,waves", [
    (hp.LOSS_SQUARED, 512, 8, 0.0, 4),      # one strip per lane, four chain waves
    (hp.LOSS_SQUARED, 1000, 8, 5e-2, 4),    # two strips per lane, ragged, frequent L2 draws
    (hp.LOSS_LOGISTIC, 200, 8, 1e-3, 2),    # two chain waves, the second partly filled
    (hp.LOSS_LOGISTIC, 300, 16, 0.0, 2),    # 16 bits, two strips per lane
])
def test_inner_loop_with_helper_waves_every_epoch_length(loss, d, b, lam, waves, T):
    """The form with helper waves hands records over two steps ahead, requests rows 16 steps
    ahead and refills the step-indexed draws every 256 steps: epoch lengths around each of
    those spans, forced on (option 1) so that no other kernel can stand in."""
    N, R = 150, 2
    seed = 900 + d + T
    case = _inner_case(loss, N, d, 1, 1, b, lam, R, T, seed, mu=0.2)
    P = _run_inner(case, loss, 1, 1, b, lam, R, T, seed, 2, mu=0.2)
    P.h.set_option(hp.OPT_INNER_WAVES, waves)
    P.h.set_option(hp.OPT_INNER_HELPERS, 1)
    P.h.inner_loop(3)
    z, w, cnt = P.get("z"), P.get("w"), P.get("counters")
    for r in range(R):
        out = _oracle_inner(case, r, T)
        assert np.array_equal(z[r].astype(np.int32), out["z"]), f"chain {r}"
        assert np.array_equal(w[r], ref.apply_offset(case["mk"](r), case["scales"][r], out["z"], case["w"][r]))
        assert np.array_equal(cnt[r].astype(np.uint64), out["counters"])
    for bad in (-1, 4):
        with pytest.raises(hp.HalpError) as e:
            P.h.set_option(hp.OPT_INNER_HELPERS, bad)
        assert e.value.code == hp.ERR_INVALID


LONE_CASES = [c for c in INNER_REG_CASES if c[3] == 8 and c[2] <= 1024] + [
    # loss, N, d, b, lam, R, T, mu
    (hp.LOSS_SQUARED, 300, 1000, 8, 5e-2, 2, 400, 0.2),     # eight strips per lane, ragged, frequent L2 draws
    (hp.LOSS_LOGISTIC, 200, 130, 8, 1e-3, 1, 300, 0.2),     # two strips per lane, ragged last lane
    (hp.LOSS_LOGISTIC, 300, 257, 8, 5e-2, 2, 333, 500.0),   # odd width, saturating, L2 draws
    (hp.LOSS_SQUARED, 100, 1024, 8, 0.0, 1, 100, 500.0),    # every lane full, saturating
]


@pytest.mark.parametrize("loss,N,d,b,lam,R,T,mu", LONE_CASES)
def test_inner_loop_one_chain_wave_bit_exact(loss, N, d, b, lam, R, T, mu):
    """The 8-bit form with a single chain wave (packed 16-bit halves) and helper waves on the
    other SIMDs, forced on (option 3) so that no other kernel can stand in: 2, 4 and 8 strips
    per lane, ragged rows, L2 draws, saturation."""
    seed = 40 + d + T
    case = _inner_case(loss, N, d, 1, 1, b, lam, R, T, seed, mu=mu)
    P = _run_inner(case, loss, 1, 1, b, lam, R, T, seed, 2, mu=mu)
    P.h.set_option(hp.OPT_INNER_HELPERS, 3)
    P.h.inner_loop(3)
    z, w, cnt = P.get("z"), P.get("w"), P.get("counters")
    assert P.h.get_stats(0).inner_variant == 2
    for r in range(R):
        out = _oracle_inner(case, r, T)
        assert np.array_equal(z[r].astype(np.int32), out["z"]), f"chain {r}"
        w_r = ref.apply_offset(case["mk"](r), case["scales"][r], out["z"], case["w"][r])
        assert np.array_equal(w[r], w_r)
        assert np.array_equal(cnt[r].astype(np.uint64), out["counters"])
    if mu > 100:
        assert cnt[0, 0] > 0


@pytest.mark.parametrize("T", [0, 1, 2, 7, 8, 9, 15, 16, 17, 23, 24, 25, 33, 255, 256, 257, 263, 264, 513])
@pytest.mark.parametrize("loss,d,lam", [
    (hp.LOSS_SQUARED, 512, 0.0),      # four strips per lane
    (hp.LOSS_SQUARED, 1000, 5e-2),    # eight, ragged, frequent L2 draws
    (hp.LOSS_LOGISTIC, 200, 1e-3),    # two
])
def test_inner_loop_one_chain_wave_every_epoch_length(loss, d, lam, T):
    """Records are handed over a window of 8 steps ahead, rows are requested three windows
    ahead and the step-indexed draws are refilled every 256 steps: epoch lengths around each
    of those spans."""
    N, R = 150, 2
    seed = 700 + d + T
    case = _inner_case(loss, N, d, 1, 1, 8, lam, R, T, seed, mu=0.2)
    P = _run_inner(case, loss, 1, 1, 8, lam, R, T, seed, 2, mu=0.2)
    P.h.set_option(hp.OPT_INNER_HELPERS, 3)
    P.h.inner_loop(3)
    z, w, cnt = P.get("z"), P.get("w"), P.get("counters")
    for r in range(R):
        out = _oracle_inner(case, r, T)
        assert np.array_equal(z[r].astype(np.int32), out["z"]), f"chain {r}"
        assert np.array_equal(w[r], ref.apply_offset(case["mk"](r), case["scales"][r], out["z"], case["w"][r]))
        assert np.array_equal(cnt[r].astype(np.uint64), out["counters"])


def test_one_chain_wave_form_is_refused_where_it_does_not_exist():
    # 16 bits, and rows of more than 1024 coordinates: forcing the form is an error, not a wrong answer
    for d, b in ((256, 16), (2048, 8)):
        case = _inner_case(hp.LOSS_SQUARED, 100, d, 1, 1, b, 0.0, 1, 20, 5, mu=0.2)
        P = _run_inner(case, hp.LOSS_SQUARED, 1, 1, b, 0.0, 1, 20, 5, 2, mu=0.2)
        P.h.set_option(hp.OPT_INNER_HELPERS, 3)
        with pytest.raises(hp.HalpError) as e:
            P.h.inner_loop(3)
        assert e.value.code == hp.ERR_UNSUPPORTED


@pytest.mark.parametrize("loss,N,d,b,lam,R,T,mu", [c for c in INNER_REG_CASES if c[3] == 8 and c[2] <= 1024])
def test_inner_loop_packed_form_bit_exact(loss, N, d, b, lam, R, T, mu):
    """The 8-bit form on packed 16-bit halves (the library's choice only when chains are many),
    forced on the same cases: one wave per chain, 1 to 8 strips per lane, L2 draws, saturation."""
    seed = 40 + d + T
    case = _inner_case(loss, N, d, 1, 1, b, lam, R, T, seed, mu=mu)
    P = _run_inner(case, loss, 1, 1, b, lam, R, T, seed, 2, mu=mu)
    P.h.set_option(hp.OPT_INNER_WAVES, 1)
    P.h.set_option(hp.OPT_INNER_PACKED, 1)
    P.h.inner_loop(3)
    z, w, cnt = P.get("z"), P.get("w"), P.get("counters")
    for r in range(R):
        out = _oracle_inner(case, r, T)
        assert np.array_equal(z[r].astype(np.int32), out["z"]), f"chain {r}"
        assert np.array_equal(w[r], ref.apply_offset(case["mk"](r), case["scales"][r], out["z"], case["w"][r]))
        assert np.array_equal(cnt[r].astype(np.uint64), out["counters"])
    if mu > 100:
        assert cnt[0, 0] > 0
    for bad in (-1, 3):
        with pytest.raises(hp.HalpError) as e:
            P.h.set_option(hp.OPT_INNER_PACKED, bad)
        assert e.value.code == hp.ERR_INVALID


@pytest.mark.parametrize("d", [200, 500])
def test_more_chains_than_cus_on_the_one_chain_wave_form(d):
    """Between one and two chains per CU the library still takes the form with one chain wave, in a
    build that fits a CU twice (at most 128 registers): 400 chains over shared data, forced, agree
    with the form that has a helper beside every chain wave, and sampled chains match the oracle."""
    N, b, T, R, seed = 128, 8, 83, 400, 91
    X, y, _ = inp.linreg(N, d, seed=6, x_var="inv_d")
    dd = inp.default_delta_d(X, b)
    Xq = ref.quantize_data(X, dd, b)
    rng = np.random.default_rng(3)
    w1 = (0.05 * rng.standard_normal((1, d))).astype(np.float32)
    probs = [ref.make_problem(N, d, b=b, alpha=0.02, mu=0.05, delta_d=dd, seed=seed + r) for r in range(R)]
    phi, g, _ = ref.full_gradient(probs[0], X, y, w1)
    phi, g = phi.astype(np.float32), g.astype(np.float32)
    rec = [ref.recenter(pr, g, 1) for pr in probs]
    res = []
    for helpers in (3, 1):
        P = GpuProblem(X, Xq, y, R=R, b=b, T=T, alpha=0.02, mu=0.05, delta_d=dd, seed=seed, share_data=True,
                       w0=np.repeat(w1[None], R, axis=0))
        P.put("phi", np.repeat(phi.reshape(1, -1), R, axis=0))
        P.put("h", np.stack([h for _, h, _ in rec]))
        P.put("scales", np.stack([s for s, _, _ in rec]))
        P.st["z"].zero_()
        P.h.set_option(hp.OPT_INNER_HELPERS, helpers)
        P.h.inner_loop(1)
        res.append({k: P.get(k).copy() for k in ("z", "w", "counters")})
    a, c = res
    assert np.array_equal(a["z"], c["z"]) and np.array_equal(a["w"], c["w"])
    assert np.array_equal(a["counters"], c["counters"])
    for r in (0, 255, 256, 399):
        s_ref, h_ref, _ = rec[r]
        out = ref.inner_loop(probs[r], Xq, phi, y, h_ref, s_ref, 1, T)
        assert np.array_equal(a["z"][r].astype(np.int32), out["z"]), f"chain {r}"
        assert np.array_equal(a["counters"][r].astype(np.uint64), out["counters"])


def test_many_chains_take_the_packed_form_by_themselves():
    """2048 chains over shared data (every SIMD holds two): the default launch and the one with
    the packed form switched off agree bit for bit, and sampled chains match the oracle."""
    N, d, b, T, R, seed = 256, 512, 8, 203, 2048, 77
    X, y, _ = inp.linreg(N, d, seed=5, x_var="inv_d")
    dd = inp.default_delta_d(X, b)
    Xq = ref.quantize_data(X, dd, b)
    rng = np.random.default_rng(2)
    w1 = (0.05 * rng.standard_normal((1, d))).astype(np.float32)
    probs = [ref.make_problem(N, d, b=b, alpha=0.02, mu=0.05, delta_d=dd, seed=seed + r) for r in range(R)]
    phi, g, _ = ref.full_gradient(probs[0], X, y, w1)   # the same for every chain
    phi, g = phi.astype(np.float32), g.astype(np.float32)
    rec = [ref.recenter(pr, g, 1) for pr in probs]       # h~ differs: its rounding is the chain's
    res = []
    for packed in (0, 2):
        P = GpuProblem(X, Xq, y, R=R, b=b, T=T, alpha=0.02, mu=0.05, delta_d=dd, seed=seed, share_data=True,
                       w0=np.repeat(w1[None], R, axis=0))
        P.put("phi", np.repeat(phi.reshape(1, -1), R, axis=0))
        P.put("h", np.stack([h for _, h, _ in rec]))
        P.put("scales", np.stack([s for s, _, _ in rec]))
        P.st["z"].zero_()
        P.h.set_option(hp.OPT_INNER_PACKED, packed)
        P.h.inner_loop(1)
        res.append({k: P.get(k).copy() for k in ("z", "w", "counters")})
    a, c = res
    assert np.array_equal(a["z"], c["z"]) and np.array_equal(a["w"], c["w"])
    assert np.array_equal(a["counters"], c["counters"])
    for r in (0, 1, 1023, 2047):
        s_ref, h_ref, _ = rec[r]
        out = ref.inner_loop(probs[r], Xq, phi, y, h_ref, s_ref, 1, T)
        assert np.array_equal(a["z"][r].astype(np.int32), out["z"]), f"chain {r}"
        assert np.array_equal(a["counters"][r].astype(np.uint64), out["counters"])
    assert len({a["z"][r].tobytes() for r in (0, 1, 1023, 2047)}) == 4   # the chains do differ


_ORACLE_CACHE = {}


def _oracle_inner(case, r, T):
    """the oracle's inner loop for chain r of a case (cached: the same case runs on several kernels)"""
    key = (id(case["Xq"]), r, T)
    prob = case["mk"](r)
    key = (prob.N, prob.d, prob.b, prob.B, prob.loss, prob.seed, prob.mu, prob.lam, T)
    if key not in _ORACLE_CACHE:
        _ORACLE_CACHE[key] = ref.inner_loop(prob, case["Xq"][r], case["phi"][r], case["y"][r],
                                            case["h"][r], case["scales"][r], 3, T)
    return _ORACLE_CACHE[key]


SOFTMAX_REG_CASES = [
    # N, d, K, b, lam, R, T, mu
    (400, 784, 10, 8, 1e-4, 2, 303, 0.05),    # the 10-class shape: 8 strips per lane, ragged wave
    (300, 100, 3, 8, 1e-2, 2, 1000, 0.05),    # one strip per lane, few classes, L2 draws
    (300, 256, 15, 16, 1e-3, 1, 203, 0.05),   # 15 classes at 16 bits
    (200, 1024, 12, 8, 0.0, 1, 150, 0.05),    # every lane full
    (250, 200, 5, 16, 0.0, 1, 520, 0.05),     # crosses two batches of draws
    (100, 64, 2, 8, 0.0, 1, 1, 0.05),         # a single step
    (100, 64, 2, 8, 0.0, 1, 0, 0.05),         # no step at all
    (2, 1, 2, 8, 0.0, 1, 40, 0.05),           # two examples, one feature
    (5, 3, 15, 16, 1e-2, 1, 33, 0.05),
    (64, 64, 4, 8, 0.0, 1, 600, 500.0),       # box far too small: z saturates
    (128, 96, 3, 16, 1e-3, 1, 400, 500.0),    # the same at 16 bits
    (300, 784, 10, 16, 1e-4, 1, 203, 0.05),   # the 10-class shape at 16 bits: 16 strips per lane, 49 lanes
    (200, 781, 4, 16, 1e-2, 2, 150, 0.05),    # the same with a ragged last lane, L2 draws
    (150, 1008, 2, 16, 0.0, 1, 120, 500.0),   # 63 lanes, saturating
    (300, 784, 16, 8, 1e-3, 2, 303, 0.05),    # 16 classes: two rows of z per class wave, 8 strips per lane
    (200, 512, 16, 16, 1e-2, 1, 270, 0.05),   # ... at 16 bits, 8 strips per lane, L2 draws
    (150, 100, 16, 8, 0.0, 1, 520, 0.05),     # ... one strip per lane, two batches of draws
    (100, 250, 16, 16, 0.0, 1, 33, 500.0),    # ... four strips per lane, saturating
    (60, 7, 16, 8, 1e-2, 1, 9, 0.05),         # ... a row inside one lane
]


@pytest.mark.parametrize("variant", [2, 1])
@pytest.mark.parametrize("N,d,K,b,lam,R,T,mu", SOFTMAX_REG_CASES)
def test_inner_loop_softmax_bit_exact(N, d, K, b, lam, R, T, mu, variant):
    loss = hp.LOSS_SOFTMAX
    seed = 70 + d + T
    case = _inner_case(loss, N, d, K, 1, b, lam, R, T, seed, mu=mu)
    P = _run_inner(case, loss, K, 1, b, lam, R, T, seed, variant, mu=mu)
    P.h.inner_loop(3)
    z, w, cnt = P.get("z"), P.get("w"), P.get("counters")
    assert P.h.get_stats(0).inner_variant == variant
    for r in range(R):
        prob = case["mk"](r)
        out = ref.inner_loop(prob, case["Xq"][r], case["phi"][r], case["y"][r], case["h"][r],
                             case["scales"][r], 3, T)
        assert np.array_equal(z[r].astype(np.int32), out["z"]), f"chain {r}"
        assert np.array_equal(w[r], ref.apply_offset(prob, case["scales"][r], out["z"], case["w"][r]))
        assert np.array_equal(cnt[r].astype(np.uint64), out["counters"])
    if mu > 100:
        assert cnt[0, 0] > 0


SOFTMAX_BATCH_CASES = [
    # N, d, K, B, b, lam, R, T, mu
    (400, 784, 10, 8, 8, 1e-4, 2, 60, 0.05),      # the 10-class shape, 12-wave build
    (300, 100, 3, 64, 8, 1e-2, 1, 100, 0.05),     # the widest minibatch, few lanes on the row, L2 draws
    (300, 256, 15, 5, 16, 1e-3, 1, 50, 0.05),     # 15 classes at 16 bits: 16 waves
    (200, 1024, 7, 4, 8, 0.0, 1, 40, 0.05),       # every lane full, 8-wave build
    (300, 784, 10, 16, 16, 1e-4, 1, 30, 0.05),    # 16 strips per lane at 16 bits
    (150, 1008, 2, 3, 16, 0.0, 1, 33, 500.0),     # ... saturating
    (200, 781, 4, 6, 16, 1e-2, 2, 25, 0.05),      # ragged last lane
    (100, 64, 2, 2, 8, 0.0, 1, 1, 0.05),          # a single step
    (100, 64, 2, 2, 8, 0.0, 1, 0, 0.05),          # no step at all
    (60, 7, 12, 64, 8, 1e-2, 1, 9, 0.05),         # a row inside one lane
    (64, 64, 4, 32, 8, 0.0, 1, 200, 500.0),       # box far too small: z saturates
    (2, 1, 2, 2, 8, 0.0, 1, 40, 0.05),            # two examples, one feature
    (300, 100, 3, 65, 8, 1e-2, 1, 30, 0.05),      # more rows than LDS holds at a time: 64 + 1
    (200, 784, 10, 130, 8, 1e-4, 1, 12, 0.05),    # ... three chunks, the last of two rows
    (150, 256, 5, 512, 16, 1e-3, 1, 6, 0.05),     # ... the widest minibatch, 16 bits
    (120, 64, 4, 200, 8, 0.0, 1, 20, 500.0),      # ... saturating
    (200, 300, 16, 7, 8, 1e-3, 1, 40, 0.05),      # 16 classes: sixteen class waves and no other
    (150, 512, 16, 64, 16, 0.0, 1, 10, 0.05),     # ... at 16 bits, 1024 (row, class) pairs per step
    (100, 96, 16, 70, 8, 1e-2, 1, 15, 0.05),      # ... in two chunks
]


@pytest.mark.parametrize("variant", [2, 0, 1])
@pytest.mark.parametrize("N,d,K,B,b,lam,R,T,mu", SOFTMAX_BATCH_CASES)
def test_inner_loop_softmax_minibatch_bit_exact(N, d, K, B, b, lam, R, T, mu, variant):
    loss = hp.LOSS_SOFTMAX
    seed = 90 + d + T + B
    case = _inner_case(loss, N, d, K, B, b, lam, R, T, seed, mu=mu)
    P = _run_inner(case, loss, K, B, b, lam, R, T, seed, variant, mu=mu)
    P.h.inner_loop(3)
    z, w, cnt = P.get("z"), P.get("w"), P.get("counters")
    assert P.h.get_stats(0).inner_variant == (1 if variant == 1 else 2)
    for r in range(R):
        prob = case["mk"](r)
        out = ref.inner_loop(prob, case["Xq"][r], case["phi"][r], case["y"][r], case["h"][r],
                             case["scales"][r], 3, T)
        assert np.array_equal(z[r].astype(np.int32), out["z"]), f"chain {r}"
        assert np.array_equal(w[r], ref.apply_offset(prob, case["scales"][r], out["z"], case["w"][r]))
        assert np.array_equal(cnt[r].astype(np.uint64), out["counters"])
    if mu > 100:
        assert cnt[0, 0] > 0


def test_softmax_minibatch_shapes_outside_the_register_kernel_fall_back():
    # rows of more than 512 strips (8 bits) do not fit a class wave at 8 strips per lane
    for K, B in ((3, 4), (16, 100)):
        loss, N, d, b, T = hp.LOSS_SOFTMAX, 150, 1100, 8, 12
        case = _inner_case(loss, N, d, K, B, b, 0.0, 1, T, 55, mu=0.05)
        P = _run_inner(case, loss, K, B, b, 0.0, 1, T, 55, 0, mu=0.05)
        P.h.inner_loop(3)
        assert P.h.get_stats(0).inner_variant == 1
        prob = case["mk"](0)
        out = ref.inner_loop(prob, case["Xq"][0], case["phi"][0], case["y"][0], case["h"][0],
                             case["scales"][0], 3, T)
        assert np.array_equal(P.get("z")[0].astype(np.int32), out["z"])
        P.h.set_option(hp.OPT_INNER_VARIANT, 2)
        with pytest.raises(hp.HalpError) as e:
            P.h.inner_loop(3)
        assert e.value.code == hp.ERR_UNSUPPORTED


def test_softmax_shapes_outside_the_register_kernel_fall_back():
    # 1600 coordinates at 16 bits need more than 16 strips per lane: the automatic choice is the
    # general kernel, and forcing the register kernel is an error, not a wrong answer
    loss, N, d, K, b, T = hp.LOSS_SOFTMAX, 120, 1600, 3, 16, 40
    case = _inner_case(loss, N, d, K, 1, b, 0.0, 1, T, 77, mu=0.05)
    P = _run_inner(case, loss, K, 1, b, 0.0, 1, T, 77, 0, mu=0.05)
    P.h.inner_loop(3)
    assert P.h.get_stats(0).inner_variant == 1
    out = ref.inner_loop(case["mk"](0), case["Xq"][0], case["phi"][0], case["y"][0], case["h"][0],
                         case["scales"][0], 3, T)
    assert np.array_equal(P.get("z")[0].astype(np.int32), out["z"])
    P.h.set_option(hp.OPT_INNER_VARIANT, 2)
    with pytest.raises(hp.HalpError):
        P.h.inner_loop(3)


BATCH_CASES = [
    # loss, N, d, B, b, lam, R, T
    (hp.LOSS_SQUARED, 400, 64, 64, 8, 0.0, 2, 200),        # one worker wave, 4-byte fragments
    (hp.LOSS_SQUARED, 300, 1000, 7, 8, 1e-2, 1, 303),      # ragged row, odd batch, L2 draws
    (hp.LOSS_LOGISTIC, 500, 256, 8, 16, 1e-5, 1, 300),
    (hp.LOSS_LOGISTIC, 300, 4096, 64, 16, 1e-5, 1, 40),    # the C5 shape: 8 worker waves, 16-byte fragments
    (hp.LOSS_SQUARED, 200, 2048, 33, 16, 0.0, 2, 100),
    (hp.LOSS_LOGISTIC, 200, 3000, 64, 16, 0.0, 1, 30),     # full-step form on six workgroups, ragged last slice
    (hp.LOSS_SQUARED, 120, 4096, 64, 8, 1e-3, 1, 25),      # ... on eight, 8-byte fragments, L2 draws
    (hp.LOSS_SQUARED, 150, 512, 40, 16, 0.0, 3, 60),       # ... one workgroup per chain, rows dealt 16-16-8
    (hp.LOSS_SQUARED, 200, 512, 2, 8, 0.0, 1, 1),
    (hp.LOSS_LOGISTIC, 1, 1, 64, 16, 0.0, 1, 20),          # every row of the batch is the only example
    (hp.LOSS_SQUARED, 5, 3, 3, 8, 1e-2, 2, 25),
    (hp.LOSS_SQUARED, 64, 64, 16, 8, 0.0, 1, 300),         # box far too small (mu below): z saturates
]


# (kernel variant, workgroups per chain of the register kernel: 0 = the library's choice)
BATCH_KERNELS = [(2, 0), (2, 1), (2, 2), (2, 4), (2, 8), (1, 0)]


@pytest.mark.parametrize("variant,parts", BATCH_KERNELS)
@pytest.mark.parametrize("loss,N,d,B,b,lam,R,T", BATCH_CASES)
def test_inner_loop_minibatch_bit_exact(loss, N, d, B, b, lam, R, T, variant, parts):
    seed = 60 + d + B
    mu = 500.0 if (N, d, B) == (64, 64, 16) else 0.05
    case = _inner_case(loss, N, d, 1, B, b, lam, R, T, seed, mu=mu)
    P = _run_inner(case, loss, 1, B, b, lam, R, T, seed, variant, mu=mu)
    P.h.set_option(hp.OPT_INNER_PARTS, parts)
    P.h.inner_loop(3)
    z, w, cnt = P.get("z"), P.get("w"), P.get("counters")
    assert P.h.get_stats(0).inner_variant == variant
    for r in range(R):
        out = _oracle_inner(case, r, T)
        assert np.array_equal(z[r].astype(np.int32), out["z"]), f"chain {r}"
        w_r = ref.apply_offset(case["mk"](r), case["scales"][r], out["z"], case["w"][r])
        assert np.array_equal(w[r], w_r)
        assert np.array_equal(cnt[r].astype(np.uint64), out["counters"])
    if mu > 100:
        assert cnt[0, 0] > 0


WIDE_BATCH_CASES = [
    # loss, N, d, B, b, lam, R, T, mu: more than 64 rows per step with a scalar margin
    (hp.LOSS_SQUARED, 400, 64, 65, 8, 0.0, 2, 40, 0.05),
    (hp.LOSS_SQUARED, 300, 1000, 100, 8, 1e-2, 1, 25, 0.05),   # ragged row, L2 draws
    (hp.LOSS_LOGISTIC, 500, 256, 512, 16, 1e-5, 1, 8, 0.05),   # the widest minibatch
    (hp.LOSS_LOGISTIC, 200, 1024, 130, 16, 0.0, 1, 12, 0.05),  # 16 strips per lane
    (hp.LOSS_SQUARED, 64, 64, 200, 8, 0.0, 1, 60, 500.0),      # box far too small: z saturates
]


@pytest.mark.parametrize("variant", [2, 0, 1])
@pytest.mark.parametrize("loss,N,d,B,b,lam,R,T,mu", WIDE_BATCH_CASES)
def test_inner_loop_wide_minibatch_bit_exact(loss, N, d, B, b, lam, R, T, mu, variant):
    seed = 40 + d + B
    case = _inner_case(loss, N, d, 1, B, b, lam, R, T, seed, mu=mu)
    P = _run_inner(case, loss, 1, B, b, lam, R, T, seed, variant, mu=mu)
    P.h.inner_loop(3)
    z, w, cnt = P.get("z"), P.get("w"), P.get("counters")
    assert P.h.get_stats(0).inner_variant == (1 if variant == 1 else 2)
    for r in range(R):
        out = _oracle_inner(case, r, T)
        assert np.array_equal(z[r].astype(np.int32), out["z"]), f"chain {r}"
        w_r = ref.apply_offset(case["mk"](r), case["scales"][r], out["z"], case["w"][r])
        assert np.array_equal(w[r], w_r)
        assert np.array_equal(cnt[r].astype(np.uint64), out["counters"])
    if mu > 100:
        assert cnt[0, 0] > 0


def test_wide_minibatch_on_rows_too_wide_for_a_class_wave_falls_back():
    loss, N, d, B, b, T = hp.LOSS_LOGISTIC, 150, 4096, 96, 16, 6
    case = _inner_case(loss, N, d, 1, B, b, 0.0, 1, T, 21, mu=0.05)
    P = _run_inner(case, loss, 1, B, b, 0.0, 1, T, 21, 0, mu=0.05)
    P.h.inner_loop(3)
    assert P.h.get_stats(0).inner_variant == 1
    assert np.array_equal(P.get("z")[0].astype(np.int32), _oracle_inner(case, 0, T)["z"])


GENERIC_CASES = [
    # loss, N, d, K, B, b, lam, R, T
    (hp.LOSS_SOFTMAX, 400, 784, 10, 1, 8, 1e-4, 1, 300),
    (hp.LOSS_SOFTMAX, 300, 100, 3, 2, 16, 1e-3, 2, 400),
    (hp.LOSS_LOGISTIC, 500, 256, 1, 8, 16, 1e-5, 1, 300),
    (hp.LOSS_SQUARED, 400, 64, 1, 64, 8, 0.0, 2, 200),
    (hp.LOSS_LOGISTIC, 300, 4096, 1, 64, 16, 1e-5, 1, 40),
]


@pytest.mark.parametrize("loss,N,d,K,B,b,lam,R,T", GENERIC_CASES)
def test_inner_loop_generic_trace_bit_exact(loss, N, d, K, B, b, lam, R, T):
    seed = 90 + d + B
    case = _inner_case(loss, N, d, K, B, b, lam, R, T, seed, mu=0.05)
    P = _run_inner(case, loss, K, B, b, lam, R, T, seed, 0, mu=0.05)
    M = min(T, 50)
    tr = dict(idx=torch.zeros((R, M, B), dtype=torch.int64, device="cuda"),
              D=torch.zeros((R, M, B, K), dtype=torch.int64, device="cuda"),
              beta=torch.zeros((R, M, B, K), dtype=torch.float64, device="cuda"),
              gamma=torch.zeros((R, M, B, K), dtype=torch.int32, device="cuda"),
              ztraj=torch.zeros((R, M, K, d), dtype=torch.int32, device="cuda"))
    P.h.inner_loop_trace(3, M, **tr)
    z, w, cnt = P.get("z"), P.get("w"), P.get("counters")
    for r in range(R):
        out = ref.inner_loop(case["mk"](r), case["Xq"][r], case["phi"][r], case["y"][r],
                             case["h"][r], case["scales"][r], 3, T, trace_steps=M)
        assert np.array_equal(tr["idx"][r].cpu().numpy(), out["idx"])
        assert np.array_equal(tr["D"][r].cpu().numpy(), out["D"])
        bg, bo = tr["beta"][r].cpu().numpy(), out["beta"]
        assert np.all(np.abs(bg - bo) <= 1e-12 * np.abs(bo).max() + 1e-9 * np.abs(bo))
        assert np.array_equal(tr["gamma"][r].cpu().numpy(), out["gamma"])
        assert np.array_equal(tr["ztraj"][r].cpu().numpy(), out["ztraj"])
        assert np.array_equal(z[r].astype(np.int32), out["z"])
        assert np.array_equal(w[r], ref.apply_offset(case["mk"](r), case["scales"][r], out["z"],
                                                     case["w"][r]))
        assert np.array_equal(cnt[r].astype(np.uint64), out["counters"])


# ------------------------------------------------------------ whole epochs

def test_epoch_bit_exact_when_fp32_sums_are_exact():
    """Small-integer data and w~ = 0 make every fp32 sum of the gradient pass exact,
    so one whole epoch (gradient, centering, inner loop, update) must match to the bit."""
    rng = np.random.default_rng(5)
    N, d, R = 256, 64, 2
    Xq = rng.integers(-100, 101, size=(R, N, d)).astype(np.int8)
    dd = 2.0 ** -6
    X = (Xq * dd).astype(np.float32)
    y = (rng.integers(-64, 65, size=(R, N)) / 16.0).astype(np.float32)
    P = GpuProblem(X, Xq, y, R=R, T=2 * N, alpha=0.01, mu=0.3, delta_d=dd, seed=21)
    P.h.epoch(0)
    for r in range(R):
        prob = ref.make_problem(N, d, alpha=0.01, mu=0.3, delta_d=dd, seed=21 + r)
        out = ref.epoch(prob, X[r], Xq[r], y[r], np.zeros((1, d), np.float32), 0, 2 * N)
        assert np.array_equal(P.get("phi")[r], out["phi"])
        assert np.array_equal(P.get("g")[r], out["g"])
        assert np.array_equal(P.get("scales")[r][[0, 1, 2, 3, 4, 5, 7]], out["scales"][[0, 1, 2, 3, 4, 5, 7]])
        assert np.array_equal(P.get("h")[r].astype(np.int64), out["h"])
        assert np.array_equal(P.get("z")[r].astype(np.int32), out["z"])
        assert np.array_equal(P.get("w")[r], out["w"])


def test_epochs_converge_like_the_oracle():
    """Config-1-shaped run (N=1000, d=64, b=8, mu=1, alpha=0.01, T=2N, 10 epochs): the GPU and
    the oracle contract the distance to the least-squares solution at the same rate."""
    N, d = 1000, 64
    X, y, _ = inp.linreg(N, d, seed=0, x_var="unit", noise=0.01)
    dd = inp.default_delta_d(X, 8)
    Xq = ref.quantize_data(X, dd, 8)
    w_star = np.linalg.lstsq(X.astype(np.float64), y.astype(np.float64), rcond=None)[0]
    P = GpuProblem(X, None, y, T=2 * N, alpha=0.01, mu=1.0, delta_d=dd, seed=0)
    P.h.quantize_data()
    prob = ref.make_problem(N, d, alpha=0.01, mu=1.0, delta_d=dd, seed=0)
    w_ref = np.zeros((1, d), np.float32)
    d_gpu, d_ref = [], []
    for k in range(10):
        P.h.epoch(k)
        w_ref = ref.epoch(prob, X, Xq, y, w_ref, k, 2 * N)["w"]
        d_gpu.append(np.linalg.norm(P.get("w")[0, 0] - w_star))
        d_ref.append(np.linalg.norm(w_ref[0] - w_star))
    d0 = np.linalg.norm(w_star)
    assert d_gpu[-1] < 0.05 * d0 and d_ref[-1] < 0.05 * d0
    ratio = np.array(d_gpu) / np.array(d_ref)
    assert np.all(ratio < 3) and np.all(ratio > 1 / 3)


def test_missing_buffers_and_bad_calls_are_errors():
    X = np.zeros((1, 8, 16), np.float32)
    P = GpuProblem(X, None, np.zeros((1, 8), np.float32))
    h2 = hp.Halp(8, 16)
    with pytest.raises(hp.HalpError) as e:
        h2.epoch(0)
    assert e.value.code == hp.ERR_NOT_BOUND
    with pytest.raises(hp.HalpError) as e:
        P.h.epoch(-1)
    assert e.value.code == hp.ERR_INVALID
    with pytest.raises(hp.HalpError) as e:
        P.h.bind(X=P.X[:, :, 1:], ldx=16, **P.st)  # misaligned base pointer
    assert e.value.code == hp.ERR_ALIGN


def test_minibatch_exchange_wait_is_bounded_and_reported():
    """Several workgroups per chain wait for each other's sums; told never to wait, the launch
    must still end, report it in counters[3], and leave the handle usable."""
    loss, N, d, B, b, T = hp.LOSS_LOGISTIC, 300, 4096, 64, 16, 40
    seed = 60 + d + B
    case = _inner_case(loss, N, d, 1, B, b, 1e-5, 1, T, seed, mu=0.05)
    P = _run_inner(case, loss, 1, B, b, 1e-5, 1, T, seed, 2, mu=0.05)
    P.h.set_option(hp.OPT_INNER_PARTS, 4)
    P.h.set_option(hp.OPT_EXCHANGE_SPIN_LIMIT, -1)
    w_before = P.get("w").copy()
    P.h.inner_loop(3)
    assert int(P.get("counters")[0, 3]) == 1
    # the model is left as it was, the status says why, and the statistics call reports it
    assert np.array_equal(P.get("w"), w_before)
    assert P.get("scales")[0, 7] == -2.0
    with pytest.raises(hp.HalpError) as e:
        P.h.get_stats(0)
    assert e.value.code == hp.ERR_EXCHANGE_TIMEOUT
    assert e.value.stats.status == -2 and e.value.stats.n_exchange_timeouts == 1
    P.st["scales"][0, 7] = 0.0  # what the next halp_recenter would do
    # with the default limit the same handle gives the oracle's result again
    P.h.set_option(hp.OPT_EXCHANGE_SPIN_LIMIT, 1 << 20)
    P.put("w", case["w"]); P.st["z"].zero_()
    P.h.inner_loop(3)
    out = _oracle_inner(case, 0, T)
    assert np.array_equal(P.get("z")[0].astype(np.int32), out["z"])
    assert int(P.get("counters")[0, 3]) == 0
    assert np.array_equal(P.get("w")[0], ref.apply_offset(case["mk"](0), case["scales"][0], out["z"], case["w"][0]))
    assert P.h.get_stats(0).n_exchange_timeouts == 0
    with pytest.raises(hp.HalpError):
        P.h.set_option(hp.OPT_EXCHANGE_SPIN_LIMIT, -2)


def test_epoch_refuses_a_shape_no_inner_kernel_covers_before_launching_anything():
    """A step of 600 rows fits no inner-loop kernel (the general one stops at 512): halp_epoch
    says so before the gradient pass or the re-scaling have written anything."""
    N, d, K, B = 700, 20, 3, 600
    X, y, _ = inp.softmax_sparse(N, d, K, seed=4)
    P = GpuProblem(X, ref.quantize_data(X, 1 / 127, 8), y, K=K, loss=hp.LOSS_SOFTMAX, B=B, T=5,
                   delta_d=1 / 127, w0=np.full((1, K, d), 0.25, np.float32))
    P.st["g"].fill_(7.0); P.st["h"].fill_(3); P.st["scales"].fill_(5.0)
    with pytest.raises(hp.HalpError) as e:
        P.h.epoch(0)
    assert e.value.code == hp.ERR_UNSUPPORTED
    assert float(P.get("g").min()) == 7.0 and int(P.get("h").min()) == 3
    assert float(P.get("scales").min()) == 5.0 and float(P.get("w").max()) == 0.25
    P.h.full_gradient()  # the gradient pass alone still covers the shape
    assert float(P.get("g").max()) != 7.0


def test_general_inner_loop_with_the_model_in_device_memory():
    """K d = 20 000 coordinates of z and h~ do not fit LDS as 32-bit integers: the general kernel
    keeps them in its device-memory workspace.  Softmax, minibatch of 3, L2 draws; bit-exact."""
    loss, N, d, K, B, b, lam, T = hp.LOSS_SOFTMAX, 150, 2000, 10, 3, 8, 1e-2, 60
    seed = 77
    case = _inner_case(loss, N, d, K, B, b, lam, 2, T, seed, mu=0.05)
    P = _run_inner(case, loss, K, B, b, lam, 2, T, seed, 1, mu=0.05)
    P.h.inner_loop(3)
    assert P.h.get_stats(0).inner_variant == 1
    for r in range(2):
        out = _oracle_inner(case, r, T)
        assert np.array_equal(P.get("z")[r].astype(np.int32), out["z"])
        assert np.array_equal(P.get("counters")[r].astype(np.uint64), out["counters"])
        assert np.array_equal(P.get("w")[r], ref.apply_offset(case["mk"](r), case["scales"][r], out["z"], case["w"][r]))


def test_step_latency_probe_runs_and_is_deterministic():
    """The latency micro-kernel of the bench line: same output on every run and for every grid
    position (all workgroups run the same chain on lane constants)."""
    import torch
    outs = [hp.debug_step_latency(w, 64, 3).cpu().numpy() for w in (4, 4, 2, 1)]
    assert np.array_equal(outs[0], outs[1])
    for o, w in zip(outs[1:], (4, 2, 1)):
        o = o.reshape(3, w * 64)
        assert np.array_equal(o[0], o[1]) and np.array_equal(o[0], o[2])
    with pytest.raises(ValueError):
        hp.debug_step_latency(4, 64, 3, out=torch.empty(10, dtype=torch.int32, device="cuda"))


@pytest.mark.parametrize("d,waves,helpers", [(64, 1, 0), (512, 4, 2), (512, 4, 1), (2048, 4, 0)])
@pytest.mark.parametrize("alpha_lam", [0.45, 0.7])
def test_sixteen_bit_update_at_the_edge_of_32_bits(d, waves, helpers, alpha_lam):
    """The register kernels keep the 16-bit update -gamma x + r - (h~ mod 2^16) - c_lambda z in
    32 bits, the oracle in 64.  Every term at its largest at once: data quantized to +-32767,
    a box so small that z sits at its ends and gamma at its clamp, and alpha lambda 2^16 near
    q_max (0.45: c_lambda ~ 29491 on every step) or beyond it (0.7: clamped to 32767)."""
    N, T, b, seed = 40, 300, 16, 5
    rng = np.random.default_rng(seed + d)
    X = rng.choice(np.array([-1.0, 1.0], np.float32), size=(N, d))
    y = (X @ rng.standard_normal(d).astype(np.float32) * 50.0).astype(np.float32)
    dd = 1.0 / 32767.0
    Xq = ref.quantize_data(X, dd, b)
    assert np.abs(Xq).min() == 32767
    alpha, lam, mu = 0.5, alpha_lam / 0.5, 2000.0
    prob = ref.make_problem(N, d, b=b, alpha=alpha, mu=mu, lam=lam, delta_d=dd, seed=seed)
    w = (rng.standard_normal((1, d)) * 3.0).astype(np.float32)
    phi, g, _ = ref.full_gradient(prob, X, y, w)
    sc, h, _ = ref.recenter(prob, g.astype(np.float32), 3)
    tr = ref.inner_loop(prob, Xq, phi.astype(np.float32), y, h, sc, 3, T, trace_steps=T)
    out = ref.inner_loop(prob, Xq, phi.astype(np.float32), y, h, sc, 3, T)
    assert np.abs(out["z"]).max() == 32768 and out["counters"][0] > 0   # z at the ends of its box
    assert out["counters"][1] > 0                                        # gamma clamped
    assert out["counters"][2] == T                                       # an L2 draw on every step
    assert np.abs(tr["gamma"]).max() >= 32767
    P = GpuProblem(X, Xq, y, b=b, T=T, alpha=alpha, mu=mu, lam=lam, delta_d=dd, seed=seed, w0=w)
    P.put("phi", phi.astype(np.float32)); P.put("h", h); P.put("scales", sc)
    P.st["z"].zero_()
    P.h.set_option(hp.OPT_INNER_VARIANT, 2)
    P.h.set_option(hp.OPT_INNER_WAVES, waves)
    P.h.set_option(hp.OPT_INNER_HELPERS, helpers)
    P.h.inner_loop(3)
    assert np.array_equal(P.get("z")[0].astype(np.int32), out["z"])
    assert np.array_equal(P.get("counters")[0].astype(np.uint64), out["counters"])


@pytest.mark.parametrize("delay", [0, 16, 64])
def test_minibatch_result_does_not_depend_on_the_poll_delay(delay):
    """A chain cut across sixteen workgroups (margins and labels shipped from part 0 with the
    tagged sums): the same bits whether the first poll of a step's exchange comes at once or late."""
    loss, N, d, B, b, T = hp.LOSS_LOGISTIC, 300, 4096, 64, 16, 40
    seed = 60 + d + B
    case = _inner_case(loss, N, d, 1, B, b, 1e-5, 1, T, seed, mu=0.05)
    P = _run_inner(case, loss, 1, B, b, 1e-5, 1, T, seed, 2, mu=0.05)
    P.h.set_option(hp.OPT_EXCHANGE_POLL_DELAY, delay)
    P.h.inner_loop(3)
    out = _oracle_inner(case, 0, T)
    assert np.array_equal(P.get("z")[0].astype(np.int32), out["z"])
    assert np.array_equal(P.get("counters")[0].astype(np.uint64), out["counters"])
    for bad in (-1, 65):
        with pytest.raises(hp.HalpError) as e:
            P.h.set_option(hp.OPT_EXCHANGE_POLL_DELAY, bad)
        assert e.value.code == hp.ERR_INVALID
