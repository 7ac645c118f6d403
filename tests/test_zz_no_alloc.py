"""halp_full_gradient_static, the gradient pass that allocates nothing (its partial sums live
in a fixed device array inside the library), against halp_full_gradient on the same inputs:
two calls in a row per case, the second on a smaller problem, so that whatever the first call
left in the shared array must not leak into the second.  Runs last in the suite (file name)
and also passes alone in a fresh process."""
import ctypes as C

import numpy as np
import pytest
import torch

import halp_inputs as inp
import paper_1803_03383_amd as hp
from gpu_util import GpuProblem, rel_l2

pytestmark = pytest.mark.gpu


def _case(loss, N, d, K, R, seed):
    rng = np.random.default_rng(seed)
    if loss == hp.LOSS_SOFTMAX:
        X, y, _ = inp.softmax_sparse(N, d, K, seed=seed)
    elif loss == hp.LOSS_LOGISTIC:
        X, y, _ = inp.logistic(N, d, seed=seed)
    else:
        X, y, _ = inp.linreg(N, d, seed=seed, x_var="inv_d", noise=0.1)
    w0 = (0.3 * rng.standard_normal((R, K, d))).astype(np.float32)
    return X, y, w0


def _run_both(loss, N, d, K, R, seed, lam=0.0):
    X, y, w0 = _case(loss, N, d, K, R, seed)
    P = GpuProblem(X, None, y, K=K, R=R, loss=loss, lam=lam, share_data=True, w0=w0)
    P.h.full_gradient()
    want = {k: P.get(k).copy() for k in ("phi", "g", "scales")}
    # fresh outputs for the allocation-free call; same inputs
    st2 = hp.alloc_state(N, d, K=K, R=R)
    st2["w"].copy_(P.st["w"])
    for k in ("phi", "g"):
        st2[k].fill_(float("nan"))
    free_before = torch.cuda.mem_get_info()[0]
    hp.full_gradient_static(P.h.params, P.X, P.y, st2["w"], st2["phi"], st2["g"], st2["scales"],
                            ldx=P.X.shape[-1])
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before  # the call took no device memory
    got = {k: st2[k].cpu().numpy() for k in ("phi", "g", "scales")}
    assert np.all(np.isfinite(got["phi"])) and np.all(np.isfinite(got["g"]))
    for r in range(R):
        assert rel_l2(got["phi"][r], want["phi"][r]) <= 1e-5
        assert rel_l2(got["g"][r], want["g"][r]) <= 1e-5
        assert abs(got["scales"][r, 6] - want["scales"][r, 6]) <= 1e-5 * abs(want["scales"][r, 6])
    return got, want


@pytest.mark.parametrize("loss,K,big,small", [
    (hp.LOSS_SQUARED, 1, (5003, 1000, 3), (777, 50, 2)),      # row-per-wave kernel, then narrow rows
    (hp.LOSS_LOGISTIC, 1, (3001, 4096, 2), (1500, 257, 1)),   # widest rows, ragged tail
    (hp.LOSS_SOFTMAX, 10, (4001, 784, 2), (333, 100, 1)),     # matrix-core kernel
    (hp.LOSS_SOFTMAX, 16, (4101, 1024, 1), (257, 64, 3)),     # partials capped by the fixed array
])
def test_static_gradient_pass_matches_the_handle_one_twice_in_a_row(loss, K, big, small):
    for k, (N, d, R) in enumerate((big, small)):
        got, want = _run_both(loss, N, d, K, R, seed=11 + k, lam=1e-3 if k == 0 else 0.0)
        if k == 0 and loss != hp.LOSS_SOFTMAX:
            # same launch shape as the handle's pass here: the same bits
            assert np.array_equal(got["g"], want["g"]) and np.array_equal(got["phi"], want["phi"])


def test_static_gradient_pass_rejects_what_does_not_fit():
    """one workgroup per chain must fit the array; nothing is launched otherwise"""
    R, K, d, N = 300, 16, 1024, 64
    assert R * (4 * K * d + 8) > hp.STATIC_SCRATCH_BYTES
    p = hp.Params(N=N, d=d, K=K, R=R, loss=hp.LOSS_SOFTMAX, b=8, B=1, share_data=1, algorithm=hp.ALG_HALP,
                  T=1, alpha=0.1, mu=1.0, lam=0.0, delta_d=1.0, seed=0, delta=0.0)
    X = torch.zeros((N, d), device="cuda")
    y = torch.zeros((N,), dtype=torch.int32, device="cuda")
    st = hp.alloc_state(N, d, K=K, R=R)
    st["g"].fill_(7.0)
    with pytest.raises(hp.HalpError) as e:
        hp.full_gradient_static(p, X, y, st["w"], st["phi"], st["g"], st["scales"])
    assert e.value.code == hp.ERR_TOO_LARGE
    torch.cuda.synchronize()
    assert float(st["g"].min()) == 7.0
