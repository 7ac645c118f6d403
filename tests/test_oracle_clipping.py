"""The clipping study (paper, appendix "Clipping Discussion") on the oracle, no GPU: 16-bit HALP
given the box of 8-bit HALP ("Clip", same mu) follows the 8-bit run; given its lattice spacing
("Scale", mu chosen so that mu_16 (2^15 - 1) = mu_8 (2^7 - 1)) it has a box 258 times wider,
never saturates and follows full-precision SVRG."""
import numpy as np

import halp_inputs as inp
from oracle import ref

N, D, LAM, ALPHA, MU8, EPOCHS = 600, 64, 1e-4, 2.0, 0.1, 10
T = 2 * N


def _run(X, y, alg, b, mu):
    w = np.zeros((1, D), np.float32)
    gn, moves, clamped, deltas = [], [], 0, []
    if alg == "svrg":
        prob = ref.make_problem(N, D, loss=ref.LOGISTIC, alpha=ALPHA, lam=LAM, seed=0, algorithm=ref.ALG_SVRG)
    else:
        dd = inp.default_delta_d(X, b)
        Xq = ref.quantize_data(X, dd, b)
        prob = ref.make_problem(N, D, loss=ref.LOGISTIC, b=b, alpha=ALPHA, mu=mu, lam=LAM, delta_d=dd, seed=0)
    for k in range(EPOCHS):
        if alg == "svrg":
            out = ref.svrg_epoch(prob, X, y, w, k, T)
        else:
            out = ref.epoch(prob, X, Xq, y, w, k, T)
            clamped += int(out["counters"][0])
            moves.append(np.abs(out["w"].astype(np.float64) - w).max())
            deltas.append(out["scales"][0])
        gn.append(np.linalg.norm(out["g"]))
        w = out["w"]
    return dict(gn=np.array(gn), moves=np.array(moves), clamped=clamped, deltas=np.array(deltas))


def test_clip_follows_8_bits_and_scale_follows_svrg():
    X, y, _ = inp.logistic(N, D, seed=3)
    mu_scale = MU8 * 127.0 / 32767.0
    svrg = _run(X, y, "svrg", 0, 1.0)
    h8 = _run(X, y, "halp", 8, MU8)
    clip = _run(X, y, "halp", 16, MU8)
    scale = _run(X, y, "halp", 16, mu_scale)
    # the two definitions: same lattice spacing / same box at the first epoch (same g~)
    assert abs(scale["deltas"][0] / h8["deltas"][0] - 1) < 1e-14
    assert abs(clip["deltas"][0] * 32767 / (h8["deltas"][0] * 127) - 1) < 1e-14
    # the box binds for 8 bits and for Clip, epoch after epoch, and never for Scale
    box8 = h8["gn"] / MU8
    assert h8["clamped"] > 1000 and clip["clamped"] > 1000 and scale["clamped"] == 0
    assert np.all(h8["moves"] <= box8 * (1 + 128 / 127 * 0.01)) and np.all(h8["moves"] > 0.9 * box8)
    assert np.all(clip["moves"] <= clip["gn"] / MU8 * 1.001) and np.all(clip["moves"] > 0.9 * clip["gn"] / MU8)
    assert np.all(scale["moves"] < 0.5 * 258 * scale["gn"] / MU8)
    # trajectories: Clip mimics 8-bit HALP, Scale mimics SVRG, and the two pairs are far apart
    assert np.all(np.abs(clip["gn"] / h8["gn"] - 1) < 0.05)
    assert np.all(np.abs(scale["gn"] / svrg["gn"] - 1) < 0.15)
    assert h8["gn"][-1] > 100 * svrg["gn"][-1]
