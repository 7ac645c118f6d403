"""Algorithms 1-3 of the paper as written, in fp64 reals (numpy).

TEST INFRASTRUCTURE ONLY (part of the CPU oracle; never imported by the HIP
package).  These are the generic forms -- SVRG (Algorithm 1), LP-SVRG
(Algorithm 2) and HALP (Algorithm 3) -- over any finite sum given by two
callables, with the quantizer Q_(delta,b) of Sec. 3 "Quantization" acting on
real numbers.  They serve the mathematical pins of the integer oracle
(identity-Q HALP equals SVRG, the linear rate of Theorem 2, unbiasedness of
the linear-model form against the generic update); they are never compared
bit-wise with the GPU.

Small problems only: every inner step is a Python-level call.
"""
import numpy as np


def quantize(x, delta, b, rng):
    """Q_(delta,b): unbiased stochastic rounding onto delta * {-2^(b-1) .. 2^(b-1)-1};
    values outside the domain go to its nearest end (Sec. 3 'Quantization')."""
    x = np.asarray(x, dtype=np.float64)
    lo, hi = -(2 ** (b - 1)), 2 ** (b - 1) - 1
    q = x / delta
    down = np.floor(q)
    up_prob = q - down
    out = down + (rng.random(x.shape) < up_prob)
    return delta * np.clip(out, lo, hi)


def identity_q(x, delta, b, rng):
    return np.asarray(x, dtype=np.float64)


def svrg(grad_i, full_grad, w0, alpha, T, epochs, index_stream, option="I", option_rng=None):
    """Algorithm 1.  index_stream(k, t) -> i.  Returns the list of outer iterates."""
    w_tilde = np.array(w0, dtype=np.float64)
    outs = [w_tilde.copy()]
    for k in range(epochs):
        g = full_grad(w_tilde)
        w = w_tilde.copy()
        hist = [w.copy()]
        for t in range(T):
            i = index_stream(k, t)
            w = w - alpha * (grad_i(i, w) - grad_i(i, w_tilde) + g)
            hist.append(w.copy())
        if option == "I":
            w_tilde = w
        else:
            w_tilde = hist[option_rng.integers(0, T)]
        outs.append(w_tilde.copy())
    return outs


def lp_svrg(grad_i, full_grad, w0, alpha, T, epochs, index_stream, delta, b, rng):
    """Algorithm 2 (option I): SVRG whose iterate is stored in (delta, b)."""
    w_tilde = quantize(np.array(w0, dtype=np.float64), delta, b, rng)
    outs = [w_tilde.copy()]
    for k in range(epochs):
        g = full_grad(w_tilde)
        w = w_tilde.copy()
        for t in range(T):
            i = index_stream(k, t)
            u = w - alpha * (grad_i(i, w) - grad_i(i, w_tilde) + g)
            w = quantize(u, delta, b, rng)
        w_tilde = w
        outs.append(w_tilde.copy())
    return outs


def halp(grad_i, full_grad, w0, alpha, T, epochs, index_stream, mu, b, rng, Q=quantize,
         option="I", option_rng=None):
    """Algorithm 3.  Returns (outer iterates, list of per-epoch delta)."""
    w_tilde = np.array(w0, dtype=np.float64)
    outs, deltas = [w_tilde.copy()], []
    for k in range(epochs):
        g = full_grad(w_tilde)
        delta = np.linalg.norm(g) / (mu * (2 ** (b - 1) - 1))
        deltas.append(delta)
        if delta == 0.0:
            outs.append(w_tilde.copy())
            continue
        z = Q(np.zeros_like(w_tilde), delta, b, rng)
        hist = [z.copy()]
        for t in range(T):
            i = index_stream(k, t)
            u = z - alpha * (grad_i(i, w_tilde + z) - grad_i(i, w_tilde) + g)
            z = Q(u, delta, b, rng)
            hist.append(z.copy())
        if option == "I":
            w_tilde = w_tilde + z
        else:
            w_tilde = w_tilde + hist[option_rng.integers(0, T)]
        outs.append(w_tilde.copy())
    return outs, deltas
