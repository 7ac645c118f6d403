"""Seeded synthetic inputs for the HALP epoch: the only module that the CPU
oracle's tests and the HIP path's tests / benchmark both import.

It holds data recipes only -- none of the method's arithmetic (no gradient,
no quantizer, no random rounding).  The recipes have the shapes and value
distributions of the workloads this build is measured on; they stand in for
the paper's data sets (its synthetic regression of Fig. 1, MNIST-shaped
10-class logistic regression and the 10 000-feature synthetic classification
set of Sec. 5.2), none of whose records are reproduced here.

Host recipes use numpy's PCG64; the two large device recipes use torch's
device generator so that multi-gigabyte inputs never cross PCIe.
"""
import numpy as np


def linreg(N, d, seed=0, x_var="unit", noise=0.01):
    """Linear regression: rows ~ N(0, I) ('unit') or N(0, I/d) ('inv_d');
    w* ~ N(0, 1); y = X w* + N(0, noise^2)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    X = rng.standard_normal((N, d))
    if x_var == "inv_d":
        X /= np.sqrt(d)
    w_star = rng.standard_normal(d)
    y = X @ w_star + noise * rng.standard_normal(N)
    return X.astype(np.float32), y.astype(np.float32), w_star.astype(np.float32)


def logistic(N, d, seed=0, noise=0.5):
    """Binary labels in {-1,+1}: sign(X w* + N(0, noise^2)), X ~ N(0, I/d)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    X = rng.standard_normal((N, d)) / np.sqrt(d)
    w_star = rng.standard_normal(d)
    s = X @ w_star + noise * rng.standard_normal(N)
    y = np.where(s >= 0, 1.0, -1.0)
    return X.astype(np.float32), y.astype(np.float32), w_star.astype(np.float32)


def softmax_sparse(N, d, K, seed=0, zero_frac=0.8):
    """Image-shaped features in [0,1]: zero_frac exact zeros, the rest U(0,1);
    labels = argmax(X W* + Gumbel), W* ~ N(0,1)^{d x K}."""
    rng = np.random.Generator(np.random.PCG64(seed))
    X = rng.random((N, d))
    X[rng.random((N, d)) < zero_frac] = 0.0
    W_star = rng.standard_normal((d, K))
    logits = X @ W_star + rng.gumbel(size=(N, K))
    y = np.argmax(logits, axis=1)
    return X.astype(np.float32), y.astype(np.int32), W_star.T.copy().astype(np.float32)


def softmax_dense(N, d, K, seed=0, margin=4.0):
    """K-class data with dense Gaussian features, the shape of a synthetic classification set
    with many informative features: X ~ N(0, I/d), W* ~ N(0,1)^{d x K},
    labels = argmax(margin X W* + Gumbel)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    X = (rng.standard_normal((N, d)) / np.sqrt(d)).astype(np.float32)
    W_star = rng.standard_normal((d, K)).astype(np.float32)
    logits = margin * (X @ W_star) + rng.gumbel(size=(N, K))
    y = np.argmax(logits, axis=1)
    return X, y.astype(np.int32), W_star.T.copy()


def linreg_conditioned(N, d, kappa, seed=0, noise=0.01):
    """Linear regression with a prescribed spectrum (the recipe of the paper's conditioning
    study): X = U S V^T with U (N x d, orthonormal columns) and V (d x d) random orthogonal,
    from QR of Gaussian matrices, and S such that the Hessian X^T X / N of the squared loss
    has eigenvalues spaced geometrically from 1 to kappa.  w* ~ N(0,1), y = X w* + N(0, noise^2).
    Returns X, y, w* as fp32 and the eigenvalues."""
    rng = np.random.Generator(np.random.PCG64(seed))
    U, _ = np.linalg.qr(rng.standard_normal((N, d)))
    V, _ = np.linalg.qr(rng.standard_normal((d, d)))
    eig = np.geomspace(1.0, float(kappa), d) if d > 1 else np.ones(1)
    X = (U * np.sqrt(N * eig)) @ V.T
    w_star = rng.standard_normal(d)
    y = X @ w_star + noise * rng.standard_normal(N)
    return X.astype(np.float32), y.astype(np.float32), w_star.astype(np.float32), eig


def default_delta_d(X, b):
    """One scalar data scale so that max|X| maps to the largest code."""
    m = float(np.max(np.abs(X)))
    return (m if m > 0 else 1.0) / float(2 ** (b - 1) - 1)


# ---------------------------------------------------------------- device recipes


def linreg_chains_device(R, N, d, seed=0, noise=0.1, device="cuda"):
    """R independent linear-regression instances generated on the device:
    X[r] ~ N(0, I/d), w*[r] ~ N(0,1), y = X w* + N(0, noise^2).
    Returns torch tensors X [R,N,d] f32, y [R,N] f32, w_star [R,d] f32."""
    import torch

    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    X = torch.empty((R, N, d), dtype=torch.float32, device=device)
    for r in range(R):  # chain by chain: bounded temporaries
        X[r].normal_(0.0, 1.0 / float(np.sqrt(d)), generator=gen)
    w_star = torch.empty((R, d), dtype=torch.float32, device=device).normal_(generator=gen)
    y = torch.bmm(X, w_star.unsqueeze(2)).squeeze(2)
    y += noise * torch.empty_like(y).normal_(generator=gen)
    return X, y, w_star


def logistic_device(N, d, seed=0, noise=0.5, device="cuda", chunk=65536):
    """Binary logistic data generated on the device (labels -1/+1 as f32)."""
    import torch

    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    X = torch.empty((N, d), dtype=torch.float32, device=device)
    w_star = torch.empty((d,), dtype=torch.float32, device=device).normal_(generator=gen)
    y = torch.empty((N,), dtype=torch.float32, device=device)
    for s in range(0, N, chunk):
        e = min(N, s + chunk)
        X[s:e].normal_(0.0, 1.0 / float(np.sqrt(d)), generator=gen)
        m = X[s:e] @ w_star + noise * torch.empty((e - s,), device=device).normal_(generator=gen)
        y[s:e] = torch.where(m >= 0, 1.0, -1.0)
    return X, y, w_star
