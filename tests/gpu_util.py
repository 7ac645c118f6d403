"""Shared plumbing of the GPU parity tests: build a handle over torch tensors
and move oracle-made inputs to the device.  Inputs always flow oracle -> GPU,
never the other way."""
import numpy as np
import torch

import paper_1803_03383_amd as hp
from oracle import ref

DEV = "cuda"


def xq_torch_dtype(b):
    return torch.int8 if b == 8 else torch.int16


def pad_cols(a, ld):
    """[.., d] -> [.., ld] with zero padding (row stride ld)."""
    if a.shape[-1] == ld:
        return np.ascontiguousarray(a)
    out = np.zeros(a.shape[:-1] + (ld,), dtype=a.dtype)
    out[..., : a.shape[-1]] = a
    return out


def xq_ld(d, b):
    """smallest row stride (elements) that is a multiple of 8 bytes"""
    per = 8 // (b // 8)
    return (d + per - 1) // per * per


class GpuProblem:
    """R chains; X [Rd,N,d] f32, Xq [Rd,N,d] int, y [Rd,N]; state buffers allocated here."""

    def __init__(self, X, Xq, y, *, K=1, R=1, loss=hp.LOSS_SQUARED, b=8, B=1, T=0, alpha=0.01,
                 mu=1.0, lam=0.0, delta_d=1.0, seed=0, share_data=False, w0=None,
                 algorithm=hp.ALG_HALP, delta=0.0):
        X = np.asarray(X, dtype=np.float32)
        if X.ndim == 2:
            X = X[None]
        Rd, N, d = X.shape
        self.N, self.d, self.K, self.R, self.b = N, d, K, R, b
        ldx = (d + 3) // 4 * 4
        ldxq = xq_ld(d, b)
        self.X = torch.from_numpy(pad_cols(X, ldx)).to(DEV)
        if Xq is not None:
            Xq = np.asarray(Xq)
            if Xq.ndim == 2:
                Xq = Xq[None]
            self.Xq = torch.from_numpy(pad_cols(Xq.astype(ref.xq_dtype(b)), ldxq)).to(DEV)
        else:
            self.Xq = torch.zeros((Rd, N, ldxq), dtype=xq_torch_dtype(b), device=DEV)
        y = np.asarray(y)
        if y.ndim == 1:
            y = y[None]
        ydt = np.int32 if loss == hp.LOSS_SOFTMAX else np.float32
        self.y = torch.from_numpy(np.ascontiguousarray(y.astype(ydt))).to(DEV)
        self.st = hp.alloc_state(N, d, K=K, R=R, b=b, device=DEV)
        if w0 is not None:
            self.st["w"].copy_(torch.from_numpy(np.asarray(w0, np.float32).reshape(R, K, d)))
        self.h = hp.Halp(N, d, K=K, R=R, loss=loss, b=b, B=B, T=T, alpha=alpha, mu=mu, lam=lam,
                         delta_d=delta_d, seed=seed, share_data=share_data, algorithm=algorithm,
                         delta=delta)
        self.h.bind(X=self.X, Xq=self.Xq, y=self.y, ldx=ldx, ldxq=ldxq, **self.st)

    # -- oracle-made inputs to the device
    def put(self, name, arr):
        t = self.st[name]
        src = torch.from_numpy(np.ascontiguousarray(arr)).to(t.dtype)
        t.copy_(src.reshape(t.shape))

    def get(self, name):
        torch.cuda.synchronize()
        return self.st[name].cpu().numpy()


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.linalg.norm(b)
    return np.linalg.norm(a - b) / (den if den > 0 else 1.0)
