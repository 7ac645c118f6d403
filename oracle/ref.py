"""ctypes front end of the CPU oracle (oracle/halp_ref.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  It never imports the HIP package.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

SQUARED, LOGISTIC, SOFTMAX = 0, 1, 2
PURPOSE_IDX, PURPOSE_GAMMA, PURPOSE_ZROUND, PURPOSE_REG, PURPOSE_HROUND, PURPOSE_OPT2 = 0, 1, 2, 3, 4, 5


class Problem(C.Structure):
    _fields_ = [
        ("N", C.c_int64), ("d", C.c_int32), ("K", C.c_int32), ("loss", C.c_int32),
        ("b", C.c_int32), ("B", C.c_int32), ("algorithm", C.c_int32),
        ("alpha", C.c_double), ("mu", C.c_double), ("lam", C.c_double),
        ("delta_d", C.c_double), ("seed", C.c_uint64), ("delta", C.c_double),
        ("scalar_path", C.c_int32),
    ]


class Trace(C.Structure):
    _fields_ = [
        ("M", C.c_int64), ("idx", C.c_void_p), ("D", C.c_void_p), ("beta", C.c_void_p),
        ("gamma", C.c_void_p), ("ztraj", C.c_void_p), ("beta_other", C.c_void_p),
        ("gamma_other", C.c_void_p),
    ]


_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        L.halp_ref_stream_word.restype = C.c_uint32
        L.halp_ref_stream_word.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint64]
        L.halp_ref_zround_bits.restype = C.c_uint32
        L.halp_ref_zround_bits.argtypes = [C.c_uint64, C.c_uint32, C.c_uint64, C.c_int32,
                                           C.c_int32, C.c_int32, C.c_int32]
        L.halp_ref_option2_steps.restype = C.c_int64
        L.halp_ref_option2_steps.argtypes = [C.c_uint64, C.c_uint32, C.c_int64]
        L.halp_ref_sample_index.restype = C.c_int64
        L.halp_ref_sample_index.argtypes = [C.c_uint64, C.c_uint32, C.c_uint64, C.c_int32,
                                            C.c_int32, C.c_int64]
        L.halp_ref_quantize_real.restype = C.c_int64
        L.halp_ref_quantize_real.argtypes = [C.c_double, C.c_double, C.c_uint32, C.c_int64,
                                             C.c_int64, C.c_void_p]
        L.halp_ref_exp_array.restype = None
        L.halp_ref_exp_array.argtypes = [C.c_void_p, C.c_int64, C.c_void_p]
        L.halp_ref_round_shift.restype = C.c_int64
        L.halp_ref_round_shift.argtypes = [C.c_int64, C.c_int64, C.c_uint32, C.c_int, C.c_void_p]
        L.halp_ref_philox4x32_10.restype = None
        L.halp_ref_philox4x32_10.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.halp_ref_quantize_data.restype = None
        L.halp_ref_quantize_data.argtypes = [C.c_void_p, C.c_int64, C.c_double, C.c_int, C.c_void_p]
        L.halp_ref_quantize_data_scaled.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_double,
                                                    C.c_void_p, C.c_int, C.c_void_p]
        L.halp_ref_full_gradient_scaled.restype = C.c_int
        L.halp_ref_full_gradient_scaled.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p,
                                                    C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                                    C.c_void_p]
        L.halp_ref_full_gradient.restype = C.c_int
        L.halp_ref_full_gradient.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p,
                                             C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.halp_ref_recenter.restype = C.c_int
        L.halp_ref_recenter.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p,
                                        C.c_void_p, C.c_void_p]
        L.halp_ref_lp_begin.restype = C.c_int
        L.halp_ref_lp_begin.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p,
                                        C.c_void_p, C.c_void_p]
        L.halp_ref_svrg_inner.restype = C.c_int
        L.halp_ref_svrg_inner.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                          C.c_void_p, C.c_uint32, C.c_int64, C.c_void_p]
        L.halp_ref_inner_loop.restype = C.c_int
        L.halp_ref_inner_loop.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                          C.c_void_p, C.c_void_p, C.c_uint32, C.c_int64, C.c_void_p,
                                          C.c_void_p, C.c_void_p]
        L.halp_ref_apply_offset.restype = None
        L.halp_ref_apply_offset.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.halp_ref_epoch.restype = C.c_int
        L.halp_ref_epoch.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64,
                                     C.c_void_p, C.c_void_p, C.c_uint32, C.c_int64, C.c_void_p,
                                     C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def xq_dtype(b):
    return np.int8 if b == 8 else (np.int16 if b == 16 else np.int32)


ALG_HALP, ALG_LPSVRG, ALG_SVRG = 0, 1, 2
# legs of the inner loop's scalar path: the reproducible reading / the plain definition
SCALAR_FIXED, SCALAR_PLAIN = 0, 1


def make_problem(N, d, K=1, loss=SQUARED, b=8, B=1, alpha=0.01, mu=1.0, lam=0.0, delta_d=1.0,
                 seed=0, algorithm=ALG_HALP, delta=0.0, scalar_path=SCALAR_FIXED):
    return Problem(N=N, d=d, K=K, loss=loss, b=b, B=B, algorithm=algorithm, alpha=alpha, mu=mu,
                   lam=lam, delta_d=delta_d, seed=seed, delta=delta, scalar_path=scalar_path)


def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().halp_ref_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def stream_word(seed, purpose, epoch, n):
    return int(lib().halp_ref_stream_word(seed, purpose, epoch, n))


def zround_bits(seed, epoch, t, d, b, c, j):
    return int(lib().halp_ref_zround_bits(seed, epoch, t, d, b, c, j))


def sample_index(seed, epoch, t, B, m, N):
    return int(lib().halp_ref_sample_index(seed, epoch, t, B, m, N))


def option2_steps(seed, epoch, T):
    """option II: the number of inner steps after which the epoch of that number ends"""
    return int(lib().halp_ref_option2_steps(seed, epoch, T))


def quantize_real(x, inv_delta, r32, lo, hi):
    hit = C.c_int(0)
    q = lib().halp_ref_quantize_real(x, inv_delta, r32, lo, hi, C.addressof(hit))
    return int(q), bool(hit.value)


def exp_inner(x):
    """exp as the inner loop's scalar path evaluates it, elementwise"""
    x = np.ascontiguousarray(x, dtype=np.float64)
    out = np.empty_like(x)
    lib().halp_ref_exp_array(x.ctypes.data, x.size, out.ctypes.data)
    return out


def round_shift(z, v, r, b):
    hit = C.c_int(0)
    q = lib().halp_ref_round_shift(z, v, r, b, C.addressof(hit))
    return int(q), bool(hit.value)


def quantize_data(X, delta_d, b):
    X = np.ascontiguousarray(X, dtype=np.float32)
    Xq = np.zeros(X.shape, dtype=xq_dtype(b))
    lib().halp_ref_quantize_data(_p(X), X.size, float(delta_d), b, _p(Xq))
    return Xq


def quantize_data_scaled(X, delta_d, s, b):
    """q_ij = clamp(rne(X_ij / (delta_d s_j))): per-feature scales s[d]"""
    X = np.ascontiguousarray(X, dtype=np.float32)
    s = np.ascontiguousarray(s, dtype=np.float32)
    assert X.ndim == 2 and s.shape == (X.shape[1],)
    Xq = np.zeros(X.shape, dtype=xq_dtype(b))
    lib().halp_ref_quantize_data_scaled(_p(X), X.shape[0], X.shape[1], float(delta_d), _p(s), b, _p(Xq))
    return Xq


def _ylike(prob, y):
    if prob.loss == SOFTMAX:
        return np.ascontiguousarray(y, dtype=np.int32)
    return np.ascontiguousarray(y, dtype=np.float32)


def full_gradient(prob, X, y, w):
    """returns (phi[N,K] f64, g[K,d] f64, loss f64)"""
    X = np.ascontiguousarray(X, dtype=np.float32)
    w = np.ascontiguousarray(w, dtype=np.float32).reshape(prob.K, prob.d)
    yy = _ylike(prob, y)
    phi = np.zeros((prob.N, prob.K), dtype=np.float64)
    g = np.zeros((prob.K, prob.d), dtype=np.float64)
    loss = np.zeros(1, dtype=np.float64)
    rc = lib().halp_ref_full_gradient(C.addressof(prob), _p(X), X.shape[1], _p(yy), _p(w), _p(phi),
                                      _p(g), _p(loss))
    if rc != 0:
        raise ValueError(f"halp_ref_full_gradient rc={rc}")
    return phi, g, float(loss[0])


def full_gradient_scaled(prob, X, y, v, s):
    """the pass for the scaled model v_j = s_j w_j: returns (phi, d f / d v, loss)"""
    X = np.ascontiguousarray(X, dtype=np.float32)
    v = np.ascontiguousarray(v, dtype=np.float32).reshape(prob.K, prob.d)
    s = np.ascontiguousarray(s, dtype=np.float32)
    yy = _ylike(prob, y)
    phi = np.zeros((prob.N, prob.K), dtype=np.float64)
    g = np.zeros((prob.K, prob.d), dtype=np.float64)
    loss = np.zeros(1, dtype=np.float64)
    rc = lib().halp_ref_full_gradient_scaled(C.addressof(prob), _p(X), X.shape[1], _p(yy), _p(v), _p(s),
                                             _p(phi), _p(g), _p(loss))
    if rc != 0:
        raise ValueError(f"halp_ref_full_gradient_scaled rc={rc}")
    return phi, g, float(loss[0])


def epoch_scaled(prob, X, Xq, y, v, s, epoch_no, T):
    """one HALP epoch on the scaled model: scaled gradient pass, then the unchanged bit
    centering, inner loop and update of v"""
    phi, g, loss = full_gradient_scaled(prob, X, y, v, s)
    phi32, g32 = phi.astype(np.float32), g.astype(np.float32)
    scales, h, z = recenter(prob, g32, epoch_no)
    out = inner_loop(prob, Xq, phi32, y, h, scales, epoch_no, T)
    v1 = apply_offset(prob, scales, out["z"], v)
    return dict(w=v1, phi=phi32, g=g32, scales=scales, h=h, z=out["z"], counters=out["counters"], loss=loss)


def recenter(prob, g32, epoch):
    """returns (scales[8] f64, h[K,d] i64, z[K,d] i32)"""
    g32 = np.ascontiguousarray(g32, dtype=np.float32)
    scales = np.zeros(8, dtype=np.float64)
    h = np.zeros((prob.K, prob.d), dtype=np.int64)
    z = np.zeros((prob.K, prob.d), dtype=np.int32)
    rc = lib().halp_ref_recenter(C.addressof(prob), _p(g32), epoch, _p(scales), _p(h), _p(z))
    if rc != 0:
        raise ValueError(f"halp_ref_recenter rc={rc}")
    return scales, h, z


def lp_begin(prob, g32, w, epoch):
    """start of an LP-SVRG epoch; returns (scales[8] f64, h[K,d] i64, z[K,d] i32)"""
    g32 = np.ascontiguousarray(g32, dtype=np.float32)
    w = np.ascontiguousarray(w, dtype=np.float32)
    scales = np.zeros(8, dtype=np.float64)
    h = np.zeros((prob.K, prob.d), dtype=np.int64)
    z = np.zeros((prob.K, prob.d), dtype=np.int32)
    rc = lib().halp_ref_lp_begin(C.addressof(prob), _p(g32), _p(w), epoch, _p(scales), _p(h), _p(z))
    if rc != 0:
        raise ValueError(f"halp_ref_lp_begin rc={rc}")
    return scales, h, z


def inner_loop(prob, Xq, phi32, y, h, scales, epoch, T, z0=None, trace_steps=0, trace_z=True,
               trace_other=False):
    """returns dict(z=..., counters=..., and trace arrays when trace_steps > 0).  trace_other adds
    beta_other / gamma_other: what the other leg of the scalar path gives at each recorded step
    (same state, same draw)"""
    Xq = np.ascontiguousarray(Xq, dtype=xq_dtype(prob.b))
    phi32 = np.ascontiguousarray(phi32, dtype=np.float32)
    yy = _ylike(prob, y)
    h = np.ascontiguousarray(h, dtype=np.int64)
    scales = np.ascontiguousarray(scales, dtype=np.float64)
    z = np.zeros((prob.K, prob.d), dtype=np.int32) if z0 is None else np.array(z0, dtype=np.int32)
    counters = np.zeros(4, dtype=np.uint64)
    out = {}
    tr = None
    if trace_steps > 0:
        M, B, K, d = trace_steps, prob.B, prob.K, prob.d
        out["idx"] = np.zeros((M, B), dtype=np.int64)
        out["D"] = np.zeros((M, B, K), dtype=np.int64)
        out["beta"] = np.zeros((M, B, K), dtype=np.float64)
        out["gamma"] = np.zeros((M, B, K), dtype=np.int32)
        if trace_z:
            out["ztraj"] = np.zeros((M, K, d), dtype=np.int32)
        if trace_other:
            out["beta_other"] = np.zeros((M, B, K), dtype=np.float64)
            out["gamma_other"] = np.zeros((M, B, K), dtype=np.int32)
        tr = Trace(M=M, idx=out["idx"].ctypes.data, D=out["D"].ctypes.data,
                   beta=out["beta"].ctypes.data, gamma=out["gamma"].ctypes.data,
                   ztraj=out["ztraj"].ctypes.data if trace_z else None,
                   beta_other=out["beta_other"].ctypes.data if trace_other else None,
                   gamma_other=out["gamma_other"].ctypes.data if trace_other else None)
    rc = lib().halp_ref_inner_loop(C.addressof(prob), _p(Xq), Xq.shape[1], _p(phi32), _p(yy), _p(h),
                                   _p(scales), epoch, T, _p(z),
                                   C.addressof(tr) if tr is not None else None, _p(counters))
    if rc != 0:
        raise ValueError(f"halp_ref_inner_loop rc={rc}")
    out["z"] = z
    out["counters"] = counters
    return out


def svrg_inner(prob, X, y, phi32, g32, w, epoch, T):
    """T steps of Algorithm 1 from w~ = w (fp64 state); returns w_T as float64 [d]"""
    X = np.ascontiguousarray(X, dtype=np.float32)
    yy = _ylike(prob, y)
    phi32 = np.ascontiguousarray(phi32, dtype=np.float32)
    g32 = np.ascontiguousarray(g32, dtype=np.float32)
    w = np.array(w, dtype=np.float64).reshape(prob.d)
    rc = lib().halp_ref_svrg_inner(C.addressof(prob), _p(X), X.shape[1], _p(yy), _p(phi32), _p(g32),
                                   epoch, T, _p(w))
    if rc != 0:
        raise ValueError(f"halp_ref_svrg_inner rc={rc}")
    return w


def svrg_epoch(prob, X, y, w, epoch, T, option2=False):
    """one SVRG epoch as the library runs it: fp64 gradient pass rounded to fp32, inner loop,
    w~ <- fp32(w_T) (option I) or fp32(w_t), t drawn (option II)"""
    if option2:
        T = option2_steps(prob.seed, epoch, T)
    phi, g, loss = full_gradient(prob, X, y, np.asarray(w, np.float32).reshape(1, prob.d))
    wT = svrg_inner(prob, X, y, phi.astype(np.float32), g.astype(np.float32),
                    np.asarray(w, np.float32).reshape(prob.d), epoch, T)
    return dict(w=wT.astype(np.float32).reshape(1, prob.d), w64=wT, phi=phi, g=g, loss=loss)


def apply_offset(prob, scales, z, w):
    w = np.array(w, dtype=np.float32).reshape(prob.K, prob.d)
    z = np.ascontiguousarray(z, dtype=np.int32)
    scales = np.ascontiguousarray(scales, dtype=np.float64)
    lib().halp_ref_apply_offset(C.addressof(prob), _p(scales), _p(z), _p(w))
    return w


def epoch(prob, X, Xq, y, w, epoch_no, T, option2=False):
    """one HALP epoch; returns dict(w, phi, g, scales, h, z, counters).  option2: the epoch ends
    at the iterate after t steps, t drawn uniformly from {0..T-1} (option II)"""
    if option2:
        T = option2_steps(prob.seed, epoch_no, T)
    X = np.ascontiguousarray(X, dtype=np.float32)
    Xq = np.ascontiguousarray(Xq, dtype=xq_dtype(prob.b))
    yy = _ylike(prob, y)
    w = np.array(w, dtype=np.float32).reshape(prob.K, prob.d)
    phi = np.zeros((prob.N, prob.K), dtype=np.float32)
    g = np.zeros((prob.K, prob.d), dtype=np.float32)
    scales = np.zeros(8, dtype=np.float64)
    h = np.zeros((prob.K, prob.d), dtype=np.int64)
    z = np.zeros((prob.K, prob.d), dtype=np.int32)
    counters = np.zeros(4, dtype=np.uint64)
    rc = lib().halp_ref_epoch(C.addressof(prob), _p(X), X.shape[1], _p(Xq), Xq.shape[1], _p(yy),
                              _p(w), epoch_no, T, _p(phi), _p(g), _p(scales), _p(h), _p(z),
                              _p(counters))
    if rc != 0:
        raise ValueError(f"halp_ref_epoch rc={rc}")
    return dict(w=w, phi=phi, g=g, scales=scales, h=h, z=z, counters=counters)
