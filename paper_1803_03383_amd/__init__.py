"""Thin Python binding of libhalp.so, the MI355X (gfx950) HALP epoch library.

Argument marshalling only: every step of the epoch runs in the library's HIP
kernels.  PyTorch is used for device memory and the stream handle.  There is
no CPU fallback: if the library has not been built, or a kernel does not cover
a shape, the call raises.
"""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhalp.so")

LOSS_SQUARED, LOSS_LOGISTIC, LOSS_SOFTMAX = 0, 1, 2
ALG_HALP, ALG_LPSVRG, ALG_SVRG = 0, 1, 2
OPT_INNER_VARIANT, OPT_TIMING, OPT_FULLGRAD_BLOCKS, OPT_INNER_WAVES, OPT_OPTION_II = 1, 2, 4, 5, 6
OPT_INNER_PARTS, OPT_EXCHANGE_SPIN_LIMIT, OPT_INNER_PACKED, OPT_INNER_HELPERS = 7, 8, 9, 10
OPT_EXCHANGE_POLL_DELAY = 11
OPT_GRADIENT_FP32 = 12
ERR_NULL, ERR_INVALID, ERR_UNSUPPORTED, ERR_NOT_BOUND, ERR_HIP, ERR_ALIGN = -1, -2, -3, -4, -5, -6
ERR_TOO_LARGE = -7
ERR_EXCHANGE_TIMEOUT = -8
STATIC_SCRATCH_BYTES = 16 << 20

EXPORTS = [
    "halp_create", "halp_destroy", "halp_bind", "halp_set_option", "halp_set_chain_hyper",
    "halp_set_feature_scale",
    "halp_quantize_data",
    "halp_full_gradient", "halp_full_gradient_static", "halp_recenter", "halp_inner_loop", "halp_epoch",
    "halp_inner_loop_trace", "halp_get_stats", "halp_debug_stream_words",
    "halp_debug_zround_bits", "halp_debug_read_bandwidth", "halp_debug_step_latency", "halp_strerror", "halp_last_error_detail", "halp_version",
]


class HalpError(RuntimeError):
    def __init__(self, code, what):
        self.code = code
        detail = lib().halp_last_error_detail().decode() if code == ERR_HIP else ""
        super().__init__(f"{what}: {strerror(code)} ({code})" + (f" [{detail}]" if detail else ""))


class Params(C.Structure):
    _fields_ = [
        ("N", C.c_int64), ("d", C.c_int32), ("K", C.c_int32), ("R", C.c_int32), ("loss", C.c_int32),
        ("b", C.c_int32), ("B", C.c_int32), ("share_data", C.c_int32), ("algorithm", C.c_int32),
        ("T", C.c_int64), ("alpha", C.c_double), ("mu", C.c_double), ("lam", C.c_double),
        ("delta_d", C.c_double), ("seed", C.c_uint64), ("delta", C.c_double),
    ]


class Buffers(C.Structure):
    _fields_ = [
        ("X", C.c_void_p), ("ldx", C.c_int64), ("Xq", C.c_void_p), ("ldxq", C.c_int64),
        ("y", C.c_void_p), ("w", C.c_void_p), ("phi", C.c_void_p), ("g", C.c_void_p),
        ("z", C.c_void_p), ("h", C.c_void_p), ("scales", C.c_void_p), ("counters", C.c_void_p),
    ]


class Stats(C.Structure):
    _fields_ = [
        ("delta_m", C.c_double), ("delta_i", C.c_double), ("delta_s", C.c_double),
        ("grad_norm", C.c_double), ("loss", C.c_double), ("status", C.c_int32),
        ("inner_variant", C.c_int32), ("n_clamped_z", C.c_uint64), ("n_clamped_gamma", C.c_uint64),
        ("n_reg_draws", C.c_uint64), ("ms_full_gradient", C.c_float), ("ms_recenter", C.c_float),
        ("ms_inner_loop", C.c_float), ("timed_epochs", C.c_int32),
        ("n_exchange_timeouts", C.c_uint64),
    ]


_lib = None


def lib():
    """Loads libhalp.so; fails loudly when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_1803_03383_amd.build`")
        # torch first: the process must end up with ONE HIP runtime, the one torch's
        # allocations and streams live in; libhalp.so then binds to that copy
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        vp, i64, i32, u64, u32 = C.c_void_p, C.c_int64, C.c_int32, C.c_uint64, C.c_uint32
        L.halp_create.argtypes = [C.POINTER(vp), C.POINTER(Params)]
        L.halp_destroy.argtypes = [vp]
        L.halp_bind.argtypes = [vp, C.POINTER(Buffers)]
        L.halp_set_option.argtypes = [vp, i32, i64]
        L.halp_set_chain_hyper.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_double)]
        L.halp_set_feature_scale.argtypes = [vp, vp]
        L.halp_quantize_data.argtypes = [vp, vp]
        L.halp_full_gradient.argtypes = [vp, vp]
        L.halp_full_gradient_static.argtypes = [C.POINTER(Params), C.POINTER(Buffers), vp]
        L.halp_recenter.argtypes = [vp, i64, vp]
        L.halp_inner_loop.argtypes = [vp, i64, vp]
        L.halp_epoch.argtypes = [vp, i64, vp]
        L.halp_inner_loop_trace.argtypes = [vp, i64, i64, vp, vp, vp, vp, vp, vp]
        L.halp_get_stats.argtypes = [vp, i32, vp, C.POINTER(Stats)]
        L.halp_debug_stream_words.argtypes = [u64, u32, u32, u64, i64, vp, vp]
        L.halp_debug_zround_bits.argtypes = [u64, u32, u64, i32, i32, i32, vp, vp]
        L.halp_debug_read_bandwidth.argtypes = [vp, i64, vp, vp]
        L.halp_debug_step_latency.argtypes = [i32, i64, i32, vp, vp]
        for name in EXPORTS:
            getattr(L, name).restype = C.c_int
        L.halp_strerror.restype = C.c_char_p
        L.halp_strerror.argtypes = [C.c_int]
        L.halp_last_error_detail.restype = C.c_char_p
        L.halp_last_error_detail.argtypes = []
        L.halp_version.restype = C.c_char_p
        L.halp_version.argtypes = []
        _lib = L
    return _lib


def strerror(code):
    return lib().halp_strerror(int(code)).decode()


def version():
    return lib().halp_version().decode()


def _check(rc, what):
    if rc != 0:
        raise HalpError(rc, what)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        return C.c_void_p(torch.cuda.current_stream().cuda_stream)
    return C.c_void_p(int(stream))


class Halp:
    """One handle: R chains of an N x d problem.  Tensors are torch CUDA tensors
    owned by the caller; the handle keeps references so they outlive it."""

    def __init__(self, N, d, K=1, R=1, loss=LOSS_SQUARED, b=8, B=1, T=0, alpha=0.01, mu=1.0,
                 lam=0.0, delta_d=1.0, seed=0, share_data=False, algorithm=ALG_HALP, delta=0.0):
        self.params = Params(N=N, d=d, K=K, R=R, loss=loss, b=b, B=B, share_data=int(share_data),
                             algorithm=algorithm, T=T, alpha=alpha, mu=mu, lam=lam,
                             delta_d=delta_d, seed=seed, delta=delta)
        self._h = C.c_void_p()
        _check(lib().halp_create(C.byref(self._h), C.byref(self.params)), "halp_create")
        self._keep = {}

    def close(self):
        if self._h:
            lib().halp_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def bind(self, X=None, Xq=None, y=None, w=None, phi=None, g=None, z=None, h=None, scales=None,
             counters=None, ldx=None, ldxq=None):
        self._keep = dict(X=X, Xq=Xq, y=y, w=w, phi=phi, g=g, z=z, h=h, scales=scales,
                          counters=counters, fscale=self._keep.get("fscale"))
        b = Buffers()
        b.X, b.Xq, b.y, b.w, b.phi, b.g = _ptr(X), _ptr(Xq), _ptr(y), _ptr(w), _ptr(phi), _ptr(g)
        b.z, b.h, b.scales, b.counters = _ptr(z), _ptr(h), _ptr(scales), _ptr(counters)
        b.ldx = int(ldx if ldx is not None else (X.stride(-2) if X is not None else self.params.d))
        b.ldxq = int(ldxq if ldxq is not None else (Xq.stride(-2) if Xq is not None else self.params.d))
        _check(lib().halp_bind(self._h, C.byref(b)), "halp_bind")

    def set_option(self, option, value):
        _check(lib().halp_set_option(self._h, option, value), "halp_set_option")

    def set_chain_hyper(self, alpha=None, mu=None):
        """Per-chain step size and mu (sequences of R floats, or None for the handle's)."""
        def arr(v):
            if v is None:
                return None
            v = [float(x) for x in v]
            if len(v) != self.params.R:
                raise ValueError("one value per chain expected")
            return (C.c_double * len(v))(*v)
        _check(lib().halp_set_chain_hyper(self._h, arr(alpha), arr(mu)), "halp_set_chain_hyper")

    def set_feature_scale(self, s=None):
        """Per-feature data scales: a float32 CUDA tensor of d entries, or None to switch off."""
        self._keep["fscale"] = s
        _check(lib().halp_set_feature_scale(self._h, _ptr(s)), "halp_set_feature_scale")

    def quantize_data(self, stream=None):
        _check(lib().halp_quantize_data(self._h, _stream(stream)), "halp_quantize_data")

    def full_gradient(self, stream=None):
        _check(lib().halp_full_gradient(self._h, _stream(stream)), "halp_full_gradient")

    def recenter(self, epoch, stream=None):
        _check(lib().halp_recenter(self._h, epoch, _stream(stream)), "halp_recenter")

    def inner_loop(self, epoch, stream=None):
        _check(lib().halp_inner_loop(self._h, epoch, _stream(stream)), "halp_inner_loop")

    def epoch(self, epoch, stream=None):
        _check(lib().halp_epoch(self._h, epoch, _stream(stream)), "halp_epoch")

    def inner_loop_trace(self, epoch, M, idx=None, D=None, beta=None, gamma=None, ztraj=None,
                         stream=None):
        _check(lib().halp_inner_loop_trace(self._h, epoch, M, _ptr(idx), _ptr(D), _ptr(beta),
                                           _ptr(gamma), _ptr(ztraj), _stream(stream)),
               "halp_inner_loop_trace")

    def get_stats(self, chain=0, stream=None):
        s = Stats()
        rc = lib().halp_get_stats(self._h, chain, _stream(stream), C.byref(s))
        if rc == ERR_EXCHANGE_TIMEOUT:  # the statistics are complete; the caller sees both
            err = HalpError(rc, "halp_get_stats")
            err.stats = s
            raise err
        _check(rc, "halp_get_stats")
        return s


def full_gradient_static(params, X, y, w, phi, g, scales, ldx=None, stream=None):
    """halp_full_gradient without a handle and without any allocation: the partial sums go
    through the library's fixed device array.  params: a Params; the rest torch CUDA tensors."""
    b = Buffers()
    b.X, b.y, b.w, b.phi, b.g, b.scales = _ptr(X), _ptr(y), _ptr(w), _ptr(phi), _ptr(g), _ptr(scales)
    b.ldx = int(ldx if ldx is not None else X.stride(-2))
    _check(lib().halp_full_gradient_static(C.byref(params), C.byref(b), _stream(stream)),
           "halp_full_gradient_static")


def alloc_state(N, d, K=1, R=1, b=8, device="cuda"):
    """Allocates the library's output / state buffers as torch tensors."""
    import torch

    zt = torch.int8 if b == 8 else torch.int16
    ht = torch.int16 if b == 8 else torch.int32
    return dict(
        w=torch.zeros((R, K, d), dtype=torch.float32, device=device),
        phi=torch.zeros((R, N, K), dtype=torch.float32, device=device),
        g=torch.zeros((R, K, d), dtype=torch.float32, device=device),
        z=torch.zeros((R, K, d), dtype=zt, device=device),
        h=torch.zeros((R, K, d), dtype=ht, device=device),
        scales=torch.zeros((R, 8), dtype=torch.float64, device=device),
        counters=torch.zeros((R, 4), dtype=torch.int64, device=device),
    )


def debug_stream_words(seed, purpose, epoch, n0, count, stream=None):
    import torch

    out = torch.zeros((count,), dtype=torch.int32, device="cuda")
    _check(lib().halp_debug_stream_words(seed, purpose, epoch, n0, count, _ptr(out),
                                         _stream(stream)), "halp_debug_stream_words")
    return out


def debug_zround_bits(seed, epoch, t, d, b, K, stream=None):
    import torch

    out = torch.zeros((K, d), dtype=torch.int32, device="cuda")
    _check(lib().halp_debug_zround_bits(seed, epoch, t, d, b, K, _ptr(out), _stream(stream)),
           "halp_debug_zround_bits")
    return out


def debug_read_bandwidth(t, out=None, stream=None):
    """Reads tensor t (contiguous, a multiple of 16 bytes) once; returns the checksum tensor."""
    import torch
    if out is None:
        out = torch.empty(2048, dtype=torch.int32, device=t.device)
    nbytes = t.numel() * t.element_size()
    _check(lib().halp_debug_read_bandwidth(_ptr(t), nbytes, _ptr(out), _stream(stream)),
           "halp_debug_read_bandwidth")
    return out


def debug_step_latency(waves, steps, blocks, out=None, stream=None):
    """Runs the isolated dependent chain of an 8-bit inner-loop step; returns its output tensor."""
    import torch
    if out is None:
        out = torch.empty(blocks * waves * 64, dtype=torch.int32, device="cuda")
    if out.numel() < blocks * waves * 64:
        raise ValueError("out holds fewer than blocks * waves * 64 words")
    _check(lib().halp_debug_step_latency(waves, steps, blocks, _ptr(out), _stream(stream)),
           "halp_debug_step_latency")
    return out
