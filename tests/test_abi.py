"""The C ABI without a GPU: the built library loads, exports every function include/halp.h
declares (and the binding lists the same names), and the host-side argument checks answer
before anything touches a device.  No kernel is launched here."""
import ctypes as C
import os
import re

import pytest

import paper_1803_03383_amd as hp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "halp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"^\s*(?:int|const char\s*\*)\s*(halp_\w+)\s*\(", text, flags=re.M)))


def test_header_declares_the_four_epoch_calls():
    names = _declared()
    for n in ("halp_full_gradient", "halp_recenter", "halp_inner_loop", "halp_epoch", "halp_create",
              "halp_destroy", "halp_bind", "halp_set_chain_hyper"):
        assert n in names
    assert len(names) >= 17


def test_library_exports_every_declared_symbol():
    L = hp.lib()
    for n in _declared():
        assert hasattr(L, n), f"{n} is declared in include/halp.h but not exported"
    assert sorted(hp.EXPORTS) == _declared()   # the binding wraps exactly the header


def test_binding_constants_follow_the_header():
    """Every HALP_ERR_*, HALP_LOSS_*, HALP_ALG_* and HALP_OPT_* macro has the same value under the
    same name (without the prefix) in the binding, and the binding has no option the header lacks."""
    text = open(os.path.join(ROOT, "include", "halp.h")).read()
    macros = {m.group(1): int(m.group(2)) for m in
              re.finditer(r"^#define HALP_((?:ERR|LOSS|ALG|OPT)_\w+)\s+\(?(-?\d+)\)?", text, flags=re.M)}
    assert len(macros) >= 20 and "OPT_INNER_PACKED" in macros
    for name, value in macros.items():
        assert getattr(hp, name) == value, name
    for name in dir(hp):
        if name.startswith(("OPT_", "ERR_", "LOSS_", "ALG_")):
            assert name in macros, f"{name} is not in include/halp.h"
    opts = [v for k, v in macros.items() if k.startswith("OPT_")]
    assert len(set(opts)) == len(opts)


def test_error_strings_and_version():
    for code in (hp.ERR_NULL, hp.ERR_INVALID, hp.ERR_UNSUPPORTED, hp.ERR_NOT_BOUND, hp.ERR_HIP, hp.ERR_ALIGN,
                 hp.ERR_TOO_LARGE, hp.ERR_EXCHANGE_TIMEOUT, 0):
        assert len(hp.strerror(code)) >= 2
    assert len({hp.strerror(c) for c in range(-8, 1)}) == 9
    assert hp.version()


def _params(**kw):
    base = dict(N=100, d=8, K=1, R=1, loss=hp.LOSS_SQUARED, b=8, B=1, share_data=0, algorithm=hp.ALG_HALP,
                T=10, alpha=0.1, mu=1.0, lam=0.0, delta_d=1.0, seed=0, delta=0.0)
    base.update(kw)
    return hp.Params(**base)


@pytest.mark.parametrize("kw,code", [
    (dict(N=0), hp.ERR_INVALID), (dict(d=0), hp.ERR_INVALID), (dict(R=0), hp.ERR_INVALID),
    (dict(B=0), hp.ERR_INVALID), (dict(b=7), hp.ERR_UNSUPPORTED), (dict(b=32), hp.ERR_UNSUPPORTED),
    (dict(T=-1), hp.ERR_INVALID), (dict(T=2 ** 32), hp.ERR_INVALID), (dict(loss=3), hp.ERR_INVALID),
    (dict(K=2), hp.ERR_INVALID), (dict(loss=hp.LOSS_SOFTMAX, K=1), hp.ERR_INVALID),
    (dict(loss=hp.LOSS_SOFTMAX, K=17), hp.ERR_UNSUPPORTED), (dict(alpha=0.0), hp.ERR_INVALID),
    (dict(alpha=float("nan")), hp.ERR_INVALID), (dict(mu=0.0), hp.ERR_INVALID),
    (dict(lam=-1.0), hp.ERR_INVALID), (dict(delta_d=0.0), hp.ERR_INVALID), (dict(share_data=2), hp.ERR_INVALID),
    (dict(algorithm=3), hp.ERR_INVALID), (dict(algorithm=hp.ALG_LPSVRG, delta=0.0), hp.ERR_INVALID),
    (dict(algorithm=hp.ALG_LPSVRG, delta=0.1, lam=0.1), hp.ERR_INVALID),
    (dict(algorithm=hp.ALG_SVRG, B=2), hp.ERR_UNSUPPORTED),
    (dict(algorithm=hp.ALG_SVRG, loss=hp.LOSS_SOFTMAX, K=3), hp.ERR_UNSUPPORTED),
])
def test_create_rejects_bad_parameters_on_the_host(kw, code):
    h = C.c_void_p()
    p = _params(**kw)
    assert hp.lib().halp_create(C.byref(h), C.byref(p)) == code
    assert not h.value


def test_null_arguments():
    L = hp.lib()
    h = C.c_void_p()
    assert L.halp_create(None, C.byref(_params())) == hp.ERR_NULL
    assert L.halp_create(C.byref(h), None) == hp.ERR_NULL
    assert L.halp_destroy(None) == hp.ERR_NULL
    assert L.halp_bind(None, None) == hp.ERR_NULL
    assert L.halp_set_option(None, hp.OPT_TIMING, 1) == hp.ERR_NULL
    assert L.halp_set_chain_hyper(None, None, None) == hp.ERR_NULL


def test_allocation_free_gradient_pass_checks_on_the_host():
    """halp_full_gradient_static answers bad arguments, and a problem beyond its fixed scratch,
    before it touches a device (the pointers here are never dereferenced)."""
    L = hp.lib()
    fake = 0x10000
    def bufs(**kw):
        b = hp.Buffers(X=fake, ldx=8, y=fake, w=fake, phi=fake, g=fake, scales=fake)
        for k, v in kw.items():
            setattr(b, k, v)
        return b
    ok = _params()
    assert L.halp_full_gradient_static(None, C.byref(bufs()), None) == hp.ERR_NULL
    assert L.halp_full_gradient_static(C.byref(ok), None, None) == hp.ERR_NULL
    assert L.halp_full_gradient_static(C.byref(_params(N=0)), C.byref(bufs()), None) == hp.ERR_INVALID
    assert L.halp_full_gradient_static(C.byref(ok), C.byref(bufs(g=None)), None) == hp.ERR_NOT_BOUND
    assert L.halp_full_gradient_static(C.byref(ok), C.byref(bufs(ldx=4)), None) == hp.ERR_INVALID
    assert L.halp_full_gradient_static(C.byref(ok), C.byref(bufs(ldx=10)), None) == hp.ERR_ALIGN
    assert L.halp_full_gradient_static(C.byref(ok), C.byref(bufs(X=fake + 4)), None) == hp.ERR_ALIGN
    # one workgroup per chain needs R (4 K d + 8) bytes: 4096 chains of 16 x 1024 do not fit 16 MiB
    big = _params(R=4096, loss=hp.LOSS_SOFTMAX, K=16, d=1024)
    assert 4096 * (4 * 16 * 1024 + 8) > hp.STATIC_SCRATCH_BYTES
    assert L.halp_full_gradient_static(C.byref(big), C.byref(bufs(ldx=1024)), None) == hp.ERR_TOO_LARGE


def test_step_latency_probe_checks_its_arguments_on_the_host():
    """halp_debug_step_latency refuses wave counts it has no kernel for, step counts that are
    not whole windows and a missing output before any launch."""
    L = hp.lib()
    fake = 0x10000
    assert L.halp_debug_step_latency(4, 64, 1, None, None) == hp.ERR_INVALID
    assert L.halp_debug_step_latency(3, 64, 1, fake, None) == hp.ERR_INVALID
    assert L.halp_debug_step_latency(4, 60, 1, fake, None) == hp.ERR_INVALID
    assert L.halp_debug_step_latency(4, 0, 1, fake, None) == hp.ERR_INVALID
    assert L.halp_debug_step_latency(4, 64, 0, fake, None) == hp.ERR_INVALID
    assert L.halp_debug_step_latency(4, 64, 70000, fake, None) == hp.ERR_INVALID
