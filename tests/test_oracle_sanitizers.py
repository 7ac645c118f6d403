"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: every entry point once
on small ragged, strided inputs (primitives, all three losses, minibatches, L2 draws, both legs
of the scalar path, a softmax epoch, LP-SVRG epochs), every report fatal."""
import os
import subprocess

from oracle import build as obuild


def test_oracle_runs_clean_under_asan_and_ubsan():
    exe = obuild.build_sanitized()
    env = dict(os.environ)
    env.pop("LD_PRELOAD", None)  # the sanitizer runtime has to come first in the link order
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.strip() == "ok"
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr
