"""Compile the CPU oracle (oracle/halp_ref.c) into oracle/libhalp_ref.so with gcc.

Test infrastructure only.  Contraction is switched off so that every fp64
operation of the oracle is rounded on its own, as its header states.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "halp_ref.c")
OUT = os.path.join(HERE, "libhalp_ref.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(OUT) and os.path.getmtime(OUT) >= max(
        os.path.getmtime(SRC), os.path.getmtime(os.path.join(HERE, "halp_ref.h"))
    ):
        return OUT
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
           "-Wall", "-Wextra", "-o", OUT, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return OUT


SAN_DIR = os.path.join(HERE, "_san")
SAN_OUT = os.path.join(SAN_DIR, "halp_ref_san")


def build_sanitized() -> str:
    """The oracle and its driver (sanitize_main.c) as one executable under AddressSanitizer and
    UndefinedBehaviorSanitizer, every report fatal.  Same floating-point flags as the library."""
    os.makedirs(SAN_DIR, exist_ok=True)
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fno-fast-math",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           "-Wall", "-Wextra", "-o", SAN_OUT, SRC, os.path.join(HERE, "sanitize_main.c"), "-lm"]
    subprocess.run(cmd, check=True)
    return SAN_OUT


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
