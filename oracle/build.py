"""Compile the C oracle into oracle/libmom_oracle.so with gcc.

Test infrastructure only; the product never imports this package.
`-ffp-contract=off` and no `-march` keep every product rounded before its add,
as the oracle's header promises; `-fopenmp` only spreads independent rows.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "mom_oracle.c")
LIB = os.path.join(HERE, "libmom_oracle.so")

LIB_SANITIZED = os.path.join(HERE, "libmom_oracle_san.so")

FLAGS = ["-O2", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra"]
SANITIZE_FLAGS = ["-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"]


def build(force=True, sanitize=False):
    """Compile; with force=False only when the library is missing or stale.  sanitize=True builds a
    second library with AddressSanitizer and UndefinedBehaviorSanitizer (same arithmetic flags)
    for the sanitizer run of the oracle's tests; it needs gcc's libasan preloaded to be loaded."""
    lib = LIB_SANITIZED if sanitize else LIB
    if not force and os.path.exists(lib) and os.path.getmtime(lib) >= os.path.getmtime(SRC):
        return lib
    cmd = ["gcc"] + FLAGS + (SANITIZE_FLAGS if sanitize else []) + ["-o", lib, SRC, "-lm"]
    subprocess.run(cmd, check=True, cwd=HERE)
    return lib


if __name__ == "__main__":
    print(build())
