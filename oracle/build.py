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

CMD = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
       "-Wall", "-Wextra", "-o", LIB, SRC, "-lm"]


def build(force=True):
    """Compile; with force=False only when the library is missing or stale."""
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    subprocess.run(CMD, check=True, cwd=HERE)
    return LIB


if __name__ == "__main__":
    print(build())
