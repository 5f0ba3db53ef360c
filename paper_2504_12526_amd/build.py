"""Build libmom.so (the C-ABI HIP library) in-tree with hipcc for gfx950."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmom.so")
SOURCES = [os.path.join(CSRC, "mom.hip")]
DEPS = SOURCES + [os.path.join(CSRC, "mom_gemm.hip.inc"), os.path.join(CSRC, "mom_gemm_schedule.h"),
                  os.path.join(CSRC, "mom_gemv.hip.inc"), os.path.join(CSRC, "mom_probe.hip.inc"),
                  os.path.join(ROOT, "include", "mom.h")]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def build(force=True, extra_flags=(), out=None):
    """Compile; with force=False only when the library is missing or older than a source."""
    lib = out or LIB
    if not force and os.path.exists(lib) and all(os.path.getmtime(lib) >= os.path.getmtime(d) for d in DEPS):
        return lib
    cmd = [HIPCC] + FLAGS + list(extra_flags) + ["-o", lib] + SOURCES
    subprocess.run(cmd, check=True, cwd=CSRC)
    return lib


if __name__ == "__main__":
    print(build())
