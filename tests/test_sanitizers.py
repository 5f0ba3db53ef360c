"""Sanitizer runs of the host code (no GPU): the oracle's pins under gcc's AddressSanitizer +
UndefinedBehaviorSanitizer, and the C ABI's host side (argument validation, status paths) under
clang's, each in a child process with the matching sanitizer runtime preloaded."""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _child_env(runtime):
    env = dict(os.environ)
    # the sanitizer runtime must come first in the initial library list; whatever is preloaded already stays
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1:abort_on_error=0"      # the interpreter itself leaks
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    return env


def _check(r):
    tail = (r.stdout + r.stderr)[-4000:]
    assert r.returncode == 0, tail
    for bad in ("ERROR: AddressSanitizer", "runtime error:", "SUMMARY: UndefinedBehaviorSanitizer"):
        assert bad not in r.stdout + r.stderr, tail
    assert " passed" in r.stdout, tail


def test_oracle_pins_under_asan_and_ubsan():
    from oracle import build as oracle_build
    oracle_build.build(force=True, sanitize=True)
    runtime = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("gcc's libasan.so is not installed")
    env = _child_env(os.path.realpath(runtime))
    env["MOM_ORACLE_SANITIZED"] = "1"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                       capture_output=True, text=True, cwd=ROOT, env=env, timeout=900)
    _check(r)


def test_abi_host_side_under_asan_and_ubsan():
    from paper_2504_12526_amd import build as lib_build
    found = glob.glob("/opt/rocm/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    if not found:
        pytest.skip("clang's shared AddressSanitizer runtime is not installed")
    san = os.path.join(ROOT, "paper_2504_12526_amd", "libmom_san.so")
    # host code only: every -fsanitize directly behind -Xarch_host; the device code is built as usual
    lib_build.build(force=True, out=san,
                    extra_flags=["-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                                 "-Xarch_host", "-fno-sanitize-recover=undefined", "-shared-libsan"])
    runner = ("import sys; sys.path.insert(0, %r); from paper_2504_12526_amd import binding; "
              "binding.LIB_PATH = %r; import pytest; "
              "sys.exit(pytest.main(['-x', '-q', '-p', 'no:cacheprovider', %r]))"
              % (ROOT, san, os.path.join(ROOT, "tests", "test_abi_host.py")))
    r = subprocess.run([sys.executable, "-c", runner], capture_output=True, text=True, cwd=ROOT,
                       env=_child_env(found[0]), timeout=900)
    _check(r)
