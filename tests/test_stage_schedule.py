"""The chained stage schedule of the 256-row GEMM tiles, checked on the host: tests/stage_schedule_check.cpp walks
the same functions the kernel asks (paper_2504_12526_amd/csrc/mom_gemm_schedule.h) and verifies index ranges,
what each barrier's wait covers, ring-slot reuse and the contents of the operand registers at every MFMA."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2504_12526_amd", "csrc")
CHECK = os.path.join(ROOT, "tests", "stage_schedule_check.cpp")
HEADER = os.path.join(CSRC, "mom_gemm_schedule.h")


def _build_and_run(tmp_path, include_dir):
    exe = os.path.join(tmp_path, "stage_schedule_check")
    subprocess.run(["g++", "-std=c++17", "-O1", "-Wall", "-Werror", "-I", include_dir, "-o", exe, CHECK], check=True)
    return subprocess.run([exe], capture_output=True, text=True)


def test_schedule_as_shipped_passes(tmp_path):
    r = _build_and_run(str(tmp_path), CSRC)
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.count(": ok") == 5, r.stdout          # the five tile widths


@pytest.mark.parametrize("old,new,what", [
    # the barrier one row late: row 1 reads stage T+1 before anybody waited for it
    ("MOM_SCHED_FN int barrier_row() { return 1; }", "MOM_SCHED_FN int barrier_row() { return 2; }", "barrier"),
    # the wait lets one load too many stay in flight
    ("MOM_SCHED_FN int barrier_loads_in_flight(int MB) { return MB; }",
     "MOM_SCHED_FN int barrier_loads_in_flight(int MB) { return MB + 1; }", "wait"),
    # token fragments refilled one row early: the row still multiplies with them
    ("return {TOK, khalf, mb - 1, 1, 2};", "return {TOK, khalf, mb, 1, 2};", "register"),
    # a ring load index past the wavefront's blocks
    ("if (mb == 0) return {TOK, MB - 2 + h, 2, 4};", "if (mb == 0) return {TOK, MB - 1 + h, 2, 4};", "index"),
    # the weights of stage T+2 into the slot that stage T+1 is still read from
    ("if (mb <= MB / 2) return {WGT, 2 * (mb - 1) + h, 2, 0};", "if (mb <= MB / 2) return {WGT, 2 * (mb - 1) + h, 2, 2};", "slot"),
    # the token pointer moved too late for the first token loads of stage T+3
    ("MOM_SCHED_FN int token_pointer_row(int MB) { return MB - 3; }", "MOM_SCHED_FN int token_pointer_row(int MB) { return MB - 2; }",
     "pointer"),
])
def test_a_planted_mistake_is_caught(tmp_path, old, new, what):
    """The checker is worth something only if it fails on a wrong schedule: plant one mistake at a time in a
    copy of the header (on the CPU; nothing of this reaches a GPU)."""
    inc = os.path.join(str(tmp_path), "inc")
    os.makedirs(inc)
    text = open(HEADER).read()
    assert text.count(old) == 1, f"header text changed: {old}"
    with open(os.path.join(inc, "mom_gemm_schedule.h"), "w") as f:
        f.write(text.replace(old, new))
    r = _build_and_run(str(tmp_path), inc)
    assert r.returncode != 0, f"planted {what} mistake not caught:\n{r.stdout}"
