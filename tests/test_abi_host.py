"""Host-side checks that need no GPU: the C-ABI library loads, exports every symbol the header
declares, sizes its workspace per Eq. 3, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2504_12526_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "mom.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mom_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = binding.lib()
    names = _declared_symbols()
    assert set(names) == set(binding.SYMBOLS)
    for n in names:
        assert getattr(L, n) is not None


def test_status_strings():
    seen = {binding.status_string(s) for s in range(8)}
    assert len(seen) == 8 and "unknown status" not in seen
    assert binding.status_string(99) == "unknown status"


def test_workspace_bytes_is_eq3():
    wb = binding.mom_mlp_workspace_bytes
    for wl in synth.WORKLOADS.values():
        assert wb(wl.S, wl.H, wl.I, wl.mini_seq) == wl.mini_seq * wl.I * 2        # Eq. 3: C*I
        assert wb(wl.S, wl.H, wl.I, 0) == wl.S * wl.I * 2                         # Eq. 1: S*I
        assert wb(wl.S, wl.H, wl.I, wl.S + 1) == wl.S * wl.I * 2
    assert wb(100, 64, 96, 33) == 33 * 96 * 2
    assert wb(0, 64, 96, 8) == 0 and wb(10, 64, 96, -1) == 0


def _call(x=0x1000, wg=0x2000000, wu=0x3000000, wd=0x4000000, S=64, H=64, I=96, C=16, out=0x5000000,
          ws=0x6000000, wsb=None):
    if wsb is None:
        wsb = binding.mom_mlp_workspace_bytes(S, H, I, C)
    vp = ctypes.c_void_p
    return binding.lib().mom_mlp_prefill(vp(x), vp(wg), vp(wu), vp(wd), S, H, I, C, vp(out), vp(ws), wsb, None)


def test_mlp_argument_validation_happens_before_any_launch():
    # fake, never-dereferenced addresses: every case must return before touching HIP
    assert _call(S=-1) == binding.MOM_ERR_SHAPE
    assert _call(H=0) == binding.MOM_ERR_SHAPE
    assert _call(H=48) == binding.MOM_ERR_SHAPE
    assert _call(I=100) == binding.MOM_ERR_SHAPE
    assert _call(C=-2) == binding.MOM_ERR_SHAPE
    assert _call(x=0) == binding.MOM_ERR_NULL
    assert _call(ws=0) == binding.MOM_ERR_NULL
    assert _call(x=0x1008) == binding.MOM_ERR_ALIGN
    assert _call(out=0x5000004) == binding.MOM_ERR_ALIGN
    assert _call(wsb=15 * 96 * 2) == binding.MOM_ERR_WORKSPACE
    assert _call(out=0x1000) == binding.MOM_ERR_ALIAS                       # out == x
    assert _call(ws=0x2000000 + 64) == binding.MOM_ERR_ALIAS                # workspace inside W_gate
    assert _call(out=0x6000000 + 32) == binding.MOM_ERR_ALIAS               # out inside workspace
    assert _call(S=0, x=0, out=0, ws=0) == binding.MOM_OK                   # empty input: no-op


def test_pipelined_workspace_and_argument_validation():
    pb, wb = binding.mom_mlp_pipelined_workspace_bytes, binding.mom_mlp_workspace_bytes
    for wl in synth.WORKLOADS.values():
        assert pb(wl.S, wl.H, wl.I, wl.mini_seq) == 2 * wb(wl.S, wl.H, wl.I, wl.mini_seq)   # two halves, still O(C*I)
        assert pb(wl.S, wl.H, wl.I, 0) == wb(wl.S, wl.H, wl.I, 0)                           # one mini-sequence: one half
    assert pb(0, 64, 96, 8) == 0 and pb(10, 64, 96, -1) == 0
    vp = ctypes.c_void_p

    def call(x=0x1000, wg=0x2000000, wu=0x3000000, wd=0x4000000, S=64, H=64, I=96, C=16, out=0x5000000,
             ws=0x6000000, wsb=None, events=True, n_events=5):
        if wsb is None:
            wsb = pb(S, H, I, C)
        ev = (vp * 5)(*[vp(0x10 + i) for i in range(5)]) if events else None
        return binding.lib().mom_mlp_prefill_pipelined(vp(x), vp(wg), vp(wu), vp(wd), S, H, I, C, vp(out), vp(ws),
                                                       wsb, None, None, ev, n_events)
    assert call(H=48) == binding.MOM_ERR_SHAPE
    assert call(wu=0) == binding.MOM_ERR_NULL
    assert call(out=0x5000004) == binding.MOM_ERR_ALIGN
    assert call(wsb=wb(64, 64, 96, 16)) == binding.MOM_ERR_WORKSPACE          # one half is not enough
    assert call(ws=0x5000000 - 16 * 96 * 2 - 32) == binding.MOM_ERR_ALIAS    # second half runs into out
    assert call(events=False) == binding.MOM_ERR_NULL                         # several mini-sequences need events
    assert call(n_events=4) == binding.MOM_ERR_SHAPE                          # ... five of them
    assert call(S=0, x=0, out=0, ws=0) == binding.MOM_OK


def test_lmhead_and_offload_argument_validation():
    vp = ctypes.c_void_p
    L = binding.lib()
    assert L.mom_lmhead_last(vp(0x1000), vp(0x2000), 16, vp(0x900000), 40, None) == binding.MOM_ERR_SHAPE
    assert L.mom_lmhead_last(vp(0x1000), vp(0x2000), -1, vp(0x900000), 64, None) == binding.MOM_ERR_SHAPE
    assert L.mom_lmhead_last(vp(0x1000), vp(0x2000), 16, vp(0x900000), 65536, None) == binding.MOM_ERR_SHAPE
    assert L.mom_lmhead_last(None, vp(0x2000), 16, vp(0x900000), 64, None) == binding.MOM_ERR_NULL
    assert L.mom_lmhead_last(vp(0x1002), vp(0x2000), 16, vp(0x900000), 64, None) == binding.MOM_ERR_ALIGN
    assert L.mom_lmhead_last(vp(0x1000), vp(0x2000), 16, vp(0x2010), 64, None) == binding.MOM_ERR_ALIAS
    assert L.mom_lmhead_last(None, None, 0, None, 64, None) == binding.MOM_OK
    # last-token MLP: x [64], weights [96,64] / [64,96] at fake addresses
    def last(x=0x1000, wg=0x200000, wu=0x300000, wd=0x400000, H=64, I=96, out=0x500000, ws=0x600000, wsb=192):
        return L.mom_mlp_last(vp(x), vp(wg), vp(wu), vp(wd), H, I, vp(out), vp(ws), wsb, None)
    assert last(H=40) == binding.MOM_ERR_SHAPE
    assert last(I=65536) == binding.MOM_ERR_SHAPE
    assert last(wd=0) == binding.MOM_ERR_NULL
    assert last(out=0x500008) == binding.MOM_ERR_ALIGN
    assert last(wsb=191) == binding.MOM_ERR_WORKSPACE
    assert last(out=0x200010) == binding.MOM_ERR_ALIAS
    assert last(ws=0x500000 + 64) == binding.MOM_ERR_ALIAS
    assert L.mom_kv_reload(None, vp(0x10), vp(0x20), None, 16, None) == binding.MOM_ERR_NULL
    assert L.mom_kv_offload(None, vp(0x10), vp(0x20), None, 16, None, None, None) == binding.MOM_ERR_NULL
    assert L.mom_kv_offload(vp(0x10), vp(0x20), vp(0x30), None, 16, vp(0x1), None, None) == binding.MOM_ERR_NULL


def test_debug_overrides_validate_their_arguments():
    L = binding.lib()
    for ok in ((256, 0, 0), (256, 5, 0), (128, 5, 0), (128, 10, 0), (64, 5, 0), (64, 10, 0), (64, 20, 0), (128, 0, 0),
               (64, 0, 0), (256, 0, 224), (256, 5, 224), (256, 5, 192), (256, 5, 160), (256, 5, 128), (256, 5, 256),
               (0, 0, 0)):
        assert L.mom_debug_force_gemm_form(*ok) == binding.MOM_OK
    for bad in ((100, 0, 0), (256, 10, 0), (128, 20, 0), (64, 3, 0), (0, 5, 0), (-64, 0, 0), (224, 5, 0), (128, 5, 128),
                (256, 5, 96), (0, 0, 224)):
        assert L.mom_debug_force_gemm_form(*bad) == binding.MOM_ERR_SHAPE
    assert L.mom_debug_force_pipeline(1) == binding.MOM_OK and L.mom_debug_force_pipeline(0) == binding.MOM_OK


def test_product_reads_no_environment_variables():
    pkg = os.path.join(ROOT, "paper_2504_12526_amd", "csrc")
    for f in os.listdir(pkg):
        assert "getenv" not in open(os.path.join(pkg, f)).read(), f


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2504_12526_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".inc", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"import\s+oracle|from\s+oracle|oracle\.|oracle/|mom_oracle", text), f


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)
