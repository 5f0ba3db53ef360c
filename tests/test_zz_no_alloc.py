"""mom_mlp_prefill_static - the entry point for callers that cannot allocate - against
mom_mlp_prefill, through the C ABI: the same kernels on the library's static workspace must give
the same bits, call after call, whatever the previous call left in that workspace."""
import ctypes

import pytest
import torch

from paper_2504_12526_amd import binding, synth

pytestmark = pytest.mark.gpu


def _raw_static(x, wg, wu, wd, mini_seq, out):
    """Straight through ctypes (no binding helper): pointers and sizes only."""
    S, H = x.shape
    vp = ctypes.c_void_p
    return binding.lib().mom_mlp_prefill_static(vp(x.data_ptr()), vp(wg.data_ptr()), vp(wu.data_ptr()),
                                                vp(wd.data_ptr()), S, H, wg.shape[0], mini_seq, vp(out.data_ptr()),
                                                vp(torch.cuda.current_stream().cuda_stream))


def _reference(x, wg, wu, wd, mini_seq):
    S, H = x.shape
    out = torch.empty_like(x)
    ws = torch.empty(binding.mom_mlp_workspace_bytes(S, H, wg.shape[0], mini_seq), dtype=torch.uint8, device=x.device)
    binding.mom_mlp_prefill(x, wg, wu, wd, mini_seq, out, ws)
    torch.cuda.synchronize()
    return out


def test_static_workspace_entry_point_matches_mom_mlp_prefill():
    assert torch.cuda.is_available(), "needs the MI355X"
    dev = torch.device("cuda:0")
    # first call: 3000 rows in mini-sequences of 1024 (ragged tail), I = 2048 -> 4 MiB of the static workspace
    big = synth.Workload("static_big", S=3000, H=512, I=2048, mini_seq=1024, seed=41, w_std=0.04)
    xb, wgb, wub, wdb = synth.mlp_inputs(big, device=dev)
    ref_big = _reference(xb, wgb, wub, wdb, big.mini_seq)
    # second call: a smaller input with other shapes, so it finds the first call's intermediate in the workspace
    small = synth.Workload("static_small", S=333, H=128, I=448, mini_seq=100, seed=42, w_std=0.05)
    xs, wgs, wus, wds = synth.mlp_inputs(small, device=dev)
    ref_small = _reference(xs, wgs, wus, wds, small.mini_seq)

    out_big = torch.zeros_like(xb)
    out_small = torch.zeros_like(xs)
    out_small0 = torch.zeros_like(xs)
    # set-up, once per device: the address of the static workspace is looked up here (the runtime
    # may map the array on this first use); nothing below may allocate
    assert binding.mom_init() == binding.MOM_OK
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    peak0 = torch.cuda.max_memory_allocated()
    # three calls in a row, nothing but the library between the two readings of the device's free
    # memory (torch's own comparisons below allocate temporaries, so they come afterwards)
    rc = [_raw_static(xb, wgb, wub, wdb, big.mini_seq, out_big),
          _raw_static(xs, wgs, wus, wds, small.mini_seq, out_small),
          _raw_static(xs, wgs, wus, wds, 0, out_small0)]           # the small one again, unchunked
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    peak1 = torch.cuda.max_memory_allocated()
    assert rc == [binding.MOM_OK] * 3
    assert free1 == free0 and peak1 == peak0                        # nothing was allocated
    assert torch.equal(out_big.view(torch.int16), ref_big.view(torch.int16))
    assert torch.equal(out_small.view(torch.int16), ref_small.view(torch.int16))
    assert torch.equal(out_small0.view(torch.int16), ref_small.view(torch.int16))

    # beyond the limit: refused, nothing enqueued, output untouched
    I_big = 14336
    C = binding.MOM_STATIC_WORKSPACE_BYTES // (2 * I_big) + 1
    wl = synth.Workload("static_over", S=C, H=64, I=I_big, mini_seq=0, seed=43)
    xo, wgo, wuo, wdo = synth.mlp_inputs(wl, device=dev)
    oo = torch.zeros_like(xo)
    assert _raw_static(xo, wgo, wuo, wdo, 0, oo) == binding.MOM_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert torch.count_nonzero(oo.view(torch.int16)).item() == 0
    # the same rows fit once they are cut into mini-sequences: exactly at the limit is accepted
    assert _raw_static(xo, wgo, wuo, wdo, C - 1, oo) == binding.MOM_OK
    torch.cuda.synchronize()
    assert torch.equal(oo.view(torch.int16), _reference(xo, wgo, wuo, wdo, C - 1).view(torch.int16))
    # empty input and bad shapes behave as in mom_mlp_prefill
    assert _raw_static(xo[:0], wgo, wuo, wdo, 16, oo[:0]) == binding.MOM_OK
    assert binding.mom_mlp_prefill_static(xo, wgo, wuo, wdo, -1, oo, check=False) == binding.MOM_ERR_SHAPE
    assert binding.mom_init() == binding.MOM_OK
