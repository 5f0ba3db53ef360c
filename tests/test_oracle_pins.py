"""Pins for the CPU oracle (no GPU).  Each check ties the oracle to something other than
itself: a closed form, a library routine in float64, a brute-force evaluation in pure Python,
or an invariant the method must have (row independence of Algorithm 1, linearity in W_down)."""
import math
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2504_12526_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_bits(rng, shape, std=1.0):
    t = torch.from_numpy(rng.standard_normal(shape).astype(np.float32) * std).to(torch.bfloat16)
    return synth.bits(t)


def _ref_mlp_f64(x, wg, wu, wd):
    """float64 library evaluation of Section 3.3's formula: three matmuls and an elementwise map."""
    X = synth.bits_to_f64(x); G = synth.bits_to_f64(wg); U = synth.bits_to_f64(wu); D = synth.bits_to_f64(wd)
    g = X @ G.T
    u = X @ U.T
    h = g / (1.0 + np.exp(-g)) * u
    return h @ D.T


# ---------------------------------------------------------------- bf16 conversion

def test_bf16_widen_all_patterns_match_library():
    allb = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    ref = synth.from_bits(allb).to(torch.float32).numpy()
    got = np.array([oracle.bf16_to_f32(int(b)) for b in allb], dtype=np.float32)
    nan = np.isnan(ref)           # NaN payloads do not survive the trip through a Python float
    assert np.array_equal(np.isnan(got), nan) and nan.sum() == 2 * 127
    assert np.array_equal(got.view(np.uint32)[~nan], ref.view(np.uint32)[~nan])


def test_f32_to_bf16_is_round_to_nearest_even():
    rng = np.random.default_rng(1)
    vals = np.concatenate([
        rng.standard_normal(20000).astype(np.float32),
        (rng.standard_normal(2000) * 1e-39).astype(np.float32),      # subnormals
        (rng.standard_normal(2000) * 1e38).astype(np.float32),
        np.array([0.0, -0.0, np.inf, -np.inf, 3.3895314e38, 65280.0], dtype=np.float32),
    ])
    # exact ties: bf16 value plus half a bf16 ulp
    base = rng.integers(0, 0x7f00, size=4000).astype(np.uint32)
    ties = ((base << 16) | 0x8000).view(np.float32)
    vals = np.concatenate([vals, ties, -ties])
    ref = synth.bits(torch.from_numpy(vals).to(torch.bfloat16))
    got = np.array([oracle.f32_to_bf16(v) for v in vals], dtype=np.uint16)
    assert np.array_equal(got, ref)
    # hand cases: 1 + 2^-8 is a tie -> even (1.0); 1 + 3*2^-8 is a tie -> rounds up to 1 + 2^-6
    assert oracle.f32_to_bf16(1.0 + 2.0 ** -8) == 0x3F80
    assert oracle.f32_to_bf16(1.0 + 3 * 2.0 ** -8) == 0x3F82
    assert oracle.f32_to_bf16(1.0 + 2.0 ** -8 + 2.0 ** -20) == 0x3F81
    nan_b = oracle.f32_to_bf16(float("nan"))
    assert (nan_b & 0x7F80) == 0x7F80 and (nan_b & 0x7F) != 0


# ---------------------------------------------------------------- SiLU closed forms

def _golden_silu():
    d = {}
    for line in open(os.path.join(GOLDEN, "silu_constants.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split()
        d[k] = float(v)
    return d


def test_silu_closed_forms():
    g = _golden_silu()
    assert oracle.silu_f32(0.0) == 0.0 and oracle.silu_f64(0.0) == 0.0
    for name, x in [("s(1)", 1.0), ("s(-1)", -1.0), ("s(20)", 20.0), ("s(-20)", -20.0)]:
        assert oracle.silu_f64(x) == pytest.approx(g[name], rel=1e-15)
        assert oracle.silu_f32(x) == pytest.approx(g[name], rel=3e-7)
    # minimum: value and location (scan around the stationary point)
    assert oracle.silu_f64(g["argmin"]) == pytest.approx(g["min"], rel=1e-15)
    xs = np.linspace(-3, 1, 4001)
    ys = np.array([oracle.silu_f64(x) for x in xs])
    assert abs(xs[ys.argmin()] - g["argmin"]) < 1e-3
    assert ys.min() >= g["min"] - 1e-15
    # antisymmetric part: s(x) - s(-x) = x
    for x in np.linspace(-30, 30, 121):
        assert oracle.silu_f64(x) - oracle.silu_f64(-x) == pytest.approx(x, abs=1e-14)
        assert oracle.silu_f32(x) - oracle.silu_f32(-x) == pytest.approx(x, abs=4e-6 * max(1, abs(x)))
    # slope 1/2 at the origin
    assert oracle.silu_f64(1e-6) / 1e-6 == pytest.approx(0.5, abs=1e-6)


def test_silu_matches_library_and_has_no_nan():
    xs = np.linspace(-40, 40, 1601).astype(np.float32).astype(np.float64)   # exact in float
    ref = torch.nn.functional.silu(torch.from_numpy(xs)).numpy()
    got64 = np.array([oracle.silu_f64(x) for x in xs])
    got32 = np.array([oracle.silu_f32(x) for x in xs])
    assert np.allclose(got64, ref, rtol=1e-14, atol=1e-300)
    assert np.allclose(got32, ref, rtol=1e-6, atol=1e-30)
    for x in [88.0, 89.0, 104.0, 1e4, 3e38, -88.0, -89.0, -104.0, -1e4, -3e38]:
        y = oracle.silu_f32(x)
        assert not math.isnan(y)
        assert (y == pytest.approx(x, rel=1e-6)) if x > 0 else (abs(y) < 1e-30)


# ---------------------------------------------------------------- MLP definition

def test_mlp_brute_force_pure_python():
    rng = np.random.default_rng(2)
    S, H, I = 3, 5, 4      # no dimension equals another: a transposed operand cannot pass
    x = _rand_bits(rng, (S, H)); wg = _rand_bits(rng, (I, H), 0.5)
    wu = _rand_bits(rng, (I, H), 0.5); wd = _rand_bits(rng, (H, I), 0.5)
    X = synth.bits_to_f64(x).tolist(); G = synth.bits_to_f64(wg).tolist()
    U = synth.bits_to_f64(wu).tolist(); D = synth.bits_to_f64(wd).tolist()
    ref = [[0.0] * H for _ in range(S)]
    for m in range(S):
        h = []
        for j in range(I):
            g = sum(X[m][k] * G[j][k] for k in range(H))
            u = sum(X[m][k] * U[j][k] for k in range(H))
            h.append(g / (1.0 + math.exp(-g)) * u)
        for i in range(H):
            ref[m][i] = sum(h[j] * D[i][j] for j in range(I))
    ref = np.array(ref)
    assert np.allclose(oracle.mlp_rows(x, wg, wu, wd, acc64=True), ref, rtol=2e-7, atol=1e-9)
    assert np.allclose(oracle.mlp_rows(x, wg, wu, wd, acc64=False), ref, rtol=2e-5, atol=1e-6)


@pytest.mark.parametrize("S,H,I", [(5, 32, 64), (17, 96, 160), (64, 256, 1024)])
def test_mlp_matches_float64_library_matmul(S, H, I):
    rng = np.random.default_rng(S + H + I)
    x = _rand_bits(rng, (S, H)); wg = _rand_bits(rng, (I, H), 0.05)
    wu = _rand_bits(rng, (I, H), 0.05); wd = _rand_bits(rng, (H, I), 0.05)
    ref = _ref_mlp_f64(x, wg, wu, wd)
    scale = np.abs(ref).max()
    e64 = np.abs(oracle.mlp_rows(x, wg, wu, wd, acc64=True) - ref).max() / scale
    e32 = np.abs(oracle.mlp_rows(x, wg, wu, wd, acc64=False) - ref).max() / scale
    assert e64 < 2e-7          # only the final float rounding
    assert e32 < 1e-5          # float sums: ~sqrt(K)*2^-24 typical, K*2^-24 worst case
    # the bf16-rounded-intermediate diagnostic stays within one bf16 rounding of h
    er = np.abs(oracle.mlp_rows(x, wg, wu, wd, acc64=True, round_h=True) - ref).max() / scale
    assert 0 < er < 2 ** -8


def test_mlp_tiny_workload_against_float64():
    wl = synth.WORKLOADS["tiny"]
    x, wg, wu, wd = (synth.bits(t) for t in synth.mlp_inputs(wl, S=48))
    ref = _ref_mlp_f64(x, wg, wu, wd)
    got = oracle.mlp_rows(x, wg, wu, wd)
    assert np.abs(got - ref).max() / np.abs(ref).max() < 1e-5


def test_mlp_one_hot_row_is_hand_checkable():
    rng = np.random.default_rng(3)
    S, H, I = 2, 8, 6
    wg = _rand_bits(rng, (I, H)); wu = _rand_bits(rng, (I, H)); wd = _rand_bits(rng, (H, I))
    x = np.zeros((S, H), dtype=np.uint16)
    k0 = 5
    x[1, k0] = 0x3F80                     # 1.0 in bf16; row 0 stays zero
    g = synth.bits_to_f64(wg)[:, k0]; u = synth.bits_to_f64(wu)[:, k0]
    h = g / (1 + np.exp(-g)) * u
    ref1 = synth.bits_to_f64(wd) @ h
    got = oracle.mlp_rows(x, wg, wu, wd, acc64=True)
    assert np.all(got[0] == 0.0)
    assert np.allclose(got[1], ref1, rtol=2e-7, atol=1e-9)


def test_mlp_zero_and_scaling_invariants():
    rng = np.random.default_rng(4)
    S, H, I = 6, 32, 48
    x = _rand_bits(rng, (S, H)); wg = _rand_bits(rng, (I, H), 0.1)
    wu = _rand_bits(rng, (I, H), 0.1); wd = _rand_bits(rng, (H, I), 0.1)
    base = oracle.mlp_rows(x, wg, wu, wd)
    assert np.all(oracle.mlp_rows(x, wg, np.zeros_like(wu), wd) == 0.0)
    assert np.all(oracle.mlp_rows(np.zeros_like(x), wg, wu, wd) == 0.0)
    # doubling W_down (exponent + 1 on every bf16) doubles the output exactly
    wd2 = synth.bits((synth.from_bits(wd).to(torch.float32) * 2).to(torch.bfloat16))
    assert np.array_equal(oracle.mlp_rows(x, wg, wu, wd2), 2.0 * base)
    # negating W_up negates the output exactly; negating W_gate does not (Swish is not odd)
    wun = wu ^ np.uint16(0x8000)
    assert np.array_equal(oracle.mlp_rows(x, wg, wun, wd), -base)
    assert not np.allclose(oracle.mlp_rows(x, wg ^ np.uint16(0x8000), wu, wd), -base)


def test_mlp_row_independence_and_subsets():
    rng = np.random.default_rng(5)
    S, H, I = 11, 32, 40
    x = _rand_bits(rng, (S, H)); wg = _rand_bits(rng, (I, H), 0.1)
    wu = _rand_bits(rng, (I, H), 0.1); wd = _rand_bits(rng, (H, I), 0.1)
    full = oracle.mlp_rows(x, wg, wu, wd)
    perm = rng.permutation(S)
    assert np.array_equal(oracle.mlp_rows(x[perm], wg, wu, wd), full[perm])
    rows = [10, 0, 3, 3]
    assert np.array_equal(oracle.mlp_rows(x, wg, wu, wd, rows=rows), full[rows])
    x2 = x.copy(); x2[4] = _rand_bits(rng, (H,))
    out2 = oracle.mlp_rows(x2, wg, wu, wd)
    changed = np.any(out2 != full, axis=1)
    assert changed[4] and changed.sum() == 1
    # permuting the intermediate index (rows of W_gate/W_up with columns of W_down) only reassociates
    p = rng.permutation(I)
    outp = oracle.mlp_rows(x, wg[p], wu[p], np.ascontiguousarray(wd[:, p]))
    assert np.allclose(outp, full, rtol=0, atol=1e-5 * np.abs(full).max())


@pytest.mark.parametrize("C", [0, 1, 3, 4, 7, 13, 14, 100])
def test_miniseq_equals_unchunked_bitwise(C):
    """Algorithm 1's loop over mini-sequences gives the very same numbers as the full-sequence
    formula (the paper's equivalence claim), and its intermediate is min(C,S)*I (Eq. 3 vs Eq. 1)."""
    rng = np.random.default_rng(6)
    S, H, I = 13, 24, 36
    x = _rand_bits(rng, (S, H)); wg = _rand_bits(rng, (I, H), 0.1)
    wu = _rand_bits(rng, (I, H), 0.1); wd = _rand_bits(rng, (H, I), 0.1)
    full = oracle.mlp_rows(x, wg, wu, wd)
    out, peak = oracle.mlp_miniseq(x, wg, wu, wd, C)
    assert np.array_equal(out.view(np.uint32), full.view(np.uint32))
    assert peak == (S if (C <= 0 or C > S) else C) * I


def test_memory_model_fixture_matches_eq1_eq3():
    for line in open(os.path.join(GOLDEN, "memory_model.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, S, I, C, full_b, mini_b = line.split()
        S, I, C, full_b, mini_b = int(S), int(I), int(C), int(full_b), int(mini_b)
        wl = synth.WORKLOADS[name]
        assert (wl.S, wl.I, wl.mini_seq) == (S, I, C)
        assert full_b == 2 * S * I and mini_b == 2 * S * I // math.ceil(S / C)


# ---------------------------------------------------------------- LM head / last token

def test_lmhead_identity_and_library():
    rng = np.random.default_rng(7)
    H, V = 48, 112
    xl = _rand_bits(rng, (H,))
    eye = np.zeros((V, H), dtype=np.uint16)
    for k in range(H):
        eye[2 * k + 1, k] = 0x3F80           # row 2k+1 selects x[k]; other rows are zero
    lg = oracle.lmhead(xl, eye)
    assert np.array_equal(lg[1:2 * H:2], synth.bits_to_f64(xl).astype(np.float32))
    assert np.all(lg[0::2] == 0) and np.all(lg[2 * H:] == 0)
    w = _rand_bits(rng, (V, H), 0.1)
    ref = synth.bits_to_f64(w) @ synth.bits_to_f64(xl)
    assert np.allclose(oracle.lmhead(xl, w, acc64=True), ref, rtol=2e-7, atol=1e-9)
    assert np.allclose(oracle.lmhead(xl, w, acc64=False), ref, rtol=0, atol=1e-5 * np.abs(ref).max())


def test_last_token_branch():
    """Algorithm 1 if-branch: only the last row of A reaches the MLP and the LM head."""
    rng = np.random.default_rng(8)
    S, H, I, V = 9, 32, 56, 80
    A = _rand_bits(rng, (S, H)); wg = _rand_bits(rng, (I, H), 0.1); wu = _rand_bits(rng, (I, H), 0.1)
    wd = _rand_bits(rng, (H, I), 0.1); wl = _rand_bits(rng, (V, H), 0.1)
    o, lg = oracle.last_token(A, wg, wu, wd, wl, acc64=True)
    ref_o = _ref_mlp_f64(A[-1:], wg, wu, wd)[0]
    assert np.allclose(o, ref_o, rtol=2e-7, atol=1e-9)
    ob = synth.bits(torch.from_numpy(ref_o.astype(np.float32)).to(torch.bfloat16))
    ref_l = synth.bits_to_f64(wl) @ synth.bits_to_f64(ob)
    assert np.allclose(lg, ref_l, rtol=0, atol=3e-3 * np.abs(ref_l).max())   # one bf16 ulp of o may flip
    A2 = A.copy(); A2[:-1] = _rand_bits(rng, (S - 1, H))
    o2, lg2 = oracle.last_token(A2, wg, wu, wd, wl, acc64=True)
    assert np.array_equal(o2, o) and np.array_equal(lg2, lg)


def test_oracle_rejects_bad_arguments():
    rng = np.random.default_rng(9)
    x = _rand_bits(rng, (4, 8)); wg = _rand_bits(rng, (6, 8)); wd = _rand_bits(rng, (8, 6))
    with pytest.raises(ValueError):
        oracle.mlp_rows(x, wg, wg, wd, rows=[4])
    with pytest.raises(ValueError):
        oracle.mlp_rows(x, wg, wg, wd.T)
    with pytest.raises(TypeError):
        oracle.mlp_rows(x.astype(np.float32), wg, wg, wd)


def test_synth_is_seeded_and_shaped():
    wl = synth.WORKLOADS["tiny"]
    a = synth.bits(synth.mlp_inputs(wl, S=16)[0]); b = synth.bits(synth.mlp_inputs(wl, S=16)[0])
    assert np.array_equal(a, b) and a.shape == (16, wl.H)
    wl2 = synth.WORKLOADS["llama3_8b_32k"]
    xr = synth.normal_bf16("x", (8, wl2.H), 0, rms_norm_rows=True).to(torch.float32)
    assert torch.allclose(xr.pow(2).mean(dim=1).sqrt(), torch.ones(8), atol=5e-3)
    w = synth.normal_bf16("W_gate", (512, 256), 0, std=0.02).to(torch.float32)
    assert abs(float(w.std()) - 0.02) < 1e-3
    rows = synth.parity_rows(1000, 256, n_random=16)
    for r in (0, 255, 256, 511, 512, 767, 768, 999):
        assert r in rows
