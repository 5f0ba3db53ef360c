"""Seeded synthetic inputs for the MOM prefill path.

Input generation only: nothing here evaluates any step of the method.  Both the
GPU tests/benchmark and the CPU oracle's tests draw their tensors from this
module, so that the two sides see the same bits.

Recipe.  Tensor number t (x=0, W_gate=1, W_up=2, W_down=3, W_lm=4, k=5, v=6,
x_last=7) of a workload with seed s is drawn from its own
`torch.Generator(device).manual_seed(1000*s + t)` as float32 standard normals,
in row blocks, scaled by the tensor's standard deviation, optionally
row-normalised to unit RMS (x / sqrt(mean(x^2) + 1e-5), float32), and rounded
once to bf16 with round-to-nearest-even (torch's conversion).  The same
(seed, device kind) always gives the same bits; CPU and GPU generators give
different streams, so a test draws each tensor once and hands copies of those
very bits to both sides.

The shapes are the MLP / LM-head / KV shapes of the model families the paper
evaluates (Llama-3-8B, Qwen2.5-7B, Mistral); the values are synthetic stand-ins
for trained weights and real activations, which are not available offline.
"""
from dataclasses import dataclass

import numpy as np
import torch

TENSOR_IDS = {"x": 0, "W_gate": 1, "W_up": 2, "W_down": 3, "W_lm": 4, "k": 5, "v": 6, "x_last": 7}


@dataclass(frozen=True)
class Workload:
    name: str
    S: int
    H: int
    I: int
    mini_seq: int
    V: int = 0            # 0: no LM head in this workload
    kv_heads: int = 0     # 0: no KV offload in this workload
    head_dim: int = 128
    rms_norm_x: bool = False
    seed: int = 0
    w_std: float = 0.02


# The benchmark configurations, in order: a tiny correctness case, then layer shapes of the model families the paper evaluates.
WORKLOADS = {
    "tiny": Workload("tiny", S=512, H=256, I=1024, mini_seq=128, V=4096),
    "llama3_8b_32k": Workload("llama3_8b_32k", S=32768, H=4096, I=14336, mini_seq=4096,
                              rms_norm_x=True),
    "llama3_8b_128k": Workload("llama3_8b_128k", S=131072, H=4096, I=14336, mini_seq=8192,
                               V=128256, kv_heads=8),
    "qwen25_7b_256k": Workload("qwen25_7b_256k", S=262144, H=3584, I=18944, mini_seq=8192,
                               V=152064),
    "mistral_7b_448k": Workload("mistral_7b_448k", S=458752, H=4096, I=14336, mini_seq=16384,
                                kv_heads=8),
}


def normal_bf16(name, shape, seed, std=1.0, device="cpu", rms_norm_rows=False, block_rows=16384):
    """bf16 tensor `name` of a workload, per the module recipe."""
    shape = tuple(int(d) for d in shape)
    gen = torch.Generator(device=device)
    gen.manual_seed(1000 * int(seed) + TENSOR_IDS[name])
    out = torch.empty(shape, dtype=torch.bfloat16, device=device)
    if out.numel() == 0:
        return out
    flat = out.view(shape[0], -1) if len(shape) > 1 else out.view(1, -1)
    rows = flat.shape[0]
    for r0 in range(0, rows, block_rows):
        r1 = min(rows, r0 + block_rows)
        blk = torch.randn((r1 - r0, flat.shape[1]), generator=gen, device=device, dtype=torch.float32)
        if std != 1.0:
            blk *= std
        if rms_norm_rows:
            blk /= torch.sqrt(torch.mean(blk * blk, dim=1, keepdim=True) + 1e-5)
        flat[r0:r1] = blk.to(torch.bfloat16)
    return out


def mlp_inputs(wl, device="cpu", S=None):
    """x [S,H], W_gate [I,H], W_up [I,H], W_down [H,I] for workload `wl` (bf16 tensors)."""
    S = wl.S if S is None else int(S)
    x = normal_bf16("x", (S, wl.H), wl.seed, 1.0, device, rms_norm_rows=wl.rms_norm_x)
    wg = normal_bf16("W_gate", (wl.I, wl.H), wl.seed, wl.w_std, device)
    wu = normal_bf16("W_up", (wl.I, wl.H), wl.seed, wl.w_std, device)
    wd = normal_bf16("W_down", (wl.H, wl.I), wl.seed, wl.w_std, device)
    return x, wg, wu, wd


def lmhead_inputs(wl, device="cpu"):
    """x_last [H] ~ N(0,1), W_lm [V,H] ~ N(0, w_std) (bf16 tensors)."""
    xl = normal_bf16("x_last", (wl.H,), wl.seed, 1.0, device)
    w = normal_bf16("W_lm", (wl.V, wl.H), wl.seed, wl.w_std, device)
    return xl, w


def kv_inputs(wl, device="cpu", S=None):
    """k, v [S, kv_heads, head_dim] ~ N(0,1) (bf16 tensors)."""
    S = wl.S if S is None else int(S)
    k = normal_bf16("k", (S, wl.kv_heads, wl.head_dim), wl.seed, 1.0, device)
    v = normal_bf16("v", (S, wl.kv_heads, wl.head_dim), wl.seed, 1.0, device)
    return k, v


def bits(t):
    """bf16 torch tensor -> numpy uint16 bit patterns (host copy)."""
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def from_bits(a, device="cpu"):
    """numpy uint16 bit patterns -> bf16 torch tensor on `device`."""
    a = np.ascontiguousarray(a, dtype=np.uint16)
    return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).to(device)


def bits_to_f64(a):
    """numpy uint16 bf16 bit patterns -> float64 values (exact widening)."""
    a = np.ascontiguousarray(a, dtype=np.uint16)
    return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def parity_rows(S, mini_seq, n_random=128, seed=0, residues=256):
    """Row sample for big-S parity: first/last row of every mini-sequence (both sides of
    every boundary), seeded random rows, and for every residue class r mod `residues` one seeded
    random row of that class (so that a sample covers every row position of a `residues`-row tile
    of whoever computes the rows); sorted, unique."""
    C = S if (mini_seq <= 0 or mini_seq > S) else mini_seq
    rows = {0, S - 1}
    for r0 in range(0, S, C):
        rows.add(r0)
        rows.add(min(S, r0 + C) - 1)
    rng = np.random.default_rng(seed)
    rows.update(int(r) for r in rng.integers(0, S, size=n_random))
    for rho in range(min(residues, S)):
        n_in_class = (S - 1 - rho) // residues + 1
        rows.add(rho + residues * int(rng.integers(0, n_in_class)))
    return np.array(sorted(r for r in rows if 0 <= r < S), dtype=np.int64)
