"""CPU oracle for the MOM prefill hot path (test infrastructure only).

Thin ctypes wrapper over `mom_oracle.c`; all arithmetic lives in the C file,
whose header states what it follows in the paper.  bf16 tensors travel as
numpy uint16 bit patterns.  Only tests, the smoke check and the benchmark's
cpu_baseline leg may import this package; the product path never does.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        # MOM_ORACLE_SANITIZED=1: the AddressSanitizer / UBSan build (the sanitizer run of the tests)
        lib = ctypes.CDLL(_build.build(force=False, sanitize=os.environ.get("MOM_ORACLE_SANITIZED") == "1"))
        u16p = ctypes.POINTER(ctypes.c_uint16)
        f32p = ctypes.POINTER(ctypes.c_float)
        i64p = ctypes.POINTER(ctypes.c_int64)
        i64 = ctypes.c_int64
        lib.oracle_bf16_to_f32.restype = ctypes.c_float
        lib.oracle_bf16_to_f32.argtypes = [ctypes.c_uint16]
        lib.oracle_f32_to_bf16.restype = ctypes.c_uint16
        lib.oracle_f32_to_bf16.argtypes = [ctypes.c_float]
        lib.oracle_silu_f32.restype = ctypes.c_float
        lib.oracle_silu_f32.argtypes = [ctypes.c_float]
        lib.oracle_silu_f64.restype = ctypes.c_double
        lib.oracle_silu_f64.argtypes = [ctypes.c_double]
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_set_num_threads.argtypes = [ctypes.c_int]
        lib.oracle_mlp_rows.restype = ctypes.c_int
        lib.oracle_mlp_rows.argtypes = [u16p, u16p, u16p, u16p, i64, i64, i64, i64p, i64,
                                        ctypes.c_int, ctypes.c_int, f32p]
        lib.oracle_mlp_miniseq.restype = ctypes.c_int
        lib.oracle_mlp_miniseq.argtypes = [u16p, u16p, u16p, u16p, i64, i64, i64, i64, f32p, i64p]
        lib.oracle_lmhead.restype = ctypes.c_int
        lib.oracle_lmhead.argtypes = [u16p, u16p, i64, i64, ctypes.c_int, f32p]
        lib.oracle_last_token.restype = ctypes.c_int
        lib.oracle_last_token.argtypes = [u16p, u16p, u16p, u16p, u16p, i64, i64, i64, i64,
                                          ctypes.c_int, f32p, f32p]
        _lib = lib
    return _lib


def _u16(a, shape):
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16:
        raise TypeError("bf16 tensors are passed as uint16 bit patterns")
    if tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(a.shape)}")
    return a


def _p(a, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def bf16_to_f32(b):
    return float(_load().oracle_bf16_to_f32(int(b)))


def f32_to_bf16(f):
    return int(_load().oracle_f32_to_bf16(float(np.float32(f))))


def silu_f32(g):
    return float(_load().oracle_silu_f32(float(np.float32(g))))


def silu_f64(g):
    return float(_load().oracle_silu_f64(float(g)))


def num_threads():
    return int(_load().oracle_num_threads())


def set_num_threads(n):
    _load().oracle_set_num_threads(int(n))


def mlp_rows(x, W_gate, W_up, W_down, rows=None, acc64=False, round_h=False):
    """Unchunked SwiGLU MLP (Section 3.3) on all rows, or on `rows` only.

    x [S,H], W_gate/W_up [I,H], W_down [H,I] as uint16 bf16 bits -> float32 [n,H].
    """
    lib = _load()
    S, H = x.shape
    I = W_gate.shape[0]
    x = _u16(x, (S, H)); wg = _u16(W_gate, (I, H)); wu = _u16(W_up, (I, H)); wd = _u16(W_down, (H, I))
    if rows is None:
        n, rp = S, None
    else:
        r = np.ascontiguousarray(np.asarray(rows, dtype=np.int64))
        n, rp = int(r.size), _p(r, ctypes.c_int64)
    out = np.empty((n, H), dtype=np.float32)
    rc = lib.oracle_mlp_rows(_p(x, ctypes.c_uint16), _p(wg, ctypes.c_uint16), _p(wu, ctypes.c_uint16),
                             _p(wd, ctypes.c_uint16), S, H, I, rp, n, int(acc64), int(round_h),
                             _p(out, ctypes.c_float))
    if rc:
        raise ValueError("oracle_mlp_rows rejected its arguments")
    return out


def mlp_miniseq(x, W_gate, W_up, W_down, mini_seq):
    """Algorithm 1 else-branch: loop over mini-sequences of `mini_seq` rows with one
    reused intermediate.  Returns (out float32 [S,H], peak intermediate elements)."""
    lib = _load()
    S, H = x.shape
    I = W_gate.shape[0]
    x = _u16(x, (S, H)); wg = _u16(W_gate, (I, H)); wu = _u16(W_up, (I, H)); wd = _u16(W_down, (H, I))
    out = np.empty((S, H), dtype=np.float32)
    peak = ctypes.c_int64(0)
    rc = lib.oracle_mlp_miniseq(_p(x, ctypes.c_uint16), _p(wg, ctypes.c_uint16), _p(wu, ctypes.c_uint16),
                                _p(wd, ctypes.c_uint16), S, H, I, int(mini_seq),
                                _p(out, ctypes.c_float), ctypes.byref(peak))
    if rc:
        raise ValueError("oracle_mlp_miniseq rejected its arguments")
    return out, int(peak.value)


def lmhead(x_last, W_lm, acc64=False):
    """logits[v] = sum_k x_last[k] W_lm[v,k]; x_last [H], W_lm [V,H] uint16 -> float32 [V]."""
    lib = _load()
    V, H = W_lm.shape
    xl = _u16(x_last, (H,)); w = _u16(W_lm, (V, H))
    out = np.empty((V,), dtype=np.float32)
    rc = lib.oracle_lmhead(_p(xl, ctypes.c_uint16), _p(w, ctypes.c_uint16), V, H, int(acc64),
                           _p(out, ctypes.c_float))
    if rc:
        raise ValueError("oracle_lmhead rejected its arguments")
    return out


def last_token(A, W_gate, W_up, W_down, W_lm, acc64=False):
    """Algorithm 1 if-branch: last row of A -> MLP -> (bf16) -> LM head.
    Returns (o_last float32 [H], logits float32 [V])."""
    lib = _load()
    S, H = A.shape
    I = W_gate.shape[0]
    V = W_lm.shape[0]
    A = _u16(A, (S, H)); wg = _u16(W_gate, (I, H)); wu = _u16(W_up, (I, H)); wd = _u16(W_down, (H, I))
    wl = _u16(W_lm, (V, H))
    o = np.empty((H,), dtype=np.float32)
    lg = np.empty((V,), dtype=np.float32)
    rc = lib.oracle_last_token(_p(A, ctypes.c_uint16), _p(wg, ctypes.c_uint16), _p(wu, ctypes.c_uint16),
                               _p(wd, ctypes.c_uint16), _p(wl, ctypes.c_uint16), S, H, I, V, int(acc64),
                               _p(o, ctypes.c_float), _p(lg, ctypes.c_float))
    if rc:
        raise ValueError("oracle_last_token rejected its arguments")
    return o, lg
