"""ctypes binding of libmom.so: same names as the C ABI, argument marshalling only.

Tensors are torch tensors used purely as device (or pinned host) buffers; every step of the
path runs in the library's HIP kernels.  There is no fallback: if the library has not been
built (`python -m paper_2504_12526_amd.build` or `__graft_entry__.build()`), importing the
symbols raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmom.so")

SYMBOLS = ("mom_status_string", "mom_mlp_workspace_bytes", "mom_mlp_prefill", "mom_mlp_prefill_events",
           "mom_mlp_pipelined_workspace_bytes", "mom_mlp_prefill_pipelined",
           "mom_lmhead_last", "mom_mlp_last", "mom_kv_offload", "mom_kv_reload",
           "mom_init", "mom_debug_force_gemm_form", "mom_debug_force_pipeline", "mom_mlp_prefill_static",
           "mom_debug_mfma_probe")

MOM_STATIC_WORKSPACE_BYTES = 64 << 20

(MOM_OK, MOM_ERR_NULL, MOM_ERR_SHAPE, MOM_ERR_ALIGN, MOM_ERR_ALIAS, MOM_ERR_WORKSPACE, MOM_ERR_HIP,
 MOM_ERR_HOST) = range(8)

_lib = None


class MomError(RuntimeError):
    def __init__(self, status, what):
        self.status = int(status)
        super().__init__(f"{what}: status {status} ({status_string(status)})")


def lib():
    """The loaded C-ABI library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build the HIP library first (python -m paper_2504_12526_amd.build)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_size_t
        L.mom_status_string.restype = ctypes.c_char_p
        L.mom_status_string.argtypes = [ctypes.c_int]
        L.mom_mlp_workspace_bytes.restype = sz
        L.mom_mlp_workspace_bytes.argtypes = [i64, i64, i64, i64]
        L.mom_mlp_prefill.restype = ctypes.c_int
        L.mom_mlp_prefill.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, vp, vp, sz, vp]
        L.mom_mlp_prefill_events.restype = ctypes.c_int
        L.mom_mlp_prefill_events.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, vp, vp, sz, vp,
                                             ctypes.POINTER(vp), i64]
        L.mom_mlp_pipelined_workspace_bytes.restype = sz
        L.mom_mlp_pipelined_workspace_bytes.argtypes = [i64, i64, i64, i64]
        L.mom_mlp_prefill_pipelined.restype = ctypes.c_int
        L.mom_mlp_prefill_pipelined.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, vp, vp, sz, vp, vp,
                                                ctypes.POINTER(vp), i64]
        L.mom_lmhead_last.restype = ctypes.c_int
        L.mom_lmhead_last.argtypes = [vp, vp, i64, vp, i64, vp]
        L.mom_kv_offload.restype = ctypes.c_int
        L.mom_kv_offload.argtypes = [vp, vp, vp, vp, sz, vp, vp, vp]
        L.mom_mlp_last.restype = ctypes.c_int
        L.mom_mlp_last.argtypes = [vp, vp, vp, vp, i64, i64, vp, vp, sz, vp]
        L.mom_kv_reload.restype = ctypes.c_int
        L.mom_kv_reload.argtypes = [vp, vp, vp, vp, sz, vp]
        L.mom_mlp_prefill_static.restype = ctypes.c_int
        L.mom_mlp_prefill_static.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, vp, vp]
        L.mom_init.restype = ctypes.c_int
        L.mom_init.argtypes = []
        L.mom_debug_force_gemm_form.restype = ctypes.c_int
        L.mom_debug_force_gemm_form.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int]
        L.mom_debug_mfma_probe.restype = ctypes.c_int
        L.mom_debug_mfma_probe.argtypes = [vp, sz, vp, sz, i64, ctypes.c_int, ctypes.c_int, vp, vp]
        L.mom_debug_force_pipeline.restype = ctypes.c_int
        L.mom_debug_force_pipeline.argtypes = [ctypes.c_int]
        _lib = L
    return _lib


def status_string(status):
    return lib().mom_status_string(int(status)).decode()


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _nbytes(t):
    return t.numel() * t.element_size()


def mom_mlp_workspace_bytes(S, H, I, mini_seq):
    return int(lib().mom_mlp_workspace_bytes(S, H, I, mini_seq))


def mom_mlp_prefill(x, W_gate, W_up, W_down, mini_seq, out, workspace, stream=None, check=True):
    """x [S,H], W_gate/W_up [I,H], W_down [H,I], out [S,H] bf16 device tensors; workspace any
    device tensor of at least mom_mlp_workspace_bytes bytes.  Enqueues on `stream`."""
    S, H = x.shape
    I = W_gate.shape[0]
    rc = lib().mom_mlp_prefill(_ptr(x), _ptr(W_gate), _ptr(W_up), _ptr(W_down), S, H, I, int(mini_seq),
                               _ptr(out), _ptr(workspace), _nbytes(workspace), _stream(stream))
    if check and rc != MOM_OK:
        raise MomError(rc, "mom_mlp_prefill")
    return rc


def mom_mlp_prefill_static(x, W_gate, W_up, W_down, mini_seq, out, stream=None, check=True):
    """mom_mlp_prefill with the library's own static workspace (at most MOM_STATIC_WORKSPACE_BYTES)."""
    S, H = x.shape
    I = W_gate.shape[0]
    rc = lib().mom_mlp_prefill_static(_ptr(x), _ptr(W_gate), _ptr(W_up), _ptr(W_down), S, H, I, int(mini_seq),
                                      _ptr(out), _stream(stream))
    if check and rc != MOM_OK:
        raise MomError(rc, "mom_mlp_prefill_static")
    return rc


def mom_mlp_prefill_events(x, W_gate, W_up, W_down, mini_seq, out, workspace, events, stream=None):
    """As mom_mlp_prefill, recording `events` (list of torch.cuda.Event(enable_timing=True),
    already recorded once so that their handles exist) around every kernel."""
    S, H = x.shape
    I = W_gate.shape[0]
    arr = (ctypes.c_void_p * len(events))(*[e.cuda_event for e in events])
    rc = lib().mom_mlp_prefill_events(_ptr(x), _ptr(W_gate), _ptr(W_up), _ptr(W_down), S, H, I, int(mini_seq),
                                      _ptr(out), _ptr(workspace), _nbytes(workspace), _stream(stream),
                                      arr, len(events))
    if rc != MOM_OK:
        raise MomError(rc, "mom_mlp_prefill_events")
    return rc


def mom_mlp_pipelined_workspace_bytes(S, H, I, mini_seq):
    return int(lib().mom_mlp_pipelined_workspace_bytes(int(S), int(H), int(I), int(mini_seq)))


def mom_mlp_prefill_pipelined(x, W_gate, W_up, W_down, mini_seq, out, workspace, stream, stream2, events,
                              check=True):
    """As mom_mlp_prefill with down(c) on stream2 beside gate/up(c+1) on stream; workspace of
    mom_mlp_pipelined_workspace_bytes; events: at least 5 torch.cuda.Event whose handles exist."""
    S, H = x.shape
    I = W_gate.shape[0]
    arr = None if events is None else (ctypes.c_void_p * len(events))(*[e.cuda_event for e in events])
    rc = lib().mom_mlp_prefill_pipelined(_ptr(x), _ptr(W_gate), _ptr(W_up), _ptr(W_down), S, H, I, int(mini_seq),
                                         _ptr(out), _ptr(workspace), _nbytes(workspace), _stream(stream),
                                         _stream(stream2), arr, 0 if events is None else len(events))
    if check and rc != MOM_OK:
        raise MomError(rc, "mom_mlp_prefill_pipelined")
    return rc


def mom_lmhead_last(x_last, W_lm, logits, stream=None, check=True):
    """x_last [H] bf16, W_lm [V,H] bf16, logits [V] fp32 device tensors."""
    V, H = W_lm.shape
    rc = lib().mom_lmhead_last(_ptr(x_last), _ptr(W_lm), V, _ptr(logits), H, _stream(stream))
    if check and rc != MOM_OK:
        raise MomError(rc, "mom_lmhead_last")
    return rc


def mom_init():
    rc = lib().mom_init()
    if rc != MOM_OK:
        raise MomError(rc, "mom_init")
    return rc


def mom_debug_force_gemm_form(tile_edge=0, ring_slots=0, tile_width=0):
    """Testing aid: force the tile form of the matrix-core kernels; (0, 0, 0) = the library's choice."""
    rc = lib().mom_debug_force_gemm_form(int(tile_edge), int(ring_slots), int(tile_width))
    if rc != MOM_OK:
        raise MomError(rc, "mom_debug_force_gemm_form")
    return rc


def mom_debug_force_pipeline(on):
    """Testing aid: make mom_mlp_prefill_pipelined always use its two-stream schedule."""
    return lib().mom_debug_force_pipeline(1 if on else 0)


def mom_debug_mfma_probe(a, b, iters, workgroups, sink, stream=None, order=0):
    """Measurement aid: register-only MFMA loop on operand fragments taken from bf16 tensors a and b
    (order 0: the kernels' back-to-back pairs, 1: K-half by K-half); returns the flop of the launch
    (time it with events on the stream)."""
    if sink.numel() < workgroups * 256 or sink.dtype != torch.float32:
        raise ValueError("sink must hold workgroups*256 float32")
    rc = lib().mom_debug_mfma_probe(_ptr(a), _nbytes(a), _ptr(b), _nbytes(b), int(iters), int(workgroups),
                                    int(order), _ptr(sink), _stream(stream))
    if rc != MOM_OK:
        raise MomError(rc, "mom_debug_mfma_probe")
    return float(workgroups) * 4 * int(iters) * 128 * 16384


def mom_kv_offload(k, v, pinned_host, stream, producer_stream=None, order_event=None, done_event=None,
                   check=True):
    """Copy device k, v (same byte size) to the pinned host tensor (k then v) on `stream`.
    With order_event the copy is ordered after the work already enqueued on producer_stream
    (None = the default stream); done_event is recorded after both copies."""
    nb = _nbytes(k)
    if _nbytes(v) != nb or _nbytes(pinned_host) < 2 * nb:
        raise ValueError("k and v must have equal byte size and pinned_host must hold both")
    rc = lib().mom_kv_offload(_ptr(k), _ptr(v), _ptr(pinned_host), _stream(stream), nb,
                              None if producer_stream is None else _stream(producer_stream),
                              None if order_event is None else ctypes.c_void_p(order_event.cuda_event),
                              None if done_event is None else ctypes.c_void_p(done_event.cuda_event))
    if check and rc != MOM_OK:
        raise MomError(rc, "mom_kv_offload")
    return rc


def mom_mlp_last(x_last, W_gate, W_up, W_down, out_last, workspace, stream=None, check=True):
    """x_last [H], W_gate/W_up [I,H], W_down [H,I], out_last [H] bf16 device tensors; workspace >= I*2 bytes."""
    I, H = W_gate.shape
    rc = lib().mom_mlp_last(_ptr(x_last), _ptr(W_gate), _ptr(W_up), _ptr(W_down), H, I, _ptr(out_last),
                            _ptr(workspace), _nbytes(workspace), _stream(stream))
    if check and rc != MOM_OK:
        raise MomError(rc, "mom_mlp_last")
    return rc


def mom_kv_reload(pinned_host, k, v, stream, done_event=None, check=True):
    """Copy k then v back from the pinned host tensor into the device tensors on `stream`."""
    nb = _nbytes(k)
    if _nbytes(v) != nb or _nbytes(pinned_host) < 2 * nb:
        raise ValueError("k and v must have equal byte size and pinned_host must hold both")
    rc = lib().mom_kv_reload(_ptr(pinned_host), _ptr(k), _ptr(v), _stream(stream), nb,
                             None if done_event is None else ctypes.c_void_p(done_event.cuda_event))
    if check and rc != MOM_OK:
        raise MomError(rc, "mom_kv_reload")
    return rc
