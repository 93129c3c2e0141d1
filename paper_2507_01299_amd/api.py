"""ctypes binding over liblarosa.so: argument marshalling only.

Every function mirrors the C entry point of the same name (include/larosa.h).  Tensors are
torch CUDA tensors used purely as device buffers: 16-bit data as torch.float16 /
torch.bfloat16 (or uint16/int16 bit patterns), indices as torch.int32.  Work is enqueued on
torch's current stream.  A missing library is an error; there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblarosa.so")

F16, BF16 = 0, 1
OK, EINVAL, EUNSUPPORTED, EWORKSPACE, EHIP = 0, -1, -2, -3, -4

_lib = None


class LarosaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


class _Layer(ctypes.Structure):
    _fields_ = [
        ("d", ctypes.c_int), ("d_q", ctypes.c_int), ("d_kv", ctypes.c_int), ("d_ff", ctypes.c_int),
        ("head_dim", ctypes.c_int),
        ("K1", ctypes.c_int), ("K2", ctypes.c_int), ("K3", ctypes.c_int), ("K4", ctypes.c_int),
        ("Wqkv", ctypes.c_void_p), ("Wo", ctypes.c_void_p), ("Wgu", ctypes.c_void_p), ("Wdown", ctypes.c_void_p),
        ("Q_attn", ctypes.c_void_p), ("Q_mlp", ctypes.c_void_p), ("adapter", ctypes.c_void_p),
        ("rms_attn", ctypes.c_void_p), ("rms_mlp", ctypes.c_void_p),
        ("rms_eps", ctypes.c_float), ("attn_mode", ctypes.c_int), ("dtype", ctypes.c_int),
        ("shortcut_attn", ctypes.c_void_p), ("shortcut_mlp", ctypes.c_void_p),
    ]


TRACE_FIELDS = ("h1", "qkv", "h2", "o", "x1", "h3", "gu", "h4", "down", "x2", "idx1", "idx2", "idx3", "idx4",
                "s1", "s2")


class _Trace(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in TRACE_FIELDS] + [("stage_events", ctypes.c_void_p * 8)]


def lib() -> ctypes.CDLL:
    """Load liblarosa.so (built in-tree by paper_2507_01299_amd.build); raise if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2507_01299_amd.build` "
                               "(or __graft_entry__.build()) first; there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        L.larosa_status_string.restype = ctypes.c_char_p
        L.larosa_status_string.argtypes = [i]
        L.larosa_version.restype = i
        L.larosa_workspace_bytes.restype = sz
        L.larosa_workspace_bytes.argtypes = [i, i, i, i]
        L.larosa_workspace_init.argtypes = [vp, sz, vp]
        L.larosa_rotate.argtypes = [vp, vp, vp, i, i, i, vp, sz, vp]
        L.larosa_dense_gemv.argtypes = [vp, vp, vp, i, i, i, i, vp, sz, vp]
        L.larosa_topk.argtypes = [vp, i, i, i, vp, vp, i, vp, sz, vp]
        L.larosa_sparse_gemv.argtypes = [vp, vp, vp, vp, i, i, i, i, i, vp, sz, vp]
        L.larosa_sparse_gemv_static.argtypes = [vp, vp, vp, vp, i, i, i, i, i, vp]
        L.larosa_layer_workspace_bytes.restype = sz
        L.larosa_layer_workspace_bytes.argtypes = [ctypes.POINTER(_Layer), i]
        L.larosa_layer_forward.argtypes = [ctypes.POINTER(_Layer), vp, vp, i, ctypes.POINTER(_Trace), vp, sz, vp]
        L.larosa_layer_qkv.argtypes = [ctypes.POINTER(_Layer), vp, vp, vp, i, ctypes.POINTER(_Trace), vp, sz, vp]
        L.larosa_layer_after_attention.argtypes = [ctypes.POINTER(_Layer), vp, vp, vp, i, ctypes.POINTER(_Trace), vp,
                                                   sz, vp]
        L.larosa_set_tuning.argtypes = [i, i]
        L.larosa_quantize_w4.argtypes = [vp, i, i, i, vp, vp, vp]
        L.larosa_sparse_gemv_w4.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, vp, sz, vp]
        L.larosa_threshold_select.argtypes = [vp, i, i, ctypes.c_float, i, vp, vp, vp]
        L.larosa_offline_workspace_bytes.restype = sz
        L.larosa_offline_workspace_bytes.argtypes = [i, i]
        L.larosa_second_moment.argtypes = [vp, i, i, i, vp, i, vp]
        L.larosa_fold_input.argtypes = [vp, vp, i, i, i, vp, vp, sz, vp]
        L.larosa_fold_output.argtypes = [vp, vp, i, i, i, vp, vp, sz, vp]
        L.larosa_residual_adapter.argtypes = [vp, vp, i, i, vp, vp, sz, vp]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().larosa_status_string(int(status)).decode()


def version() -> int:
    return lib().larosa_version()


def dtype_code(t) -> int:
    if t in (F16, "f16", torch.float16):
        return F16
    if t in (BF16, "bf16", torch.bfloat16):
        return BF16
    raise ValueError(f"unsupported dtype {t}")


def torch_dtype(code) -> torch.dtype:
    return torch.float16 if dtype_code(code) == F16 else torch.bfloat16


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc: int, where: str):
    if rc != OK:
        raise LarosaError(rc, where)


class Workspace:
    """A caller-owned device buffer passed once through larosa_workspace_init."""

    def __init__(self, nbytes: int, device="cuda:0"):
        self.nbytes = int(nbytes)
        self.buf = torch.empty(self.nbytes + 256, dtype=torch.uint8, device=device)
        off = (-self.buf.data_ptr()) % 256
        self.ptr = self.buf.data_ptr() + off
        _check(lib().larosa_workspace_init(ctypes.c_void_p(self.ptr), self.nbytes, _stream()), "larosa_workspace_init")


def workspace_bytes(B: int, d_in_max: int, d_out_max: int, K_max: int) -> int:
    return lib().larosa_workspace_bytes(B, d_in_max, d_out_max, K_max)


def workspace(B: int, d_in_max: int, d_out_max: int, K_max: int, device="cuda:0") -> Workspace:
    return Workspace(workspace_bytes(B, d_in_max, d_out_max, K_max), device)


def set_tuning(key: int, value: int):
    _check(lib().larosa_set_tuning(key, value), "larosa_set_tuning")


def rotate(x, Q, h, dtype, ws: Workspace):
    B, d = x.shape
    _check(lib().larosa_rotate(_ptr(x), _ptr(Q), _ptr(h), B, d, dtype_code(dtype),
                               ctypes.c_void_p(ws.ptr), ws.nbytes, _stream()), "larosa_rotate")
    return h


def dense_gemv(Wp, x, y, dtype, ws: Workspace):
    B, d_in = x.shape
    d_out = Wp.shape[1]
    _check(lib().larosa_dense_gemv(_ptr(Wp), _ptr(x), _ptr(y), B, d_in, d_out, dtype_code(dtype),
                                   ctypes.c_void_p(ws.ptr), ws.nbytes, _stream()), "larosa_dense_gemv")
    return y


def topk(h, K: int, idx, dtype, vals=None, ws: Workspace | None = None):
    B, d = h.shape
    _check(lib().larosa_topk(_ptr(h), B, d, K, _ptr(idx), _ptr(vals), dtype_code(dtype),
                             ctypes.c_void_p(ws.ptr) if ws else None, ws.nbytes if ws else 0, _stream()),
           "larosa_topk")
    return idx


def sparse_gemv(Wp, h, idx, y, dtype, ws: Workspace):
    B, d_in = h.shape
    d_out = Wp.shape[1]
    K = idx.shape[1]
    _check(lib().larosa_sparse_gemv(_ptr(Wp), _ptr(h), _ptr(idx), _ptr(y), B, d_in, d_out, K, dtype_code(dtype),
                                    ctypes.c_void_p(ws.ptr), ws.nbytes, _stream()), "larosa_sparse_gemv")
    return y


def sparse_gemv_static(Wp, h, idx, y, dtype):
    """larosa_sparse_gemv without a workspace: the scratch is a fixed device array inside the library."""
    B, d_in = h.shape
    d_out = Wp.shape[1]
    K = idx.shape[1]
    _check(lib().larosa_sparse_gemv_static(_ptr(Wp), _ptr(h), _ptr(idx), _ptr(y), B, d_in, d_out, K,
                                           dtype_code(dtype), _stream()), "larosa_sparse_gemv_static")
    return y


def quantize_w4(W, dtype):
    """Round-to-nearest 4-bit codes (int32 [d_in, d_out/8], eight nibbles per dword) and 16-bit scales
    [d_in, ceil(d_out/128)] of W [d_in, d_out]."""
    d_in, d_out = W.shape
    Wq = torch.empty(d_in, d_out // 8, dtype=torch.int32, device=W.device)
    scales = torch.empty(d_in, (d_out + 127) // 128, dtype=W.dtype, device=W.device)
    _check(lib().larosa_quantize_w4(_ptr(W), d_in, d_out, dtype_code(dtype), _ptr(Wq), _ptr(scales), _stream()),
           "larosa_quantize_w4")
    return Wq, scales


def sparse_gemv_w4(Wq, scales, h, idx, y, dtype, ws: Workspace):
    B, d_in = h.shape
    d_out = Wq.shape[1] * 8
    K = d_in if idx is None else idx.shape[1]
    _check(lib().larosa_sparse_gemv_w4(_ptr(Wq), _ptr(scales), _ptr(h), _ptr(idx), _ptr(y), B, d_in, d_out, K,
                                       dtype_code(dtype), ctypes.c_void_p(ws.ptr), ws.nbytes, _stream()),
           "larosa_sparse_gemv_w4")
    return y


def threshold_select(h, eps: float, idx, count, dtype):
    """idx [B, d] int32, count [B] int32: per token the ascending channels with |h| > eps."""
    B, d = h.shape
    _check(lib().larosa_threshold_select(_ptr(h), B, d, float(eps), dtype_code(dtype), _ptr(idx), _ptr(count),
                                         _stream()), "larosa_threshold_select")
    return idx, count


class OfflineScratch:
    """Device scratch for the folding calls (16-bit terms of the fp32 rotations)."""

    def __init__(self, d: int, dtype, device="cuda:0"):
        self.nbytes = int(lib().larosa_offline_workspace_bytes(d, dtype_code(dtype)))
        self.buf = torch.empty(self.nbytes + 256, dtype=torch.uint8, device=device)
        self.ptr = self.buf.data_ptr() + (-self.buf.data_ptr()) % 256


def second_moment(X, C, dtype, accumulate: bool = False):
    """C [d,d] fp32 (+)= X^T X for X [n,d] 16-bit."""
    n, d = X.shape
    _check(lib().larosa_second_moment(_ptr(X), n, d, dtype_code(dtype), _ptr(C), int(accumulate), _stream()),
           "larosa_second_moment")
    return C


def fold_input(Q, W, W_out, dtype, scratch: OfflineScratch):
    """W_out [d,d_out] = Q^T W with Q [d,d] fp32."""
    d, d_out = W.shape
    _check(lib().larosa_fold_input(_ptr(Q), _ptr(W), d, d_out, dtype_code(dtype), _ptr(W_out),
                                   ctypes.c_void_p(scratch.ptr), scratch.nbytes, _stream()), "larosa_fold_input")
    return W_out


def fold_output(W, Q, W_out, dtype, scratch: OfflineScratch):
    """W_out [d_in,d] = W Q with Q [d,d] fp32."""
    d_in, d = W.shape
    _check(lib().larosa_fold_output(_ptr(W), _ptr(Q), d_in, d, dtype_code(dtype), _ptr(W_out),
                                    ctypes.c_void_p(scratch.ptr), scratch.nbytes, _stream()), "larosa_fold_output")
    return W_out


def residual_adapter(Q_l, Q_next, A_out, dtype, scratch: OfflineScratch):
    """A_out [d,d] = Q_l^T Q_next, both fp32."""
    d = Q_l.shape[0]
    _check(lib().larosa_residual_adapter(_ptr(Q_l), _ptr(Q_next), d, dtype_code(dtype), _ptr(A_out),
                                         ctypes.c_void_p(scratch.ptr), scratch.nbytes, _stream()),
           "larosa_residual_adapter")
    return A_out


class Layer:
    """Holds the device tensors of one decoder layer and the matching C struct."""

    def __init__(self, d, d_q, d_kv, d_ff, head_dim, K1, K2, K3, K4, Wqkv, Wo, Wgu, Wdown, dtype,
                 Q_attn=None, Q_mlp=None, adapter=None, rms_attn=None, rms_mlp=None, rms_eps=-1.0, attn_mode=0,
                 shortcut_attn=None, shortcut_mlp=None):
        self.tensors = dict(Wqkv=Wqkv, Wo=Wo, Wgu=Wgu, Wdown=Wdown, Q_attn=Q_attn, Q_mlp=Q_mlp,
                            adapter=adapter, rms_attn=rms_attn, rms_mlp=rms_mlp, shortcut_attn=shortcut_attn,
                            shortcut_mlp=shortcut_mlp)   # keep alive
        self.dtype = dtype_code(dtype)
        self.c = _Layer(d, d_q, d_kv, d_ff, head_dim, K1, K2, K3, K4,
                        *[None if t is None else t.data_ptr() for t in
                          (Wqkv, Wo, Wgu, Wdown, Q_attn, Q_mlp, adapter, rms_attn, rms_mlp)],
                        float(rms_eps), int(attn_mode), self.dtype,
                        None if shortcut_attn is None else shortcut_attn.data_ptr(),
                        None if shortcut_mlp is None else shortcut_mlp.data_ptr())

    def workspace_bytes(self, B: int) -> int:
        return lib().larosa_layer_workspace_bytes(ctypes.byref(self.c), B)

    def trace_buffers(self, B: int, device="cuda:0") -> dict:
        c, td = self.c, torch_dtype(self.dtype)
        w = dict(h1=c.d, qkv=c.d_q + 2 * c.d_kv, h2=c.d_q, o=c.d, x1=c.d, h3=c.d, gu=2 * c.d_ff, h4=c.d_ff,
                 down=c.d, x2=c.d)
        if c.shortcut_attn:
            w["s1"] = c.d
        if c.shortcut_mlp:
            w["s2"] = c.d
        out = {k: torch.zeros(B, v, dtype=td, device=device) for k, v in w.items()}
        for k, K in (("idx1", c.K1), ("idx2", c.K2), ("idx3", c.K3), ("idx4", c.K4)):
            out[k] = torch.full((B, K), -1, dtype=torch.int32, device=device)
        return out


def _trace_struct(trace: dict | None, stage_events=None):
    if trace is None and stage_events is None:
        return None
    trace = trace or {}
    tr = _Trace(*[None if trace.get(n) is None else trace[n].data_ptr() for n in TRACE_FIELDS])
    if stage_events is not None:
        for i, ev in enumerate(stage_events[:8]):
            tr.stage_events[i] = None if ev is None else ev.cuda_event
    return tr


def layer_forward(layer: Layer, x, x_out, ws: Workspace, trace: dict | None = None, stage_events=None):
    """stage_events: optional list of up to 8 torch.cuda.Event(enable_timing=True) that have been
    recorded once already (so their handles exist); the library records them at stage boundaries."""
    B = x.shape[0]
    tr = _trace_struct(trace, stage_events)
    _check(lib().larosa_layer_forward(ctypes.byref(layer.c), _ptr(x), _ptr(x_out), B,
                                      ctypes.byref(tr) if tr is not None else None,
                                      ctypes.c_void_p(ws.ptr), ws.nbytes, _stream()), "larosa_layer_forward")
    return x_out


def layer_qkv(layer: Layer, x, qkv, s1, ws: Workspace, trace: dict | None = None):
    """First half of the layer for a caller with its own attention core: writes q|k|v and, if the
    layer has shortcut_attn, the shortcut value s1 (else pass None)."""
    tr = _trace_struct(trace)
    _check(lib().larosa_layer_qkv(ctypes.byref(layer.c), _ptr(x), _ptr(qkv), _ptr(s1), x.shape[0],
                                  ctypes.byref(tr) if tr is not None else None,
                                  ctypes.c_void_p(ws.ptr), ws.nbytes, _stream()), "larosa_layer_qkv")
    return qkv


def layer_after_attention(layer: Layer, residual, attn, x_out, ws: Workspace, trace: dict | None = None):
    """Rest of the layer from the attention core's output attn [B, d_q]; residual is the layer input x,
    or the s1 written by layer_qkv when the layer has shortcut_attn."""
    tr = _trace_struct(trace)
    _check(lib().larosa_layer_after_attention(ctypes.byref(layer.c), _ptr(residual), _ptr(attn), _ptr(x_out),
                                              residual.shape[0], ctypes.byref(tr) if tr is not None else None,
                                              ctypes.c_void_p(ws.ptr), ws.nbytes, _stream()),
           "larosa_layer_after_attention")
    return x_out
