"""Thin ctypes binding of libmsla.so (the C ABI of include/msla.h).

Argument marshalling only: every step of the module runs in the HIP kernels.
PyTorch appears here solely as the owner of device memory and of the stream.
There is no CPU fallback: if the library is missing or not built for this GPU
the import of the symbols fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# MSLA_LIBRARY_PATH lets a tuning run point at another build of the same library
LIB_PATH = os.environ.get("MSLA_LIBRARY_PATH") or os.path.join(_HERE, "libmsla.so")

MSLA_OK = 0
MSLA_ERR_INVALID_ARG = -1
MSLA_ERR_UNSUPPORTED = -2
MSLA_ERR_WORKSPACE = -3
MSLA_ERR_LAUNCH = -4

MSLA_F32, MSLA_F16, MSLA_BF16 = 0, 1, 2
MSLA_NHWC, MSLA_NCHW = 0, 1

MSLA_OPT_GENERAL_AGGREGATION = 1
MSLA_OPT_STAGE_PROJECT, MSLA_OPT_STAGE_AGGREGATE, MSLA_OPT_STAGE_FINALIZE, MSLA_OPT_STAGE_APPLY = 2, 4, 8, 16
MSLA_OPT_STATE_VALU = 32

EXPORTS = ("msla_error_string", "msla_workspace_bytes", "msla_forward", "msla_forward_opts", "msla_forward_profiled",
           "msla_core_forward",
           "msla_multiscale_state", "msla_multiscale_state_static", "msla_linear",
           "msla_ffn_workspace_bytes", "msla_ffn_forward", "msla_block_workspace_bytes", "msla_block_forward",
           "msla_softmax_attention", "msla_linear_attention_backward_workspace_bytes",
           "msla_linear_attention_backward")

MSLA_ACT_RELU, MSLA_ACT_HSWISH = 0, 1

_DTYPES = {torch.float32: MSLA_F32, torch.float16: MSLA_F16, torch.bfloat16: MSLA_BF16}

_lib = None


class MslaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {error_string(status)}")


def load_library() -> ctypes.CDLL:
    """Load libmsla.so (building it first only if no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build(True)
    lib = ctypes.CDLL(LIB_PATH)
    vp, ip, i, f, sz = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int), ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    lib.msla_error_string.argtypes = [i]
    lib.msla_error_string.restype = ctypes.c_char_p
    lib.msla_workspace_bytes.argtypes = [i, i, i, i, i, i, ip, i, i, ctypes.POINTER(sz)]
    lib.msla_workspace_bytes.restype = i
    lib.msla_forward.argtypes = [vp, vp, vp, vp, vp, vp, vp, sz, i, i, i, i, i, i, ip, i, f, i, i, vp]
    lib.msla_forward.restype = i
    lib.msla_forward_opts.argtypes = lib.msla_forward.argtypes + [ctypes.c_uint]
    lib.msla_forward_opts.restype = i
    lib.msla_forward_profiled.argtypes = lib.msla_forward.argtypes + [ctypes.POINTER(vp)]
    lib.msla_forward_profiled.restype = i
    lib.msla_core_forward.argtypes = [vp, vp, vp, vp, vp, sz, i, i, i, i, i, ip, i, f, i, vp]
    lib.msla_core_forward.restype = i
    lib.msla_multiscale_state.argtypes = [vp, vp, vp, vp, vp, vp, sz, i, i, i, i, i, ip, i, i, vp]
    lib.msla_multiscale_state.restype = i
    lib.msla_multiscale_state_static.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, ip, i, i, vp]
    lib.msla_multiscale_state_static.restype = i
    lib.msla_ffn_workspace_bytes.argtypes = [i, i, i, i, i, i, ctypes.POINTER(sz)]
    lib.msla_ffn_workspace_bytes.restype = i
    lib.msla_ffn_forward.argtypes = [vp, vp, vp, vp, vp, vp, sz, i, i, i, i, i, i, i, vp]
    lib.msla_ffn_forward.restype = i
    lib.msla_block_workspace_bytes.argtypes = [i, i, i, i, i, i, ip, i, i, i, ctypes.POINTER(sz)]
    lib.msla_block_workspace_bytes.restype = i
    lib.msla_block_forward.argtypes = [vp] * 10 + [sz, i, i, i, i, i, i, ip, i, f, i, i, i, vp]
    lib.msla_block_forward.restype = i
    lib.msla_softmax_attention.argtypes = [vp, vp, i, i, i, i, i, vp]
    lib.msla_softmax_attention.restype = i
    lib.msla_linear_attention_backward_workspace_bytes.argtypes = [i, i, i, i, i, ctypes.POINTER(sz)]
    lib.msla_linear_attention_backward_workspace_bytes.restype = i
    lib.msla_linear_attention_backward.argtypes = [vp, vp, vp, vp, sz, i, i, i, i, f, i, vp]
    lib.msla_linear_attention_backward.restype = i
    lib.msla_linear.argtypes = [vp, vp, vp, ctypes.c_long, i, i, i, vp]
    lib.msla_linear.restype = i
    _lib = lib
    return lib


def error_string(status: int) -> str:
    return load_library().msla_error_string(int(status)).decode()


def _scales(scales: Sequence[int]):
    scales = [int(k) for k in scales]
    return (ctypes.c_int * max(1, len(scales)))(*scales), len(scales)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _dev(*ts):
    for t in ts:
        if t is not None:
            if not t.is_cuda:
                raise ValueError("msla: tensors must live in GPU memory")
            if not t.is_contiguous():
                raise ValueError("msla: tensors must be contiguous")


def _stream(stream) -> ctypes.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def msla_workspace_bytes(B, C, H, W, heads, head_dim, scales, dtype) -> int:
    sc, ns = _scales(scales)
    out = ctypes.c_size_t(0)
    st = load_library().msla_workspace_bytes(B, C, H, W, heads, head_dim, sc, ns, _DTYPES[dtype],
                                             ctypes.byref(out))
    if st != MSLA_OK:
        raise MslaError(st, "msla_workspace_bytes")
    return int(out.value)


def new_workspace(B, C, H, W, heads, head_dim, scales, dtype, device="cuda") -> torch.Tensor:
    n = msla_workspace_bytes(B, C, H, W, heads, head_dim, scales, dtype)
    return torch.empty(n, dtype=torch.uint8, device=device)


def msla_forward(x, w_qkv, w_dw, w_gpw, w_proj, heads, head_dim, scales, eps=1e-15, out=None,
                 workspace=None, stream=None, layout=MSLA_NHWC, options=0):
    """out = MSLA(x): x [B,H,W,C] -> out [B,H,W,C], or [B,C,H,W] both with layout=MSLA_NCHW
    (see include/msla.h for every shape).  options != 0 goes through msla_forward_opts."""
    _dev(x, w_qkv, w_dw, w_gpw, w_proj, out, workspace)
    if layout == MSLA_NCHW:
        B, C, H, W = x.shape
    else:
        B, H, W, C = x.shape
    if out is None:
        out = torch.empty_like(x)
    if workspace is None:
        workspace = new_workspace(B, C, H, W, heads, head_dim, scales, x.dtype, x.device)
    sc, ns = _scales(scales)
    args = (_ptr(x), _ptr(w_qkv), _ptr(w_dw), _ptr(w_gpw), _ptr(w_proj), _ptr(out), _ptr(workspace),
            workspace.numel(), B, C, H, W, heads, head_dim, sc, ns, float(eps), _DTYPES[x.dtype], layout,
            _stream(stream))
    if options:
        st = load_library().msla_forward_opts(*args, int(options))
    else:
        st = load_library().msla_forward(*args)
    if st != MSLA_OK:
        raise MslaError(st, "msla_forward")
    return out


def msla_forward_opts(x, w_qkv, w_dw, w_gpw, w_proj, heads, head_dim, scales, eps, options, out=None,
                      workspace=None, stream=None, layout=MSLA_NHWC):
    """msla_forward with a choice of code path / stages (MSLA_OPT_* bits, see include/msla.h)."""
    return msla_forward(x, w_qkv, w_dw, w_gpw, w_proj, heads, head_dim, scales, eps, out=out,
                        workspace=workspace, stream=stream, layout=layout, options=options)


def msla_forward_profiled(x, w_qkv, w_dw, w_gpw, w_proj, heads, head_dim, scales, eps, out, workspace,
                          events, stream=None, layout=MSLA_NHWC):
    """msla_forward that also records 5 caller-created hipEvent_t handles (ints) between its stages."""
    _dev(x, w_qkv, w_dw, w_gpw, w_proj, out, workspace)
    if layout == MSLA_NCHW:
        B, C, H, W = x.shape
    else:
        B, H, W, C = x.shape
    sc, ns = _scales(scales)
    ev = (ctypes.c_void_p * 5)(*[ctypes.c_void_p(int(e)) for e in events])
    st = load_library().msla_forward_profiled(_ptr(x), _ptr(w_qkv), _ptr(w_dw), _ptr(w_gpw), _ptr(w_proj),
                                              _ptr(out), _ptr(workspace), workspace.numel(), B, C, H, W, heads,
                                              head_dim, sc, ns, float(eps), _DTYPES[x.dtype], layout,
                                              _stream(stream), ev)
    if st != MSLA_OK:
        raise MslaError(st, "msla_forward_profiled")
    return out


def msla_core_forward(qkv, w_dw, w_gpw, heads, head_dim, scales, eps=1e-15, att=None, workspace=None,
                      stream=None):
    """att = concat over branches of ReLU linear attention on qkv [B,H,W,3*heads*d]."""
    _dev(qkv, w_dw, w_gpw, att, workspace)
    B, H, W, ch = qkv.shape
    Ct = heads * head_dim
    if att is None:
        att = torch.empty((B, H, W, (1 + len(scales)) * Ct), dtype=qkv.dtype, device=qkv.device)
    if workspace is None:
        workspace = new_workspace(B, Ct, H, W, heads, head_dim, scales, qkv.dtype, qkv.device)
    sc, ns = _scales(scales)
    st = load_library().msla_core_forward(_ptr(qkv), _ptr(w_dw), _ptr(w_gpw), _ptr(att), _ptr(workspace),
                                          workspace.numel(), B, H, W, heads, head_dim, sc, ns, float(eps),
                                          _DTYPES[qkv.dtype], _stream(stream))
    if st != MSLA_OK:
        raise MslaError(st, "msla_core_forward")
    return att


def msla_multiscale_state(qkv, w_dw, w_gpw, heads, head_dim, scales, workspace=None, stream=None,
                          want_q=True):
    """(q_ms [B,H,W,S*Ct], kv [B,S,heads,d,d+1] fp32): multi-scale Q tokens and Eq. (3) states."""
    _dev(qkv, w_dw, w_gpw, workspace)
    B, H, W, ch = qkv.shape
    Ct = heads * head_dim
    S = 1 + len(scales)
    q_ms = torch.empty((B, H, W, S * Ct), dtype=qkv.dtype, device=qkv.device) if want_q else None
    kv = torch.empty((B, S, heads, head_dim, head_dim + 1), dtype=torch.float32, device=qkv.device)
    if workspace is None:
        workspace = new_workspace(B, Ct, H, W, heads, head_dim, scales, qkv.dtype, qkv.device)
    sc, ns = _scales(scales)
    st = load_library().msla_multiscale_state(_ptr(qkv), _ptr(w_dw), _ptr(w_gpw), _ptr(q_ms), _ptr(kv),
                                              _ptr(workspace), workspace.numel(), B, H, W, heads, head_dim,
                                              sc, ns, _DTYPES[qkv.dtype], _stream(stream))
    if st != MSLA_OK:
        raise MslaError(st, "msla_multiscale_state")
    return q_ms, kv


def msla_multiscale_state_static(qkv, w_dw, w_gpw, heads, head_dim, scales, q_ms, kv, stream=None):
    """msla_multiscale_state without a workspace and without any allocation: the caller passes the
    outputs q_ms [B,H,W,S*Ct] and kv [B,S,heads,d,d+1] fp32; the library's own device array is the scratch."""
    _dev(qkv, w_dw, w_gpw, q_ms, kv)
    B, H, W, ch = qkv.shape
    sc, ns = _scales(scales)
    st = load_library().msla_multiscale_state_static(_ptr(qkv), _ptr(w_dw), _ptr(w_gpw), _ptr(q_ms), _ptr(kv),
                                                     B, H, W, heads, head_dim, sc, ns, _DTYPES[qkv.dtype],
                                                     _stream(stream))
    if st != MSLA_OK:
        raise MslaError(st, "msla_multiscale_state_static")
    return q_ms, kv


def msla_linear(x, w, y=None, stream=None):
    """y[..., o] = sum_c x[..., c] * w[o, c]."""
    _dev(x, w, y)
    c_out, c_in = w.shape
    n = x.numel() // c_in
    if y is None:
        y = torch.empty(x.shape[:-1] + (c_out,), dtype=x.dtype, device=x.device)
    st = load_library().msla_linear(_ptr(x), _ptr(w), _ptr(y), n, c_in, c_out, _DTYPES[x.dtype],
                                    _stream(stream))
    if st != MSLA_OK:
        raise MslaError(st, "msla_linear")
    return y


def msla_ffn_workspace_bytes(B, C, H, W, hidden, dtype) -> int:
    out = ctypes.c_size_t(0)
    st = load_library().msla_ffn_workspace_bytes(B, C, H, W, hidden, _DTYPES[dtype], ctypes.byref(out))
    if st != MSLA_OK:
        raise MslaError(st, "msla_ffn_workspace_bytes")
    return int(out.value)


def msla_ffn_forward(y, w1, w_dw, w2, act=MSLA_ACT_RELU, out=None, workspace=None, stream=None):
    """out = y + W2 . act(DW3x3(act(W1 . y))): y [B,H,W,C], w1 [hidden,C], w_dw [hidden,3,3], w2 [C,hidden]."""
    _dev(y, w1, w_dw, w2, out, workspace)
    B, H, W, C = y.shape
    hidden = w1.shape[0]
    if out is None:
        out = torch.empty_like(y)
    if workspace is None:
        workspace = torch.empty(msla_ffn_workspace_bytes(B, C, H, W, hidden, y.dtype), dtype=torch.uint8, device=y.device)
    st = load_library().msla_ffn_forward(_ptr(y), _ptr(w1), _ptr(w_dw), _ptr(w2), _ptr(out), _ptr(workspace),
                                         workspace.numel(), B, C, H, W, hidden, int(act), _DTYPES[y.dtype],
                                         _stream(stream))
    if st != MSLA_OK:
        raise MslaError(st, "msla_ffn_forward")
    return out


def msla_block_workspace_bytes(B, C, H, W, heads, head_dim, scales, hidden, dtype) -> int:
    sc, ns = _scales(scales)
    out = ctypes.c_size_t(0)
    st = load_library().msla_block_workspace_bytes(B, C, H, W, heads, head_dim, sc, ns, hidden, _DTYPES[dtype],
                                                   ctypes.byref(out))
    if st != MSLA_OK:
        raise MslaError(st, "msla_block_workspace_bytes")
    return int(out.value)


def msla_block_forward(x, w_qkv, w_dw, w_gpw, w_proj, w1, w_ffn_dw, w2, heads, head_dim, scales, eps=1e-15,
                       act=MSLA_ACT_RELU, out=None, workspace=None, stream=None):
    """The whole building block: y = x + MSLA(x); out = y + FFN(y).  x, out [B,H,W,C]."""
    _dev(x, w_qkv, w_dw, w_gpw, w_proj, w1, w_ffn_dw, w2, out, workspace)
    B, H, W, C = x.shape
    hidden = w1.shape[0]
    if out is None:
        out = torch.empty_like(x)
    if workspace is None:
        workspace = torch.empty(msla_block_workspace_bytes(B, C, H, W, heads, head_dim, scales, hidden, x.dtype),
                                dtype=torch.uint8, device=x.device)
    sc, ns = _scales(scales)
    st = load_library().msla_block_forward(_ptr(x), _ptr(w_qkv), _ptr(w_dw), _ptr(w_gpw), _ptr(w_proj), _ptr(w1),
                                           _ptr(w_ffn_dw), _ptr(w2), _ptr(out), _ptr(workspace), workspace.numel(),
                                           B, C, H, W, heads, head_dim, sc, ns, float(eps), hidden, int(act),
                                           _DTYPES[x.dtype], _stream(stream))
    if st != MSLA_OK:
        raise MslaError(st, "msla_block_forward")
    return out


def msla_softmax_attention(qkv, heads, head_dim, att=None, stream=None):
    """Softmax attention per image and head: qkv [B, ..., 3*heads*d] -> att [B, ..., heads*d]."""
    _dev(qkv, att)
    B = qkv.shape[0]
    N = qkv.numel() // (B * qkv.shape[-1])
    if att is None:
        att = torch.empty(qkv.shape[:-1] + (heads * head_dim,), dtype=qkv.dtype, device=qkv.device)
    st = load_library().msla_softmax_attention(_ptr(qkv), _ptr(att), B, N, heads, head_dim, _DTYPES[qkv.dtype],
                                               _stream(stream))
    if st != MSLA_OK:
        raise MslaError(st, "msla_softmax_attention")
    return att


def msla_linear_attention_backward_workspace_bytes(B, N, heads, head_dim, dtype) -> int:
    out = ctypes.c_size_t(0)
    st = load_library().msla_linear_attention_backward_workspace_bytes(B, N, heads, head_dim, _DTYPES[dtype],
                                                                       ctypes.byref(out))
    if st != MSLA_OK:
        raise MslaError(st, "msla_linear_attention_backward_workspace_bytes")
    return int(out.value)


def msla_linear_attention_backward(qkv, d_att, heads, head_dim, eps=1e-15, d_qkv=None, workspace=None, stream=None):
    """Gradient of ReLU linear attention: qkv [B, ..., 3*heads*d], d_att [B, ..., heads*d] -> d_qkv like qkv."""
    _dev(qkv, d_att, d_qkv, workspace)
    B = qkv.shape[0]
    N = qkv.numel() // (B * qkv.shape[-1])
    if d_qkv is None:
        d_qkv = torch.empty_like(qkv)
    if workspace is None:
        workspace = torch.empty(msla_linear_attention_backward_workspace_bytes(B, N, heads, head_dim, qkv.dtype),
                                dtype=torch.uint8, device=qkv.device)
    st = load_library().msla_linear_attention_backward(_ptr(qkv), _ptr(d_att), _ptr(d_qkv), _ptr(workspace),
                                                       workspace.numel(), B, N, heads, head_dim, float(eps),
                                                       _DTYPES[qkv.dtype], _stream(stream))
    if st != MSLA_OK:
        raise MslaError(st, "msla_linear_attention_backward")
    return d_qkv
