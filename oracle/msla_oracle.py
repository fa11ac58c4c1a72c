"""ctypes loader for the fp64 CPU oracle (``msla_oracle.c``).

TEST INFRASTRUCTURE, NOT PRODUCT CODE: only ``tests/``, the smoke check and the
bench's ``cpu_baseline`` leg may import this.  The GPU library never does, and
this module imports nothing from the GPU package.

All arrays are C-contiguous ``numpy.float64``; shapes follow the comments in
``msla_oracle.c`` (token maps ``[B, H, W, channels]``, projected channel order
``o = (h*3 + t)*d + e``).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "msla_oracle.c")
_LIB = os.path.join(_HERE, "libmsla_oracle.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP on) next to its source."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
             "-ffp-contract=off", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        P = ctypes.POINTER(ctypes.c_double)
        I = ctypes.c_int
        L = ctypes.c_long
        D = ctypes.c_double
        PI = ctypes.POINTER(ctypes.c_int)
        lib.msla_oracle_num_threads.restype = I
        lib.msla_oracle_linear.argtypes = [P, P, P, L, I, I]
        lib.msla_oracle_linear.restype = None
        lib.msla_oracle_dwconv.argtypes = [P, P, P, I, I, I, I, I]
        lib.msla_oracle_dwconv.restype = None
        lib.msla_oracle_grouped_pw.argtypes = [P, P, P, L, I, I]
        lib.msla_oracle_grouped_pw.restype = None
        lib.msla_oracle_kv_state.argtypes = [P, P, L, I, I]
        lib.msla_oracle_kv_state.restype = None
        lib.msla_oracle_apply.argtypes = [P, P, P, L, I, I, D, L, L]
        lib.msla_oracle_apply.restype = None
        lib.msla_oracle_attention_nxn.argtypes = [P, P, P, P, L, I, D]
        lib.msla_oracle_attention_nxn.restype = None
        lib.msla_oracle_core_forward.argtypes = [P, P, P, P, P, I, I, I, I, I, PI, I, D]
        lib.msla_oracle_core_forward.restype = I
        lib.msla_oracle_forward.argtypes = [P, P, P, P, P, P, I, I, I, I, I, I, PI, I, D]
        lib.msla_oracle_forward.restype = I
        _lib = lib
    return _lib


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _scales(scales):
    arr = (ctypes.c_int * max(1, len(scales)))(*scales)
    return arr, len(scales)


def num_threads() -> int:
    return int(_load().msla_oracle_num_threads())


def linear(x, w) -> np.ndarray:
    """``y[..., o] = sum_c x[..., c] * w[o, c]``."""
    x = _f64(x); w = _f64(w)
    c_out, c_in = w.shape
    assert x.shape[-1] == c_in
    n = x.size // c_in
    y = np.empty(x.shape[:-1] + (c_out,), dtype=np.float64)
    _load().msla_oracle_linear(_p(x), _p(w), _p(y), n, c_in, c_out)
    return y


def dwconv(inp, w) -> np.ndarray:
    """Depthwise k x k, stride 1, zero pad; ``inp [B,H,W,ch]``, ``w [ch,k,k]``."""
    inp = _f64(inp); w = _f64(w)
    B, H, W, ch = inp.shape
    k = w.shape[1]
    assert w.shape == (ch, k, k) and k % 2 == 1
    out = np.empty_like(inp)
    _load().msla_oracle_dwconv(_p(inp), _p(w), _p(out), B, H, W, ch, k)
    return out


def grouped_pw(inp, w) -> np.ndarray:
    """Grouped 1x1; ``inp [..., ch]``, ``w [ch, d]``, groups of ``d`` channels."""
    inp = _f64(inp); w = _f64(w)
    ch, d = w.shape
    assert inp.shape[-1] == ch and ch % d == 0
    out = np.empty_like(inp)
    _load().msla_oracle_grouped_pw(_p(inp), _p(w), _p(out), inp.size // ch, ch, d)
    return out


def kv_state(tokens, heads: int, d: int) -> np.ndarray:
    """``tokens [N, 3*heads*d]`` of one image/branch -> ``[heads, d, d+1]``."""
    tokens = _f64(tokens)
    N = tokens.shape[0]
    assert tokens.shape == (N, 3 * heads * d)
    kv = np.empty((heads, d, d + 1), dtype=np.float64)
    _load().msla_oracle_kv_state(_p(tokens), _p(kv), N, heads, d)
    return kv


def apply(tokens, kv, eps: float) -> np.ndarray:
    """Eq. (3) given the state: ``tokens [N, 3*heads*d]`` -> ``[N, heads*d]``."""
    tokens = _f64(tokens); kv = _f64(kv)
    heads, d, d1 = kv.shape
    assert d1 == d + 1
    N = tokens.shape[0]
    att = np.empty((N, heads * d), dtype=np.float64)
    _load().msla_oracle_apply(_p(tokens), _p(kv), _p(att), N, heads, d, float(eps),
                              heads * d, 0)
    return att


def relu_linear_attention(tokens, heads: int, d: int, eps: float) -> np.ndarray:
    """Linear form of Eq. (3) on one image/branch map ``[N, 3*heads*d]``."""
    return apply(tokens, kv_state(tokens, heads, d), eps)


def attention_nxn(Q, K, V, eps: float) -> np.ndarray:
    """Quadratic form of Eq. (1)+(2), one head; ``Q, K, V [N, d]``."""
    Q = _f64(Q); K = _f64(K); V = _f64(V)
    N, d = Q.shape
    O = np.empty((N, d), dtype=np.float64)
    _load().msla_oracle_attention_nxn(_p(Q), _p(K), _p(V), _p(O), N, d, float(eps))
    return O


def core_forward(qkv, w_dw, w_gpw, heads: int, d: int, scales, eps: float,
                 return_kv: bool = False):
    """``qkv [B,H,W,3*heads*d]`` -> ``att [B,H,W,(1+A)*heads*d]`` (and the
    ``[B, 1+A, heads, d, d+1]`` states if ``return_kv``)."""
    qkv = _f64(qkv)
    B, H, W, ch = qkv.shape
    assert ch == 3 * heads * d
    scales = [int(k) for k in scales]
    A = len(scales)
    w_dw = _f64(w_dw).reshape(-1)
    w_gpw = _f64(w_gpw).reshape(-1)
    assert w_dw.size == sum(ch * k * k for k in scales)
    assert w_gpw.size == A * ch * d
    if A == 0:
        w_dw = np.zeros(1); w_gpw = np.zeros(1)
    att = np.empty((B, H, W, (1 + A) * heads * d), dtype=np.float64)
    kv = np.empty((B, 1 + A, heads, d, d + 1), dtype=np.float64) if return_kv else None
    sc, ns = _scales(scales)
    rc = _load().msla_oracle_core_forward(
        _p(qkv), _p(w_dw), _p(w_gpw), _p(att), _p(kv) if return_kv else None,
        B, H, W, heads, d, sc, ns, float(eps))
    if rc != 0:
        raise MemoryError("msla_oracle_core_forward: out of memory")
    return (att, kv) if return_kv else att


def forward(x, w_qkv, w_dw, w_gpw, w_proj, heads: int, d: int, scales, eps: float) -> np.ndarray:
    """Whole module: ``x [B,H,W,C]`` -> ``out [B,H,W,C]``."""
    x = _f64(x); w_qkv = _f64(w_qkv); w_proj = _f64(w_proj)
    B, H, W, C = x.shape
    ch = 3 * heads * d
    scales = [int(k) for k in scales]
    A = len(scales)
    assert w_qkv.shape == (ch, C)
    assert w_proj.shape == (C, (1 + A) * heads * d)
    w_dw = _f64(w_dw).reshape(-1)
    w_gpw = _f64(w_gpw).reshape(-1)
    assert w_dw.size == sum(ch * k * k for k in scales)
    assert w_gpw.size == A * ch * d
    if A == 0:
        w_dw = np.zeros(1); w_gpw = np.zeros(1)
    out = np.empty((B, H, W, C), dtype=np.float64)
    sc, ns = _scales(scales)
    rc = _load().msla_oracle_forward(
        _p(x), _p(w_qkv), _p(w_dw), _p(w_gpw), _p(w_proj), _p(out),
        B, C, H, W, heads, d, sc, ns, float(eps))
    if rc != 0:
        raise MemoryError("msla_oracle_forward: out of memory")
    return out


# ----------------------------------------------------------------------------
# The same module composed stage by stage (Fig. 2 right) from the stage
# functions above, with every intermediate returned.  Nothing is rounded and
# nothing is taken from outside: this is the paper's definition, only split at
# the arrows of the figure (a test pins it to the one-call forms).
# ----------------------------------------------------------------------------

def branch_maps(qkv, w_dw, w_gpw, heads: int, d: int, scales):
    """[raw map, aggregated map per scale], each [B,H,W,3*heads*d]; every
    aggregated branch reads the raw map (Section 3.1, last paragraph)."""
    qkv = _f64(qkv)
    ch = 3 * heads * d
    w_dw = _f64(w_dw).reshape(-1)
    maps = [qkv]
    off = 0
    for a, k in enumerate(scales):
        w = w_dw[off:off + ch * k * k].reshape(ch, k, k)
        off += ch * k * k
        maps.append(grouped_pw(dwconv(qkv, w), _f64(w_gpw)[a]))
    return maps


def q_tokens_of(maps, heads: int, d: int) -> np.ndarray:
    """The Q tokens of every branch, [B,H,W,S*heads*d], column (s*heads+h)*d+e."""
    B, H, W, _ = maps[0].shape
    return np.concatenate([m.reshape(B, H, W, heads, 3, d)[..., 0, :].reshape(B, H, W, heads * d)
                           for m in maps], axis=-1)


def attention_of_maps(maps, heads: int, d: int, eps: float):
    """Eq. (3) per image / branch / head on the given branch maps.
    Returns (att [B,H,W,S*heads*d], kv [B,S,heads,d,d+1])."""
    B, H, W, ch = maps[0].shape
    S = len(maps)
    N = H * W
    Ct = heads * d
    att = np.empty((B, N, S * Ct), dtype=np.float64)
    kv = np.empty((B, S, heads, d, d + 1), dtype=np.float64)
    for s, m in enumerate(maps):
        m = _f64(m).reshape(B, N, ch)
        for b in range(B):
            tok = np.ascontiguousarray(m[b])
            kv[b, s] = kv_state(tok, heads, d)
            att[b, :, s * Ct:(s + 1) * Ct] = apply(tok, kv[b, s], eps)
    return att.reshape(B, H, W, S * Ct), kv


def forward_staged(x, w_qkv, w_dw, w_gpw, w_proj, heads: int, d: int, scales, eps: float):
    """Whole module, stage by stage: (out, parts) with parts = the projected
    map, the branch maps, the attention rows, the Eq. (3) states and the Q
    tokens of every branch.  `out` is exactly `forward` (pinned by a test)."""
    qkv = linear(x, w_qkv)
    maps = branch_maps(qkv, w_dw, w_gpw, heads, d, scales)
    att, kv = attention_of_maps(maps, heads, d, eps)
    out = linear(att, w_proj)
    return out, {"qkv": qkv, "maps": maps, "att": att, "kv": kv, "q_tokens": q_tokens_of(maps, heads, d)}
