"""fp64 CPU oracle of the backward pass of ReLU linear attention (paper Section 3.1, Eq. (3); the
paper trains its models, Section 4.1, but prints nothing about gradients, so the definition is
the derivative of Eq. (3) itself).

TEST INFRASTRUCTURE, NOT PRODUCT CODE: only ``tests/``, the smoke check and the bench's CPU legs may
import this.

Forward, per image and head (Q, K, V [N, d], rq = max(Q, 0), rk = max(K, 0)):
    S = sum_n rk_n^T [V_n, 1]                      (d x (d+1))
    den_n = rq_n . S[:, d] + eps,   att_n = rq_n S[:, :d] / den_n
Given dA = dL/d att, the chain rule gives (g_n = dA_n / den_n, c_n = -(dA_n . att_n) / den_n):
    dS      = sum_n rq_n^T [g_n, c_n]
    d rq_n  = S[:, :d] g_n + S[:, d] c_n           dQ_n = d rq_n * [Q_n > 0]
    d rk_n  = dS[:, :d] V_n + dS[:, d]             dK_n = d rk_n * [K_n > 0]
    dV_n    = rk_n dS[:, :d]
(the rectifier's derivative is taken as 0 at 0).  Written out with numpy in fp64, nothing rounded.

Pins (tests/test_backward_oracle_pins.py) that do not use these formulas: central finite
differences of the forward oracle (msla_oracle.relu_linear_attention) on small inputs; torch
autograd in fp64 on Eq. (3) re-stated in torch; the gradient of a loss that ignores att is zero;
dV is linear in dA; a dead query gets no gradient.  Parity unpinned: the derivative at exactly 0.
"""
from __future__ import annotations

import numpy as np


def linear_attention_backward_head(Q, K, V, dA, eps: float):
    """One head: Q, K, V, dA [N, d] -> (dQ, dK, dV), each [N, d]."""
    Q, K, V, dA = (np.asarray(a, dtype=np.float64) for a in (Q, K, V, dA))
    d = Q.shape[1]
    rq, rk = np.maximum(Q, 0.0), np.maximum(K, 0.0)
    S = rk.T @ np.concatenate([V, np.ones((V.shape[0], 1))], axis=1)          # [d, d+1]
    den = rq @ S[:, d] + eps                                                 # [N]
    att = (rq @ S[:, :d]) / den[:, None]
    g = dA / den[:, None]
    c = -(dA * att).sum(1) / den
    dS = rq.T @ np.concatenate([g, c[:, None]], axis=1)                      # [d, d+1]
    dQ = (g @ S[:, :d].T + np.outer(c, S[:, d])) * (Q > 0)
    dK = (V @ dS[:, :d].T + dS[:, d][None, :]) * (K > 0)
    dV = rk @ dS[:, :d]
    return dQ, dK, dV


def linear_attention_backward(qkv, d_att, heads: int, d: int, eps: float) -> np.ndarray:
    """qkv [B, N, 3*heads*d] (channel (h*3 + t)*d + e), d_att [B, N, heads*d] -> d_qkv like qkv."""
    qkv = np.asarray(qkv, dtype=np.float64)
    d_att = np.asarray(d_att, dtype=np.float64)
    B, N, ch = qkv.shape
    assert ch == 3 * heads * d and d_att.shape == (B, N, heads * d)
    out = np.empty_like(qkv)
    v = qkv.reshape(B, N, heads, 3, d)
    o = out.reshape(B, N, heads, 3, d)
    for b in range(B):
        for h in range(heads):
            dQ, dK, dV = linear_attention_backward_head(v[b, :, h, 0], v[b, :, h, 1], v[b, :, h, 2],
                                                        d_att[b, :, h * d:(h + 1) * d], eps)
            o[b, :, h, 0], o[b, :, h, 1], o[b, :, h, 2] = dQ, dK, dV
    return out
