"""fp64 CPU oracle of softmax attention, the comparison point of the paper's ReLU linear attention
(Section 3.1: Eq. (1) with Sim(Q, K) = exp(Q K^T / sqrt(d)); Fig. 3 compares the latency of the two).

TEST INFRASTRUCTURE, NOT PRODUCT CODE: only ``tests/``, the smoke check and the bench's CPU legs may
import this.  It is the definition written out with numpy in fp64, one head at a time:

    O_i = sum_j exp(Q_i . K_j / sqrt(d)) V_j  /  sum_j exp(Q_i . K_j / sqrt(d))

(the largest score of a row is subtracted before exponentiation, which cancels in the quotient and
only keeps exp() in range).  Channel order of the projected map as everywhere in this library:
``o = (h*3 + t)*d + e`` with t = 0:Q, 1:K, 2:V.

Pins (tests/test_softmax_oracle_pins.py): a two-token example worked by hand; rows of the similarity
sum to one (constant V returns the constant; outputs stay inside the hull of V); Q = 0 gives the mean
of V; a sharply peaked score picks one V row; torch's scaled_dot_product_attention in fp64.
Parity unpinned: nothing.
"""
from __future__ import annotations

import numpy as np


def softmax_attention_head(Q, K, V) -> np.ndarray:
    """One head: Q, K, V [N, d] -> O [N, d] (Eq. (1) with the exponential similarity)."""
    Q = np.asarray(Q, dtype=np.float64); K = np.asarray(K, dtype=np.float64); V = np.asarray(V, dtype=np.float64)
    d = Q.shape[1]
    s = (Q @ K.T) / np.sqrt(d)
    s = s - s.max(axis=1, keepdims=True)
    p = np.exp(s)
    return (p @ V) / p.sum(axis=1, keepdims=True)


def softmax_attention(qkv, heads: int, d: int) -> np.ndarray:
    """qkv [B, N, 3*heads*d] -> att [B, N, heads*d]: every image and head on its own."""
    qkv = np.asarray(qkv, dtype=np.float64)
    B, N, ch = qkv.shape
    assert ch == 3 * heads * d
    out = np.empty((B, N, heads * d))
    v = qkv.reshape(B, N, heads, 3, d)
    for b in range(B):
        for h in range(heads):
            out[b, :, h * d:(h + 1) * d] = softmax_attention_head(v[b, :, h, 0], v[b, :, h, 1], v[b, :, h, 2])
    return out
