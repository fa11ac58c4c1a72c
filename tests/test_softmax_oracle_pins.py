"""CPU pins of oracle/softmax_oracle.py (Section 3.1, Eq. (1) with the exponential similarity)."""
import os

import numpy as np
import torch

from oracle import softmax_oracle as sm

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def test_hand_worked_two_token_example():
    want = np.array([l.split() for l in open(os.path.join(GOLDEN, "softmax_attention_n2_d2.txt"))
                     if l.strip() and not l.startswith("#")], dtype=np.float64)
    Q = np.array([[np.sqrt(2.0) * np.log(2.0), 0.0], [0.0, 0.0]])
    K = np.array([[1.0, 0.0], [0.0, 0.0]])
    V = np.array([[3.0, 0.0], [0.0, 6.0]])
    assert np.allclose(sm.softmax_attention_head(Q, K, V), want, rtol=0, atol=1e-14)


def test_rows_of_the_similarity_sum_to_one():
    rng = np.random.default_rng(0)
    N, d = 40, 16
    Q, K, V = (rng.standard_normal((N, d)) for _ in range(3))
    const = np.tile(rng.standard_normal(d), (N, 1))
    assert np.allclose(sm.softmax_attention_head(Q, K, const), const, rtol=0, atol=1e-13)
    O = sm.softmax_attention_head(Q, K, V)
    assert (O <= V.max(0) + 1e-12).all() and (O >= V.min(0) - 1e-12).all()
    # Q = 0: uniform weights, the mean of V; invariant to permuting the (K, V) tokens together
    assert np.allclose(sm.softmax_attention_head(np.zeros((N, d)), K, V), np.tile(V.mean(0), (N, 1)), atol=1e-13)
    perm = rng.permutation(N)
    assert np.allclose(sm.softmax_attention_head(Q, K[perm], V[perm]), O, atol=1e-12)
    # unlike the ReLU form it is NOT invariant to scaling Q and K: a large scale picks the best-matching key
    big = sm.softmax_attention_head(2000.0 * Q, K, V)
    scores = np.sort(Q @ K.T, axis=1)
    clear = scores[:, -1] - scores[:, -2] > 0.05          # rows whose best key leads by a clear margin
    assert clear.sum() > N // 2
    assert np.allclose(big[clear], V[np.argmax(Q @ K.T, axis=1)][clear], atol=1e-6)


def test_against_torch_scaled_dot_product_attention():
    rng = np.random.default_rng(1)
    B, N, heads, d = 2, 33, 3, 16
    qkv = rng.standard_normal((B, N, 3 * heads * d))
    got = sm.softmax_attention(qkv, heads, d)
    v = torch.from_numpy(qkv).reshape(B, N, heads, 3, d).permute(3, 0, 2, 1, 4)       # [3, B, heads, N, d]
    ref = torch.nn.functional.scaled_dot_product_attention(v[0], v[1], v[2])           # scale 1/sqrt(d)
    ref = ref.permute(0, 2, 1, 3).reshape(B, N, heads * d).numpy()
    assert np.allclose(got, ref, rtol=1e-11, atol=1e-12)
    # the heads and images do not mix: changing head 1 of image 0 changes only that block
    qkv2 = qkv.copy(); qkv2[0, :, 3 * d:6 * d] += 1.0
    got2 = sm.softmax_attention(qkv2, heads, d)
    changed = np.abs(got2 - got) > 1e-9
    assert changed[0, :, d:2 * d].any() and not changed[1].any() and not changed[0, :, :d].any() and not changed[0, :, 2 * d:].any()
