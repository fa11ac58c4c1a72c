"""CPU pins of oracle/backward_oracle.py: the gradient of Eq. (3) against things that do not use its
formulas -- finite differences of the forward oracle and torch autograd in fp64."""
import numpy as np
import torch

from oracle import backward_oracle as bwd
from oracle import msla_oracle as orc


def _pack(Q, K, V):
    return np.ascontiguousarray(np.concatenate([Q, K, V], axis=-1))


def _loss(Q, K, V, dA, eps):
    att = orc.relu_linear_attention(_pack(Q, K, V), 1, Q.shape[1], eps)
    return float((att * dA).sum())


def test_central_finite_differences_of_the_forward_oracle():
    rng = np.random.default_rng(0)
    N, d, eps = 7, 16, 1e-15
    Q, K, V, dA = (rng.standard_normal((N, d)) for _ in range(4))
    # keep every entry away from the kink of the rectifier, so the difference quotient is the derivative
    Q[np.abs(Q) < 0.05] = 0.3; K[np.abs(K) < 0.05] = -0.3
    dQ, dK, dV = bwd.linear_attention_backward_head(Q, K, V, dA, eps)
    hstep = 1e-6
    for name, X, G in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV)):
        num = np.zeros_like(X)
        for idx in np.ndindex(*X.shape):
            keep = X[idx]
            X[idx] = keep + hstep; up = _loss(Q, K, V, dA, eps)
            X[idx] = keep - hstep; dn = _loss(Q, K, V, dA, eps)
            X[idx] = keep
            num[idx] = (up - dn) / (2 * hstep)
        assert np.allclose(G, num, rtol=1e-6, atol=1e-7), f"d{name} differs from the difference quotient"


def test_against_torch_autograd():
    rng = np.random.default_rng(1)
    B, N, heads, d, eps = 2, 19, 3, 16, 1e-15
    qkv = rng.standard_normal((B, N, 3 * heads * d))
    dA = rng.standard_normal((B, N, heads * d))
    got = bwd.linear_attention_backward(qkv, dA, heads, d, eps)
    t = torch.from_numpy(qkv).requires_grad_(True)
    v = t.reshape(B, N, heads, 3, d)
    rq, rk, V = torch.relu(v[..., 0, :]), torch.relu(v[..., 1, :]), v[..., 2, :]
    kv = torch.einsum("bnhe,bnhf->bhef", rk, V)
    ks = rk.sum(1)                                                  # [B, heads, d]
    att = torch.einsum("bnhe,bhef->bnhf", rq, kv) / (torch.einsum("bnhe,bhe->bnh", rq, ks)[..., None] + eps)
    (att.reshape(B, N, heads * d) * torch.from_numpy(dA)).sum().backward()
    assert np.allclose(got, t.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_structure_of_the_gradient():
    rng = np.random.default_rng(2)
    N, d, eps = 12, 16, 1e-15
    Q, K, V, dA = (rng.standard_normal((N, d)) for _ in range(4))
    Q[4] = -np.abs(Q[4])                                            # a dead query
    dQ, dK, dV = bwd.linear_attention_backward_head(Q, K, V, dA, eps)
    assert np.array_equal(dQ[4], np.zeros(d))
    assert np.array_equal(dQ[Q <= 0], np.zeros((Q <= 0).sum())) and np.array_equal(dK[K <= 0], np.zeros((K <= 0).sum()))
    z = bwd.linear_attention_backward_head(Q, K, V, np.zeros_like(dA), eps)
    assert all(np.array_equal(a, np.zeros((N, d))) for a in z)
    # linear in dA
    dA2 = rng.standard_normal((N, d))
    a = bwd.linear_attention_backward_head(Q, K, V, dA + 2 * dA2, eps)
    b2 = bwd.linear_attention_backward_head(Q, K, V, dA2, eps)
    for x, y, zz in zip(a, (dQ, dK, dV), b2):
        assert np.allclose(x, y + 2 * zz, rtol=1e-11, atol=1e-12)
    # att does not change when V gets a constant row added to every token only through the convex weights:
    # a constant dA (same row for every token) gives dQ = 0 when ... the rows of the similarity sum to one
    const = np.tile(rng.standard_normal(d), (N, 1))
    dQc, dKc, dVc = bwd.linear_attention_backward_head(Q, K, const, dA, eps)
    assert np.allclose(dQc, 0, atol=1e-12) and np.allclose(dKc, 0, atol=1e-12)       # constant V: att = const whatever Q, K
