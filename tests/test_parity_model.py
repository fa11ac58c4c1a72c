"""CPU tests of the parity protocol itself (tests/parity_model.py): what the GPU tests rely on is
shown here without a GPU -- the margin, the admissible set of Eq. (3), the threshold THETA, and that
the judgement rejects planted mistakes."""
import numpy as np
import pytest

import parity_model as pm
from oracle import msla_oracle as orc
from paper_2205_14756_amd import workloads as wk


def _pack(Q, K, V):
    return np.ascontiguousarray(np.concatenate([Q, K, V], axis=-1))


def test_gate_margin_marks_the_tokens_whose_gate_hangs_on_a_rounding_sized_component():
    d = 16
    rng = np.random.default_rng(4)
    N = 12
    Q, K, V = (rng.standard_normal((1, N, d)) for _ in range(3))
    Q[0, 3] = -np.abs(Q[0, 3]); Q[0, 3, 5] = 1e-9
    Q[0, 6] = np.abs(Q[0, 6])
    Q[0, 9] = -np.abs(Q[0, 9])
    m = _pack(Q, K, V).reshape(1, 3, 4, 3 * d)
    att, kv = orc.attention_of_maps([m], 1, d, 1e-15)
    margin = pm.gate_margin(orc.q_tokens_of([m], 1, d), kv, 1, d).reshape(N)
    assert margin[6] == 1.0 and 0 < margin[3] < 1e-8 and margin[9] == 0.0
    assert (margin >= 0).all() and (margin <= 1).all()
    # such a row IS one of the hull's vertices; its neighbour across the gate is exactly 0
    att = att.reshape(N, d)
    assert np.allclose(att[3], kv[0, 0, 0, 5, :d] / kv[0, 0, 0, 5, d], rtol=1e-6)
    assert np.array_equal(att[9], np.zeros(d))
    for n in range(N):
        assert pm.att_row_validity(att[n], kv[0, 0, 0]) <= 1e-6 * np.abs(att).max()


def test_admissible_set_of_eq3():
    d = 16
    rng = np.random.default_rng(5)
    state = np.abs(rng.standard_normal((d, d + 1)))
    state[:, :d] = rng.standard_normal((d, d)) * 3
    R = pm.hull_rows(state)
    lam = rng.random(d); lam /= lam.sum()
    inside = lam @ R
    assert pm.att_row_validity(inside, state) < 1e-6
    assert pm.att_row_validity(np.zeros(d), state) == 0.0
    assert pm.att_row_validity(R[7], state) < 1e-6
    outside = R.max(0) + 1.0                      # beyond every vertex in every coordinate
    assert pm.att_row_validity(outside, state) > 0.5
    state[3, d] = 0.0                              # a row with Ksum = 0 is no vertex
    assert pm.hull_rows(state).shape[0] == d - 1


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_theta_covers_what_storage_rounding_alone_does_to_the_benchmark_workloads(cfg):
    """Storage rounding of the token maps (and nothing else) vs the plain oracle, all tokens: every
    token it moves past the bar has a gate margin below THETA, and is an admissible value of Eq. (3).
    Counts: none on the fp32 / fp16 workloads, one token on the bf16 one."""
    wl = wk.WORKLOADS[cfg]
    t = wk.make_inputs(wl)
    out_s, _ = pm.storage_reading(t, wl.dtype, wl.heads, wl.head_dim, wl.scales, wl.eps)
    got = wk.round_to_dtype(out_s, wl.dtype)
    j = pm.judge_module(got, t, wl.dtype, wl.heads, wl.head_dim, wl.scales, wl.eps)
    print(f"{wl.name}: {j}")
    assert len(j.listed) == len(j.predicted) == (1 if cfg == 4 else 0)
    assert j.worst_ok <= pm.TOL[wl.dtype]
    for tok, err, margin, dist in j.listed:
        assert margin < pm.theta(wl.dtype) and dist <= pm.TOL[wl.dtype]


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_theta_on_small_shapes(dtype):
    """The same on many small modules (more draws of the rare event)."""
    listed = 0
    for seed in range(12):
        heads, d, scales = 2, 16, (3, 5)
        t = wk.random_module(7000 + seed, dtype, 2, 32, 24, 31, heads, d, scales)
        out_s, _ = pm.storage_reading(t, dtype, heads, d, scales, 1e-15)
        j = pm.judge_module(wk.round_to_dtype(out_s, dtype), t, dtype, heads, d, scales, 1e-15)
        listed += len(j.listed)
    print(f"{dtype}: {listed} ill-conditioned tokens in 12 modules of 1488 tokens")


def test_judgement_rejects_planted_mistakes():
    wl = wk.WORKLOADS[2]
    t = wk.make_inputs(wl)
    args = (t, wl.dtype, wl.heads, wl.head_dim, wl.scales, wl.eps)
    plain, parts = orc.forward_staged(t["x"], t["w_qkv"], t["w_dw"], t["w_gpw"], t["w_proj"], wl.heads, wl.head_dim,
                                      wl.scales, wl.eps)
    scale = np.abs(plain).max()
    pm.judge_module(plain.copy(), *args)
    # (1) an error above the bar at a well-conditioned token
    bad = plain.copy(); bad[0, 10, 10, 3] += 2 * pm.TOL["f16"] * scale
    with pytest.raises(AssertionError, match="well-conditioned"):
        pm.judge_module(bad, *args)
    # (2) an ill-conditioned token filled with something Eq. (3) cannot give
    margin = pm.gate_margin(parts["q_tokens"], parts["kv"], wl.heads, wl.head_dim)
    tok = tuple(int(i) for i in np.argwhere(margin.min(-1) < pm.theta("f16"))[0])
    junk = plain.copy(); junk[tok] += 10 * scale
    with pytest.raises(AssertionError, match="not an admissible|predicts"):
        pm.judge_module(junk, *args, slack=1)
    # (3) the same token with its ill-conditioned head-branch row flipped to exactly 0 IS admissible,
    #     but is one more listed token than the storage reading predicts
    m = int(np.argmin(margin[tok]))
    d = wl.head_dim
    flipped = plain.copy()
    flipped[tok] -= t["w_proj"][:, m * d:(m + 1) * d] @ parts["att"][tok][m * d:(m + 1) * d]
    if np.abs(flipped[tok] - plain[tok]).max() > pm.TOL["f16"] * scale:
        with pytest.raises(AssertionError, match="predicts"):
            pm.judge_module(flipped, *args)
        j = pm.judge_module(flipped, *args, slack=1)
        assert len(j.listed) == 1 and j.listed[0][0] == tok and j.listed[0][3] <= pm.TOL["f16"]
    # (4) a transposed projection weight, a dropped branch: far over the bar everywhere
    t2 = dict(t); t2["w_proj"] = np.ascontiguousarray(t["w_proj"][:, ::-1])
    wrong = orc.forward(t2["x"], t2["w_qkv"], t2["w_dw"], t2["w_gpw"], t2["w_proj"], wl.heads, wl.head_dim, wl.scales, wl.eps)
    with pytest.raises(AssertionError):
        pm.judge_module(wrong, *args)


def test_heads_of_eight_in_bf16_need_the_first_order_rule():
    """bf16 storage, heads of 8 channels: the storage reading alone (CPU) moves tokens past the bar whose
    margins are above THETA; each of them has a head-branch whose first-order bound reaches the bar, and a
    value planted at such a token that is not the storage reading's is still rejected."""
    dtype, heads, d, scales = "bf16", 8, 8, (3, 5)
    hits = 0
    for seed in range(6):
        t = wk.random_module(8100 + seed, dtype, 2, 64, 24, 31, heads, d, scales)
        out_s, _ = pm.storage_reading(t, dtype, heads, d, scales, 1e-15)
        got = wk.round_to_dtype(out_s, dtype)
        j = pm.judge_module(got, t, dtype, heads, d, scales, 1e-15)
        assert len(j.listed) == len(j.predicted)
        above = [l for l in j.listed if l[2] >= pm.theta(dtype)]
        hits += len(above)
        if above:
            tok = above[0][0]
            plain = orc.forward(t["x"], t["w_qkv"], t["w_dw"], t["w_gpw"], t["w_proj"], heads, d, scales, 1e-15)
            bad = got.copy()
            bad[tok] = plain[tok] + 3 * (got[tok] - plain[tok])          # three times as far from the oracle
            with pytest.raises(AssertionError, match="away from the storage reading"):
                pm.judge_module(bad, t, dtype, heads, d, scales, 1e-15)
    print(f"{hits} tokens over the bar with a margin above THETA in 6 modules")
    assert hits > 0


def test_core_judgement():
    dtype, heads, d, scales = "bf16", 2, 16, (5,)
    t = wk.random_module(123, dtype, 1, 32, 20, 20, heads, d, scales)
    qkv = wk.round_to_dtype(orc.linear(t["x"], t["w_qkv"]), dtype)
    att = orc.core_forward(qkv, t["w_dw"], t["w_gpw"], heads, d, scales, 1e-15)
    j = pm.judge_core(wk.round_to_dtype(att, dtype), qkv, t, dtype, heads, d, scales, 1e-15)
    assert not j.listed
    bad = att.copy(); bad[0, 3, 3, 5] += 1.0
    with pytest.raises(AssertionError):
        pm.judge_core(bad, qkv, t, dtype, heads, d, scales, 1e-15)
