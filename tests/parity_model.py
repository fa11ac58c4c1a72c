"""Helpers of the parity tests (CPU only; nothing here touches the GPU library,
and nothing here is part of the oracle).

The oracle (``oracle/``) is the paper's definition in fp64 with no rounding.
The pass criterion of every parity test is the plain oracle at the stated bar
(max|gpu - oracle| <= tol * max|oracle|, tol = 1e-4 fp32, 5e-3 fp16 / bf16) on
EVERY token, except an explicit, printed and counted list of tokens at which
Eq. (3) itself is ill-posed under any finite-precision storage of Q:

  att = relu(Q) KV[:, :d] / (relu(Q) Ksum + eps)

is a convex combination of the rows KV[e, :] / Ksum[e] with weights
relu(Q_e) Ksum_e, or exactly 0 when no component of Q passes the rectifier.
Where the rectified part of Q is a rounding-sized remainder, the storage
rounding of the 16-bit token maps (which the stated precision "16-bit storage,
fp32 sums" prescribes) decides which of those rows the result is, and the
result moves by O(1).  Such a token is judged differently, with NO value taken
from the GPU other than the output under test:

  (i)  it must be *predicted*: its gate margin (below), computed from the plain
       oracle alone, is under THETA units roundoff of the storage type; and
  (ii) it must be *valid*: the output is what Eq. (3) gives for SOME admissible
       Q -- each ill-conditioned head-branch row is exactly 0 or lies in the
       convex hull of the oracle's rows KV[e, :] / Ksum[e] -- with everything
       else of that token equal to the plain oracle's within the bar.

The number of listed tokens is checked against a CPU prediction: the oracle's
own stage functions composed with the storage rounding (``storage_reading``).
THETA is not tuned on the GPU: ``tests/test_parity_model.py`` shows on the CPU
that every token the storage reading moves past the bar has a margin below it.

That holds for the benchmark workloads (heads of 16 channels).  With heads of 8
channels and bf16 storage a gate has half as many terms, and the CPU's storage
reading alone moves tokens whose margins are a few THETA past the bar: not a
flip between hull vertices, but the first-order effect of one rounding of Q,
(2u / margin) times the spread of the hull, which the projection carries into
the output.  A token over the bar is therefore also accepted when

  (iii) that first-order bound for one of its head-branches
        (``first_order_bound``, in units of max|out|, computed from the plain
        oracle alone) is at least the bar, AND the output is within the bar of
        the CPU's storage reading at that token.

(iii) takes no value from the GPU either, cannot excuse a well-conditioned
token, and still pins the GPU's value to within the bar of a CPU-computed one.
The count check covers the tokens of (i)-(ii) and of (iii) together.
"""
from __future__ import annotations

import itertools

import numpy as np
from scipy.optimize import nnls

from oracle import msla_oracle as orc
from paper_2205_14756_amd import workloads as wk

TOL = {"f32": 1e-4, "f16": 5e-3, "bf16": 5e-3}
UNIT_ROUNDOFF = {"f32": 2.0 ** -24, "f16": 2.0 ** -11, "bf16": 2.0 ** -8}
THETA_UNITS = 4.0      # a token-head is ill-conditioned when gate_margin < THETA_UNITS * u


def theta(dtype: str) -> float:
    return THETA_UNITS * UNIT_ROUNDOFF[dtype]


def storage_reading(t, dtype, heads, d, scales, eps):
    """The module under the reading "storage in `dtype`, every sum exact": the
    oracle's stage functions, with the token maps that a two-pass evaluation of
    Eq. (3) keeps between its passes (projected Q/K/V; aggregated Q) rounded
    once to the storage type.  Returns (out, parts) like orc.forward_staged."""
    r = lambda a: wk.round_to_dtype(a, dtype)
    qkv = r(orc.linear(t["x"], t["w_qkv"]))
    maps = orc.branch_maps(qkv, t["w_dw"], t["w_gpw"], heads, d, scales)
    for m in maps[1:]:
        B, H, W, _ = m.shape
        v = m.reshape(B, H, W, heads, 3, d)
        v[..., 0, :] = r(np.ascontiguousarray(v[..., 0, :]))
    att, kv = orc.attention_of_maps(maps, heads, d, eps)
    out = orc.linear(att, t["w_proj"])
    return out, {"qkv": qkv, "maps": maps, "att": att, "kv": kv, "q_tokens": orc.q_tokens_of(maps, heads, d)}


def gate_margin(q_tokens, kv, heads: int, d: int) -> np.ndarray:
    """Conditioning of Eq. (3) per (token, head-branch): (relu(Q).Ksum) / (|Q|.Ksum) in [0, 1].
    0 = no component passes the rectifier; tiny = the denominator is a rounding-sized remainder.
    q_tokens [B,H,W,S*heads*d], kv [B,S,heads,d,d+1] -> [B,H,W,S*heads]."""
    q = np.asarray(q_tokens, dtype=np.float64)
    B, H, W, _ = q.shape
    S = kv.shape[1]
    q = q.reshape(B, H * W, S, heads, d)
    ks = np.asarray(kv, dtype=np.float64)[..., d]
    num = np.einsum("bnshe,bshe->bnsh", np.maximum(q, 0.0), ks)
    den = np.einsum("bnshe,bshe->bnsh", np.abs(q), ks)
    out = np.where(den > 0, num / np.where(den > 0, den, 1.0), 1.0)
    return out.reshape(B, H, W, S * heads)


def hull_rows(state: np.ndarray) -> np.ndarray:
    """The rows KV[e, :d] / Ksum[e] (Ksum[e] > 0) of one Eq. (3) state [d, d+1]."""
    d = state.shape[0]
    live = state[:, d] > 0
    return state[live, :d] / state[live, d:d + 1]


def _fit_convex(A_blocks, target, scale):
    """min over lambda >= 0 with sum(lambda_block) = 1 per block of max|sum_block A_block lambda - target|.
    A_blocks: list of [m, k_i].  Returns the max-norm residual."""
    if not A_blocks:
        return float(np.abs(target).max()) if target.size else 0.0
    m = target.shape[0]
    w = 1e3 * max(scale, 1e-300)
    k = sum(a.shape[1] for a in A_blocks)
    A = np.zeros((m + len(A_blocks), k))
    b = np.concatenate([target, np.full(len(A_blocks), w)])
    c0 = 0
    for i, a in enumerate(A_blocks):
        A[:m, c0:c0 + a.shape[1]] = a
        A[m + i, c0:c0 + a.shape[1]] = w
        c0 += a.shape[1]
    lam, _ = nnls(A, b, maxiter=50 * k + 100)
    c0 = 0
    for a in A_blocks:                      # renormalise each block exactly onto the simplex
        s = lam[c0:c0 + a.shape[1]].sum()
        if s > 0:
            lam[c0:c0 + a.shape[1]] /= s
        c0 += a.shape[1]
    return float(np.abs(A[:m] @ lam - target).max())


def att_row_validity(row: np.ndarray, state: np.ndarray) -> float:
    """Distance (max-norm) of one attention row [d] from the admissible set of Eq. (3):
    {0} united with the convex hull of the state's rows KV[e,:]/Ksum[e]."""
    best = float(np.abs(row).max())         # the all-rectified-away answer: exactly 0
    R = hull_rows(state)
    if R.shape[0]:
        best = min(best, _fit_convex([R.T], row, np.abs(R).max()))
    return best


def token_validity(out_row, plain_out_row, plain_att_row, w_proj, states, ill, d, scale):
    """Distance of one output token [C] from the set Eq. (3) admits when the head-branches `ill`
    (indices m into the S*heads attention groups) may each be 0 or any point of their hull, and all
    other groups are the plain oracle's.  states[m] = that group's [d, d+1] state."""
    fixed = plain_out_row.copy()
    blocks = []
    for m in ill:
        cols = slice(m * d, (m + 1) * d)
        fixed -= w_proj[:, cols] @ plain_att_row[cols]
        blocks.append(w_proj[:, cols] @ hull_rows(states[m]).T)           # [C, live rows]
    target = out_row - fixed
    best = np.inf
    for alive in itertools.product((False, True), repeat=len(ill)):
        use = [b for b, a in zip(blocks, alive) if a and b.shape[1]]
        if len(use) != sum(alive):
            continue
        best = min(best, _fit_convex(use, target, scale))
    return float(best)


def first_order_bound(att_row, w_proj, kv_b, margin_row, heads, d, u, scale):
    """What the storage rounding of Q can do to one output token through ONE head-branch, to first order,
    in units of `scale`: the largest over the head-branches m of
    (2u / margin_m) * max_e |W_proj[:, m] (KV[e,:]/Ksum[e] - att_m)|_inf
    -- perturbations of size u|Q| move the denominator of Eq. (3) by u / margin of itself, and the row by that
    fraction of the way to a hull vertex.  kv_b [S, heads, d, d+1] are the states of the token's image;
    inf where a margin is 0."""
    worst = 0.0
    for m in range(margin_row.shape[0]):
        state = kv_b[m // heads, m % heads]
        rows = hull_rows(state)
        if rows.shape[0] == 0:
            continue
        cols = slice(m * d, (m + 1) * d)
        spread = np.abs(w_proj[:, cols] @ (rows - att_row[cols]).T).max()
        if spread <= 0:
            continue
        if margin_row[m] <= 0:
            return np.inf
        worst = max(worst, 2.0 * u / margin_row[m] * spread / scale)
    return float(worst)


class Judgement:
    """Outcome of judge_module / judge_core, printable."""

    def __init__(self, worst_ok, n_tokens, listed, predicted, tol):
        self.worst_ok, self.n_tokens, self.listed, self.predicted, self.tol = worst_ok, n_tokens, listed, predicted, tol

    def __str__(self):
        s = (f"plain oracle: max err {self.worst_ok:.2e} of max|out| over {self.n_tokens - len(self.listed)} of "
             f"{self.n_tokens} tokens (bar {self.tol:.0e}); ill-conditioned tokens listed {len(self.listed)}, "
             f"CPU-predicted {len(self.predicted)}")
        for tok, err, margin, dist in self.listed:
            s += f"\n    token {tok}: err {err:.3e}, gate margin {margin:.3e}, distance from admissible set {dist:.3e}"
        return s


def predicted_tokens(t, dtype, heads, d, scales, eps, plain_out, return_reading=False):
    """Tokens that the storage reading (CPU only) moves past the bar."""
    out_s, _ = storage_reading(t, dtype, heads, d, scales, eps)
    out_s = wk.round_to_dtype(out_s, dtype)
    err = np.abs(out_s - plain_out).max(-1) / np.abs(plain_out).max()
    toks = [tuple(int(i) for i in idx) for idx in np.argwhere(err > TOL[dtype])]
    return (toks, out_s) if return_reading else toks


def judge_module(got, t, dtype, heads, d, scales, eps, slack: int = 0) -> Judgement:
    """Judge a whole-module output `got` [B,H,W,C] (fp64 array of the GPU's values).  Raises
    AssertionError with the full list when a token is over the bar and not a predicted, valid
    ill-conditioned token, or when more tokens are listed than the CPU predicts (+ slack)."""
    tol = TOL[dtype]
    assert np.isfinite(got).all(), "non-finite values in GPU output"
    plain, parts = orc.forward_staged(t["x"], t["w_qkv"], t["w_dw"], t["w_gpw"], t["w_proj"], heads, d, scales, eps)
    assert got.shape == plain.shape
    scale = np.abs(plain).max()
    err = np.abs(got - plain).max(-1) / scale                          # [B,H,W]
    margin = gate_margin(parts["q_tokens"], parts["kv"], heads, d)     # [B,H,W,S*heads]
    over = [tuple(int(i) for i in idx) for idx in np.argwhere(err > tol)]
    predicted, reading = predicted_tokens(t, dtype, heads, d, scales, eps, plain, return_reading=True)
    listed, problems = [], []
    for tok in over:
        b = tok[0]
        ill = [int(m) for m in np.nonzero(margin[tok] < theta(dtype))[0]]
        states = {m: parts["kv"][b, m // heads, m % heads] for m in ill}
        dist = (token_validity(got[tok], plain[tok], parts["att"][tok], t["w_proj"], states, ill, d, scale) / scale
                if ill and len(ill) <= 4 else np.inf)
        listed.append((tok, float(err[tok]), float(margin[tok].min()), dist))
        if ill and dist <= tol:
            continue                                    # (i) + (ii)
        bound = first_order_bound(parts["att"][tok], t["w_proj"], parts["kv"][b], margin[tok], heads, d,
                                  UNIT_ROUNDOFF[dtype], scale)
        off_reading = float(np.abs(got[tok] - reading[tok]).max() / scale)
        if bound >= tol and off_reading <= tol:
            continue                                    # (iii)
        if not ill and bound < tol:
            problems.append(f"token {tok}: err {err[tok]:.3e} with a well-conditioned gate (margin {margin[tok].min():.3e}, "
                            f"first-order bound {bound:.3e})")
        elif bound >= tol and not ill:
            problems.append(f"token {tok}: err {err[tok]:.3e}, ill-conditioned to first order (bound {bound:.3e}) but "
                            f"{off_reading:.3e} away from the storage reading")
        else:
            problems.append(f"token {tok}: err {err[tok]:.3e}, not an admissible value of Eq. (3) (distance {dist:.3e}; "
                            f"{off_reading:.3e} away from the storage reading)")
    ok = np.ones(err.shape, dtype=bool)
    for tok in over:
        ok[tok] = False
    j = Judgement(float(err[ok].max()) if ok.any() else 0.0, int(err.size), listed, predicted, tol)
    if len(listed) > len(predicted) + slack:
        problems.append(f"{len(listed)} tokens over the bar, the storage reading predicts {len(predicted)}")
    assert not problems, "parity failed:\n  " + "\n  ".join(problems) + "\n  " + str(j)
    return j


def judge_core(att, qkv, t, dtype, heads, d, scales, eps, slack: int = 0) -> Judgement:
    """The same for the attention rows of msla_core_forward on a given projected map `qkv`:
    att [B,H,W,S*heads*d].  A row over the bar must belong to an ill-conditioned token-head and be
    exactly 0 or inside the hull of the oracle's state rows."""
    tol = TOL[dtype]
    assert np.isfinite(att).all(), "non-finite values in GPU output"
    plain, kv = orc.core_forward(qkv, t["w_dw"], t["w_gpw"], heads, d, scales, eps, return_kv=True)
    maps = orc.branch_maps(qkv, t["w_dw"], t["w_gpw"], heads, d, scales)
    margin = gate_margin(orc.q_tokens_of(maps, heads, d), kv, heads, d)           # [B,H,W,M]
    scale = np.abs(plain).max()
    B, H, W, M = margin.shape
    err = np.abs(att - plain).reshape(B, H, W, M, d).max(-1) / scale
    over = [tuple(int(i) for i in idx) for idx in np.argwhere(err > tol)]
    # CPU prediction: aggregated Q rounded once to the storage type, nothing else
    for m_ in maps[1:]:
        v = m_.reshape(B, H, W, heads, 3, d)
        v[..., 0, :] = wk.round_to_dtype(np.ascontiguousarray(v[..., 0, :]), dtype)
    att_s, _ = orc.attention_of_maps(maps, heads, d, eps)
    err_s = np.abs(wk.round_to_dtype(att_s, dtype) - plain).reshape(B, H, W, M, d).max(-1) / scale
    predicted = [tuple(int(i) for i in idx) for idx in np.argwhere(err_s > tol)]
    listed, problems = [], []
    for tok in over:
        b, y, x, m = tok
        row = att[b, y, x, m * d:(m + 1) * d]
        dist = att_row_validity(row, kv[b, m // heads, m % heads]) / scale
        listed.append((tok, float(err[tok]), float(margin[tok]), dist))
        if margin[tok] >= theta(dtype):
            problems.append(f"row {tok}: err {err[tok]:.3e} with a well-conditioned gate (margin {margin[tok]:.3e})")
        elif dist > tol:
            problems.append(f"row {tok}: err {err[tok]:.3e}, neither 0 nor in the hull (distance {dist:.3e})")
    ok = np.ones(err.shape, dtype=bool)
    for tok in over:
        ok[tok] = False
    j = Judgement(float(err[ok].max()) if ok.any() else 0.0, int(err.size), listed, predicted, tol)
    if len(listed) > len(predicted) + slack:
        problems.append(f"{len(listed)} rows over the bar, the storage reading predicts {len(predicted)}")
    assert not problems, "parity failed:\n  " + "\n  ".join(problems) + "\n  " + str(j)
    return j
