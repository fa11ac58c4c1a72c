"""Seeded synthetic inputs and the benchmark shapes.

This module holds NONE of the method's arithmetic: it only names the workload
shapes and draws random tensors.  It is the one module that both the GPU tests
and the CPU oracle's callers use, so that both sides see identical inputs.

Recipe (per workload index i, 1-based): ``rng = numpy.random.default_rng(1000+i)``;
drawn in fp64 in this order: ``x ~ N(0,1)`` ``[B,H,W,C]``; ``w_qkv ~ N(0,1/C)``
``[3*heads*d, C]``; per aggregated scale ``w_dw ~ N(0,1/k^2)`` ``[3*heads*d,k,k]``;
``w_gpw ~ N(0,1/d)`` ``[A, 3*heads*d, d]``; ``w_proj ~ N(0,1/(S*heads*d))``
``[C, S*heads*d]``; workloads with ``zero_frac`` then zero ``x`` where a further
``rng.random(x.shape) < zero_frac``.  Every tensor is rounded once to the
storage dtype; the fp64 arrays returned hold exactly those rounded values.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Tuple

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str                      # "f32" | "f16" | "bf16" (storage; sums are fp32 on the GPU)
    B: int
    C: int
    H: int
    W: int
    heads: int
    head_dim: int
    scales: Tuple[int, ...]         # aggregated kernel sizes; the raw branch is always present
    eps: float = 1e-15
    zero_frac: float = 0.0
    seed: int = 0

    @property
    def tokens(self) -> int:
        return self.B * self.H * self.W

    @property
    def branches(self) -> int:
        return 1 + len(self.scales)

    @property
    def qkv_channels(self) -> int:
        return 3 * self.heads * self.head_dim

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def algorithmic_bytes(self, core_only: bool = False) -> int:
        """HBM bytes the two-pass method itself must move with ideal fusion
        inside each pass: read x, write qkv; read qkv, write the aggregated Q
        maps; read raw + aggregated Q, write out  ->  e*C*T*(9+2A)
        (qkv -> att only: e*C*T*(5+3A))."""
        A = len(self.scales)
        units = (5 + 3 * A) if core_only else (9 + 2 * A)
        return self.elem_bytes * self.heads * self.head_dim * self.tokens * units


WORKLOADS: Dict[int, Workload] = {
    1: Workload("cfg1_f32_1x64x32x32_h4_s5", "f32", 1, 64, 32, 32, 4, 16, (5,), seed=1001),
    2: Workload("cfg2_f16_1x128x64x128_h8_s5", "f16", 1, 128, 64, 128, 8, 16, (5,), seed=1002),
    3: Workload("cfg3_f16_1x512x32x64_h32_s5", "f16", 1, 512, 32, 64, 32, 16, (5,), seed=1003),
    4: Workload("cfg4_bf16_1x128x256x256_h8_s35", "bf16", 1, 128, 256, 256, 8, 16, (3, 5), seed=1004),
    5: Workload("cfg5_f16_8x256x64x128_h16_s5_z10", "f16", 8, 256, 64, 128, 16, 16, (5,),
                zero_frac=0.1, seed=1005),
}


def round_to_dtype(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round an fp64 array once to the storage dtype; return the values as fp64."""
    a = np.asarray(a, dtype=np.float64)
    if dtype == "f32":
        return a.astype(np.float32).astype(np.float64)
    if dtype == "f16":
        return a.astype(np.float16).astype(np.float64)
    if dtype == "bf16":
        # round-to-nearest-even on the upper 16 bits of the fp32 pattern
        f = a.astype(np.float32)
        u = f.view(np.uint32).astype(np.uint64)
        u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
        return u.astype(np.uint32).view(np.float32).reshape(a.shape).astype(np.float64)
    raise ValueError(f"unknown dtype {dtype!r}")


def make_inputs(wl: Workload, batch: int | None = None) -> Dict[str, np.ndarray]:
    """Draw the workload's tensors (fp64 arrays holding storage-rounded values).

    ``batch`` (<= wl.B) keeps only the first images of ``x``; the draw itself is
    always the full one so a sub-batch sees the same values as the full batch.
    """
    rng = np.random.default_rng(wl.seed)
    ch = wl.qkv_channels
    d = wl.head_dim
    S = wl.branches
    x = rng.standard_normal((wl.B, wl.H, wl.W, wl.C))
    w_qkv = rng.standard_normal((ch, wl.C)) / np.sqrt(wl.C)
    w_dw = [rng.standard_normal((ch, k, k)) / k for k in wl.scales]
    w_gpw = rng.standard_normal((len(wl.scales), ch, d)) / np.sqrt(d)
    w_proj = rng.standard_normal((wl.C, S * wl.heads * d)) / np.sqrt(S * wl.heads * d)
    if wl.zero_frac > 0.0:
        x = np.where(rng.random(x.shape) < wl.zero_frac, 0.0, x)
    if batch is not None:
        x = x[:batch]
    w_dw_flat = (np.concatenate([w.reshape(-1) for w in w_dw])
                 if w_dw else np.zeros(0, dtype=np.float64))
    r = lambda a: round_to_dtype(a, wl.dtype)
    return {"x": r(x), "w_qkv": r(w_qkv), "w_dw": r(w_dw_flat), "w_gpw": r(w_gpw),
            "w_proj": r(w_proj)}


def random_module(seed: int, dtype: str, B: int, C: int, H: int, W: int, heads: int,
                  head_dim: int, scales, zero_token_frac: float = 0.0) -> Dict[str, np.ndarray]:
    """Same distributions at an arbitrary shape (for ragged / edge-case tests).
    ``zero_token_frac`` zeroes whole tokens of x (all channels), which makes
    Q = K = V = 0 for them in the raw branch."""
    wl = Workload("adhoc", dtype, B, C, H, W, heads, head_dim, tuple(scales), seed=seed)
    t = make_inputs(wl)
    if zero_token_frac > 0.0:
        rng = np.random.default_rng(seed + 7919)
        mask = rng.random((B, H, W, 1)) < zero_token_frac
        t["x"] = np.where(mask, 0.0, t["x"])
    return t


def ffn_weights(seed: int, dtype: str, C: int, hidden: int) -> Dict[str, np.ndarray]:
    """Seeded weights of the FFN+DWConv half of the building block (the same recipe: N(0, 1/fan_in),
    fan_in = C, 9 and hidden; rounded once to the storage dtype): w1 [hidden, C], w_ffn_dw [hidden, 3, 3],
    w2 [C, hidden]."""
    rng = np.random.default_rng(seed)
    w1 = rng.standard_normal((hidden, C)) / np.sqrt(C)
    w_dw = rng.standard_normal((hidden, 3, 3)) / 3.0
    w2 = rng.standard_normal((C, hidden)) / np.sqrt(hidden)
    r = lambda a: round_to_dtype(a, dtype)
    return {"w1": r(w1), "w_ffn_dw": r(w_dw), "w2": r(w2)}
