"""fp64 CPU oracle of the other half of the EfficientViT building block: the FFN with a
depthwise convolution (FFN+DWConv) and the block that chains it behind the multi-scale linear
attention module (paper Section 3.1, first paragraph below "Enhancing ReLU linear attention", and
Fig. 2 left; Section 3.2 places the block in stages 3 and 4).

TEST INFRASTRUCTURE, NOT PRODUCT CODE: only ``tests/``, the smoke check and the bench's CPU legs
may import this.  It composes the plain stage functions of ``msla_oracle`` (1x1 projection,
depthwise convolution: each a direct loop nest in fp64) with numpy elementwise operations; nothing
is rounded, blocked or fused.

What the paper fixes: the block is the MSLA module followed by an FFN into which a depthwise
convolution is inserted.  What it does not print (its figure is not in the text, its
configurations live in a repository that is not here) and is therefore a declared reading, shared
with the GPU path by specification only:
  - the FFN is  1x1 expand (C -> E)  ->  activation  ->  depthwise 3x3 (stride 1, zero padding 1,
    cross-correlation)  ->  activation  ->  1x1 project (E -> C), no activation after the projection
    (the inverted-bottleneck convention the paper's MBConv blocks follow);
  - E ("hidden") and the activation (ReLU, or hard-swish  a * clip(a + 3, 0, 6) / 6) are arguments;
  - both halves are residual:  y = x + MSLA(x),  out = y + FFN(y);
  - no bias and no normalisation anywhere.

Pins (tests/test_block_oracle_pins.py): hand-counted 3x3 box sums on a small map
(tests/golden/dwconv_box3_counts_3x4.txt); closed-form activation values; identity weights reduce
the FFN to out = y + relu(y); a recomposition with torch.nn.functional.conv2d / hardswish / relu;
zero projection weights reduce the block to its residual paths.  Parity unpinned: only the
declared readings above, which are definitions.
"""
from __future__ import annotations

import numpy as np

from . import msla_oracle as orc

ACT_RELU, ACT_HSWISH = 0, 1


def activation(a, act: int) -> np.ndarray:
    a = np.asarray(a, dtype=np.float64)
    if act == ACT_RELU:
        return np.maximum(a, 0.0)
    if act == ACT_HSWISH:
        return a * np.clip(a + 3.0, 0.0, 6.0) / 6.0
    raise ValueError(f"unknown activation {act}")


def ffn_forward(y, w1, w_dw, w2, act: int = ACT_RELU, return_parts: bool = False):
    """out = y + W2 . act(DW3x3(act(W1 . y))).
    y [B,H,W,C]; w1 [E,C]; w_dw [E,3,3]; w2 [C,E]."""
    y = np.asarray(y, dtype=np.float64)
    E, C = np.asarray(w1).shape
    assert y.shape[-1] == C and np.asarray(w_dw).shape == (E, 3, 3) and np.asarray(w2).shape == (C, E)
    h = activation(orc.linear(y, w1), act)
    g = activation(orc.dwconv(h, w_dw), act)
    out = y + orc.linear(g, w2)
    return (out, {"h": h, "g": g}) if return_parts else out


def block_forward(x, w_qkv, w_dw, w_gpw, w_proj, heads: int, d: int, scales, eps: float,
                  w1, w_ffn_dw, w2, act: int = ACT_RELU, return_parts: bool = False):
    """The whole building block: y = x + MSLA(x); out = y + FFN(y)."""
    x = np.asarray(x, dtype=np.float64)
    y = x + orc.forward(x, w_qkv, w_dw, w_gpw, w_proj, heads, d, scales, eps)
    out = ffn_forward(y, w1, w_ffn_dw, w2, act)
    return (out, {"y": y}) if return_parts else out
