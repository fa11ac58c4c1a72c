"""CPU pins of oracle/block_oracle.py (the FFN+DWConv half and the whole building block:
Section 3.1, Fig. 2 left)."""
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import block_oracle as blk
from oracle import msla_oracle as orc
from paper_2205_14756_amd import workloads as wk

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _table(name):
    rows = [l.split() for l in open(os.path.join(GOLDEN, name)) if l.strip() and not l.startswith("#")]
    return np.array(rows, dtype=np.float64)


def test_box3_counts_match_the_hand_counted_table():
    want = _table("dwconv_box3_counts_3x4.txt")
    E = 5
    h = np.ones((1, 3, 4, E))
    got = orc.dwconv(h, np.ones((E, 3, 3)))
    for c in range(E):
        assert np.array_equal(got[0, :, :, c], want)
    # through the FFN: identity expand (E = C), relu, box filter, relu, W2 picks channel 0 -> y + counts
    C = 3
    y = np.ones((1, 3, 4, C))
    w2 = np.zeros((C, C)); w2[:, 0] = 1.0
    out = blk.ffn_forward(y, np.eye(C), np.ones((C, 3, 3)), w2, blk.ACT_RELU)
    for c in range(C):
        assert np.array_equal(out[0, :, :, c], 1.0 + want)


def test_activation_closed_forms():
    a = np.array([-4.0, -3.0, -1.0, 0.0, 1.0, 3.0, 5.0])
    assert np.array_equal(blk.activation(a, blk.ACT_RELU), [0, 0, 0, 0, 1, 3, 5])
    # hard-swish: 0 below -3, identity above 3, a(a+3)/6 between: -1 -> -1/3, 1 -> 2/3
    assert np.allclose(blk.activation(a, blk.ACT_HSWISH), [0.0, 0.0, -1.0 / 3.0, 0.0, 2.0 / 3.0, 3.0, 5.0], rtol=0, atol=1e-15)
    with pytest.raises(ValueError):
        blk.activation(a, 7)


def test_identity_weights_reduce_the_ffn_to_y_plus_relu_y():
    rng = np.random.default_rng(3)
    C = 6
    y = rng.standard_normal((2, 5, 7, C))
    delta = np.zeros((C, 3, 3)); delta[:, 1, 1] = 1.0
    out = blk.ffn_forward(y, np.eye(C), delta, np.eye(C), blk.ACT_RELU)
    assert np.allclose(out, y + np.maximum(y, 0.0), rtol=0, atol=1e-15)
    # a delta one tap to the right reads the token at x + 1 (cross-correlation), zero beyond the edge
    right = np.zeros((C, 3, 3)); right[:, 1, 2] = 1.0
    out = blk.ffn_forward(y, np.eye(C), right, np.eye(C), blk.ACT_RELU)
    shifted = np.zeros_like(y); shifted[:, :, :-1] = np.maximum(y, 0.0)[:, :, 1:]
    assert np.allclose(out, y + shifted, rtol=0, atol=1e-15)
    # ... and one tap down reads the token at y + 1
    down = np.zeros((C, 3, 3)); down[:, 2, 1] = 1.0
    out = blk.ffn_forward(y, np.eye(C), down, np.eye(C), blk.ACT_RELU)
    shifted = np.zeros_like(y); shifted[:, :-1] = np.maximum(y, 0.0)[:, 1:]
    assert np.allclose(out, y + shifted, rtol=0, atol=1e-15)


@pytest.mark.parametrize("act", [blk.ACT_RELU, blk.ACT_HSWISH])
def test_ffn_against_a_library_recomposition(act):
    rng = np.random.default_rng(11 + act)
    B, H, W, C, E = 2, 6, 9, 8, 24
    y = rng.standard_normal((B, H, W, C))
    w = wk.ffn_weights(5, "f32", C, E)
    out, parts = blk.ffn_forward(y, w["w1"], w["w_ffn_dw"], w["w2"], act, return_parts=True)
    f = F.relu if act == blk.ACT_RELU else F.hardswish
    t = torch.from_numpy(y).permute(0, 3, 1, 2)                                   # NCHW, fp64
    h = f(F.conv2d(t, torch.from_numpy(w["w1"])[:, :, None, None]))
    g = f(F.conv2d(h, torch.from_numpy(w["w_ffn_dw"])[:, None], padding=1, groups=E))
    ref = t + F.conv2d(g, torch.from_numpy(w["w2"])[:, :, None, None])
    assert np.allclose(parts["h"], h.permute(0, 2, 3, 1).numpy(), rtol=1e-12, atol=1e-13)
    assert np.allclose(parts["g"], g.permute(0, 2, 3, 1).numpy(), rtol=1e-12, atol=1e-13)
    assert np.allclose(out, ref.permute(0, 2, 3, 1).numpy(), rtol=1e-12, atol=1e-13)
    # a transposed w2 or a dropped residual would not pass
    assert not np.allclose(out - y, ref.permute(0, 2, 3, 1).numpy(), atol=1e-3)


def test_block_reduces_to_its_residual_paths():
    heads, d, scales = 2, 16, (5,)
    C, E = 32, 64
    t = wk.random_module(77, "f32", 2, C, 6, 7, heads, d, scales)
    w = wk.ffn_weights(78, "f32", C, E)
    args = (t["x"], t["w_qkv"], t["w_dw"], t["w_gpw"], t["w_proj"], heads, d, scales, 1e-15)
    m = orc.forward(*args)
    # FFN projection zero: out = x + MSLA(x)
    out = blk.block_forward(*args, w["w1"], w["w_ffn_dw"], np.zeros_like(w["w2"]))
    assert np.allclose(out, t["x"] + m, rtol=0, atol=1e-14)
    # attention projection zero as well: out = x
    args0 = (t["x"], t["w_qkv"], t["w_dw"], t["w_gpw"], np.zeros_like(t["w_proj"]), heads, d, scales, 1e-15)
    out = blk.block_forward(*args0, w["w1"], w["w_ffn_dw"], np.zeros_like(w["w2"]))
    assert np.array_equal(out, t["x"])
    # the general case is the composition of the two halves, residuals included
    out, parts = blk.block_forward(*args, w["w1"], w["w_ffn_dw"], w["w2"], blk.ACT_HSWISH, return_parts=True)
    assert np.allclose(parts["y"], t["x"] + m, rtol=0, atol=1e-14)
    assert np.allclose(out, blk.ffn_forward(t["x"] + m, w["w1"], w["w_ffn_dw"], w["w2"], blk.ACT_HSWISH), rtol=0, atol=1e-14)
    assert np.abs(out - parts["y"]).max() > 0.1
