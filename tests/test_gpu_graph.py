"""The entry points under HIP graph capture: a caller with a launch-bound loop (the small workloads are
25-50 us of four or five kernels) records the module once and replays it.  Every entry point only
launches kernels on the caller's stream -- no allocation, no memset, no synchronisation -- so it can be
captured; what is checked here is that each replay reproduces the eager result bit for bit, with eager
work and synchronisations between the replays, and that a replay picks up new contents of the input
buffer."""
import numpy as np
import pytest
import torch

from paper_2205_14756_amd import msla
from paper_2205_14756_amd import workloads as wk

pytestmark = pytest.mark.gpu

TDT = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a)).to(TDT[dtype]).cuda().contiguous()


def same_bits(a, b):
    return bool((a.view(torch.uint8) == b.view(torch.uint8)).all())


@pytest.mark.parametrize("index", [1, 2, 3])
def test_forward_replays_match_eager(index):
    wl = wk.WORKLOADS[index]
    print(f"graph capture of msla_forward: {wl.name}", flush=True)
    t = wk.make_inputs(wl)
    tdt = TDT[wl.dtype]
    x, w_qkv, w_dw, w_gpw, w_proj = (dev(t[k], wl.dtype) for k in ("x", "w_qkv", "w_dw", "w_gpw", "w_proj"))
    x2 = dev(np.roll(t["x"], 3, axis=1) * 0.5, wl.dtype)
    ws = msla.new_workspace(wl.B, wl.C, wl.H, wl.W, wl.heads, wl.head_dim, wl.scales, tdt)
    out = torch.empty_like(x)
    xin = x.clone()

    def call(stream=None):
        msla.msla_forward(xin, w_qkv, w_dw, w_gpw, w_proj, wl.heads, wl.head_dim, wl.scales, wl.eps, out=out,
                          workspace=ws, stream=stream)

    # eager results for both inputs (these calls also do the per-kernel set-up a first call does)
    call()
    torch.cuda.synchronize()
    ref1 = out.clone()
    xin.copy_(x2)
    call()
    torch.cuda.synchronize()
    ref2 = out.clone()
    assert not same_bits(ref1, ref2)
    xin.copy_(x)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        call(torch.cuda.current_stream())
    torch.cuda.synchronize()

    other = wk.WORKLOADS[2 if index != 2 else 1]       # eager work of another shape between the replays
    ot = wk.make_inputs(other)
    oargs = [dev(ot[k], other.dtype) for k in ("x", "w_qkv", "w_dw", "w_gpw", "w_proj")]
    for rep, (src, ref) in enumerate(((x, ref1), (x2, ref2), (x, ref1), (x2, ref2))):
        xin.copy_(src)
        out.fill_(float("nan"))
        ws.fill_(0xFF)                                  # nothing may depend on what the last call left
        graph.replay()
        torch.cuda.synchronize()
        assert same_bits(out, ref), f"replay {rep} differs from the eager result"
        msla.msla_forward(*oargs, other.heads, other.head_dim, other.scales, other.eps)
        torch.cuda.synchronize()


def test_block_replays_match_eager():
    """The whole building block (attention module + FFN, residuals in the epilogues) recorded once."""
    B, C, H, W, heads, hidden, dtype = 1, 128, 32, 64, 8, 512, "f16"
    print(f"graph capture of msla_block_forward: {dtype} {B}x{H}x{W}x{C} hidden {hidden}", flush=True)
    wl = wk.Workload("graph_block", dtype, B, C, H, W, heads, 16, (5,), seed=4242)
    t = wk.make_inputs(wl)
    f = wk.ffn_weights(4243, dtype, C, hidden)
    args = [dev(t[k], dtype) for k in ("w_qkv", "w_dw", "w_gpw", "w_proj")] + [dev(f[k], dtype) for k in ("w1", "w_ffn_dw", "w2")]
    x = dev(t["x"], dtype)
    xin = x.clone()
    out = torch.empty_like(x)
    ws = torch.empty(msla.msla_block_workspace_bytes(B, C, H, W, heads, 16, (5,), hidden, TDT[dtype]), dtype=torch.uint8,
                     device="cuda")

    def call(stream=None):
        msla.msla_block_forward(xin, *args, heads, 16, (5,), 1e-15, msla.MSLA_ACT_HSWISH, out=out, workspace=ws,
                                stream=stream)

    call()
    torch.cuda.synchronize()
    ref = out.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        call(torch.cuda.current_stream())
    torch.cuda.synchronize()
    for rep in range(3):
        out.fill_(float("nan"))
        ws.fill_(0xFF)
        graph.replay()
        torch.cuda.synchronize()
        assert same_bits(out, ref), f"replay {rep} differs from the eager result"
        (xin * 2).sum().item()                          # eager work and a synchronisation in between
