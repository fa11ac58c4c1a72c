"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle,
element by element on the same seeded inputs.

Bar (max over all elements): |gpu - oracle| <= tol * max|oracle| with
tol = 1e-4 for fp32 storage and 5e-3 for fp16 / bf16 storage (fp32 sums).

The expected value is always the PLAIN oracle (``oracle/``: the paper's definition in fp64, no
rounding, nothing taken from the GPU), on every token.  The only tokens judged differently are an
explicit, printed, counted list of tokens where Eq. (3) itself is ill-posed under 16-bit storage of Q
(the rectified part of a Q row is a rounding-sized remainder); each of them must be predicted by the
plain oracle's gate margin and be an admissible value of Eq. (3), and their number must not exceed
what storage rounding alone does on the CPU -- see tests/parity_model.py, which holds that protocol
and whose own CPU tests (tests/test_parity_model.py) derive its threshold.
Continuous intermediates (the projected map, the multi-scale Q tokens, the Eq. (3) states) are
compared with the plain oracle's as well.
"""
import numpy as np
import pytest
import torch

import parity_model as pm
from oracle import msla_oracle as orc
from paper_2205_14756_amd import msla
from paper_2205_14756_amd import workloads as wk

pytestmark = pytest.mark.gpu

TOL = pm.TOL
TDT = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a)).to(TDT[dtype]).cuda().contiguous()


def host(t):
    torch.cuda.synchronize()
    return t.detach().to(torch.float64).cpu().numpy()


def rel_err(got, ref):
    assert got.shape == ref.shape
    assert np.isfinite(got).all(), "non-finite values in GPU output"
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-300))


def poisoned_workspace(B, C, H, W, heads, d, scales, dtype):
    ws = msla.new_workspace(B, C, H, W, heads, d, scales, TDT[dtype])
    ws.fill_(0xFF)      # NaN pattern for every float type: unwritten reads show up
    return ws


def weights(t, dtype, scales):
    return (dev(t["w_dw"], dtype) if len(scales) else None, dev(t["w_gpw"], dtype) if len(scales) else None)


def run_forward(t, dtype, heads, d, scales, eps=1e-15, options=0):
    x = dev(t["x"], dtype)
    B, H, W, C = x.shape
    wdw, wg = weights(t, dtype, scales)
    out = torch.full_like(x, float("nan"))
    msla.msla_forward(x, dev(t["w_qkv"], dtype), wdw, wg, dev(t["w_proj"], dtype), heads, d, scales, eps,
                      out=out, workspace=poisoned_workspace(B, C, H, W, heads, d, scales, dtype), options=options)
    return host(out)


def gpu_stage_chain(t, dtype, heads, d, scales):
    """The stored intermediates of the GPU path, through its stage entry points."""
    x = dev(t["x"], dtype)
    B, H, W, C = x.shape
    wdw, wg = weights(t, dtype, scales)
    qkv = msla.msla_linear(x, dev(t["w_qkv"], dtype))
    q_ms, kv = msla.msla_multiscale_state(qkv, wdw, wg, heads, d, scales,
                                          workspace=poisoned_workspace(B, heads * d, H, W, heads, d, scales, dtype))
    return host(qkv), host(q_ms), host(kv)


def check_states(kv, kv_ref, tol):
    """Every Eq. (3) state against its own maximum (branches and heads differ in size)."""
    assert kv.shape == kv_ref.shape
    B, S, heads = kv.shape[:3]
    worst = 0.0
    for b in range(B):
        for s in range(S):
            for h in range(heads):
                worst = max(worst, rel_err(kv[b, s, h], kv_ref[b, s, h]))
    assert worst <= tol, f"Eq. (3) state off by {worst:.3e}"
    return worst


def check_module(t, dtype, heads, d, scales, eps=1e-15, options=0, stages=True):
    """msla_forward against the plain oracle on every token (pm.judge_module), and -- through the
    stage entry points -- the continuous intermediates against the plain oracle's."""
    tol = TOL[dtype]
    got = run_forward(t, dtype, heads, d, scales, eps, options)
    j = pm.judge_module(got, t, dtype, heads, d, scales, eps)
    print(f"  {j}", flush=True)
    if stages:
        _, parts = orc.forward_staged(t["x"], t["w_qkv"], t["w_dw"], t["w_gpw"], t["w_proj"], heads, d, scales, eps)
        qkv_g, q_g, kv_g = gpu_stage_chain(t, dtype, heads, d, scales)
        e_qkv = rel_err(qkv_g, parts["qkv"])
        e_q = rel_err(q_g, parts["q_tokens"])
        e_kv = check_states(kv_g, parts["kv"], tol)
        print(f"  stages vs plain oracle: qkv {e_qkv:.2e}  q_ms {e_q:.2e}  kv {e_kv:.2e}  (bar {tol:.0e})", flush=True)
        assert e_qkv <= tol and e_q <= tol
    return j


# ----------------------------------------------------------------- S0 / S5 stage

@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("n,c_in,c_out", [(1000, 64, 192), (128, 256, 768), (777, 80, 48),
                                          (300, 512, 272), (1, 16, 16), (2049, 128, 384),
                                          # output channels a multiple of 256: 64 channels a wave
                                          (1031, 256, 1024), (77, 96, 256), (2049, 128, 512)])
def test_linear(dtype, n, c_in, c_out):
    rng = np.random.default_rng(n + c_in)
    x = wk.round_to_dtype(rng.standard_normal((n, c_in)), dtype)
    w = wk.round_to_dtype(rng.standard_normal((c_out, c_in)) / np.sqrt(c_in), dtype)
    print(f"linear {dtype} n={n} {c_in}->{c_out}", flush=True)
    y = host(msla.msla_linear(dev(x, dtype), dev(w, dtype)))
    assert rel_err(y, orc.linear(x, w)) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("n,c_in,c_out", [(2049, 128, 384), (1000, 256, 768), (24, 256, 768), (777, 80, 48),
                                          (40, 512, 272), (1031, 256, 1024), (77, 96, 256)])
def test_linear_writes_only_its_own_rows(dtype, n, c_in, c_out):
    """Token counts that leave the last tile ragged: the rows behind the last token, which the same
    allocation holds, keep their contents."""
    import torch
    rng = np.random.default_rng(7 * n + c_out)
    x = wk.round_to_dtype(rng.standard_normal((n, c_in)), dtype)
    w = wk.round_to_dtype(rng.standard_normal((c_out, c_in)) / np.sqrt(c_in), dtype)
    print(f"linear, guard rows: {dtype} n={n} {c_in}->{c_out}", flush=True)
    guard = 64
    whole = torch.full((n + guard, c_out), 123.0, dtype=TDT[dtype], device="cuda")
    msla.msla_linear(dev(x, dtype), dev(w, dtype), y=whole[:n])
    assert rel_err(host(whole[:n]), orc.linear(x, w)) <= TOL[dtype]
    assert bool((whole[n:] == 123.0).all()), "rows past the last token were written"


def test_linear_repeated_launches_agree():
    """The same projection launched many times gives the same bits every time (a store whose data
    registers were overwritten one instruction later once corrupted a word in a few launches of a
    hundred at this shape)."""
    import torch
    n, c_in, c_out = 3 * 64 * 96, 256, 768
    rng = np.random.default_rng(5)
    x = wk.round_to_dtype(rng.standard_normal((n, c_in)), "f16")
    w = wk.round_to_dtype(rng.standard_normal((c_out, c_in)) / np.sqrt(c_in), "f16")
    print(f"linear, 150 launches: f16 n={n} {c_in}->{c_out}", flush=True)
    xd, wd = dev(x, "f16"), dev(w, "f16")
    first = msla.msla_linear(xd, wd)
    assert rel_err(host(first), orc.linear(x, w)) <= TOL["f16"]
    differing = sum(int(not torch.equal(first, msla.msla_linear(xd, wd))) for _ in range(150))
    assert differing == 0, f"{differing} of 150 launches differ from the first"


# -------------------------------------- S1-S4: aggregation, state, normalise-and-apply

STATE_CASES = [
    # B, H, W, heads, scales
    (1, 32, 32, 4, (5,)),
    (2, 13, 37, 2, (5,)),      # ragged in both directions, several tiles
    (1, 8, 32, 1, (3,)),       # exactly one tile
    (1, 3, 2, 2, (5,)),        # smaller than the kernel
    (1, 1, 1, 1, (3, 5)),      # single token
    (2, 19, 70, 3, (3, 5)),    # two aggregated scales, ragged
    (1, 9, 5, 2, ()),          # no aggregated scale
    (3, 40, 33, 2, (5,)),
    (8, 64, 64, 16, (5,)),     # enough (image, head) pairs that a workgroup walks over several tiles
    (1, 20, 41, 2, (7,)),      # 7x7 aggregation (general kernel for every storage type)
    (2, 5, 4, 1, (7,)),        # ... on a map smaller than the kernel
    (1, 33, 35, 3, (5, 7)),    # a matrix-core scale and a general-kernel scale in one module
]


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("B,H,W,heads,scales", STATE_CASES)
def test_multiscale_state_and_core(dtype, B, H, W, heads, scales):
    d = 16
    C = heads * d
    tol = TOL[dtype]
    print(f"state+core {dtype} B={B} {H}x{W} heads={heads} scales={scales}", flush=True)
    t = wk.random_module(B * 1000 + H * 10 + W, dtype, B, C, H, W, heads, d, scales)
    qkv = wk.round_to_dtype(orc.linear(t["x"], t["w_qkv"]), dtype)         # the given projected map
    maps = orc.branch_maps(qkv, t["w_dw"], t["w_gpw"], heads, d, scales)
    _, kv_ref = orc.attention_of_maps(maps, heads, d, 1e-15)
    q_ref = orc.q_tokens_of(maps, heads, d)
    wdw, wg = weights(t, dtype, scales)

    q_ms, kv = msla.msla_multiscale_state(dev(qkv, dtype), wdw, wg, heads, d, scales,
                                          workspace=poisoned_workspace(B, C, H, W, heads, d, scales, dtype))
    q_ms, kv = host(q_ms), host(kv)
    assert rel_err(q_ms, q_ref) <= tol
    assert np.array_equal(q_ms[..., :C], q_ref[..., :C])          # the raw branch is a copy
    check_states(kv, kv_ref, tol)

    att = host(msla.msla_core_forward(dev(qkv, dtype), wdw, wg, heads, d, scales, 1e-15,
                                      workspace=poisoned_workspace(B, C, H, W, heads, d, scales, dtype)))
    print(f"  {pm.judge_core(att, qkv, t, dtype, heads, d, scales, 1e-15)}", flush=True)


# ------------------------------------------------------------- whole module

@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("B,C,H,W,heads,scales", [
    (1, 64, 32, 32, 4, (5,)),
    (2, 32, 13, 37, 2, (5,)),
    (1, 48, 5, 7, 3, (3, 5)),
    (2, 80, 20, 9, 5, (3,)),
    (1, 16, 1, 1, 1, (5,)),
    (1, 32, 6, 6, 2, ()),
    (1, 272, 17, 40, 17, (5,)),     # more than one output-channel block in the projection
    (1, 48, 12, 20, 2, (5,)),       # C != heads * head_dim: narrower attention than the module
    (2, 32, 9, 31, 4, (3,)),        # ... and wider
    (1, 272, 9, 13, 17, (3, 5)),    # 51 head-branches (816 contraction slots), 272 input channels: long-contraction kernels
    (2, 512, 7, 9, 32, (5,)),       # 64 head-branches (1024 slots), 512 input channels
    (1, 384, 6, 11, 24, (5,)),      # 48 head-branches (768 slots), ragged 32-token tiles
    (1, 640, 5, 8, 40, (5,)),       # 80 head-branches: beyond the long-contraction kernel, tiled forms
    (2, 64, 19, 23, 4, (3, 5, 7)),  # four branches, 7x7 among them
])
def test_forward_small(dtype, B, C, H, W, heads, scales):
    d = 16
    print(f"forward {dtype} B={B} C={C} {H}x{W} heads={heads} scales={scales}", flush=True)
    t = wk.random_module(C * 100 + H + W, dtype, B, C, H, W, heads, d, scales)
    check_module(t, dtype, heads, d, scales)


@pytest.mark.parametrize("dtype,B,C,H,W,heads,scales", [
    ("f16", 4, 128, 64, 64, 8, (5,)),      # 16 head-branches, 128 output channels, two tiles per workgroup
    ("f16", 8, 128, 33, 35, 8, (3, 5)),    # 24 head-branches, ragged tiles, workgroups that cross images
    ("bf16", 8, 128, 33, 35, 8, (5,)),     # the hi/lo path over several ragged tiles
    ("f16", 3, 256, 64, 96, 16, (5,)),     # 32 head-branches, 256 output channels, three tiles per workgroup
    ("bf16", 2, 256, 64, 128, 16, (5,)),
    ("f16", 2, 64, 96, 96, 4, ()),         # no aggregated scale: 4 head-branches
])
def test_forward_several_tiles_per_workgroup(dtype, B, C, H, W, heads, scales):
    """Shapes at which the persistent projection and apply workgroups walk over several token
    tiles each (more than 256 tiles of 32 tokens), in every register-resident-weight variant."""
    d = 16
    print(f"forward, several tiles per workgroup: {dtype} B={B} C={C} {H}x{W} heads={heads} scales={scales}", flush=True)
    t = wk.random_module(C * 1000 + B * 100 + H + W, dtype, B, C, H, W, heads, d, scales)
    check_module(t, dtype, heads, d, scales)


@pytest.mark.parametrize("dtype,B,C,H,W,heads,scales", [
    ("f16", 1, 64, 5, 7, 4, (5,)),          # 35 tokens: every kernel's only tile is ragged
    ("bf16", 3, 128, 9, 11, 8, (3, 5)),     # 297 tokens, tiles that cross images
    ("f32", 2, 64, 9, 5, 4, (5,)),
    ("f16", 2, 256, 13, 17, 16, (5,)),      # the weight-stationary kernels of the headline shape, 442 tokens
])
def test_forward_writes_only_its_own_rows(dtype, B, C, H, W, heads, scales):
    """The output and the workspace each lie at the start of a larger allocation: what follows the last
    token, and the bytes behind the size msla_workspace_bytes reports, stay as they were."""
    d = 16
    print(f"forward, guard rows: {dtype} B={B} C={C} {H}x{W} heads={heads} scales={scales}", flush=True)
    t = wk.random_module(99 + C + H * W, dtype, B, C, H, W, heads, d, scales)
    x = dev(t["x"], dtype)
    wdw, wg = weights(t, dtype, scales)
    T, guard = B * H * W, 64
    whole = torch.full((T + guard, C), 123.0, dtype=TDT[dtype], device="cuda")
    out = whole[:T].view(B, H, W, C)
    n_ws = msla.msla_workspace_bytes(B, C, H, W, heads, d, scales, TDT[dtype])
    ws_whole = torch.full((n_ws + 4096,), 0xFF, dtype=torch.uint8, device="cuda")
    msla.msla_forward(x, dev(t["w_qkv"], dtype), wdw, wg, dev(t["w_proj"], dtype), heads, d, scales, 1e-15,
                      out=out, workspace=ws_whole[:n_ws])
    assert bool((ws_whole[n_ws:] == 0xFF).all()), "bytes past the workspace were written"
    # (parity of such shapes is the business of the tests above)
    assert np.isfinite(host(out)).all()
    assert bool((whole[T:] == 123.0).all()), "rows past the last token were written"


@pytest.mark.parametrize("dtype,B,C,H,W,heads,scales", [
    ("f16", 1, 272, 17, 40, 17, (5,)),      # tiled projection: its 128-token tiles overhang the head-major K|V map's padding
    ("f16", 3, 256, 64, 96, 16, (5,)),      # weight-stationary kernels, several tiles per workgroup
    ("bf16", 2, 128, 33, 35, 8, (3, 5)),
])
def test_forward_repeated_launches_agree(dtype, B, C, H, W, heads, scales):
    """The whole module launched many times on the same input gives the same bits every time: a
    write that lands where another workgroup also writes (a row past the last token, a piece of a
    neighbouring head) shows up as a difference between launches sooner or later."""
    d = 16
    print(f"forward, 60 launches: {dtype} B={B} C={C} {H}x{W} heads={heads} scales={scales}", flush=True)
    t = wk.random_module(31 + C + H, dtype, B, C, H, W, heads, d, scales)
    x = dev(t["x"], dtype)
    wdw, wg = weights(t, dtype, scales)
    wq, wp = dev(t["w_qkv"], dtype), dev(t["w_proj"], dtype)
    ws = poisoned_workspace(B, C, H, W, heads, d, scales, dtype)
    first = msla.msla_forward(x, wq, wdw, wg, wp, heads, d, scales, 1e-15, workspace=ws).clone()
    differing = 0
    for _ in range(60):
        out = msla.msla_forward(x, wq, wdw, wg, wp, heads, d, scales, 1e-15, workspace=ws)
        differing += int(not torch.equal(first, out))
    assert differing == 0, f"{differing} of 60 launches differ from the first"


@pytest.mark.parametrize("dtype,B,C,H,W,heads,scales", [
    ("f16", 2, 64, 37, 70, 4, (3, 5)),
    ("bf16", 1, 128, 64, 64, 8, (5,)),
])
def test_forward_general_aggregation_kernel_for_16_bit_types(dtype, B, C, H, W, heads, scales):
    """An image whose maps span 2 GiB or more leaves the matrix-core aggregation kernel for the
    general one (half-height tiles, same chunks); msla_forward_opts takes that path at any size."""
    d = 16
    print(f"forward, general aggregation kernel: {dtype} B={B} C={C} {H}x{W} heads={heads} scales={scales}", flush=True)
    t = wk.random_module(4242 + C + H, dtype, B, C, H, W, heads, d, scales)
    check_module(t, dtype, heads, d, scales, options=msla.MSLA_OPT_GENERAL_AGGREGATION, stages=False)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("B,C,H,W,heads", [(1, 32, 6, 6, 2), (2, 64, 96, 96, 4), (3, 80, 9, 20, 5)])
def test_forward_raw_branch_state_on_the_vector_alus(dtype, B, C, H, W, heads):
    """No aggregated scale, the Eq. (3) state accumulated with vector FMAs and wavefront shuffles
    (MSLA_OPT_STATE_VALU) instead of the matrix cores: the same bar."""
    print(f"forward, vector-ALU state: {dtype} B={B} C={C} {H}x{W} heads={heads}", flush=True)
    t = wk.random_module(515 + C + H, dtype, B, C, H, W, heads, 16, ())
    check_module(t, dtype, heads, 16, (), options=msla.MSLA_OPT_STATE_VALU, stages=False)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("B,C,H,W,heads,d,scales", [
    (1, 64, 9, 13, 8, 8, (5,)),         # head size 8
    (2, 64, 12, 21, 2, 32, (5,)),       # head size 32
    (1, 32, 1, 1, 4, 8, (3, 5)),        # a single token
    (2, 96, 17, 10, 3, 32, (3, 7)),     # three branches, ragged 64-token groups, C != heads * head size
    (1, 128, 30, 40, 16, 8, ()),        # no aggregated scale
    (1, 128, 64, 64, 4, 32, (5,)),      # several chunks per state
    (3, 128, 40, 72, 16, 8, (3, 5)),    # head size 8 as pairs on the head-size-16 kernels, several tiles, ragged
    (1, 64, 20, 20, 6, 8, (7,)),        # ... with a 7x7 scale; C != heads * head size
])
def test_forward_other_head_sizes(dtype, B, C, H, W, heads, d, scales):
    """Head sizes 8 and 32: the same bar, the same protocol.  Heads of size 8 run as pairs on the
    head-size-16 kernels (heads * 8 is a multiple of 16, so their number is even), heads of size 32 on the
    plain kernels of k_generic.hip."""
    print(f"forward {dtype} B={B} C={C} {H}x{W} heads={heads} head size {d} scales={scales}", flush=True)
    t = wk.random_module(C * 10 + H + d, dtype, B, C, H, W, heads, d, scales)
    check_module(t, dtype, heads, d, scales, stages=False)


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_forward_benchmark_configs_full_size(cfg):
    """The five workload shapes at full size, in the launch configuration the bench times."""
    wl = wk.WORKLOADS[cfg]
    print(f"full-size {wl.name}", flush=True)
    check_module(wk.make_inputs(wl), wl.dtype, wl.heads, wl.head_dim, wl.scales, wl.eps)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("B,C,H,W,heads,d,scales", [(2, 32, 13, 37, 2, 16, (5,)), (1, 128, 70, 65, 8, 16, (3, 5)),
                                                     (3, 80, 9, 20, 5, 16, ()), (2, 64, 21, 30, 8, 8, (5,)),
                                                     (2, 64, 19, 34, 2, 32, (5,)), (1, 96, 7, 9, 1, 32, ())])
def test_forward_channel_planar_layout(dtype, B, C, H, W, heads, d, scales):
    """x and out as [B, C, H, W]: bit for bit the token-major result, transposed (the token-major
    result itself is checked against the oracle above).  Heads of 16 channels, of 8 (as pairs) and of 32
    (the last case: C = 3 * heads * 32, the widest the parked result allows)."""
    print(f"forward NCHW {dtype} B={B} C={C} {H}x{W} heads={heads} head size {d} scales={scales}", flush=True)
    t = wk.random_module(77 + C + H, dtype, B, C, H, W, heads, d, scales)
    ref = run_forward(t, dtype, heads, d, scales)
    x = dev(np.ascontiguousarray(np.transpose(t["x"], (0, 3, 1, 2))), dtype)
    wdw, wg = weights(t, dtype, scales)
    out = torch.full_like(x, float("nan"))
    msla.msla_forward(x, dev(t["w_qkv"], dtype), wdw, wg, dev(t["w_proj"], dtype), heads, d, scales, 1e-15,
                      out=out, workspace=poisoned_workspace(B, C, H, W, heads, d, scales, dtype),
                      layout=msla.MSLA_NCHW)
    assert np.array_equal(np.transpose(host(out), (0, 2, 3, 1)), ref)


def test_forward_replays_from_a_hip_graph():
    """The module allocates nothing and records only kernel launches, so it can be captured into a
    HIP graph: every replay -- with eager work and synchronisations of the program's own between
    them -- must reproduce the eager result bit for bit."""
    wl = wk.WORKLOADS[2]
    t = wk.make_inputs(wl)
    dtype = wl.dtype
    x = dev(t["x"], dtype)
    B, H, W, C = x.shape
    wdw, wg = weights(t, dtype, wl.scales)
    wq, wp = dev(t["w_qkv"], dtype), dev(t["w_proj"], dtype)
    ws = poisoned_workspace(B, C, H, W, wl.heads, wl.head_dim, wl.scales, dtype)
    eager = torch.full_like(x, float("nan"))
    msla.msla_forward(x, wq, wdw, wg, wp, wl.heads, wl.head_dim, wl.scales, wl.eps, out=eager, workspace=ws)
    torch.cuda.synchronize()
    out = torch.full_like(x, float("nan"))
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        graph.capture_begin()
        msla.msla_forward(x, wq, wdw, wg, wp, wl.heads, wl.head_dim, wl.scales, wl.eps, out=out, workspace=ws,
                          stream=side)
        graph.capture_end()
    torch.cuda.current_stream().wait_stream(side)
    for i in range(3):
        out.fill_(float("nan"))
        ws.fill_(0xFF if i % 2 else 0x7F)                 # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), f"replay {i} differs from the eager result"


def test_zeroed_tokens_give_exact_zero_in_raw_branch():
    # whole tokens of x set to zero: Q = K = V = 0 there, so the raw-branch rows of those
    # tokens are 0 / (0 + eps) = 0 exactly, never NaN
    dtype, B, C, H, W, heads, d, scales = "f16", 2, 64, 16, 40, 4, 16, (5,)
    t = wk.random_module(4242, dtype, B, C, H, W, heads, d, scales, zero_token_frac=0.1)
    qkv = wk.round_to_dtype(orc.linear(t["x"], t["w_qkv"]), dtype)
    wdw, wg = weights(t, dtype, scales)
    att = host(msla.msla_core_forward(dev(qkv, dtype), wdw, wg, heads, d, scales, 1e-15))
    dead = (t["x"] == 0).all(-1)
    assert dead.sum() > 20
    assert np.array_equal(att[dead][:, :C], np.zeros((int(dead.sum()), C)))
    check_module(t, dtype, heads, d, scales)


def test_forward_is_deterministic_and_batch_independent():
    wl = wk.WORKLOADS[2]
    t = wk.make_inputs(wl)
    a = run_forward(t, wl.dtype, wl.heads, wl.head_dim, wl.scales)
    b = run_forward(t, wl.dtype, wl.heads, wl.head_dim, wl.scales)
    assert np.array_equal(a, b)
    t2 = dict(t)
    t2["x"] = np.concatenate([t["x"], t["x"][:, ::-1].copy()], 0)
    c = run_forward(t2, wl.dtype, wl.heads, wl.head_dim, wl.scales)
    assert np.array_equal(c[:1], a)


def test_large_magnitude_keys_do_not_overflow_fp16_state():
    # sum_n relu(K_n) exceeds the fp16 range here; the state operands are rescaled, the output is not
    dtype, B, C, H, W, heads, d = "f16", 1, 32, 64, 64, 2, 16
    t = wk.random_module(31337, dtype, B, C, H, W, heads, d, (5,))
    qkv = wk.round_to_dtype(orc.linear(t["x"], t["w_qkv"]) * 60.0, dtype)
    maps = orc.branch_maps(qkv, t["w_dw"], t["w_gpw"], heads, d, (5,))
    _, kv = orc.attention_of_maps(maps, heads, d, 1e-15)
    assert kv[..., d].max() > 65504
    wdw, wg = weights(t, dtype, (5,))
    _, kv_g = msla.msla_multiscale_state(dev(qkv, dtype), wdw, wg, heads, d, (5,))
    check_states(host(kv_g), kv, TOL[dtype])
    att = host(msla.msla_core_forward(dev(qkv, dtype), wdw, wg, heads, d, (5,), 1e-15))
    print(f"  {pm.judge_core(att, qkv, t, dtype, heads, d, (5,), 1e-15)}", flush=True)
