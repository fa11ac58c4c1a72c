"""CPU-only checks of the C-ABI library: it loads, exports every symbol that
include/msla.h declares, and rejects bad arguments on the host before any
launch (so none of these calls touches a GPU)."""
import ctypes
import os
import re

import pytest

from paper_2205_14756_amd import build as msla_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

OK, INVALID, UNSUPPORTED, WORKSPACE = 0, -1, -2, -3
F32, F16, BF16 = 0, 1, 2


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(msla_build.LIB):
        msla_build.build(True)
    return ctypes.CDLL(msla_build.LIB)


def declared_functions():
    text = open(os.path.join(ROOT, "include", "msla.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(msla_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert set(names) == {"msla_error_string", "msla_workspace_bytes", "msla_forward", "msla_forward_opts", "msla_forward_profiled",
                          "msla_core_forward",
                          "msla_multiscale_state", "msla_multiscale_state_static", "msla_linear",
                          "msla_ffn_workspace_bytes", "msla_ffn_forward", "msla_block_workspace_bytes", "msla_block_forward",
                          "msla_softmax_attention", "msla_linear_attention_backward_workspace_bytes",
                          "msla_linear_attention_backward"}
    for n in names:
        assert getattr(lib, n) is not None
    from paper_2205_14756_amd import msla
    assert set(msla.EXPORTS) == set(names)
    for n in names:
        if n != "msla_error_string":
            assert callable(getattr(msla, n))


def test_error_strings(lib):
    lib.msla_error_string.restype = ctypes.c_char_p
    seen = set()
    for code in (0, -1, -2, -3, -4, 17):
        s = lib.msla_error_string(code)
        assert s and len(s) > 3
        seen.add(s)
    assert len(seen) == 6


def _ws(lib, B, C, H, W, heads, d, scales, dt):
    arr = (ctypes.c_int * max(1, len(scales)))(*scales)
    out = ctypes.c_size_t(12345)
    st = lib.msla_workspace_bytes(B, C, H, W, heads, d, arr, len(scales), dt, ctypes.byref(out))
    return st, out.value


def test_workspace_bytes(lib):
    st, n = _ws(lib, 8, 256, 64, 128, 16, 16, [5], F16)
    assert st == OK
    T, Ct, S = 8 * 64 * 128, 256, 2
    # at least the multi-scale Q map and the raw K/V map, and not absurdly more
    assert T * S * Ct * 2 + T * 2 * Ct * 2 <= n <= T * S * Ct * 2 + T * 2 * Ct * 2 + (64 << 20)
    st32, n32 = _ws(lib, 1, 64, 32, 32, 4, 16, [5], F32)
    assert st32 == OK and n32 >= 1024 * (2 * 64 + 2 * 64) * 4
    assert _ws(lib, 1, 64, 32, 32, 4, 16, [], F32)[0] == OK
    # invalid
    assert _ws(lib, 0, 64, 32, 32, 4, 16, [5], F32)[0] == INVALID
    assert _ws(lib, 1, 64, 32, 32, 4, 16, [4], F32)[0] == INVALID      # even kernel
    assert _ws(lib, 1, 64, 32, 32, 4, 16, [5], 9)[0] == INVALID        # bad dtype
    assert _ws(lib, 1, 64, -3, 32, 4, 16, [5], F32)[0] == INVALID
    assert lib.msla_workspace_bytes(1, 64, 32, 32, 4, 16, None, 1, F32, ctypes.byref(ctypes.c_size_t())) == INVALID
    assert lib.msla_workspace_bytes(1, 64, 32, 32, 4, 16, None, 0, F32, None) == INVALID
    # unsupported
    assert _ws(lib, 1, 64, 32, 32, 8, 8, [5], F32)[0] == OK            # head_dim 8 and 32: the plain kernels
    assert _ws(lib, 1, 64, 32, 32, 2, 32, [5], F16)[0] == OK
    assert _ws(lib, 1, 96, 32, 32, 4, 24, [5], F32)[0] == UNSUPPORTED  # head_dim not in {8, 16, 32}
    assert _ws(lib, 1, 64, 32, 32, 4, 16, [9], F32)[0] == UNSUPPORTED   # kernel sizes other than 3, 5, 7
    assert _ws(lib, 1, 64, 32, 32, 4, 16, [7], F32)[0] == OK
    assert _ws(lib, 1, 60, 32, 32, 4, 16, [5], F32)[0] == UNSUPPORTED  # C not a multiple of 16
    # a failed query leaves *bytes alone
    assert _ws(lib, 1, 64, 32, 32, 4, 16, [9], F32)[1] == 12345


def _fwd(lib, x=0x1000, wq=0x1000, wd=0x1000, wg=0x1000, wp=0x1000, out=0x2000, ws=0x3000, ws_bytes=1 << 40,
         B=1, C=64, H=32, W=32, heads=4, d=16, scales=(5,), eps=1e-15, dt=F32, layout=0):
    lib.msla_forward.argtypes = [ctypes.c_void_p] * 7 + [ctypes.c_size_t] + [ctypes.c_int] * 6 + \
        [ctypes.POINTER(ctypes.c_int), ctypes.c_int, ctypes.c_float, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    arr = (ctypes.c_int * max(1, len(scales)))(*scales)
    return lib.msla_forward(x, wq, wd, wg, wp, out, ws, ws_bytes, B, C, H, W, heads, d, arr, len(scales),
                            eps, dt, layout, None)


def test_forward_rejects_bad_arguments_before_launching(lib):
    # every call below fails validation, so the fake pointers are never dereferenced or passed to HIP
    assert _fwd(lib, x=None) == INVALID
    assert _fwd(lib, out=None) == INVALID
    assert _fwd(lib, ws=None) == INVALID
    assert _fwd(lib, wd=None) == INVALID
    assert _fwd(lib, x=0x1004) == INVALID            # misaligned
    assert _fwd(lib, eps=-1.0) == INVALID
    assert _fwd(lib, eps=float("nan")) == INVALID
    assert _fwd(lib, layout=5) == INVALID
    assert _fwd(lib, scales=(2,)) == INVALID
    assert _fwd(lib, H=0) == INVALID
    assert _fwd(lib, layout=1, C=256) == UNSUPPORTED  # channel-planar needs C <= 2 * heads * head_dim
    assert _fwd(lib, d=24, C=96) == UNSUPPORTED
    assert _fwd(lib, d=32, heads=2, C=256, layout=1) == UNSUPPORTED   # ... with heads of 32: C <= 3 * heads * head_dim
    assert _fwd(lib, d=8, heads=3, C=32, layout=1) == UNSUPPORTED      # an odd number of heads of 8: not at all
    assert _fwd(lib, d=32, heads=2, ws_bytes=1024) == WORKSPACE
    assert _fwd(lib, scales=(9,)) == UNSUPPORTED
    assert _fwd(lib, ws_bytes=1024) == WORKSPACE


def test_other_entry_points_reject_bad_arguments(lib):
    vp, i = ctypes.c_void_p, ctypes.c_int
    ip = ctypes.POINTER(ctypes.c_int)
    lib.msla_core_forward.argtypes = [vp] * 5 + [ctypes.c_size_t] + [i] * 5 + [ip, i, ctypes.c_float, i, vp]
    lib.msla_multiscale_state.argtypes = [vp] * 6 + [ctypes.c_size_t] + [i] * 5 + [ip, i, i, vp]
    lib.msla_linear.argtypes = [vp, vp, vp, ctypes.c_long, i, i, i, vp]
    sc = (ctypes.c_int * 1)(5)
    assert lib.msla_core_forward(None, 0x1000, 0x1000, 0x1000, 0x1000, 1 << 40, 1, 8, 8, 2, 16, sc, 1, 1e-15, F16, None) == INVALID
    assert lib.msla_core_forward(0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 16, 1, 8, 8, 2, 16, sc, 1, 1e-15, F16, None) == WORKSPACE
    assert lib.msla_core_forward(0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 1 << 40, 1, 8, 8, 2, 24, sc, 1, 1e-15, F16, None) == UNSUPPORTED
    assert lib.msla_multiscale_state(0x1000, 0x1000, 0x1000, None, None, 0x1000, 1 << 40, 1, 8, 8, 2, 16, sc, 1, F16, None) == INVALID
    assert lib.msla_multiscale_state(0x1000, 0x1000, 0x1000, None, 0x1000, 0x1000, 8, 1, 8, 8, 2, 16, sc, 1, F16, None) == WORKSPACE
    assert lib.msla_linear(None, 0x1000, 0x1000, 10, 16, 16, F16, None) == INVALID
    assert lib.msla_linear(0x1000, 0x1000, 0x1000, 0, 16, 16, F16, None) == INVALID
    assert lib.msla_linear(0x1000, 0x1000, 0x1000, 10, 24, 16, F16, None) == UNSUPPORTED
    assert lib.msla_linear(0x1000, 0x1000, 0x1000, 10, 16, 16, 7, None) == INVALID


def test_product_path_does_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_2205_14756_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".h", ".hip", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "msla_oracle" not in text, os.path.join(dirpath, f)
                assert not re.search(r"^\s*(import|from)\s+\S*oracle", text, flags=re.M), os.path.join(dirpath, f)


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU; asked for more, the bench says so and does not start."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)
    assert not any(line.startswith("{") for line in r.stdout.splitlines())


def test_forward_opts_rejects_unknown_bits_and_stage_bits_with_nchw(lib):
    sc = (ctypes.c_int * 1)(5)
    vp = ctypes.c_void_p
    lib.msla_forward_opts.argtypes = [vp] * 7 + [ctypes.c_size_t] + [ctypes.c_int] * 6 + [ctypes.POINTER(ctypes.c_int), ctypes.c_int,
                                                                                          ctypes.c_float, ctypes.c_int, ctypes.c_int, vp, ctypes.c_uint]
    lib.msla_forward_opts.restype = ctypes.c_int
    p = vp(0x1000)      # never dereferenced: every check below fails on the host
    call = lambda layout, opts: lib.msla_forward_opts(p, p, p, p, p, p, p, 1 << 40, 1, 64, 8, 8, 4, 16, sc, 1, 1e-15, F16,
                                                      layout, None, opts)
    assert call(0, 64) == INVALID and call(0, 0x80000000) == INVALID
    assert call(1, 2) == UNSUPPORTED and call(1, 16 | 1) == UNSUPPORTED
