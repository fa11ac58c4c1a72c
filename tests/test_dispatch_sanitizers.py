"""The library's host side (argument checks, workspace carving, launch order: csrc/msla_api.cpp) built for
the CPU with AddressSanitizer + UndefinedBehaviorSanitizer against launcher stand-ins that check, for every
launch of every entry point over a list of shapes and all storage types, that each pointer with the extent
the kernel would touch lies inside a buffer of the call, aligned, and that the buffers of one launch do not
overlap (tests/sanitize_dispatch_driver.cpp).  No GPU code runs."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIP_INCLUDE = "/opt/rocm/include"


@pytest.mark.skipif(shutil.which("g++") is None or not os.path.isdir(os.path.join(HIP_INCLUDE, "hip")),
                    reason="needs g++ and the HIP headers")
def test_dispatcher_hands_every_kernel_pointers_inside_the_callers_buffers(tmp_path):
    exe = str(tmp_path / "sanitize_dispatch")
    cmd = ["g++", "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-D__HIP_PLATFORM_AMD__", "-I" + HIP_INCLUDE, "-Wno-unused-result",
           os.path.join(ROOT, "tests", "sanitize_dispatch_driver.cpp"),
           os.path.join(ROOT, "paper_2205_14756_amd", "csrc", "msla_api.cpp"), "-o", exe]
    build = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    if build.returncode != 0 and "asan" in (build.stderr + build.stdout).lower():
        pytest.skip("this toolchain has no sanitizer runtime: " + build.stderr[-300:])
    assert build.returncode == 0, build.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0")
    run = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
    assert run.returncode == 0, (run.stdout + run.stderr)[-4000:]
    assert "dispatch driver ok" in run.stdout
