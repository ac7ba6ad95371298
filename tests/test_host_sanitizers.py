"""The host-side code of the library (plan construction, plan generators, cost model, their argument
checks) under AddressSanitizer and UndefinedBehaviorSanitizer, on the CPU.  plan.hip holds no kernel; its
host pass is compiled with the sanitizers and linked with host stand-ins for the four HIP runtime calls it
makes, so the copies into "device" arrays are checked too.  No GPU is involved."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "host_asan")


def test_plan_host_code_under_asan_and_ubsan(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    exe = tmp_path / "plan_asan"
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
    cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", *san,
           os.path.join(ROOT, "paper_2507_05228_amd", "csrc", "plan.hip"),
           os.path.join(HERE, "hip_host_stub.cpp"), os.path.join(HERE, "plan_asan_main.cpp"), "-o", str(exe)]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-3000:])
    assert "HOST_SANITIZER_OK" in run.stdout
    assert "ERROR: AddressSanitizer" not in run.stderr and "runtime error" not in run.stderr


def test_reciprocal_division_of_the_attention_launcher_is_exact(tmp_path):
    """The fused attention kernel turns its workgroup index into (query tile, batch, head block) with multiplications
    by reciprocals the launcher computes; the launcher refuses grids outside the range where that is exact.  Checked on
    the host against the integer division, exhaustively for small indices and around every multiple of the divisor near
    the admitted maximum."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    exe = tmp_path / "div_magic"
    cmd = [hipcc, "--offload-arch=gfx950", "-x", "hip", "-O1", "-std=c++17",
           os.path.join(HERE, "div_magic_main.cpp"), "-o", str(exe)]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-3000:]
    run = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300)
    assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-2000:])
    assert "DIV_MAGIC_OK" in run.stdout
