"""Memory-safety checks that need no GPU: the CPU oracle and the library's HOST code (argument validation, launch
planning, workspace sizing) built with -fsanitize=address,undefined and run through small driver programs
(tests/sanitize/).  A report from either sanitizer makes the program exit non-zero."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")


def _run(exe, tmp_path):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1",
               OMP_NUM_THREADS="4")
    res = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, cwd=str(tmp_path),
                         timeout=300)
    assert res.returncode == 0 and res.stdout.strip().endswith("ok"), res.stdout[-4000:]
    assert "runtime error" not in res.stdout and "AddressSanitizer" not in res.stdout, res.stdout[-4000:]


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    exe = str(tmp_path / "oracle_san")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-Wall", "-Wextra", "-o", exe, os.path.join(SAN, "oracle_driver.c"), os.path.join(ROOT, "oracle", "dd_oracle.c"), "-lm"]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout
    _run(exe, tmp_path)


def test_host_layer_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    from paper_2604_05250_amd.build import CSRC, SOURCES
    exe = str(tmp_path / "host_san")
    # the sanitizers instrument the host pass only (GPU sanitizers are not available): each flag follows -Xarch_host
    cmd = [hipcc, "-O1", "-g", "-std=c++17", "--offload-arch=gfx950", "-w", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-o", exe]
    cmd += [os.path.join(CSRC, f) for f in SOURCES] + [os.path.join(SAN, "host_driver.cpp")]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout[-4000:]
    _run(exe, tmp_path)
