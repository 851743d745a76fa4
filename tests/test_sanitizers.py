"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (no GPU).

Two programs are built and run here:
  * the C oracle (oracle/gemm_oracle.c) with tests/sanitize/oracle_host_driver.c, by gcc;
  * the C ABI's host layer (csrc/api.hip: validation, dispatch, launch-table planning) compiled with the sanitizers on
    the host side only and linked with the library's other objects, driven by tests/sanitize/abi_host_driver.cpp.
Each program also has a mode in which the CALLER passes a block that is too short; that run must end in a sanitizer
report, which shows the instrumentation is live.
"""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def run(cmd, **kw):
    return subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)


def must(cmd):
    p = run(cmd)
    out = "\n".join(l for l in p.stdout.splitlines() if "packed-fp32-ops" not in l)
    assert p.returncode == 0, " ".join(cmd) + "\n" + out


@pytest.fixture(scope="module")
def oracle_program(tmp_path_factory):
    out = tmp_path_factory.mktemp("san_oracle") / "oracle_host_driver"
    must(["gcc", "-O1", "-g", "-fopenmp", *SAN, "-static-libasan", "-o", str(out),
          os.path.join(ROOT, "tests", "sanitize", "oracle_host_driver.c"), os.path.join(ROOT, "oracle", "gemm_oracle.c")])
    return str(out)


@pytest.fixture(scope="module")
def abi_program(tmp_path_factory):
    from paper_2205_09120_amd import build as hip_build
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    clangxx = "/opt/rocm/lib/llvm/bin/clang++"
    if not (os.path.exists(hipcc) and os.path.exists(clangxx)):
        pytest.skip("no ROCm toolchain")
    objs = [hip_build.object_path(s) for s in hip_build.SOURCES if s != "api.hip"]
    if not all(os.path.exists(o) for o in objs):
        hip_build.build()  # leaves the objects of every source behind
    tmp = tmp_path_factory.mktemp("san_abi")
    api_o, drv_o, exe = str(tmp / "api_san.o"), str(tmp / "driver.o"), str(tmp / "abi_host_driver")
    host_san = [x for f in SAN for x in ("-Xarch_host", f)]
    must([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
          "-packed-fp32-ops", *host_san, "-I", hip_build.CSRC, "-c", os.path.join(hip_build.CSRC, "api.hip"), "-o", api_o])
    must([clangxx, "-O1", "-g", "-std=c++17", *SAN, "-I", os.path.join(ROOT, "include"), "-c",
          os.path.join(ROOT, "tests", "sanitize", "abi_host_driver.cpp"), "-o", drv_o])
    must([hipcc, "--offload-arch=gfx950", "-fno-gpu-sanitize", *SAN, "-o", exe, drv_o, api_o, *objs])
    return exe


def test_oracle_is_clean_under_sanitizers(oracle_program):
    p = run([oracle_program], env=ENV, timeout=300)
    assert p.returncode == 0 and "all expectations hold" in p.stdout, p.stdout[-4000:]
    assert "runtime error" not in p.stdout and "AddressSanitizer" not in p.stdout, p.stdout[-4000:]


def test_oracle_sanitizer_build_reports_a_short_operand(oracle_program):
    p = run([oracle_program, "--lie"], env=ENV, timeout=60)
    assert p.returncode != 0 and "AddressSanitizer" in p.stdout and "went unnoticed" not in p.stdout, p.stdout[-2000:]


def test_abi_host_layer_is_clean_under_sanitizers(abi_program):
    p = run([abi_program], env=ENV, timeout=300)
    assert p.returncode == 0 and "all expectations hold" in p.stdout, p.stdout[-4000:]
    assert "runtime error" not in p.stdout and "AddressSanitizer" not in p.stdout, p.stdout[-4000:]


def test_abi_sanitizer_build_reports_a_short_table(abi_program):
    p = run([abi_program, "--lie"], env=ENV, timeout=60)
    assert p.returncode != 0 and "AddressSanitizer" in p.stdout and "went unnoticed" not in p.stdout, p.stdout[-2000:]
