"""Address and undefined-behaviour sanitizer builds of the CPU-only code: the fp64 oracle, the
host libraries (context index, de-duplication) and the host side of the C ABI (argument checks,
launch planning).  Each build is an executable of its own (tests/sanitize/*.cpp) that runs on
small seeded inputs and aborts on the first finding.  The device code is never instrumented and
no kernel is launched."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2511_03475_amd", "csrc")
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1",
           OMP_NUM_THREADS="2")
ENV.pop("LD_PRELOAD", None)   # the sanitizer runtime must come first in the executable's library list


def _run(cmd, **kw):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert res.returncode == 0, " ".join(cmd) + "\n" + res.stdout[-4000:]
    return res.stdout


def test_oracle_and_host_libraries_under_asan_and_ubsan(tmp_path):
    flags = ["-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]
    objs = []
    for src in ("extend_attention_oracle.c", "context_distance_oracle.c"):
        obj = str(tmp_path / (src + ".o"))
        _run(["gcc", "-std=c11", "-fopenmp", *flags, "-c", os.path.join(ROOT, "oracle", src), "-o", obj])
        objs.append(obj)
    exe = str(tmp_path / "san_host")
    _run(["g++", "-std=c++17", "-fopenmp", *flags, "-I", os.path.join(ROOT, "include"),
          os.path.join(SAN, "host_driver.cpp"), os.path.join(CSRC, "cp_context_index.cpp"),
          os.path.join(CSRC, "cp_context_dedup.cpp"), *objs, "-o", exe, "-lm"])
    assert "sanitized host run: ok" in _run([exe], env=ENV)


def test_c_abi_host_side_under_asan_and_ubsan(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not found")
    exe = str(tmp_path / "san_abi")
    # the sanitizers instrument the host pass only; the device pass is compiled as always
    _run([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
          "-Xarch_host", "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer",
          "-I", os.path.join(ROOT, "include"), os.path.join(SAN, "abi_driver.cpp"),
          os.path.join(CSRC, "cp_extend.hip"), "-o", exe])
    # the HIP runtime keeps its own allocations until exit: leaks are not what this run looks for
    env = dict(ENV, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0")
    assert "sanitized C-ABI host run: ok" in _run([exe], env=env)
