"""AddressSanitizer + UndefinedBehaviorSanitizer builds, on the CPU, of (1) the oracle and (2) the
host code of the library (argument checks, registry of live sets, allocation-failure hook), each
driven by a small program under tests/sanitize/.  A sanitizer report ends the program with a
non-zero status (-fno-sanitize-recover), which fails the test."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all"]


def _run(cmd, **kw):
    res = subprocess.run(cmd, capture_output=True, text=True, timeout=600, **kw)
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    assert res.returncode == 0, "%s\n%s\n%s" % (" ".join(cmd), res.stdout[-4000:], err[-4000:])
    return res.stdout


def test_oracle_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    _run(["g++", "-std=c++17", "-O1", "-g", *SAN, "-static-libasan", "-static-libubsan", "-pthread",
          os.path.join(ROOT, "oracle", "nezha_oracle.cpp"),
          os.path.join(ROOT, "tests", "sanitize", "oracle_driver.cpp"), "-o", exe])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    assert "oracle: clean" in _run([exe], env=env)


def test_library_host_code_under_asan_and_ubsan(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("no hipcc")
    exe = str(tmp_path / "abi_san")
    host_san = [x for flag in SAN for x in ("-Xarch_host", flag)]
    csrc = os.path.join(ROOT, "paper_2511_18793_amd", "csrc")
    # host code only: the device side is not compiled, and the two symbols that would hold its
    # code objects stay unresolved (the driver never launches a kernel)
    _run([hipcc, "--offload-arch=gfx950", "--offload-host-only", "-O1", "-g", "-std=c++17",
          "-I" + os.path.join(ROOT, "include"), "-I" + csrc, *host_san,
          "-Wno-unused-command-line-argument", "-Wl,--unresolved-symbols=ignore-all",
          os.path.join(csrc, "itemset.hip"), os.path.join(csrc, "draft.hip"),
          os.path.join(ROOT, "tests", "sanitize", "abi_driver.cpp"), "-o", exe])
    # leak checking is off here: the HIP runtime keeps its own allocations until the process ends
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("NEZHA_TEST_FAIL_ALLOC", None)
    assert "abi: clean" in _run([exe], env=env)
