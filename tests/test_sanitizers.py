"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only, no GPU code is instrumented).

Builds, into a temporary directory, (a) the host side of the library -- the C-ABI state machine (ssd_api.cpp) and the
selection / search policy (ssd_policy.cpp), linked with the regular kernel object -- and (b) the C part of the CPU
oracle, both with -fsanitize=address,undefined, and runs the existing CPU tests against those builds in a child
process that has the sanitizer runtimes preloaded.  Any report (out-of-bounds access, use after free, signed overflow,
misaligned or null access, ...) aborts the child and fails this test.
"""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2604_14612_amd", "csrc")
SAN = ["-fsanitize=address,undefined", "-fno-omit-frame-pointer", "-O2", "-g", "-fPIC"]
HOST_TESTS = ["tests/test_abi_host.py", "tests/test_oracle_confidence.py", "tests/test_oracle_select.py",
              "tests/test_oracle_decoder.py", "tests/test_oracle_golden.py"]


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, "%s\n%s\n%s" % (" ".join(cmd), r.stdout[-4000:], r.stderr[-4000:])
    return r


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++ for the host-only sanitizer build")
def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    kernels_obj = os.path.join(CSRC, "ssd_kernels.o")
    if not os.path.exists(kernels_obj):
        from paper_2604_14612_amd.build import build
        build()
    out = str(tmp_path)
    hip_inc = ["-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include"]
    _run(["g++", "-std=c++17"] + SAN + hip_inc + ["-c", os.path.join(CSRC, "ssd_api.cpp"), "-o", out + "/api.o"])
    _run(["g++", "-std=c++17", "-ffp-contract=off"] + SAN + ["-c", os.path.join(CSRC, "ssd_policy.cpp"), "-o",
                                                              out + "/policy.o"])
    lib = out + "/libssd_san.so"
    _run(["g++", "-shared", "-fsanitize=address,undefined", "-Wl,--version-script=" + os.path.join(CSRC, "libssd.map"),
          "-o", lib, out + "/api.o", out + "/policy.o", kernels_obj, "-L/opt/rocm/lib", "-lamdhip64",
          "-Wl,-rpath,/opt/rocm/lib"])
    orc = out + "/liboracle_san.so"
    _run(["gcc", "-std=c11", "-ffp-contract=off", "-fno-fast-math"] + SAN + ["-shared", "-o", orc,
                                                                            os.path.join(ROOT, "oracle", "ssd_oracle.c"), "-lm"])
    runtimes = [_run(["gcc", "-print-file-name=" + n]).stdout.strip() for n in ("libasan.so", "libubsan.so")]
    assert all(os.path.isabs(p) and os.path.exists(p) for p in runtimes), runtimes
    env = dict(os.environ)
    # the sanitizer runtimes go in front of whatever is preloaded already
    env["LD_PRELOAD"] = ":".join(runtimes + ([env["LD_PRELOAD"]] if env.get("LD_PRELOAD") else []))
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["SSD_LIB_PATH"] = lib
    env["ORACLE_LIB_PATH"] = orc
    # the longest draft lengths of the losslessness test walk the same code as the short ones, an order of magnitude
    # slower under the sanitizers: they stay in the plain run only
    long_cases = ["--deselect=tests/test_oracle_decoder.py::test_ssd_is_lossless_for_any_mask[%d]" % k for k in (4, 8)]
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + long_cases + HOST_TESTS,
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = r.stdout[-3000:] + r.stderr[-3000:]
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error:" not in tail, tail
