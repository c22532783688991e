"""The host side of the library under the address and undefined-behaviour sanitizers (no GPU).

csrc/bcr_pack.cpp -- validation, compaction into the canonical arrays, the three derived kernel layouts and
their decoders, the BCRC export -- is built with g++ -fsanitize=address,undefined against stand-ins for the
kernel launchers (tests/sanitize/device_stubs.cpp), and the host-side test files run against that build in a
child interpreter with the sanitizer runtimes preloaded.  Any out-of-bounds access, use after free or
undefined operation in the index-building code aborts the child and fails this test."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HOST_TESTS = ["tests/test_host_pack.py", "tests/test_bcrc_export.py", "tests/test_host_layouts.py"]


def _runtime(name):
    path = subprocess.run(["g++", f"-print-file-name={name}"], capture_output=True, text=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    asan, ubsan = _runtime("libasan.so"), _runtime("libubsan.so")
    if not asan or not ubsan:
        pytest.skip("g++ sanitizer runtimes not installed")
    lib = str(tmp_path / "libgrim_bcr_sanitized.so")
    build = ["g++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
             "-fno-sanitize-recover=undefined", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
             "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2108_11033_amd", "csrc"),
             "-shared", "-fPIC", "-Wl,-Bsymbolic",
             os.path.join(ROOT, "paper_2108_11033_amd", "csrc", "bcr_pack.cpp"),
             os.path.join(ROOT, "tests", "sanitize", "device_stubs.cpp"), "-o", lib]
    res = subprocess.run(build, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-4000:]
    env = dict(os.environ)
    env["GRIM_BCR_LIB"] = lib
    preload = [asan, ubsan] + ([env["LD_PRELOAD"]] if env.get("LD_PRELOAD") else [])
    env["LD_PRELOAD"] = ":".join(preload)
    # Python itself is not instrumented: no leak report at exit, and the runtime may come after other preloads
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu"] + HOST_TESTS,
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (run.stdout + run.stderr)[-4000:]
    assert run.returncode == 0, tail
    assert "passed" in run.stdout and "AddressSanitizer" not in tail and "runtime error" not in tail, tail
