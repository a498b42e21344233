"""The host half of the library (uKernel generator, planner, plan cache, argument checks) built for
the CPU with AddressSanitizer and UndefinedBehaviorSanitizer, device calls stubbed out, and the
host-side parity tests run against that build in a child process: any out-of-bounds access, use
after free, signed overflow or misaligned access in the planner fails this test."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2407_21418_amd", "csrc")


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_host_logic_is_clean_under_asan_and_ubsan(tmp_path):
    asan = subprocess.run(["g++", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("no libasan in this toolchain")
    lib = str(tmp_path / "libftuner_host_san.so")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fPIC", "-shared", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-fno-omit-frame-pointer", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           os.path.join(CSRC, "host.cpp"), os.path.join(CSRC, "host_stubs.cpp"), "-o", lib]
    subprocess.run(cmd, check=True)
    env = dict(os.environ)
    env["FTUNER_LIB"] = lib
    # the sanitizer runtime has to come first among the preloaded libraries; whatever is preloaded already stays
    env["LD_PRELOAD"] = ":".join([asan] + [p for p in env.get("LD_PRELOAD", "").split(":") if p])
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:verify_asan_link_order=0"     # (CPython itself leaks by design)
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    tests = ["tests/test_library_host.py", "tests/test_planner_second_opinion.py"]
    p = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        "--deselect", "tests/test_library_host.py::test_library_exports_every_declared_symbol"] + tests,
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (p.stdout + p.stderr)[-3000:]
    assert p.returncode == 0, tail
    assert "passed" in p.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error" not in tail, tail
