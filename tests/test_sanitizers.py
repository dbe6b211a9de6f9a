"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the code that runs on the host: the CPU
oracle, and the library's host side (validation, planning, workspace layout, tables, plans) with
its kernel launchers stubbed.  Each is a small program built here with gcc / g++ and run once; a
sanitizer report or a failed invariant in the stubs fails the test.  No GPU is involved."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-static-libasan",
       "-g", "-O1"]


def _run(exe):
    env = dict(os.environ)
    # the environment may preload a library of its own; the sanitizer runtime is linked statically
    # and need not come first
    env["ASAN_OPTIONS"] = "verify_asan_link_order=0:detect_leaks=1:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    p = subprocess.run([exe], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    sys.stdout.write(p.stdout[-4000:])
    assert p.returncode == 0, "sanitizer run failed (status %d):\n%s" % (p.returncode, p.stdout[-4000:])
    assert "runtime error" not in p.stdout and "AddressSanitizer" not in p.stdout
    return p.stdout


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    subprocess.run(["gcc", "-std=c11", *SAN, "-ffp-contract=off", "-fno-fast-math", "-frounding-math", "-fopenmp",
                    "-Wall", "-Wextra", os.path.join(ROOT, "oracle", "fq_oracle.c"),
                    os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"), "-o", exe, "-lm"], check=True)
    assert "oracle sanitizer run clean" in _run(exe)


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_library_host_side_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "host_san")
    subprocess.run(["g++", "-std=c++17", *SAN, "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-Wall", "-Wextra",
                    "-Wno-unused-parameter", os.path.join(ROOT, "paper_2511_12653_amd", "csrc", "fq_api.cpp"),
                    os.path.join(ROOT, "tests", "sanitize", "host_driver.cpp"), "-o", exe, "-lpthread"], check=True)
    out = _run(exe)
    assert "0 failures" in out
