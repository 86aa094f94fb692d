"""The CPU oracle and the library's host code under AddressSanitizer + UndefinedBehaviorSanitizer.

Builds tests/sanitize/host_sanitize.cpp together with oracle/memo_oracle.c and the three host
sources of the library with gcc -fsanitize=address,undefined (no GPU, no HIP runtime: the driver
carries fakes for the handful of HIP calls the host code makes) and runs it.  The same command is
in the README; a sanitizer report makes the program exit non-zero."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OUT = os.path.join(ROOT, "tests", "sanitize", "_build")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]


def build_and_run():
    os.makedirs(OUT, exist_ok=True)
    csrc = os.path.join(ROOT, "paper_2407_12117_amd", "csrc")
    objs = []
    run = lambda cmd: subprocess.run(cmd, check=True, capture_output=True, text=True)
    o = os.path.join(OUT, "memo_oracle.o")
    run(["gcc", "-std=c99", "-fopenmp", "-Wall", "-Wextra", *SAN, "-c", os.path.join(ROOT, "oracle", "memo_oracle.c"), "-o", o])
    objs.append(o)
    hip_inc = ["-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include"]
    for src in (os.path.join(csrc, "memo_api.cpp"), os.path.join(csrc, "memo_sched.cpp"),
                os.path.join(csrc, "memo_dsa.cpp"), os.path.join(ROOT, "tests", "sanitize", "host_sanitize.cpp")):
        o = os.path.join(OUT, os.path.basename(src) + ".o")
        run(["g++", "-std=c++17", "-Wall", *SAN, *hip_inc, "-c", src, "-o", o])
        objs.append(o)
    exe = os.path.join(OUT, "host_sanitize")
    run(["g++", *SAN, "-fopenmp", *objs, "-o", exe, "-lm"])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="4")
    return subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)


def test_oracle_and_host_code_are_clean_under_asan_and_ubsan():
    try:
        res = build_and_run()
    except subprocess.CalledProcessError as e:
        pytest.fail("sanitizer build failed:\n" + e.stderr[-4000:])
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-6000:]
    assert "host sanitizer run: ok" in res.stdout


if __name__ == "__main__":
    r = build_and_run()
    sys.stdout.write(r.stdout)
    sys.stderr.write(r.stderr)
    sys.exit(r.returncode)
