"""The library's host-only code and the CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer.

Builds tests/sanitize/host_and_oracle_cases.cpp together with paper_1907_07346_amd/csrc/dsq_host.cpp and
oracle/ds_oracle.cpp with g++ -fsanitize=address,undefined (no GPU code, no GPU call) and runs the cases:
configuration checks, topologies, message sizes, and three steps of every operator of the oracle on ragged
sizes in float and double.  A sanitizer report aborts the program; a failed check makes it return non-zero.
"""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_code_and_oracle_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "sanitize_cases")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           "-ffp-contract=off", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-I", os.path.join(ROOT, "include"),
           "-I", os.path.join(ROOT, "paper_1907_07346_amd", "csrc"),
           os.path.join(ROOT, "tests", "sanitize", "host_and_oracle_cases.cpp"),
           os.path.join(ROOT, "paper_1907_07346_amd", "csrc", "dsq_host.cpp"),
           os.path.join(ROOT, "oracle", "ds_oracle.cpp"), "-o", exe]
    subprocess.run(cmd, check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    out = subprocess.run([exe], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    sys.stdout.write(out.stdout)
    assert out.returncode == 0, out.stdout[-2000:]
    assert "sanitizer cases ok" in out.stdout
