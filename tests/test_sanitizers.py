"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the CPU-side code (no GPU needed):
the oracle (through a C driver that walks every entry point, oracle/sanitize_check.c) and the host
code of the C-ABI library (argument checks and planning of cham_api.hip, through a C driver that
calls the entry points with invalid and with well-formed arguments; without a GPU the latter end in
CHAM_E_HIP, after the host-side planning has run).  Device code is never sanitized."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def test_oracle_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "sanitize_check")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-ffp-contract=off", *SAN, "-static-libasan",
           os.path.join(ROOT, "oracle", "cham_oracle.c"), os.path.join(ROOT, "oracle", "sanitize_check.c"),
           "-lm", "-o", exe]
    subprocess.run(cmd, check=True)
    r = subprocess.run([exe], env=ENV, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-4000:]
    assert "sanitize_check ok" in r.stdout


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"), reason="no hipcc")
def test_library_host_code_under_address_and_ub_sanitizers(tmp_path):
    from paper_2001_08743_amd import build as libbuild
    lib = libbuild.build_host_sanitized(str(tmp_path))
    exe = str(tmp_path / "host_check")
    clang = "/opt/rocm/lib/llvm/bin/clang"
    cmd = [clang, "-O1", "-g", *SAN, "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "paper_2001_08743_amd", "csrc", "host_check.c"), lib,
           "-Wl,-rpath," + os.path.dirname(lib), "-Wl,-rpath,/opt/rocm/lib", "-o", exe]
    subprocess.run(cmd, check=True)
    env = dict(ENV, ASAN_OPTIONS="detect_leaks=0")     # the HIP runtime keeps its own allocations until exit
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert "host_check ok" in r.stdout
