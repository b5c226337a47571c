"""The resident matrix-core kernel updates a centroid knob as S * (1/n) with one correction step
instead of a division per knob; this runs the exhaustive host-side check that the result equals the
correctly rounded S / n on the kernel's whole domain (n <= 4096, S <= 255 n)."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _host_has_fma():
    try:
        return " fma " in open("/proc/cpuinfo").read().replace("\n", " ")
    except OSError:
        return False


@pytest.mark.skipif(not _host_has_fma(), reason="the check needs a hardware fused multiply-add on the host")
def test_reciprocal_quotient_is_correctly_rounded_on_the_whole_domain(tmp_path):
    exe = str(tmp_path / "quotient_check")
    src = os.path.join(ROOT, "paper_2001_08743_amd", "csrc", "quotient_check.c")
    subprocess.run(["gcc", "-O2", "-mfma", "-fopenmp", "-ffp-contract=off", src, "-lm", "-o", exe], check=True)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "quotient_check: 0 mismatches" in r.stdout
