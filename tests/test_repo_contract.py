"""Host-side checks of the repository's own rules: the product never reaches for the CPU oracle,
fails loudly without its library, and the bench refuses more than one GPU."""
import os
import re
import subprocess
import sys

import pytest

from paper_2001_08743_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2001_08743_amd")


def _sources(top, exts):
    for base, _, files in os.walk(top):
        if "__pycache__" in base:
            continue
        for f in files:
            if f.endswith(exts):
                yield os.path.join(base, f)


def test_the_product_package_never_uses_the_oracle():
    pat = re.compile(r"^\s*(import\s+oracle|from\s+oracle\b|#include\s+[\"<].*oracle)", re.M)
    for path in _sources(PKG, (".py", ".hip", ".h", ".cpp")):
        assert not pat.search(open(path).read()), path
    # and the oracle never uses the product's kernels or binding
    for path in _sources(os.path.join(ROOT, "oracle"), (".py", ".c", ".h")):
        text = open(path).read()
        assert "binding" not in text and "libcham" not in text and "csrc" not in text, path


_WORK = re.compile(r"""["'/]_work[/"']""")


def test_nothing_committed_reads_the_working_folder():
    for top in (PKG, os.path.join(ROOT, "tests"), os.path.join(ROOT, "oracle")):
        for path in _sources(top, (".py",)):
            if os.path.abspath(path) == os.path.abspath(__file__):
                continue
            assert not _WORK.search(open(path).read()), path
    for name in ("bench.py", "__graft_entry__.py"):
        assert not _WORK.search(open(os.path.join(ROOT, name)).read()), name


def test_a_missing_library_is_an_error_not_a_fallback(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "libcham.so"))
    with pytest.raises(binding.ChamError, match="not built"):
        binding.load()


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""
