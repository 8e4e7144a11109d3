"""Repository hygiene that the build contract depends on: the product never reaches into the CPU
checkers, nothing committed depends on the working folder, and the GPU path has no CPU fallback."""
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2605_07230_amd")


WORK = re.compile(r"(^|[^A-Za-z0-9])_work/|[\"']_work[\"']")   # the folder, not identifiers like cascade_workspace_bytes


def _sources(folder, exts):
    for base, _, files in os.walk(folder):
        if "_build" in base or "__pycache__" in base:
            continue
        for f in files:
            if f.endswith(exts):
                yield os.path.join(base, f)


def test_package_never_imports_the_checkers():
    pat = re.compile(r"^\s*(from|import)\s+oracle\b", re.M)
    for path in _sources(PKG, (".py", ".hip", ".h")):
        assert not pat.search(open(path).read()), path


def test_bench_uses_the_checkers_only_for_the_cpu_baseline():
    text = open(os.path.join(ROOT, "bench.py")).read()
    uses = [m.start() for m in re.finditer(r"from oracle import|import oracle", text)]
    assert len(uses) == 1
    start = text.index("def cpu_baseline")
    end = text.index("\ndef ", start + 1)
    assert start < uses[0] < end


def test_nothing_committed_reads_the_working_folder():
    for folder in (PKG, os.path.join(ROOT, "tests"), os.path.join(ROOT, "oracle")):
        for path in _sources(folder, (".py", ".hip", ".h")):
            if os.path.basename(path) == "test_layout.py":
                continue
            assert not WORK.search(open(path).read()), path
    for name in ("bench.py", "__graft_entry__.py"):
        assert not WORK.search(open(os.path.join(ROOT, name)).read()), name


def test_checkers_do_not_import_the_package_kernels():
    for path in _sources(os.path.join(ROOT, "oracle"), (".py",)):
        text = open(path).read()
        assert "binding" not in text and "ctypes" not in text, path
