"""Structure checks: the oracle and the product path share no code, the binding has no fallback."""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _sources(folder, exts):
    for base, _, files in os.walk(os.path.join(ROOT, folder)):
        for f in files:
            if f.endswith(exts):
                yield os.path.join(base, f)


def test_package_never_imports_the_oracle():
    for path in _sources("paper_2510_11062_amd", (".py", ".hip", ".hpp", ".c", ".h")):
        text = open(path).read()
        assert not re.search(r"^\s*(from|import)\s+oracle\b", text, re.M), path
        assert "at_grpo_oracle" not in text, path


def test_oracle_never_imports_the_package_or_torch():
    for path in _sources("oracle", (".py",)):
        text = open(path).read()
        assert "paper_2510_11062_amd" not in text, path
        assert not re.search(r"^\s*(from|import)\s+(torch|ctypes)\b", text, re.M), path


def test_only_tests_smoke_and_bench_use_the_oracle():
    allowed = {os.path.join(ROOT, "bench.py"), os.path.join(ROOT, "__graft_entry__.py")}
    for path in list(_sources(".", (".py",))):
        rel = os.path.relpath(path, ROOT)
        if rel.startswith(("tests" + os.sep, "oracle" + os.sep, "_work" + os.sep, "gpurun_out" + os.sep)):
            continue
        text = open(path).read()
        uses = re.search(r"^\s*(from|import)\s+oracle\b", text, re.M) is not None
        if uses:
            assert os.path.normpath(path) in allowed, rel
    # bench.py touches it only inside the CPU-baseline leg
    bench = open(os.path.join(ROOT, "bench.py")).read()
    assert bench.count("from oracle import") == 1
    assert bench.index("from oracle import") > bench.index("def cpu_baseline")


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    from paper_2510_11062_amd import api
    monkeypatch.setattr(api, "_LIB_PATH", str(tmp_path / "libat_grpo.so"))
    monkeypatch.setattr(api, "_lib", None, raising=False)
    with pytest.raises(api.AtGrpoError):
        api.load_library()
