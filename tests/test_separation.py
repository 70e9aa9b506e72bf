"""The product path and the oracle stay apart, and the product fails loudly without its library.

The oracle is test infrastructure: only the tests, the smoke check and the benchmark's CPU baseline may use it.
Nothing in the package imports it, it imports nothing of the package, and the binding has no fallback.
"""
import ast
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PACKAGE = os.path.join(ROOT, "paper_2003_00532_amd")
ORACLE = os.path.join(ROOT, "oracle")


def imported_modules(path):
    with open(path) as f:
        tree = ast.parse(f.read(), path)
    names = set()
    for node in ast.walk(tree):
        if isinstance(node, ast.Import):
            names.update(a.name.split(".")[0] for a in node.names)
        elif isinstance(node, ast.ImportFrom) and node.level == 0 and node.module:
            names.add(node.module.split(".")[0])
    return names


def python_files(folder):
    for base, _, files in os.walk(folder):
        if "__pycache__" in base:
            continue
        for f in files:
            if f.endswith(".py"):
                yield os.path.join(base, f)


def test_the_package_never_imports_the_oracle():
    for path in python_files(PACKAGE):
        assert "oracle" not in imported_modules(path), path


def test_the_oracle_imports_nothing_of_the_package():
    for path in python_files(ORACLE):
        assert "paper_2003_00532_amd" not in imported_modules(path), path


def test_native_sources_of_the_two_sides_include_nothing_of_each_other():
    for folder, other in ((os.path.join(PACKAGE, "csrc"), "oracle"), (ORACLE, "paper_2003_00532_amd")):
        for f in os.listdir(folder):
            if f.endswith((".c", ".h", ".hpp", ".hip")):
                with open(os.path.join(folder, f)) as src:
                    for inc in re.findall(r'#\s*include\s+"([^"]+)"', src.read()):
                        assert other not in inc, (f, inc)


def test_the_oracle_is_used_only_where_it_may_be():
    allowed = {os.path.join(ROOT, "bench.py"), os.path.join(ROOT, "__graft_entry__.py")}
    for f in os.listdir(ROOT):
        path = os.path.join(ROOT, f)
        if f.endswith(".py") and "oracle" in imported_modules(path):
            assert path in allowed, path


def test_loading_fails_loudly_when_the_library_is_not_built(monkeypatch, tmp_path):
    from paper_2003_00532_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "libgemm_f64.so"))
    with pytest.raises(FileNotFoundError, match="no CPU fallback"):
        binding.load()
    with pytest.raises(FileNotFoundError):
        binding.gemm_f64_version()
