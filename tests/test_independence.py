"""The product and the oracle stay apart, and the product has no fallback (CPU tests).

The oracle is the checker: only tests, the smoke check and the benchmark's cpu_baseline leg may
use it, and it must not lean on the library either.  The binding must refuse to work without the
built library instead of computing anything itself."""
import ast
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2406_17565_amd")
ORACLE = os.path.join(ROOT, "oracle")


def _imports(path):
    """Top-level names of every module a Python file imports, with the enclosing function (or None)."""
    tree = ast.parse(open(path).read(), path)
    found = []

    def visit(node, func):
        for child in ast.iter_child_nodes(node):
            f = child.name if isinstance(child, (ast.FunctionDef, ast.AsyncFunctionDef)) else func
            if isinstance(child, ast.Import):
                found.extend((a.name.split(".")[0], func) for a in child.names)
            elif isinstance(child, ast.ImportFrom) and child.level == 0 and child.module:
                found.append((child.module.split(".")[0], func))
            visit(child, f)

    visit(tree, None)
    return found


def _files(folder, exts):
    for base, _, names in os.walk(folder):
        if "__pycache__" in base:
            continue
        for n in names:
            if n.endswith(exts):
                yield os.path.join(base, n)


def test_product_package_never_touches_the_oracle():
    for path in _files(PKG, (".py",)):
        assert all(mod != "oracle" for mod, _ in _imports(path)), path
    for path in _files(PKG, (".hip", ".hpp", ".h", ".cc", ".cpp")):
        for line in open(path):
            if line.lstrip().startswith("#include"):
                assert "oracle" not in line, (path, line)
    for line in open(os.path.join(ROOT, "include", "mempool.h")):
        if line.lstrip().startswith("#include"):
            assert "oracle" not in line


def test_oracle_never_touches_the_product():
    for path in _files(ORACLE, (".py",)):
        assert all(mod != "paper_2406_17565_amd" for mod, _ in _imports(path)), path
    for path in _files(ORACLE, (".cc", ".cpp", ".h", ".hpp", ".c")):
        text = open(path).read()
        for line in text.splitlines():
            if line.lstrip().startswith("#include"):
                assert "mempool.h" not in line and "csrc" not in line and "kv_copy" not in line and \
                    "pool_index" not in line, (path, line)
        assert "hip/hip_runtime" not in text, path


def test_only_the_baseline_leg_and_the_smoke_check_use_the_oracle_outside_tests():
    allowed = {"bench.py": {"cpu_baseline"}, "__graft_entry__.py": {"build", "smoke"}}
    for name in os.listdir(ROOT):
        if not name.endswith(".py"):
            continue
        users = {func for mod, func in _imports(os.path.join(ROOT, name)) if mod == "oracle"}
        assert users <= allowed.get(name, set()), (name, users)


def test_binding_refuses_to_work_without_the_built_library(monkeypatch, tmp_path):
    from paper_2406_17565_amd import mempool as M
    monkeypatch.setattr(M, "_lib", None)
    monkeypatch.setattr(M._build, "LIB", str(tmp_path / "libmempool.so"))
    with pytest.raises(RuntimeError, match="not built"):
        M.lib()
    with pytest.raises(RuntimeError, match="not built"):
        M.mp_selftest()


def test_binding_holds_no_arithmetic_of_the_method():
    """mempool.py only marshals: no hash constants, no copy loops of its own."""
    text = open(os.path.join(PKG, "mempool.py")).read()
    for needle in ("cbf29ce484222325", "100000001b3", "9e3779b97f4a7c15", "bf58476d1ce4e5b9", "94d049bb133111eb"):
        assert needle not in text.lower()
    assert not re.search(r"\bfor\b.*\bin range\(", text), "a loop in the binding: marshalling only"
