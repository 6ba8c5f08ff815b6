"""The product path and the oracle stay apart: neither names the other in its sources, the oracle is
reached only from the tests, the smoke check and the benchmark's CPU-baseline leg, and the binding
refuses to work without the built library instead of falling back to anything."""
import ast
import glob
import os

import pytest

from paper_2503_06564_amd import trdq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2503_06564_amd")


def _imports(path):
    tree = ast.parse(open(path).read())
    mods = set()
    for node in ast.walk(tree):
        if isinstance(node, ast.Import):
            mods.update(a.name.split(".")[0] for a in node.names)
        elif isinstance(node, ast.ImportFrom) and node.module and node.level == 0:
            mods.add(node.module.split(".")[0])
    return mods


def test_package_never_imports_the_oracle():
    for path in glob.glob(os.path.join(PKG, "*.py")):
        assert "oracle" not in _imports(path), path
    for path in glob.glob(os.path.join(PKG, "csrc", "*")):
        text = open(path).read()
        assert "oracle/" not in text and "trdq_oracle" not in text, path


def test_oracle_never_touches_the_package():
    for path in glob.glob(os.path.join(ROOT, "oracle", "*")):
        if os.path.isdir(path) or path.endswith(".so"):
            continue
        text = open(path).read()
        assert "paper_2503_06564_amd" not in text and "trdq.h" not in text and "libtrdq.so" not in text, path


def test_bench_reaches_the_oracle_only_in_its_cpu_baseline():
    tree = ast.parse(open(os.path.join(ROOT, "bench.py")).read())
    for fn in [n for n in tree.body if isinstance(n, ast.FunctionDef)]:
        uses = any(isinstance(n, ast.ImportFrom) and n.module and n.module.split(".")[0] == "oracle"
                   for n in ast.walk(fn))
        assert uses == (fn.name == "cpu_baseline"), fn.name
    top = [n for n in tree.body if isinstance(n, (ast.Import, ast.ImportFrom))]
    assert all("oracle" not in ast.dump(n) for n in top)


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    monkeypatch.setattr(trdq, "_lib", None)
    monkeypatch.setattr(trdq, "LIB_PATH", str(tmp_path / "libtrdq.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        trdq.lib()
    with pytest.raises(RuntimeError):
        trdq.qgemm_num_variants()
