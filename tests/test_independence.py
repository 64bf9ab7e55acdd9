"""The oracle is test infrastructure: the product never reaches into it, and it
never reaches into the product.  Checked on the sources."""
import ast
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _sources(sub, exts):
    for d, _, files in os.walk(os.path.join(ROOT, sub)):
        if "__pycache__" in d:
            continue
        for f in files:
            if f.endswith(exts):
                yield os.path.join(d, f)


def _imports(path):
    tree = ast.parse(open(path).read())
    for node in ast.walk(tree):
        if isinstance(node, ast.Import):
            for a in node.names:
                yield a.name, node.lineno
        elif isinstance(node, ast.ImportFrom):
            yield (node.module or ""), node.lineno


def test_product_does_not_use_the_oracle():
    for path in _sources("paper_2601_20309_amd", (".py",)):
        for mod, line in _imports(path):
            assert not mod.split(".")[0] == "oracle", f"{path}:{line} imports {mod}"
        assert "libduplexkv_oracle" not in open(path).read(), path
    for path in _sources("paper_2601_20309_amd", (".hip", ".hpp", ".cpp", ".h")):
        text = open(path).read()
        assert not re.search(r'#include\s+"[^"]*oracle', text), path
        assert "okv_" not in text, path
    text = open(os.path.join(ROOT, "include", "duplexkv.h")).read()
    assert "okv_" not in text


def test_oracle_does_not_use_the_product():
    for path in _sources("oracle", (".py",)):
        for mod, line in _imports(path):
            assert mod.split(".")[0] != "paper_2601_20309_amd", f"{path}:{line} imports {mod}"
        assert "libduplexkv.so" not in open(path).read(), path
    for path in _sources("oracle", (".c", ".h")):
        text = open(path).read()
        assert "duplexkv.h" not in text and "kv_engine" not in text, path
        assert not re.search(r"#include\s+[<\"]hip", text), path


def test_bench_touches_the_oracle_only_in_its_cpu_baseline():
    tree = ast.parse(open(os.path.join(ROOT, "bench.py")).read())
    for fn in [n for n in ast.walk(tree) if isinstance(n, ast.FunctionDef)]:
        uses = [m for node in ast.walk(fn) for m in
                ([a.name for a in node.names] if isinstance(node, ast.Import) else
                 [node.module or ""] if isinstance(node, ast.ImportFrom) else [])
                if m.split(".")[0] == "oracle"]
        assert not uses or fn.name == "cpu_baseline", f"bench.py:{fn.name} imports the oracle"
    top = [m for node in tree.body for m in
           ([a.name for a in node.names] if isinstance(node, ast.Import) else
            [node.module or ""] if isinstance(node, ast.ImportFrom) else [])]
    assert not [m for m in top if m.split(".")[0] == "oracle"]
