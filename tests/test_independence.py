"""The oracle and the HIP path share no code, and the product path never reaches the oracle."""
import ast
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2406_03285_amd")
ORACLE = os.path.join(ROOT, "oracle")


def _files(top, suffixes):
    for base, _, names in os.walk(top):
        if "__pycache__" in base:
            continue
        for n in names:
            if n.endswith(suffixes):
                yield os.path.join(base, n)


def _imports(path):
    tree = ast.parse(open(path).read(), path)
    for node in ast.walk(tree):
        if isinstance(node, ast.Import):
            for a in node.names:
                yield a.name, node
        elif isinstance(node, ast.ImportFrom):
            yield ("." * node.level) + (node.module or ""), node


def test_package_never_imports_the_oracle():
    for path in _files(PKG, (".py",)):
        for name, _ in _imports(path):
            assert not name.lstrip(".").startswith("oracle"), f"{path} imports {name}"
    for path in _files(PKG, (".h", ".hip", ".c", ".cpp")):
        for inc in re.findall(r'#\s*include\s*[<"]([^>"]+)[>"]', open(path).read()):
            assert "oracle" not in inc and "rbo" not in inc, f"{path} includes {inc}"


def test_oracle_never_touches_the_hip_path():
    for path in _files(ORACLE, (".py",)):
        for name, _ in _imports(path):
            assert "paper_2406_03285_amd" not in name and name.lstrip(".") != "torch", f"{path} imports {name}"
    for path in _files(ORACLE, (".c", ".h")):
        for inc in re.findall(r'#\s*include\s*[<"]([^>"]+)[>"]', open(path).read()):
            assert inc.startswith(("std", "string", "math", "limits", "assert")) or inc in ("stdint.h", "stddef.h", "pthread.h"), \
                f"{path} includes {inc}: only the C library (and POSIX threads for the timing variant)"


def test_bench_reaches_the_oracle_only_in_its_cpu_baseline():
    path = os.path.join(ROOT, "bench.py")
    tree = ast.parse(open(path).read(), path)
    for node in ast.walk(tree):
        if isinstance(node, ast.FunctionDef):
            uses = [n for n, _ in _imports_in(node) if n.lstrip(".").startswith("oracle")]
            assert not uses or node.name.startswith("cpu_baseline"), f"bench.py:{node.name} imports the oracle"
    top = [n for n, node in _imports(path) if n.lstrip(".").startswith("oracle") and node.col_offset == 0]
    assert not top, "bench.py imports the oracle at module level"


def _imports_in(func):
    for node in ast.walk(func):
        if isinstance(node, ast.Import):
            for a in node.names:
                yield a.name, node
        elif isinstance(node, ast.ImportFrom):
            yield ("." * node.level) + (node.module or ""), node


def test_input_generators_hold_none_of_the_methods_arithmetic():
    # the shared module only makes mini-batches: it imports neither side and has no generator of the method's own
    path = os.path.join(ROOT, "rb_workloads.py")
    for name, _ in _imports(path):
        assert name.split(".")[0] in ("torch", "numpy", "math", "dataclasses", "typing"), f"rb_workloads.py imports {name}"
    assert "philox" not in open(path).read().lower()
