"""The oracle is test infrastructure: the product never reaches it, the oracle never reaches the
product, and nothing that is committed reads the builder's working folder."""
import ast
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2505_23725_amd")


def _python_files(folder):
    for base, dirs, files in os.walk(folder):
        dirs[:] = [d for d in dirs if d != "__pycache__"]
        for f in files:
            if f.endswith(".py"):
                yield os.path.join(base, f)


def _imported_modules(path):
    tree = ast.parse(open(path).read(), filename=path)
    for node in ast.walk(tree):
        if isinstance(node, ast.Import):
            for a in node.names:
                yield a.name
        elif isinstance(node, ast.ImportFrom) and node.module:
            yield node.module


def test_product_never_imports_the_oracle():
    for path in _python_files(PKG):
        for mod in _imported_modules(path):
            assert mod.split(".")[0] != "oracle", f"{path} imports {mod}"
        assert "oracle" not in open(path).read().lower(), f"{path} mentions the oracle"
    for name in os.listdir(os.path.join(PKG, "csrc")):
        text = open(os.path.join(PKG, "csrc", name)).read()
        assert not re.search(r'#include\s+"[^"]*oracle', text), f"csrc/{name} includes oracle code"


def test_oracle_never_imports_the_product_or_torch_gpu_code():
    for path in _python_files(os.path.join(ROOT, "oracle")):
        mods = {m.split(".")[0] for m in _imported_modules(path)}
        assert "paper_2505_23725_amd" not in mods, f"{path} imports the product"
        assert "ctypes" not in mods, f"{path} could load the HIP library"
        assert mods <= {"numpy", "math", "typing", "__future__", "oracle", "dataclasses"}, (path, mods)


def test_oracle_is_only_used_by_tests_smoke_and_the_cpu_baseline():
    users = []
    for path in list(_python_files(ROOT)):
        rel = os.path.relpath(path, ROOT)
        if rel.startswith(("tests" + os.sep, "oracle" + os.sep, "_work" + os.sep, "gpurun_out" + os.sep)):
            continue
        if any(m.split(".")[0] == "oracle" for m in _imported_modules(path)):
            users.append(rel)
    assert sorted(users) == ["__graft_entry__.py", "bench.py"], users
    # in bench.py the import sits inside the cpu_baseline leg only
    tree = ast.parse(open(os.path.join(ROOT, "bench.py")).read())
    for node in ast.walk(tree):
        if isinstance(node, ast.FunctionDef):
            uses = any(isinstance(n, (ast.Import, ast.ImportFrom)) and
                       ((getattr(n, "module", None) or "").split(".")[0] == "oracle" or
                        any(a.name.split(".")[0] == "oracle" for a in n.names))
                       for n in ast.walk(node))
            assert not uses or node.name == "cpu_baseline", f"bench.py: {node.name} imports the oracle"


def test_nothing_committed_reads_the_working_folder():
    for path in _python_files(ROOT):
        rel = os.path.relpath(path, ROOT)
        if rel.startswith(("_work" + os.sep, "gpurun_out" + os.sep)) or rel == os.path.join("tests", "test_separation.py"):
            continue
        text = open(path).read()
        assert not re.search(r"(^|[^A-Za-z0-9])_work([/\\\"' ]|$)", text, re.M), f"{rel} names the working folder"
