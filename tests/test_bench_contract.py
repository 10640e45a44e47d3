"""The benchmark's command line and the fixed parts of its JSON line, without a GPU."""
import ast
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0 and "one GPU" in (p.stderr + p.stdout)


def test_without_a_gpu_the_benchmark_fails_loudly_instead_of_falling_back():
    import torch
    if torch.cuda.is_available():
        return
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "1", "--warmup", "0", "--no-cpu"],
                       capture_output=True, text=True)
    assert p.returncode != 0 and not p.stdout.strip().startswith("{")


def test_the_product_never_imports_the_oracle():
    """Only tests, smoke() and the cpu_baseline leg of bench.py may touch oracle/."""
    pkg = os.path.join(ROOT, "paper_2601_19092_amd")
    for name in os.listdir(pkg):
        if name.endswith(".py"):
            tree = ast.parse(open(os.path.join(pkg, name)).read())
            for node in ast.walk(tree):
                if isinstance(node, ast.Import):
                    assert not any(a.name.split(".")[0] == "oracle" for a in node.names), name
                if isinstance(node, ast.ImportFrom):
                    assert (node.module or "").split(".")[0] != "oracle", name
    for name in os.listdir(os.path.join(pkg, "csrc")):
        assert "oracle" not in open(os.path.join(pkg, "csrc", name)).read().lower() or name == "README", name
    # bench.py: the oracle appears in the cpu_baseline function only
    src = open(os.path.join(ROOT, "bench.py")).read()
    tree = ast.parse(src)
    for node in tree.body:
        if isinstance(node, ast.FunctionDef):
            uses = any(isinstance(n, ast.ImportFrom) and (n.module or "").startswith("oracle") for n in ast.walk(node)) or \
                   any(isinstance(n, ast.Import) and any(a.name.startswith("oracle") for a in n.names) for n in ast.walk(node))
            assert not uses or "cpu" in node.name, node.name
    # and the oracle never imports the product's kernels or binding
    for name in os.listdir(os.path.join(ROOT, "oracle")):
        if name.endswith(".py"):
            tree = ast.parse(open(os.path.join(ROOT, "oracle", name)).read())
            for node in ast.walk(tree):
                mods = [a.name for a in node.names] if isinstance(node, ast.Import) else \
                       [node.module or ""] if isinstance(node, ast.ImportFrom) else []
                assert not any(m.startswith("paper_2601_19092_amd") for m in mods), name
                if isinstance(node, ast.Constant) and isinstance(node.value, str):
                    assert "libaxe_hip" not in node.value or node is tree.body[0].value, name
