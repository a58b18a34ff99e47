"""Structural rules of this repository, checked without a GPU: the oracle and the product path share nothing, the
benchmark refuses more than one GPU, and nothing tracked depends on untracked working files."""
import ast
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _imports(path):
    tree = ast.parse(open(path).read(), filename=path)
    names = set()
    for node in ast.walk(tree):
        if isinstance(node, ast.Import):
            names.update(a.name.split(".")[0] for a in node.names)
        elif isinstance(node, ast.ImportFrom) and node.level == 0 and node.module:
            names.add(node.module.split(".")[0])
    return names


def _py_files(*dirs):
    for d in dirs:
        for base, _sub, files in os.walk(os.path.join(ROOT, d)):
            for f in files:
                if f.endswith(".py"):
                    yield os.path.join(base, f)


def test_product_and_input_generators_never_import_the_oracle():
    for path in _py_files("paper_2602_01027_amd", "sfmp_workloads"):
        assert "oracle" not in _imports(path), path


def test_oracle_imports_neither_the_product_nor_a_gpu_library():
    for path in _py_files("oracle"):
        got = _imports(path)
        assert not got & {"paper_2602_01027_amd", "torch", "ctypes", "bench"}, (path, got)


def test_native_sources_do_not_mention_the_oracle():
    csrc = os.path.join(ROOT, "paper_2602_01027_amd", "csrc")
    for f in os.listdir(csrc) + ["../../include/sfmp.h"]:
        text = open(os.path.join(csrc, f)).read()
        assert "oracle/" not in text and "sfmp_oracle" not in text, f


def test_bench_uses_the_oracle_only_in_its_cpu_baseline():
    tree = ast.parse(open(os.path.join(ROOT, "bench.py")).read())
    for node in ast.walk(tree):
        if isinstance(node, ast.FunctionDef):
            inner = {n.module.split(".")[0] for n in ast.walk(node) if isinstance(n, ast.ImportFrom) and n.module}
            inner |= {a.name.split(".")[0] for n in ast.walk(node) if isinstance(n, ast.Import) for a in n.names}
            if "oracle" in inner:
                assert node.name == "cpu_baseline", node.name
    top = {a.name.split(".")[0] for n in tree.body if isinstance(n, ast.Import) for a in n.names}
    top |= {n.module.split(".")[0] for n in tree.body if isinstance(n, ast.ImportFrom) and n.module}
    assert "oracle" not in top


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120, cwd=ROOT)
    assert r.returncode == 2, (r.returncode, r.stderr[-300:])
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""


def test_nothing_tracked_reads_untracked_working_files():
    tracked = subprocess.run(["git", "ls-files"], capture_output=True, text=True, cwd=ROOT, timeout=60).stdout.split()
    assert tracked, "not a git checkout"
    for rel in tracked:
        assert not rel.startswith(("_work/", "gpurun_out/", "tools/", "scripts/")), rel
        if rel.endswith((".py", ".hip", ".h", ".cpp", ".sh")) and rel != "tests/test_repo_contract.py":
            text = open(os.path.join(ROOT, rel), errors="replace").read()
            assert "_work/" not in text and "/root/reference" not in text, rel


def test_binding_fails_loudly_without_the_library(tmp_path, monkeypatch):
    """No CPU fallback: with the shared object out of reach the binding raises instead of computing anything."""
    import pytest
    import paper_2602_01027_amd.binding as B
    monkeypatch.setattr(B, "_LIB", None)
    monkeypatch.setattr(B, "lib_path", lambda: str(tmp_path / "libsfmp.so"))
    with pytest.raises(FileNotFoundError, match="no CPU fallback"):
        B.load_library()
    with pytest.raises(FileNotFoundError):
        B.sfmp_check_perm(__import__("numpy").arange(4, dtype="int32"))
