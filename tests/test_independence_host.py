"""The product path and the oracle stay apart: nothing under the package imports the oracle, the oracle
imports nothing of the package, bench.py touches the oracle only inside its CPU-baseline leg, and the
input generators hold none of the method's modules."""
import ast
import os

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _imports(path):
    tree = ast.parse(open(path).read())
    found = []
    for node in ast.walk(tree):
        if isinstance(node, ast.Import):
            found += [(a.name, node.lineno) for a in node.names]
        elif isinstance(node, ast.ImportFrom):
            found.append(((node.module or "") if node.level == 0 else "." * node.level + (node.module or ""), node.lineno))
    return found


def _py_files(folder):
    for base, _, files in os.walk(os.path.join(ROOT, folder)):
        for f in files:
            if f.endswith(".py"):
                yield os.path.join(base, f)


def test_package_never_imports_the_oracle():
    for path in _py_files("paper_2306_00256_amd"):
        for name, line in _imports(path):
            assert not name.startswith("oracle"), (path, line)
    for path in os.listdir(os.path.join(ROOT, "paper_2306_00256_amd", "csrc")):
        text = open(os.path.join(ROOT, "paper_2306_00256_amd", "csrc", path)).read()
        assert "oracle" not in text, path


def test_oracle_and_generators_import_nothing_of_the_package():
    for path in list(_py_files("oracle")) + [os.path.join(ROOT, "workloads.py")]:
        for name, line in _imports(path):
            assert "paper_2306_00256_amd" not in name, (path, line)
            assert not name.startswith("torch") or path.endswith("workloads.py"), (path, line)
    for name, line in _imports(os.path.join(ROOT, "workloads.py")):
        assert not name.startswith("oracle"), line


def test_bench_uses_the_oracle_only_in_its_cpu_baseline():
    path = os.path.join(ROOT, "bench.py")
    tree = ast.parse(open(path).read())
    for node in tree.body:
        inner = [n for n in ast.walk(node) if isinstance(n, (ast.Import, ast.ImportFrom))]
        for n in inner:
            names = [a.name for a in n.names] if isinstance(n, ast.Import) else [n.module or ""]
            if any(x.startswith("oracle") for x in names):
                # the CPU-baseline leg: cpu_baseline and the worker body it runs on one thread and on all cores
                assert isinstance(node, ast.FunctionDef) and node.name in ("cpu_baseline", "_cpu_sample"), \
                    (getattr(node, "name", None), n.lineno)
