"""The oracle and the product path share no code: neither imports the other, and only the seeded input
generator (which holds none of the method's arithmetic) serves both."""
import ast
import glob
import os

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _imports(path):
    tree = ast.parse(open(path).read())
    names = set()
    for node in ast.walk(tree):
        if isinstance(node, ast.Import):
            names.update(a.name.split(".")[0] for a in node.names)
        elif isinstance(node, ast.ImportFrom) and node.module and node.level == 0:
            names.add(node.module.split(".")[0])
    return names


def test_product_package_never_imports_the_oracle():
    for path in glob.glob(os.path.join(ROOT, "paper_2503_05840_amd", "**", "*.py"), recursive=True):
        assert "oracle" not in _imports(path), path
    for path in glob.glob(os.path.join(ROOT, "paper_2503_05840_amd", "csrc", "*")):
        assert "oracle" not in open(path, errors="ignore").read(), path


def test_oracle_imports_nothing_of_the_product():
    for path in glob.glob(os.path.join(ROOT, "oracle", "*.py")):
        assert "paper_2503_05840_amd" not in _imports(path), path
        assert _imports(path) <= {"__future__", "numpy", "math"}, (path, _imports(path))


def test_bench_touches_the_oracle_only_inside_its_cpu_baseline_legs():
    src = open(os.path.join(ROOT, "bench.py")).read()
    tree = ast.parse(src)
    top = [n for n in tree.body if isinstance(n, (ast.Import, ast.ImportFrom))]
    for n in top:
        mod = getattr(n, "module", None) or ""
        assert not mod.startswith("oracle") and all(not a.name.startswith("oracle") for a in n.names)
    # every import of the oracle sits under an `if not args.no_cpu_baseline:` block
    lines = src.splitlines()
    for i, ln in enumerate(lines):
        if "from oracle" in ln or "import oracle" in ln:
            indent = len(ln) - len(ln.lstrip())
            guard = next(l for l in reversed(lines[:i]) if l.strip() and len(l) - len(l.lstrip()) < indent)
            assert "no_cpu_baseline" in guard, (i + 1, guard)
