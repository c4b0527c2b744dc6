"""Host-side contract of bench.py that needs no GPU: one GPU only, and the product path never imports the oracle."""
import ast
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in (r.stderr + r.stdout) and r.stdout.strip() == ""


def test_only_the_cpu_baseline_leg_of_bench_and_smoke_touch_the_oracle():
    """The package never imports oracle/; bench.py imports it in one place, inside the cpu_baseline leg; __graft_entry__ only in smoke()."""
    pkg = os.path.join(ROOT, "paper_2602_06183_amd")
    for name in os.listdir(pkg):
        if name.endswith(".py"):
            tree = ast.parse(open(os.path.join(pkg, name)).read())
            for node in ast.walk(tree):
                if isinstance(node, ast.Import):
                    assert all(a.name.split(".")[0] != "oracle" for a in node.names), name
                if isinstance(node, ast.ImportFrom):
                    assert (node.module or "").split(".")[0] != "oracle", name
    src = open(os.path.join(ROOT, "bench.py")).read()
    lines = [l for l in src.splitlines() if l.strip().startswith(("import oracle", "from oracle"))]
    assert lines == ["        import oracle"]
    at = src.index("        import oracle")
    assert "if not args.no_cpu_baseline:" in src[at - 200:at]
    entry = ast.parse(open(os.path.join(ROOT, "__graft_entry__.py")).read())
    for fn in entry.body:
        if isinstance(fn, ast.FunctionDef) and fn.name != "smoke":
            for node in ast.walk(fn):
                if isinstance(node, (ast.Import, ast.ImportFrom)):
                    names = [a.name for a in node.names] + [getattr(node, "module", "") or ""]
                    assert all(n.split(".")[0] != "oracle" for n in names), fn.name
    for node in entry.body:
        if isinstance(node, (ast.Import, ast.ImportFrom)):
            names = [a.name for a in node.names] + [getattr(node, "module", "") or ""]
            assert all(n.split(".")[0] != "oracle" for n in names)
