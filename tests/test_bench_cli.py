"""Host-only checks of bench.py's command line."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout == ""


def test_source_digest_is_stable_and_names_the_kernel_sources():
    sys.path.insert(0, ROOT)
    import bench
    d = bench.csrc_digest()
    assert len(d) == 16 and d == bench.csrc_digest()
    assert set(bench.MEASURED_TRAFFIC["MB_per_step"]) <= set(bench.PHASE_KERNELS)
    assert set(bench.PHASE_LAUNCHES) == set(bench.PHASE_KERNELS)


def test_every_global_name_bench_uses_is_defined():
    """bench.py runs on the GPU machine only: an undefined module-level name must not wait until then to show."""
    import ast
    import builtins
    src = open(os.path.join(ROOT, "bench.py")).read()
    tree = ast.parse(src)
    defined = set(dir(builtins)) | {"__file__", "__name__"}
    for node in ast.walk(tree):
        if isinstance(node, (ast.FunctionDef, ast.ClassDef)):
            defined.add(node.name)
            for a in node.args.args + node.args.kwonlyargs if isinstance(node, ast.FunctionDef) else []:
                defined.add(a.arg)
            if isinstance(node, ast.FunctionDef):
                for a in (node.args.vararg, node.args.kwarg):
                    if a is not None:
                        defined.add(a.arg)
        elif isinstance(node, ast.Lambda):
            for a in node.args.args + node.args.kwonlyargs:
                defined.add(a.arg)
        elif isinstance(node, (ast.Import, ast.ImportFrom)):
            for a in node.names:
                defined.add((a.asname or a.name).split(".")[0])
        elif isinstance(node, ast.Name) and isinstance(node.ctx, (ast.Store, ast.Del)):
            defined.add(node.id)
        elif isinstance(node, ast.ExceptHandler) and node.name:
            defined.add(node.name)
        elif isinstance(node, ast.arg):
            defined.add(node.arg)
    used = {node.id for node in ast.walk(tree) if isinstance(node, ast.Name) and isinstance(node.ctx, ast.Load)}
    assert used <= defined, sorted(used - defined)
