"""bench.py's command line without a GPU: more than one GPU is refused with a message."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr
    assert r.stdout.strip() == ""


def test_every_name_bench_uses_exists():
    """A misspelt helper or a call with the wrong number of arguments inside a leg that
    only runs on the GPU would otherwise first show up there: check every call of a
    module-level function of bench.py against that function's signature."""
    import ast
    import inspect
    sys.path.insert(0, ROOT)
    import bench
    tree = ast.parse(open(os.path.join(ROOT, "bench.py")).read())
    funcs = {n: f for n, f in vars(bench).items() if inspect.isfunction(f) and f.__module__ == "bench"}
    checked = 0
    for node in ast.walk(tree):
        if isinstance(node, ast.Call) and isinstance(node.func, ast.Name) and node.func.id in funcs:
            if any(isinstance(a, ast.Starred) for a in node.args) or any(k.arg is None for k in node.keywords):
                continue
            sig = inspect.signature(funcs[node.func.id])
            sig.bind(*[None] * len(node.args), **{k.arg: None for k in node.keywords})
            checked += 1
    assert checked > 30


def test_traffic_figures_are_read_from_the_committed_profile():
    sys.path.insert(0, ROOT)
    import bench
    assert bench.read_traffic("k_assign_stream", "llama3_8b_layer_32k") > 6.9e7
    assert bench.read_traffic("k_attn", "batch8_layer") > 7.0e7
    assert bench.read_traffic("k_attn", "no such workload") is None
