"""Host-side checks of bench.py's contract: it refuses more than one GPU with a message, its recorded
HBM-traffic figure is tied to the kernel sources it was measured on, and the product path never imports
the oracle outside the CPU-baseline leg."""
from __future__ import annotations

import ast
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""           # no JSON line for a run that measured nothing


def test_recorded_traffic_is_tied_to_the_kernel_sources():
    sys.path.insert(0, ROOT)
    import bench
    sha = bench.kernel_sources_sha256()
    assert len(sha) == 64
    if bench.TRAFFIC["sources_sha256"] == sha:
        t = bench.measured_traffic(bench.TRAFFIC["workload"])
        assert t is not None and 2.1e9 < t < 2.4e9      # K once (2.147 GB) plus a few per cent
    else:
        assert bench.measured_traffic(bench.TRAFFIC["workload"]) is None
    assert bench.measured_traffic("some-other-workload") is None


def test_oracle_is_imported_only_in_the_cpu_baseline_leg():
    """The library package never imports the oracle; bench.py does so only under `if not args.no_cpu_baseline`."""
    pkg = os.path.join(ROOT, "paper_2603_02631_amd")
    for name in os.listdir(pkg):
        if name.endswith(".py"):
            tree = ast.parse(open(os.path.join(pkg, name)).read())
            for node in ast.walk(tree):
                if isinstance(node, ast.Import):
                    assert all(a.name.split(".")[0] != "oracle" for a in node.names), name
                if isinstance(node, ast.ImportFrom):
                    assert (node.module or "").split(".")[0] != "oracle", name
    src = open(os.path.join(ROOT, "bench.py")).read()
    tree = ast.parse(src)
    lines = [n.lineno for n in ast.walk(tree) if isinstance(n, ast.Import) and any(a.name == "oracle" for a in n.names)]
    assert len(lines) == 1
    guard = [n for n in ast.walk(tree) if isinstance(n, ast.If) and "no_cpu_baseline" in ast.unparse(n.test)]
    assert any(g.lineno < lines[0] <= g.end_lineno for g in guard)
