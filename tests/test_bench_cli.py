"""bench.py on a box without a GPU: what it refuses, and the figures it takes from profiles/."""
import importlib.util
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args, env=None):
    e = dict(os.environ)
    e.pop("WORLD_SIZE", None)
    e.update(env or {})
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          env=e, timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run("--gpus", "2")
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
    r = run(env={"WORLD_SIZE": "4"})
    assert r.returncode == 2 and "ONE GPU" in r.stderr


def test_profile_figures_are_found_for_the_benchmarked_workloads():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    for name, alg in [("c2", 1.8e9), ("c3", 3.9e9), ("c5", 6.9e9)]:
        t = bench.profiled_traffic(name, alg)
        # counters say the kernel moves within a few percent of the algorithmic bytes
        assert t is not None and 0.98 * alg < t < 1.06 * alg, (name, t)
    assert bench.profiled_traffic("no such workload", 1.0) is None
    v = bench.profiled_valu_per_logit("c2")
    assert v is not None and 10.0 < v < 60.0
    assert bench.profiled_valu_per_logit("c9") is None
