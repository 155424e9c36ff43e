"""Host-side checks of bench.py's command-line contract (no GPU needed)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2", "--steps", "1", "--warmup", "0"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_bench_names_only_committed_inputs():
    src = open(os.path.join(ROOT, "bench.py")).read()
    assert "/root/reference" not in src and "_work/" not in src
    # the oracle is used by the cpu_baseline leg only
    assert src.count("from oracle") + src.count("import oracle") <= 1
