"""Host-side behaviour of bench.py and the entry module that needs no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_bench_line_fields_are_declared():
    """The keys the measurement contract names all appear in the line bench.py prints."""
    text = open(os.path.join(ROOT, "bench.py")).read()
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline", "bound", "achieved", "peak", "frac",
                "traffic", "cores", "kind", "sample"):
        assert f'"{key}"' in text, key


def test_nothing_committed_reads_the_working_folder_or_the_paper_copy():
    bad = []
    for base, _, files in os.walk(ROOT):
        if any(part in base for part in ("/_work", "/gpurun_out", "/.git", "__pycache__", "/.pytest_cache")):
            continue
        for f in files:
            if not f.endswith((".py", ".hip", ".h", ".c", ".inc")) or f == os.path.basename(__file__):
                continue
            text = open(os.path.join(base, f), errors="replace").read()
            if "_work/" in text or "/root/reference" in text:
                bad.append(os.path.relpath(os.path.join(base, f), ROOT))
    assert not bad, bad
