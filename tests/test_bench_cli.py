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
    """Sources under version control name neither the builder's scratch folder nor the paper's copy on this machine."""
    listed = subprocess.run(["git", "ls-files"], cwd=ROOT, capture_output=True, text=True, timeout=60)
    if listed.returncode != 0:
        import pytest
        pytest.skip("not a git checkout")
    bad = []
    for rel in listed.stdout.split():
        if not rel.endswith((".py", ".hip", ".h", ".c", ".inc")) or rel == os.path.relpath(__file__, ROOT):
            continue
        text = open(os.path.join(ROOT, rel), errors="replace").read()
        if "_work/" in text or "/root/reference" in text:
            bad.append(rel)
    assert not bad, bad
