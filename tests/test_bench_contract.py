"""bench.py's command line (no GPU needed for these paths)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0 and "one GPU" in p.stderr and p.stdout.strip() == ""


def test_planner_mode_prints_json_lines():
    import json
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--planner"], capture_output=True, text=True)
    assert p.returncode == 0
    lines = [json.loads(l) for l in p.stdout.splitlines() if l.strip()]
    assert len(lines) == 2 and all(l["matches_oracle"] for l in lines)
