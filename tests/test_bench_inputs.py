"""Host-side checks of what bench.py reads besides the library (no GPU)."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_counter_summary_for_the_alu_roofline_is_present():
    # bench.py derives its vector-ALU roofline from the measured VALU instruction count per launch
    path = os.path.join(ROOT, "profiles", "fused_block_kernel_cfg2_pmc.json")
    counters = json.load(open(path))
    assert counters["SQ_INSTS_VALU"] > 0 and counters["SQ_WAVES"] > 0


def test_traffic_summary_is_present():
    t = json.load(open(os.path.join(ROOT, "profiles", "fused_block_kernel_cfg2_hbm_traffic.json")))
    assert any(isinstance(v, (int, float)) and v > 0 for v in t.values())


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr) or "1 GPU" in (r.stdout + r.stderr) or "single" in (r.stdout + r.stderr).lower()
