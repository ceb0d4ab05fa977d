"""Host-side checks of bench.py's contract: one GPU only, the figures the roofline block is computed from, and
that nothing outside tests/, the smoke entry and bench.py's cpu_baseline leg touches the oracle."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in (r.stderr + r.stdout)


def test_published_peaks_and_algorithmic_work_per_token():
    sys.path.insert(0, ROOT)
    import bench
    assert bench.PEAK_HBM_GBS == 8000.0
    assert bench.PEAK_MFMA_TFLOPS["f16"] == bench.PEAK_MFMA_TFLOPS["bf16"] == 2500.0
    # the traffic table names the workloads the profiles cover
    for key in ("opt66b@0.5", "opt66b@1", "opt66b@0", "opt13b@0.5", "opt30b@0.7", "opt13b_step@0.5"):
        assert bench.read_traffic(key) and bench.read_traffic(key) > 0
    assert bench.read_traffic("no such workload") is None


def test_product_code_never_reaches_the_oracle():
    pkg = os.path.join(ROOT, "paper_2504_07494_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".cpp", ".hip", ".inc", ".h")):
                text = open(os.path.join(dirpath, f), errors="replace").read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", text, flags=re.M), f
                assert "apt_oracle" not in text, f
    # bench.py imports it in one place only: the cpu_baseline leg
    text = open(os.path.join(ROOT, "bench.py")).read()
    assert len(re.findall(r"^\s*from oracle import", text, flags=re.M)) == 1
    assert "if not args.no_cpu_baseline:\n        from oracle import oracle as o" in text
