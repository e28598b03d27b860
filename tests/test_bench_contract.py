"""Host-side checks of bench.py that need no GPU: the multi-GPU refusal and the workload the default line names."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "single-GPU" in r.stderr and r.stdout.strip() == ""


def test_default_workload_is_the_one_the_baseline_metric_is_quoted_on():
    sys.path.insert(0, ROOT)
    import bench
    from workload import get_config
    saved = sys.argv
    sys.argv = ["bench.py"]
    try:
        a = bench.parse()
    finally:
        sys.argv = saved
    assert a.gpus == 1 and a.workload == "olmoe_like"
    base = json.load(open(os.path.join(ROOT, "BASELINE.json")))
    cfg = get_config(a.workload)
    want = base["configs"][1]
    text = json.dumps(want).lower()
    # the second configuration of the baseline: OLMoE-like layer, 64 experts, top-8, capacity 16
    for value in (cfg.n_experts, cfg.top_k, cfg.d_model, cfg.d_ff, cfg.capacity):
        assert str(value) in text
