"""Host-side checks of bench.py that need no GPU: the multi-GPU refusal and the workloads the default run covers."""
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


def test_default_run_covers_both_configurations_the_bandwidth_target_names():
    """The baseline's metric names no configuration; its target sentence names the OLMoE-like and the Mixtral-like
    ones.  The default line is quoted on the OLMoE-like layer (the second baseline configuration) and carries a
    section for a cut of the Mixtral-like stack (the third)."""
    sys.path.insert(0, ROOT)
    import bench
    from workload import get_config
    saved = sys.argv
    sys.argv = ["bench.py"]
    try:
        a = bench.parse()
    finally:
        sys.argv = saved
    assert a.gpus == 1 and a.workload == "olmoe_like" and a.second_layers > 0
    base = json.load(open(os.path.join(ROOT, "BASELINE.json")))
    assert "OLMoE-like and Mixtral-like" in base["north_star"]
    for name, want in (("olmoe_like", base["configs"][1]), ("mixtral_like", base["configs"][2])):
        cfg = get_config(name)
        text = json.dumps(want).lower()
        for value in (cfg.n_experts, cfg.top_k, cfg.d_model, cfg.d_ff, cfg.capacity, cfg.n_layers):
            assert str(value) in text, (name, value)
