"""Host-side pieces of bench.py (no GPU): the figures it takes from the tracked profiler summaries, its refusal
to run on more than one GPU, its refusal to fall back to the CPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_profile_facts_come_from_the_tracked_summaries():
    sys.path.insert(0, ROOT)
    import bench
    facts = bench.profile_facts()
    traffic, src = facts["quantize_kernel.traffic_GB_per_launch"]
    assert src.endswith(".txt") and os.path.exists(os.path.join(ROOT, "profiles", src))
    # measured HBM traffic of the quantize launch: not below the algorithmic 8 388 608 keys x 304 B, and no re-reads
    assert 2.550 <= traffic <= 2.550 * 1.05
    valu, _ = facts["key_scores_rope_kernel.valu_per_16_keys"]
    assert 80 < valu < 400
    # every summary names the command that made it
    for name in os.listdir(os.path.join(ROOT, "profiles")):
        text = open(os.path.join(ROOT, "profiles", name)).read()
        assert "command" in text and ("rocprofv3" in text or "bench.py" in text), name


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode != 0
    assert "one GPU" in res.stderr and not res.stdout.strip()


def test_no_cpu_fallback():
    """Without a GPU the benchmark exits with an error instead of timing anything else."""
    import torch
    if torch.cuda.is_available():
        return
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--brief"], capture_output=True, text=True)
    assert res.returncode != 0 and not res.stdout.strip()
