"""Host-side checks of bench.py that need no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                         capture_output=True, text=True, timeout=120)
    assert res.returncode != 0
    assert "one GPU" in res.stderr
    assert res.stdout.strip() == ""          # no JSON line for a run that did not happen


def test_algorithmic_bytes_of_the_headline_pass():
    """bench.py's bytes per pass: canonical index and codebook bytes plus x and y of every matrix."""
    sys.path.insert(0, ROOT)
    import workloads
    total = 0
    for (_, _, s, _) in workloads.llama7b_pass_shapes():
        total += sum(workloads.canonical_sizes(s)) + 2 * s.in_features + 2 * s.out_features
    assert total == 1826373632
