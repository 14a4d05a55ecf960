"""Host-side checks of bench.py that need no GPU: the byte count it prices the roofline with, the
refusal to pretend there is more than one GPU, and that the workload generator and the oracle leg
it uses run on a tiny instance."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402
from workloads import spec_for  # noqa: E402


def test_algorithmic_bytes_match_the_stated_formula():
    """2*k*H_kv*d*e (K and V) + 2*H*d*e (q, out) + 2*H_kv*d*e (new k, v) + 2*H_kv*d*e (slot) + 8, per unit."""
    spec = spec_for("c3_mistral_gqa")
    per_unit = 2 * 1024 * 8 * 128 * 2 + 2 * 32 * 128 * 2 + 4 * 8 * 128 * 2 + 8
    assert per_unit == 4_218_888
    assert bench.algorithmic_bytes_per_step(spec) == per_unit * 64 == 270_008_832
    spec4 = spec_for("c4_llama7b_stack")
    assert bench.algorithmic_bytes_per_step(spec4) == 2048 * (2 * 4096 * 32 * 128 * 2 + 2 * 32 * 128 * 2 + 4 * 32 * 128 * 2 + 8)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one gpu" in (r.stdout + r.stderr).lower() and "--gpus" in (r.stdout + r.stderr)


def test_oracle_worker_runs_a_tiny_instance():
    spec = spec_for("c1_tiny", T=40)
    secs = bench._oracle_worker((spec, 1, 0, 24))        # (spec, seed, sequence, timed steps after the fill)
    assert secs > 0
