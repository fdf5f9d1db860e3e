"""Host-side checks of bench.py's contract that need no GPU: it refuses more than one GPU with a message, and the
committed counter summaries it reads exist, parse and carry the keys it uses."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)


def test_counter_summaries_bench_reads():
    prof = os.path.join(ROOT, "profiles")
    t = json.load(open(os.path.join(prof, "gemv_8b_layer_q2_traffic.json")))
    # measured HBM bytes per launch of the headline kernel: at least the algorithmic bytes, and not wasteful
    assert 64_913_408 <= t["hbm_bytes_per_launch"] <= 1.02 * 64_913_408
    assert os.path.exists(os.path.join(ROOT, t["source"]))
    s = json.load(open(os.path.join(prof, "gemm_small_batch_q4_counters.json")))
    assert set(s["valu_wave_insts_per_launch"]) == {"1", "2", "4", "8", "16"}
    assert set(s["kernels"]) == {"1", "2", "4", "8", "16"}
    assert os.path.exists(os.path.join(ROOT, s["source"]))
    q = json.load(open(os.path.join(prof, "quantize_alg1_8b_layer_q2_counters.json")))
    assert q["valu_wave_insts_per_layer"] > 0 and q["weights_per_layer"] == 218_103_808
    assert os.path.exists(os.path.join(ROOT, q["source"]))
    v = json.load(open(os.path.join(prof, "gemv_8b_layer_q2_table_variants_counters.json")))
    assert os.path.exists(os.path.join(ROOT, v["source"]))
