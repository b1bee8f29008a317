"""Host-side checks of bench.py that need no GPU: the one-GPU rule, the byte count of a layer-pass and the
reader of the traffic summaries under profiles/."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and "--gpus 1" in r.stderr
    assert r.stdout.strip() == ""                          # no result line


def test_algorithmic_bytes_of_the_headline_layer_pass():
    # Llama3-8B shape, 32768 tokens, bf16: 2048 B per token for K, 4 x retained rows x 256 B for the gather,
    # 64 B per token of scores (written and read once), the window queries, 12 B per unit
    N, Hkv, d, e, Hq = 32768, 8, 128, 2, 32
    kept = 188940
    b = bench.algorithmic_bytes(N, Hkv, d, e, Hq, 32, kept, 8, False)
    assert b == N * 2048 + 32 * Hq * d * e + N * 64 + 4 * kept * 256 + 96
    per_token = b / N
    rho = kept / (N * Hkv)
    assert abs(per_token - (2048 * (1 + 4 * rho) + 64)) < 10          # the per-token formula, up to the query rows
    assert bench.algorithmic_bytes(N, Hkv, d, e, Hq, 32, kept, 8, True) == b + 8 * kept   # the index list


def test_traffic_summaries_are_found_and_consistent():
    step = bench.read_traffic("step", "llama3-8b-32k")
    dom = bench.read_traffic("compact", "llama3-8b-32k")
    assert step and dom and bench.read_traffic("compact", "no-such-workload") is None
    for t in (step, dom):
        assert t["total_bytes"] == t["fetch_bytes"] + t["write_bytes"]
        assert os.path.exists(os.path.join(ROOT, t["source"]))
    # the whole pass moves more than its dominant kernel and more than the method's own byte count
    assert step["total_bytes"] > dom["total_bytes"] > 150e6
    assert step["total_bytes"] > bench.algorithmic_bytes(32768, 8, 128, 2, 32, 32, 188940, 8, False)
