"""Host-side pieces of bench.py (no GPU): the refusal of more than one GPU, the readers of the recorded
traffic summaries under profiles/, and the algorithmic work formulas against brute-force counts."""
import os
import subprocess
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_recorded_traffic_readers_parse_the_committed_summaries():
    # kernel names in the legs summary contain a space ("<128, false>"): the reader must not split on it
    for k in ("attn_verify_kernel<128, false>", "attn_chunk_kernel<128, false>", "attn_chunk_kernel<128, true>"):
        v = bench.recorded_leg_traffic(k)
        assert v is not None and v > 1e8, k
    assert bench.recorded_leg_traffic("no_such_kernel") is None
    for k in ("gemm_qkv", "gemm_o", "gemm_gateup", "gemm_down"):
        v = bench.recorded_traffic(k)
        assert v is not None and v > 1e7, k
    assert bench.recorded_traffic("no_such_kernel") is None


def test_gemm_work_counts():
    T, d, F = 7, 64, 176
    w = bench.gemm_work(T, d, F)
    assert w["gemm_qkv"][0] == 2.0 * T * 3 * d * d
    assert w["gemm_gateup"][0] == 2.0 * T * 2 * F * d
    assert w["gemm_down"][0] == 2.0 * T * d * F
    # bytes: weights once + activations in + result (fp16 | fp32 read + write | half the gate/up columns)
    assert w["gemm_o"][1] == 2.0 * d * d + 2.0 * T * d + 8.0 * T * d
    assert w["gemm_gateup"][1] == 2.0 * 2 * F * d + 2.0 * T * d + 1.0 * T * 2 * F


def test_attention_work_counts_visible_pairs_only():
    d = 256
    segs = [(0, 5), (37, 3), (100, 64)]
    flops, byts = bench.attn_work(segs, d)
    pairs = sum(sum(start + i + 1 for i in range(n)) for start, n in segs)   # row i of a segment sees start + i + 1 keys
    assert np.isclose(flops, 4.0 * d * pairs)
