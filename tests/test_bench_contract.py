"""Host-side checks of bench.py that need no GPU: the one-GPU rule, the algorithmic FLOP and byte
formulas behind the roofline figures (Eq. 8 terms, 2 m n k convention) and the counter-summary parser."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench                                            # noqa: E402  (imports no GPU code at module level)
from et_inputs import SIGLIP                            # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)


def test_flop_formulas_at_the_benchmarked_shape():
    T, L, D, Mh = 32, SIGLIP.tokens_per_frame, SIGLIP.d_model, SIGLIP.d_mlp
    assert (L, D, Mh, SIGLIP.n_heads, SIGLIP.head_dim) == (729, 1152, 4304, 16, 72)
    fl = bench.flops_tables(SIGLIP, T, 8, 364, 8)
    R = T * L
    assert fl[("gemm_fc1", 0)] == 2.0 * R * D * Mh == 2.0 * 23328 * 1152 * 4304
    assert fl[("gemm_qkv", 0)] == 2.0 * R * D * 3 * D
    assert fl[("attention", 0)] == 4.0 * T * 16 * L * L * 72
    assert fl[("gemm_fc2", 1)] == 2.0 * 8 * 364 * D * Mh
    # per token and layer, Eq. 8 doubled: 8 D^2 + 4 D Mh + 4 n D
    per_token = sum(fl[(k, 0)] for k in ("gemm_qkv", "gemm_out", "gemm_fc1", "gemm_fc2", "attention")) / R
    assert per_token == pytest.approx(8 * D * D + 4 * D * Mh + 4 * L * D)
    # the uncompressed 32-frame clip: 27 layers + patch embedding = 21.3 TFLOP
    assert bench.clip_flops(SIGLIP, T, T, L, -1) == pytest.approx(21.29e12, rel=2e-3)
    # compression after 8 blocks to 8 frames of 364 tokens
    want = 2.0 * R * 588 * D + 8 * R * per_token + 19 * 8 * 364 * (8 * D * D + 4 * D * Mh + 4 * 364 * D)
    assert bench.clip_flops(SIGLIP, T, 8, 364, 8) == pytest.approx(want)


def test_stage_bytes_of_the_merge_only_workload():
    # [64, 729, 1152] bf16, 11 segments, 218 kept tokens per frame: x twice, merged frames, kept rows in and out
    b = bench.stage_bytes(64, 729, 1152, 11, 218)
    x = 64 * 729 * 1152 * 2
    assert b == 2 * x + 11 * 729 * 1152 * 2 + 2 * 11 * 218 * 1152 * 2 + 2 * 64 * 729 * 4
    assert round(b / 1e6, 1) == 244.9


def test_traffic_is_quoted_only_for_the_kernel_the_summary_names():
    value, source = bench.measured_traffic("gemm_fc1@all")
    assert value and value > 2.6e8 and source.startswith("profiles/")
    assert bench.measured_traffic("attention@all") == (None, None)
