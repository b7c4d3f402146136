"""Host-side checks of bench.py that need no GPU: the flop counts it prices the kernels with
against the layer's dimensions (Table "shard versions" sizes; a layer is four projections per
shard plus attention), and that it refuses more than one GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench           # noqa: E402
import sti_synth as S  # noqa: E402


def test_layer_flops_from_the_dimensions():
    # per token and full layer: 2 (4 d^2 + 2 d d_ff) + 4 L d
    d, dff, L = 768, 3072, 128
    assert bench.layer_flops_per_token(S.BERT_BASE, L, 12) == 2 * (4 * d * d + 2 * d * dff) + 4 * L * d == 14548992
    d, dff, L = 1024, 4096, 256
    assert bench.layer_flops_per_token(S.BERT_LARGE_SHAPED, L, 16) == 2 * (4 * d * d + 2 * d * dff) + 4 * L * d == 26214400
    # absent shards are not counted: 9 of 12 present is three quarters of the layer
    assert bench.layer_flops_per_token(S.BERT_BASE, 128, 9) * 4 == bench.layer_flops_per_token(S.BERT_BASE, 128, 12) * 3


def test_gemm_flops_add_up_to_the_projections():
    kinds = ("gemm_qkv", "gemm_out", "gemm_ffn_up", "gemm_ffn_down")
    total = sum(bench.gemm_flops(S.BERT_BASE, 4096, 12, k) for k in kinds)
    assert total == 4096 * 2 * (4 * 768 * 768 + 2 * 768 * 3072)
    # the average per launch that the roofline object reports for configuration 4
    assert total / 4 == 14495514624.0


def test_measured_traffic_is_dropped_when_the_sources_change(monkeypatch):
    good = bench.TRAFFIC["gemm"]
    assert bench.sources_sha256(good["files"]) == bench.sources_sha256(good["files"])   # deterministic
    monkeypatch.setitem(bench.TRAFFIC, "gemm", dict(good, sha256="0" * 64))
    assert bench.measured_traffic("gemm") is None


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
