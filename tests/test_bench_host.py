"""Host-side checks of bench.py that need no GPU: the flop counts it prices the kernels with
against the layer's dimensions (Table "shard versions" sizes; a layer is four projections per
shard plus attention), and that it refuses more than one GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import numpy as np     # noqa: E402

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


def test_parity_measures_agree_with_the_test_helper():
    """bench.py states the same two measures the GPU tests assert (tests/parity.py), and they see
    what they are meant to see: a small element far off in relative terms, a non-finite value."""
    from parity import parity
    rng = np.random.default_rng(3)
    want = rng.normal(0, 1, (4, 50, 64))
    got = want + rng.normal(0, 1e-3, want.shape)
    a, b = bench.parity(got, want, 2e-2), parity(got, want, 2e-2)
    assert a["max_rel_err"] == b["max_rel"] and a["elementwise_violations"] == b["violations"] == 0.0
    i = np.unravel_index(np.argmin(np.abs(want)), want.shape)
    got[i] = want[i] + 0.05          # tiny next to the tensor's maximum, large next to rms and to the element
    a = bench.parity(got, want, 2e-2)
    assert a["max_rel_err"] < 2e-2 and a["elementwise_violations"] == 1.0 / want.size
    got[i] = np.nan
    assert bench.parity(got, want, 2e-2)["elementwise_violations"] == 1.0 / want.size


def test_packed_bytes_of_configuration_0():
    # 12 shards at 4 bits: 12 * 589824 / 2 bytes of indexes + 12 codebooks of 16 float32
    assert bench.packed_bytes(S.config0()) == 12 * 294912 + 12 * 64
