"""GPU parity of sti_quantize_layer (Section "quantization per shard"; Section "Implementation")
against the reference quantizer: codebook, packed index streams and outlier dictionaries must
be identical bit for bit; the fitted moments agree to float64 rounding; and the library's own
decoder turns the quantizer's output back into the reference's dequantized weights."""
import ctypes as C

import numpy as np
import pytest

import sti_synth as S

pytestmark = pytest.mark.gpu

MID = S.Dims(128, 4, 64, 64, 1e-12)                # Wsh = 49,152 = 48 chunks of 1024


def layer_weights(seed, dims, sigma=0.03, tail=0.0015):
    """Gaussian weights with a sparse heavy tail (the paper reports 0.14-0.17 % outliers)."""
    rng = np.random.default_rng(seed)
    M, wsh = dims.n_heads, dims.weights_per_shard
    w = rng.normal(0.0, sigma, size=(M, wsh))
    mask = rng.random((M, wsh)) < tail
    w[mask] = rng.choice([-1.0, 1.0], size=int(mask.sum())) * rng.uniform(5 * sigma, 10 * sigma, size=int(mask.sum()))
    return w.astype(np.float32)


def run_gpu(dims, w, k, max_out):
    import torch
    import paper_2207_05022_amd as P
    M, wsh = dims.n_heads, dims.weights_per_shard
    wd = torch.from_numpy(w).cuda()
    packed = torch.full((M, wsh * k // 8), 0xAA, dtype=torch.uint8, device="cuda")
    cb = torch.full((1 << k,), float("nan"), device="cuda")
    pos = torch.full((M, max_out), -1, dtype=torch.int32, device="cuda")
    val = torch.full((M, max_out), float("nan"), device="cuda")
    cnt = torch.full((M,), -1, dtype=torch.int32, device="cuda")
    stats = torch.zeros(32, dtype=torch.uint8, device="cuda")
    ws = torch.empty(P.sti_quantize_workspace_bytes(dims), dtype=torch.uint8, device="cuda")
    P.sti_quantize_layer(dims, wd, k, packed, cb, pos, val, cnt, stats, ws)
    torch.cuda.synchronize()
    st = P.StiQuantStats.from_buffer_copy(stats.cpu().numpy().tobytes())
    return dict(packed=packed, codebook=cb, pos=pos, val=val, cnt=cnt, stats=st, wd=wd)


def check_against_reference(dims, w, k, g):
    from oracle import sti_quantizer_oracle as Q
    q = Q.quantize_layer(w, k)
    M = dims.n_heads
    assert g["stats"].status == 0
    assert abs(g["stats"].mean - q["mu"]) <= 1e-12 * max(1.0, abs(q["mu"])) + 1e-15
    assert abs(g["stats"].variance - q["var"]) <= 1e-11 * q["var"]
    assert g["stats"].n_outliers == sum(len(p) for p in q["outlier_pos"])
    assert np.array_equal(g["codebook"].cpu().numpy().view(np.uint32), q["codebook"].view(np.uint32))
    cnt = g["cnt"].cpu().numpy()
    for s in range(M):
        assert np.array_equal(g["packed"][s].cpu().numpy(), Q.pack_indexes(q["indexes"][s], k)), (k, s)
        n = len(q["outlier_pos"][s])
        assert cnt[s] == n
        assert np.array_equal(g["pos"][s, :n].cpu().numpy().view(np.uint32), q["outlier_pos"][s])
        assert np.array_equal(g["val"][s, :n].cpu().numpy().view(np.uint32), q["outlier_val"][s].view(np.uint32))
    return q


@pytest.mark.parametrize("k", [2, 3, 4, 5, 6])
def test_quantizer_matches_reference(k):
    w = layer_weights(50 + k, MID)
    g = run_gpu(MID, w, k, max_out=512)
    check_against_reference(MID, w, k, g)


def test_quantizer_repeats_bit_for_bit():
    """The same input gives the same codebook, streams and dictionaries on every call, at the
    BERT-base shard size (576 chunks per shard, 6-bit: 64 clusters per LDS accumulator set)."""
    dims = S.Dims(768, 2, 64, 256, 1e-12)
    w = layer_weights(77, dims)
    a = run_gpu(dims, w, 6, max_out=4096)
    for _ in range(3):
        b = run_gpu(dims, w, 6, max_out=4096)
        assert np.array_equal(a["codebook"].cpu().numpy().view(np.uint32), b["codebook"].cpu().numpy().view(np.uint32))
        assert bool((a["packed"] == b["packed"]).all())
        assert bool((a["cnt"] == b["cnt"]).all())
    check_against_reference(dims, w, 6, a)


def test_quantize_then_decode_round_trip():
    """Quantizer output -> sti_decode_shards (substitution + outliers written back) equals the
    reference's dequantized weights bit for bit."""
    import torch
    import paper_2207_05022_amd as P
    from oracle import sti_quantizer_oracle as Q
    k = 5
    w = layer_weights(61, MID)
    g = run_gpu(MID, w, k, max_out=512)
    q = check_against_reference(MID, w, k, g)
    M, wsh = MID.n_heads, MID.weights_per_shard
    cnt = g["cnt"].cpu().numpy()
    shards = [P.binding.make_shard(k, g["packed"][s], g["codebook"], g["pos"][s, :int(cnt[s])].contiguous(),
                                   g["val"][s, :int(cnt[s])].contiguous()) for s in range(M)]
    out = torch.empty(M, wsh, device="cuda")
    P.sti_decode_shards(shards, wsh, out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy().view(np.uint32), Q.dequantize(q, k).view(np.uint32))


def test_quantizer_bert_base_layer_and_repeatability():
    dims = S.BERT_BASE
    w = layer_weights(62, dims, sigma=0.04)
    g1 = run_gpu(dims, w, 4, max_out=2048)
    check_against_reference(dims, w, 4, g1)
    g2 = run_gpu(dims, w, 4, max_out=2048)
    import torch
    assert torch.equal(g1["packed"], g2["packed"]) and torch.equal(g1["codebook"], g2["codebook"])
    assert 0.0005 < g1["stats"].n_outliers / w.size < 0.004


def test_quantizer_duplicates_zeros_and_truncated_dictionary():
    """Many exact duplicates (values on a coarse grid, +-0 included) and a dictionary that is
    too small: counts still report the true numbers, the stored prefix is correct."""
    rng = np.random.default_rng(7)
    M, wsh = MID.n_heads, MID.weights_per_shard
    w = (np.round(rng.normal(0.0, 0.03, size=(M, wsh)) * 200.0) / 200.0).astype(np.float32)
    w[0, :5] = -0.0
    w[1, 100:110] = np.float32(0.5)
    g = run_gpu(MID, w, 3, max_out=4)
    from oracle import sti_quantizer_oracle as Q
    q = Q.quantize_layer(w, 3)
    assert np.array_equal(g["codebook"].cpu().numpy().view(np.uint32), q["codebook"].view(np.uint32))
    cnt = g["cnt"].cpu().numpy()
    for s in range(M):
        assert np.array_equal(g["packed"][s].cpu().numpy(), Q.pack_indexes(q["indexes"][s], 3))
        n = len(q["outlier_pos"][s])
        assert cnt[s] == n
        keep = min(n, 4)
        assert np.array_equal(g["pos"][s, :keep].cpu().numpy().view(np.uint32), q["outlier_pos"][s][:keep])
    assert cnt[1] >= 10 > 4


def test_quantizer_random_layers_and_distributions():
    """Twenty-four seeded random layers: 1-12 shards, three widths, every bitwidth; Gaussian,
    heavy-tailed, rounded (many duplicates), uniform, far from zero, and minute weights."""
    rng = np.random.default_rng(31337)
    for case in range(24):
        M = int(rng.choice([1, 2, 3, 4, 8, 12]))
        dims = S.Dims(int(rng.choice([64, 128, 192])), M, 64, int(rng.choice([64, 128, 256])), 1e-12)
        k = int(rng.choice([2, 3, 4, 5, 6]))
        kind = str(rng.choice(["gauss", "tails", "dups", "uniform", "shifted", "tiny"]))
        wsh = dims.weights_per_shard
        if kind == "gauss":
            w = rng.normal(0, 0.03, (M, wsh))
        elif kind == "tails":
            w = layer_weights(case, dims, sigma=float(rng.choice([0.01, 0.05])), tail=float(rng.choice([0.0005, 0.003])))
        elif kind == "dups":
            w = np.round(rng.normal(0, 0.03, (M, wsh)), int(rng.choice([2, 3])))
        elif kind == "uniform":
            w = rng.uniform(-0.1, 0.1, (M, wsh))
        elif kind == "shifted":
            w = rng.normal(0.5, 0.02, (M, wsh))
        else:
            w = rng.normal(0, 1e-6, (M, wsh))
        w = np.asarray(w, dtype=np.float32)
        check_against_reference(dims, w, k, run_gpu(dims, w, k, max_out=4096))


def test_quantizer_reports_a_layer_without_inliers():
    """The outlier rule is an absolute log likelihood (below -4): with a standard deviation above
    e^4 / sqrt(2 pi) = 21.8 even the mean is an outlier.  The call then reports status 1, counts
    every weight as an outlier and fills the dictionaries, in offset order, as far as they have
    room (the reference quantizer refuses such a layer)."""
    w = np.random.default_rng(1).normal(0, 100.0, (4, MID.weights_per_shard)).astype(np.float32)
    g = run_gpu(MID, w, 4, max_out=512)
    assert g["stats"].status == 1 and g["stats"].n_outliers == w.size
    assert np.array_equal(g["cnt"].cpu().numpy(), np.full(4, MID.weights_per_shard))
    assert abs(g["stats"].mean - float(np.mean(w.astype(np.float64)))) <= 1e-12 * 100
    for s in range(4):
        assert np.array_equal(g["pos"][s].cpu().numpy(), np.arange(512))
        assert np.array_equal(g["val"][s].cpu().numpy().view(np.uint32), w[s, :512].view(np.uint32))
