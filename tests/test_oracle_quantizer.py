"""Pins of the reference quantizer (Section "quantization per shard"; Section "Implementation").
CPU only."""
import numpy as np
import pytest

from oracle import sti_quantizer_oracle as Q


def heavy_tailed(seed, M=3, wsh=4096, sigma=0.03):
    rng = np.random.default_rng(seed)
    w = rng.normal(0.0, sigma, size=(M, wsh))
    tail = rng.random((M, wsh)) < 0.002                       # a few weights far outside the Gaussian
    w[tail] = rng.choice([-1.0, 1.0], size=int(tail.sum())) * rng.uniform(5 * sigma, 9 * sigma, size=int(tail.sum()))
    return w.astype(np.float32)


def test_fit_and_likelihood_match_the_mixture_model_fit():
    """The paper fits a one-component Gaussian mixture; that library routine is the pin."""
    from sklearn.mixture import GaussianMixture
    w = heavy_tailed(1)
    flat = w.ravel().astype(np.float64).reshape(-1, 1)
    gm = GaussianMixture(1).fit(flat)
    mu, var = Q.fit_gaussian(w.ravel())
    assert abs(mu - gm.means_.ravel()[0]) < 1e-12 and abs(var - gm.covariances_.ravel()[0]) < 1e-12
    assert np.max(np.abs(Q.log_likelihood(w.ravel(), mu, var) - gm.score_samples(flat))) < 1e-9
    q = Q.quantize_layer(w, 4)
    n_out = sum(len(p) for p in q["outlier_pos"])
    assert n_out == int((gm.score_samples(flat) < -4).sum())
    assert 0.001 < n_out / w.size < 0.004                       # the planted tail, same order as the paper's 0.14-0.17 %


def test_outlier_rule_closed_form():
    """log N(x) < -4  <=>  (x - mu)^2 > 2 var (4 - log sqrt(2 pi var))."""
    w = heavy_tailed(2)
    mu, var = Q.fit_gaussian(w.ravel())
    r = 2.0 * var * (4.0 - 0.5 * np.log(2.0 * np.pi * var))
    q = Q.quantize_layer(w, 3)
    mask = np.zeros(w.shape, dtype=bool)
    for s, p in enumerate(q["outlier_pos"]):
        mask[s, p] = True
    assert np.array_equal(mask, (w.astype(np.float64) - mu) ** 2 > r)
    for s, (p, v) in enumerate(zip(q["outlier_pos"], q["outlier_val"])):
        assert np.array_equal(v, w[s, p]) and np.all(np.diff(p.astype(np.int64)) > 0)


@pytest.mark.parametrize("k", [2, 3, 4, 5, 6])
def test_equal_population_clusters_and_mean_centroids(k):
    w = heavy_tailed(10 + k, M=4, wsh=8192)
    q = Q.quantize_layer(w, k)
    C = 1 << k
    mask = np.ones(w.shape, dtype=bool)
    for s, p in enumerate(q["outlier_pos"]):
        mask[s, p] = False
    idx, vals = q["indexes"][mask], w[mask].astype(np.float64)
    counts = np.bincount(idx, minlength=C)
    assert counts.sum() == q["n_inliers"] and counts.max() - counts.min() <= 1      # distinct values: exact split
    order = np.argsort(vals, kind="stable")
    assert np.all(np.diff(idx[order].astype(int)) >= 0)           # clusters are contiguous in sorted order
    for c in range(C):
        assert q["codebook"][c] == np.float32(vals[idx == c].mean())
    assert np.all(np.diff(q["codebook"]) > 0)
    # a k-bit code stores nothing outside 0 .. 2^k - 1; the index histogram is flat (what the
    # synthetic shard generator assumes)
    assert q["indexes"].max() < C


def test_reconstruction_error_shrinks_with_bitwidth_and_outliers_are_exact():
    w = heavy_tailed(3, M=2, wsh=16384)
    errs = []
    for k in (2, 3, 4, 5, 6):
        q = Q.quantize_layer(w, k)
        r = Q.dequantize(q, k)
        for s, p in enumerate(q["outlier_pos"]):
            assert np.array_equal(r[s, p], w[s, p])
        errs.append(float(np.sqrt(np.mean((r.astype(np.float64) - w) ** 2))))
        # a centroid is the mean of its cluster: the reconstruction preserves the sum of the non-outliers
        mask = np.ones(w.shape, dtype=bool)
        for s, p in enumerate(q["outlier_pos"]):
            mask[s, p] = False
        assert abs(r[mask].astype(np.float64).sum() - w[mask].astype(np.float64).sum()) < 1e-3
    assert all(a > 1.4 * b for a, b in zip(errs, errs[1:]))      # equal-population clusters: x1.5-1.6 per extra bit


def test_duplicates_stay_in_one_cluster_and_negative_zero():
    w = np.array([[0.0, -0.0, 0.01, 0.01, 0.01, 0.01, -0.02, 0.03]], dtype=np.float32)
    q = Q.quantize_layer(w, 2, threshold=-1e9)
    idx = q["indexes"][0]
    assert idx[0] == idx[1] and len({idx[2], idx[3], idx[4], idx[5]}) == 1
    assert idx[6] == 0 and idx[7] == 3 and sum(len(p) for p in q["outlier_pos"]) == 0


def test_packing_matches_the_stream_format_and_the_decoder(oracle_mod):
    """pack -> the reference decoder of the shard format gives back the dequantized weights."""
    import sti_synth as S
    w = heavy_tailed(4, M=2, wsh=2048)
    for k in (2, 3, 5, 6):
        q = Q.quantize_layer(w, k)
        want = Q.dequantize(q, k)
        for s in range(2):
            stream = Q.pack_indexes(q["indexes"][s], k)
            assert stream.size == 2048 * k // 8
            for j in (0, 1, 7, 8, 1000, 2047):
                assert oracle_mod.unpack_index(stream, k, j) == q["indexes"][s][j]
            sh = S.Shard(k, stream, q["codebook"], q["outlier_pos"][s], q["outlier_val"][s])
            got = oracle_mod.decode_shards([sh], 2048, oracle_mod.F32)
            assert np.array_equal(np.asarray(got).ravel().view(np.uint32), want[s].view(np.uint32))
