"""TEST INFRASTRUCTURE ONLY - slow reference of the outlier-aware shard quantizer.

Only tests/ may import this module; it shares no code with the library's quantizer.

What it computes (Section "quantization per shard"; Section "Implementation", preprocessing):
all weights of one layer, as one flat array, are fitted with a single Gaussian (mean and
biased variance, plus the 1e-6 that the mixture-model fit the paper uses adds to the
variance); a weight whose log likelihood under the fit is below -4 is an outlier; the other
weights are sorted and cut into 2^k clusters of equal population; the centroid of a cluster
is the arithmetic mean of its members; every weight is replaced by the k-bit index of its
cluster; outliers keep a k-bit placeholder in the stream and their original value and offset
inside the shard are kept in a dictionary.  Decompression substitutes centroids and then
writes the outliers back.

Readings: cluster c starts at sorted rank floor(c*n/2^k) of the n non-outliers and clusters are
separated by VALUE (all copies of a value fall into the same cluster; populations are equal up
to such duplicates); an outlier's placeholder is the index of the cluster whose value range it
falls into (0 or 2^k-1 for the usual far outliers); an empty cluster takes its lower boundary
value as centroid; -0.0 counts as +0.0.  All statistics in float64; centroids are rounded to
float32 once.
"""
from __future__ import annotations

import numpy as np


def fit_gaussian(flat32: np.ndarray, reg_covar: float = 1e-6):
    x = flat32.astype(np.float64)
    mu = x.mean()
    var = ((x - mu) ** 2).mean() + reg_covar
    return float(mu), float(var)


def log_likelihood(flat32: np.ndarray, mu: float, var: float) -> np.ndarray:
    x = flat32.astype(np.float64)
    return -0.5 * np.log(2.0 * np.pi * var) - (x - mu) ** 2 / (2.0 * var)


def quantize_layer(w: np.ndarray, k: int, threshold: float = -4.0, reg_covar: float = 1e-6):
    """w: float32 [M][Wsh].  Returns dict(mu, var, codebook f32[2^k], indexes u8 [M][Wsh],
    outlier_pos list of uint32 arrays, outlier_val list of f32 arrays, thresholds f32[2^k - 1])."""
    assert w.dtype == np.float32 and w.ndim == 2 and 2 <= k <= 6
    flat = w.ravel() + np.float32(0.0)          # -0.0 -> +0.0
    mu, var = fit_gaussian(flat, reg_covar)
    outlier = log_likelihood(flat, mu, var) < threshold
    inl = np.sort(flat[~outlier])
    n, C = inl.size, 1 << k
    assert n > 0
    starts = [(c * n) // C for c in range(C)]
    edges = inl[starts[1:]]                      # lower boundary values of clusters 1..C-1
    idx = np.searchsorted(edges, flat, side="right").astype(np.uint8)
    codebook = np.empty(C, dtype=np.float32)
    x64 = flat.astype(np.float64)
    for c in range(C):
        members = x64[(idx == c) & ~outlier]
        if members.size:
            codebook[c] = np.float32(members.mean())
        else:
            codebook[c] = edges[c - 1] if c > 0 else inl[0]
    idx2 = idx.reshape(w.shape)
    out_mask = outlier.reshape(w.shape)
    pos = [np.flatnonzero(out_mask[s]).astype(np.uint32) for s in range(w.shape[0])]
    val = [w[s][p].astype(np.float32) for s, p in enumerate(pos)]
    return dict(mu=mu, var=var, codebook=codebook, indexes=idx2, outlier_pos=pos, outlier_val=val,
                thresholds=edges.astype(np.float32), n_inliers=n)


def pack_indexes(idx: np.ndarray, k: int) -> np.ndarray:
    """Index j in bits [j*k, j*k+k) of a gap-free little-endian bitstream (stream format of the
    library's header)."""
    bits = ((idx.astype(np.uint32)[:, None] >> np.arange(k, dtype=np.uint32)) & 1).astype(np.uint8).ravel()
    pad = (-bits.size) % 8
    if pad:
        bits = np.concatenate([bits, np.zeros(pad, dtype=np.uint8)])
    return np.packbits(bits, bitorder="little")


def dequantize(q, k: int) -> np.ndarray:
    """float32 [M][Wsh]: centroids substituted, outliers written back."""
    out = q["codebook"][q["indexes"]]
    for s, (p, v) in enumerate(zip(q["outlier_pos"], q["outlier_val"])):
        out[s, p] = v
    return out
