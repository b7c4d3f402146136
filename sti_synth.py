"""Seeded synthetic inputs for the shard-decode + encoder-layer path.

This module only *draws data*: packed index streams, codebooks, resident
parameters, activations and plans.  It contains none of the method's
arithmetic (no unpacking, no lookup, no layer math) and imports neither the
HIP binding nor the CPU oracle, so both sides can be fed from it.

Shapes follow the paper's Table 1 (one shard = one attention head's Q, K, V,
O slices plus a 1/M slice of both FFN matrices) and its set of fidelity
versions K = {2..6, 32} (Section "storing shards per version").  Values follow
the structure its quantizer produces (Section "Implementation"): weights are
Gaussian and clusters are equal-population, so the index histogram of a k-bit
shard is uniform and the centroids sit at Gaussian quantiles.

Recipe
------
* ``numpy.random.Generator(PCG64(...))`` everywhere; base seed 220705022,
  per-configuration seed ``base + 1000 * config``.
* From the configuration's ``SeedSequence`` two children are spawned: one for
  the plan/activations/resident parameters, one that is spawned again into one
  child per (layer, shard) in row-major order.
* A k-bit shard draws, in this order: ``u ~ U[0,1)`` (codebook scale
  ``sigma = 0.02 * (0.8 + 0.4 u)``), then ``Wsh * k / 8`` uniform bytes.  The
  bytes *are* the bitstream, so every k-bit code is uniform.
* Codebook entry j of a k-bit shard is ``sigma * Phi^-1((j + 1/2) / 2^k)``
  evaluated in float64 and rounded once to float32.
* A 32-bit shard draws ``Wsh`` values from N(0, 0.02^2), rounded to float32.
* Biases and LayerNorm shifts are N(0, 0.02^2) float32; LayerNorm gains are 1.
* Activations are N(0, 1), float32 (or rounded to float16 where stated).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from statistics import NormalDist
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

BASE_SEED = 220705022
BITWIDTHS = (2, 3, 4, 5, 6, 32)
PACKED_BITWIDTHS = (2, 3, 4, 5, 6)
SIGMA = 0.02


@dataclass(frozen=True)
class Dims:
    """Geometry of one encoder layer cut into ``n_heads`` shards (Table 1)."""

    d_model: int
    n_heads: int
    d_head: int
    ffn_per_shard: int
    ln_eps: float = 1e-12

    @property
    def weights_per_shard(self) -> int:
        return self.d_model * (4 * self.d_head + 2 * self.ffn_per_shard)

    def packed_bytes(self, k: int) -> int:
        if k == 32:
            return 4 * self.weights_per_shard
        return (self.weights_per_shard * k + 7) // 8

    # element offsets of the six row-major sub-blocks inside a shard
    def offsets(self) -> Dict[str, int]:
        d, dh, f = self.d_model, self.d_head, self.ffn_per_shard
        return {
            "q": 0,
            "k": dh * d,
            "v": 2 * dh * d,
            "o": 3 * dh * d,
            "ffn1": 4 * dh * d,
            "ffn2": 4 * dh * d + f * d,
        }


BERT_BASE = Dims(768, 12, 64, 256)
BERT_LARGE_SHAPED = Dims(1024, 16, 64, 256)


@dataclass
class Shard:
    """One fidelity version of one shard, in host memory."""

    bitwidth: int                      # 2..6 packed indices, 32 raw float32
    data: np.ndarray                   # uint8 stream (k-bit) or float32 (32-bit)
    codebook: Optional[np.ndarray]     # float32[2**k], None for 32-bit
    outlier_pos: Optional[np.ndarray] = None   # uint32, distinct increasing offsets in the shard
    outlier_val: Optional[np.ndarray] = None   # float32 original weights at those offsets


@dataclass
class LayerParams:
    """Resident full-fidelity parameters of one layer (all float32)."""

    bq: np.ndarray
    bk: np.ndarray
    bv: np.ndarray
    bo: np.ndarray
    b1: np.ndarray
    b2: np.ndarray
    ln1_g: np.ndarray
    ln1_b: np.ndarray
    ln2_g: np.ndarray
    ln2_b: np.ndarray

    NAMES = ("bq", "bk", "bv", "bo", "b1", "b2", "ln1_g", "ln1_b", "ln2_g", "ln2_b")


@dataclass
class Workload:
    """A model (or single layer) plus its plan and one batch of activations."""

    name: str
    dims: Dims
    batch: int
    seq: int
    plan: np.ndarray                       # int8 [n_layers][M]: 0 absent | 2..6 | 32
    shards: List[List[Optional[Shard]]]    # [n_layers][M]; None where the plan says absent
    params: List[LayerParams]
    x: np.ndarray                          # [batch, seq, d] float32 or float16
    io_dtype: str = "f32"
    extra: dict = field(default_factory=dict)

    @property
    def n_layers(self) -> int:
        return len(self.shards)

    @property
    def tokens(self) -> int:
        return self.batch * self.seq


_QUANTILES: Dict[int, np.ndarray] = {}


def unit_quantiles(k: int) -> np.ndarray:
    """Phi^-1((j + 1/2) / 2^k) for j = 0 .. 2^k - 1, float64."""
    if k not in _QUANTILES:
        n = 1 << k
        nd = NormalDist()
        _QUANTILES[k] = np.array([nd.inv_cdf((j + 0.5) / n) for j in range(n)], dtype=np.float64)
    return _QUANTILES[k]


def make_codebook(k: int, sigma: float) -> np.ndarray:
    return (unit_quantiles(k) * np.float64(sigma)).astype(np.float32)


def make_shard(rng: np.random.Generator, n_weights: int, k: int) -> Shard:
    if k == 32:
        w = rng.normal(0.0, SIGMA, size=n_weights).astype(np.float32)
        return Shard(32, w, None)
    if k not in PACKED_BITWIDTHS:
        raise ValueError(f"bitwidth {k}")
    u = rng.random()
    sigma = SIGMA * (0.8 + 0.4 * u)
    nbytes = (n_weights * k + 7) // 8
    stream = rng.integers(0, 256, size=nbytes, dtype=np.uint8)
    tail_bits = nbytes * 8 - n_weights * k
    if tail_bits:
        # bits past the last index carry no information; keep them zero
        stream[-1] &= np.uint8(0xFF >> tail_bits)
    return Shard(k, stream, make_codebook(k, sigma))


def add_outliers(rng: np.random.Generator, shard: Shard, n_weights: int, fraction: float = 0.0015) -> Shard:
    """Give a k-bit shard an outlier dictionary: ``fraction`` of its weights (the paper reports
    0.14-0.17 %) at distinct uniform offsets, with magnitudes beyond the codebook's range
    (3 to 6 times 0.02, random sign).  The k-bit placeholders in the stream stay as drawn."""
    if shard.bitwidth == 32:
        return shard
    count = max(1, int(round(n_weights * fraction)))
    pos = np.sort(rng.choice(n_weights, size=count, replace=False)).astype(np.uint32)
    mag = rng.uniform(3 * SIGMA, 6 * SIGMA, size=count)
    sign = rng.choice(np.array([-1.0, 1.0]), size=count)
    shard.outlier_pos = pos
    shard.outlier_val = (mag * sign).astype(np.float32)
    return shard


def make_layer_params(rng: np.random.Generator, dims: Dims) -> LayerParams:
    d, M, dh, f = dims.d_model, dims.n_heads, dims.d_head, dims.ffn_per_shard

    def nrm(n):
        return rng.normal(0.0, SIGMA, size=n).astype(np.float32)

    bq, bk, bv = nrm(M * dh), nrm(M * dh), nrm(M * dh)
    bo, b1, b2 = nrm(d), nrm(M * f), nrm(d)
    ln1_b, ln2_b = nrm(d), nrm(d)
    ones = np.ones(d, dtype=np.float32)
    return LayerParams(bq, bk, bv, bo, b1, b2, ones.copy(), ln1_b, ones.copy(), ln2_b)


def _seed_children(root: np.random.SeedSequence, n_layers: int, M: int):
    misc_ss, shard_root = root.spawn(2)
    shard_ss = shard_root.spawn(n_layers * M)
    return np.random.default_rng(np.random.PCG64(misc_ss)), shard_ss


def config_root(config: int) -> np.random.SeedSequence:
    return np.random.SeedSequence(BASE_SEED + 1000 * config)


def build_workload(
    name: str,
    root: np.random.SeedSequence,
    dims: Dims,
    n_layers: int,
    batch: int,
    seq: int,
    bit_choices: Sequence[int],
    n_absent: int,
    io_dtype: str = "f32",
    fixed_bitwidth: Optional[int] = None,
    plan: Optional[np.ndarray] = None,
) -> Workload:
    """Draw a model of ``n_layers`` layers with a random mixed-bitwidth plan.

    Per layer the plan first draws M bitwidths uniformly from ``bit_choices``
    (or uses ``fixed_bitwidth``), then marks ``n_absent`` distinct shard ids
    absent (uniform without replacement).  A caller-supplied ``plan`` replaces
    the drawn one (nothing is drawn for it).
    """
    M = dims.n_heads
    rng, shard_ss = _seed_children(root, n_layers, M)
    if plan is not None:
        plan = np.asarray(plan, dtype=np.int8).reshape(n_layers, M).copy()
    else:
        plan = np.zeros((n_layers, M), dtype=np.int8)
        for l in range(n_layers):
            if fixed_bitwidth is not None:
                row = np.full(M, fixed_bitwidth, dtype=np.int8)
            else:
                row = rng.choice(np.asarray(bit_choices, dtype=np.int8), size=M)
            if n_absent:
                gone = rng.choice(M, size=n_absent, replace=False)
                row[gone] = 0
            plan[l] = row
    params = [make_layer_params(rng, dims) for _ in range(n_layers)]
    x = rng.normal(0.0, 1.0, size=(batch, seq, dims.d_model)).astype(np.float32)
    if io_dtype == "f16":
        x = x.astype(np.float16)
    shards: List[List[Optional[Shard]]] = []
    for l in range(n_layers):
        row_shards: List[Optional[Shard]] = []
        for i in range(M):
            k = int(plan[l, i])
            if k == 0:
                row_shards.append(None)
                continue
            srng = np.random.default_rng(np.random.PCG64(shard_ss[l * M + i]))
            row_shards.append(make_shard(srng, dims.weights_per_shard, k))
        shards.append(row_shards)
    return Workload(name, dims, batch, seq, plan, shards, params, x, io_dtype)


# ---------------------------------------------------------------------------
# The five evaluation configurations
# ---------------------------------------------------------------------------

def config0() -> Workload:
    """One BERT-base layer, all 12 shards at 4 bits, batch 1, seq 128."""
    return build_workload("config0_bert_base_layer_4bit", config_root(0), BERT_BASE, 1, 1, 128,
                          (4,), 0, fixed_bitwidth=4)


def config2(n_layers: int = 12) -> Workload:
    """BERT-base, k ~ U{2,3,4,5,6,32}, 3 of 12 shards absent per layer."""
    return build_workload("config2_bert_base_mixed", config_root(2), BERT_BASE, n_layers, 1, 128,
                          (2, 3, 4, 5, 6, 32), 3)


def config3(n_layers: int = 24) -> Workload:
    """BERT-large-shaped, k ~ U{2..6}, 4 of 16 shards absent per layer, seq 256."""
    return build_workload("config3_bert_large_shaped", config_root(3), BERT_LARGE_SHAPED, n_layers, 1, 256,
                          (2, 3, 4, 5, 6), 4)


def config4(n_layers: int = 12, batch: int = 32) -> Workload:
    """Batched BERT-base, k ~ U{2,3,4,6,32}, full shard set, fp16 activations."""
    return build_workload("config4_bert_base_batched", config_root(4), BERT_BASE, n_layers, batch, 128,
                          (2, 3, 4, 6, 32), 0, io_dtype="f16")


@dataclass
class DecodeStream:
    """Decode-only workload: shards grouped by bitwidth, stored back to back."""

    name: str
    weights_per_shard: int
    bitwidths: np.ndarray          # int8 [n_shards]
    offsets: np.ndarray            # int64 [n_shards] byte offset of each stream in ``packed``
    packed: np.ndarray             # uint8, all streams back to back
    codebooks: List[np.ndarray]    # float32[2**k] per shard

    @property
    def n_shards(self) -> int:
        return len(self.bitwidths)

    def shard(self, s: int) -> Shard:
        k = int(self.bitwidths[s])
        nb = (self.weights_per_shard * k + 7) // 8
        o = int(self.offsets[s])
        return Shard(k, self.packed[o:o + nb], self.codebooks[s])


def decode_stream_counts(total_bytes: int, weights_per_shard: int) -> Dict[int, int]:
    """Whole shards per bitwidth when ``total_bytes`` is split evenly over k = 2..6."""
    share = total_bytes / len(PACKED_BITWIDTHS)
    return {k: int(share // (weights_per_shard * k // 8)) for k in PACKED_BITWIDTHS}


def config1(total_bytes: int = 1 << 30, dims: Dims = BERT_BASE) -> DecodeStream:
    """Decode-only stream: ``total_bytes`` of packed indices split evenly over k = 2..6.

    At the default size this is 1456/970/728/582/485 shards for k = 2..6
    (4221 shards, 1,073,037,312 packed bytes, 2,489,647,104 weights).
    """
    wsh = dims.weights_per_shard
    counts = decode_stream_counts(total_bytes, wsh)
    n = sum(counts.values())
    root = np.random.SeedSequence(BASE_SEED + 1000 * 1)
    misc_ss, bytes_ss = root.spawn(2)
    rng = np.random.default_rng(np.random.PCG64(misc_ss))
    bitwidths = np.concatenate([np.full(counts[k], k, dtype=np.int8) for k in PACKED_BITWIDTHS])
    sizes = np.array([wsh * int(k) // 8 for k in bitwidths], dtype=np.int64)
    offsets = np.concatenate([[0], np.cumsum(sizes)[:-1]]).astype(np.int64)
    total = int(sizes.sum())
    # one bulk draw for the whole stream (uniform bytes = uniform codes for every k)
    brng = np.random.default_rng(np.random.PCG64(bytes_ss))
    packed = brng.integers(0, 256, size=total, dtype=np.uint8)
    us = rng.random(n)
    codebooks = [make_codebook(int(bitwidths[s]), SIGMA * (0.8 + 0.4 * us[s])) for s in range(n)]
    return DecodeStream(f"config1_decode_stream_{total}B", wsh, bitwidths, offsets, packed, codebooks)


def small_workload(seed: int, dims: Dims, n_layers: int, batch: int, seq: int,
                   plan: Optional[np.ndarray] = None,
                   bit_choices: Sequence[int] = (2, 3, 4, 5, 6, 32),
                   n_absent: int = 0, io_dtype: str = "f32") -> Workload:
    """Free-form small case for tests, on a seed tree of its own."""
    root = np.random.SeedSequence([BASE_SEED, 7, seed])
    return build_workload(f"small_{seed}", root, dims, n_layers, batch, seq, bit_choices,
                          n_absent, io_dtype=io_dtype, plan=plan)


def make_every_term_matter(wl: Workload, seed: int, amp: float = 6.0) -> None:
    """Rescale a workload in place so that every term of the layer moves its output.

    With the configurations' recipe (weights N(0, 0.02), biases N(0, 0.02), LayerNorm gains
    of exactly 1) the attention block changes the layer output by a few per cent only, and a
    gain of 1 hides a dropped gain altogether.  Here all weights (codebooks and float32
    shards) are multiplied by `amp`, gains become N(1, 0.3), shifts N(0, 0.3) and the six bias
    vectors N(0, 0.2).  Input data only: what a layer computes from it is not this module's
    business."""
    rng = np.random.default_rng([BASE_SEED, 11, seed])
    for layer in wl.shards:
        for sh in layer:
            if sh is None or sh.bitwidth == 0:
                continue
            if sh.bitwidth == 32:
                sh.data *= np.float32(amp)
            else:
                sh.codebook *= np.float32(amp)
            if sh.outlier_val is not None:
                sh.outlier_val *= np.float32(amp)
    d = wl.dims.d_model
    for prm in wl.params:
        for name in ("ln1_g", "ln2_g"):
            getattr(prm, name)[:] = rng.normal(1.0, 0.3, d).astype(np.float32)
        for name in ("ln1_b", "ln2_b"):
            getattr(prm, name)[:] = rng.normal(0.0, 0.3, d).astype(np.float32)
        for name in ("bq", "bk", "bv", "bo", "b1", "b2"):
            v = getattr(prm, name)
            v[:] = rng.normal(0.0, 0.2, v.shape).astype(np.float32)
