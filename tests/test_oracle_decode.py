"""Pins for the oracle's decode (index unpacking, centroid substitution, rounding).

Every check here compares the oracle with something that is not the oracle:
hand-written byte patterns, Python big-integer extraction, numpy's bit
unpacking, numpy/torch rounding, set membership and size arithmetic from the
paper (Table 1, the 32/k size reduction, the storage totals of its evaluation).
"""
import os

import numpy as np
import pytest

import sti_synth as S

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def read_stream_fixture(name):
    k = data = idx = None
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            key, *vals = line.split()
            if key == "k":
                k = int(vals[0])
            elif key == "bytes":
                data = np.array([int(v, 16) for v in vals], dtype=np.uint8)
            elif key == "indexes":
                idx = [int(v) for v in vals]
    return k, data, idx


def bigint_indexes(stream: np.ndarray, k: int, n: int):
    """Independent extraction: the stream is one little-endian integer."""
    big = int.from_bytes(stream.tobytes(), "little")
    mask = (1 << k) - 1
    return [(big >> (j * k)) & mask for j in range(n)]


def pack_indexes(idx, k: int) -> np.ndarray:
    """Independent packer used for round trips (least significant bit first)."""
    big = 0
    for j, v in enumerate(idx):
        big |= int(v) << (j * k)
    nbytes = (len(idx) * k + 7) // 8
    return np.frombuffer(big.to_bytes(nbytes, "little"), dtype=np.uint8).copy()


@pytest.mark.parametrize("name", ["unpack_k3.txt", "unpack_k5.txt"])
def test_hand_written_streams(oracle_mod, name):
    k, data, idx = read_stream_fixture(name)
    got = [oracle_mod.unpack_index(data, k, j) for j in range(len(idx))]
    assert got == idx
    # substitution: codebook entry i is the value 100+i
    cb = (100 + np.arange(1 << k)).astype(np.float32)
    out = oracle_mod.decode_shards([S.Shard(k, data, cb)], len(idx))
    assert out[0].tolist() == [100.0 + i for i in idx]


def test_nibble_order_low_first(oracle_mod):
    # "packed uint4": byte 0xA3 holds index 3 first, then index 10
    data = np.array([0xA3, 0x0F], dtype=np.uint8)
    assert [oracle_mod.unpack_index(data, 4, j) for j in range(4)] == [3, 10, 15, 0]
    # 2-bit: 0b11_10_01_00 -> 0,1,2,3
    data = np.array([0b11100100], dtype=np.uint8)
    assert [oracle_mod.unpack_index(data, 2, j) for j in range(4)] == [0, 1, 2, 3]
    # 6-bit: indexes 63,0,63,0 -> bits 0-5 set, 12-17 set -> 0x3F, 0xF0, 0x03
    data = np.array([0x3F, 0xF0, 0x03], dtype=np.uint8)
    assert [oracle_mod.unpack_index(data, 6, j) for j in range(4)] == [63, 0, 63, 0]


@pytest.mark.parametrize("k", [2, 3, 4, 5, 6])
@pytest.mark.parametrize("n", [1, 7, 8, 33, 257, 4099])
def test_bigint_bruteforce(oracle_mod, k, n):
    rng = np.random.default_rng(1000 * k + n)
    sh = S.make_shard(rng, n, k)
    want = bigint_indexes(sh.data, k, n)
    got = [oracle_mod.unpack_index(sh.data, k, j) for j in range(n)]
    assert got == want
    out = oracle_mod.decode_shards([sh], n)[0]
    assert np.array_equal(out.view(np.uint32), sh.codebook[np.array(want)].view(np.uint32))


@pytest.mark.parametrize("k", [2, 3, 4, 5, 6])
def test_numpy_unpackbits_and_roundtrip(oracle_mod, k):
    n = 8 * 4096 + 8 * 3
    rng = np.random.default_rng(k)
    sh = S.make_shard(rng, n, k)
    bits = np.unpackbits(sh.data, bitorder="little")[: n * k].reshape(n, k)
    want = (bits.astype(np.uint32) << np.arange(k, dtype=np.uint32)).sum(axis=1)
    out = oracle_mod.decode_shards([sh], n)[0]
    # exact-codebook: every decoded value is bitwise one of the centroids
    cb_bits = set(sh.codebook.view(np.uint32).tolist())
    assert set(out.view(np.uint32).tolist()) <= cb_bits
    # strictly increasing distinct centroids -> recover the indexes from the values
    rec = np.searchsorted(sh.codebook, out)
    assert np.array_equal(rec, want)
    assert np.array_equal(np.bincount(rec, minlength=1 << k), np.bincount(want, minlength=1 << k))
    assert np.array_equal(pack_indexes(rec, k), sh.data)


def test_multi_shard_layout_and_passthrough(oracle_mod):
    n = 1000
    rng = np.random.default_rng(5)
    shards = [S.make_shard(rng, n, k) for k in (6, 32, 2, 32, 3)]
    out = oracle_mod.decode_shards(shards, n)
    assert out.shape == (5, n)
    for s, sh in enumerate(shards):
        if sh.bitwidth == 32:
            assert np.array_equal(out[s].view(np.uint32), sh.data.view(np.uint32))
        else:
            want = sh.codebook[np.array(bigint_indexes(sh.data, sh.bitwidth, n))]
            assert np.array_equal(out[s].view(np.uint32), want.view(np.uint32))


def _edge_values():
    vals = [0.0, -0.0, 1.0, -1.0, 65504.0, 65519.99, 65520.0, 65536.0, 1e10, -1e10,
            np.inf, -np.inf, 2.0 ** -14, 2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.0000001,
            2.0 ** -26, 3 * 2.0 ** -25, 2.0 ** -24 * 1.5, 1e-30, 1e-45, 0.1, 1 / 3,
            1.0 + 2.0 ** -11, 1.0 + 2.0 ** -11 + 2.0 ** -23, 1.0 + 3 * 2.0 ** -11,
            2047.5, 2048.5, 2049.5, 6.1e-5, 6.0e-5, 5.96e-8, 2.98e-8]
    return np.array(vals, dtype=np.float32)


def test_f16_rounding_matches_numpy(oracle_mod):
    rng = np.random.default_rng(11)
    bits = rng.integers(0, 2 ** 32, size=200000, dtype=np.uint64).astype(np.uint32)
    vals = np.concatenate([_edge_values(), bits.view(np.float32),
                           rng.normal(0, 0.02, 50000).astype(np.float32),
                           (rng.normal(0, 1, 20000) * 1e-6).astype(np.float32)])
    vals = vals[~np.isnan(vals)]
    got = oracle_mod.decode_shards([S.Shard(32, vals, None)], vals.size, oracle_mod.F16)[0]
    with np.errstate(over="ignore"):
        want = vals.astype(np.float16).view(np.uint16)
    assert np.array_equal(got, want)


def test_bf16_rounding_matches_torch(oracle_mod):
    import torch
    rng = np.random.default_rng(12)
    bits = rng.integers(0, 2 ** 32, size=200000, dtype=np.uint64).astype(np.uint32)
    vals = np.concatenate([_edge_values(), bits.view(np.float32)])
    vals = vals[~np.isnan(vals)]
    got = oracle_mod.decode_shards([S.Shard(32, vals, None)], vals.size, oracle_mod.BF16)[0]
    want = torch.from_numpy(vals).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, want)


def test_nan_rounding_is_quiet_with_sign(oracle_mod):
    for pattern, f16, bf16 in [(0x7FC00000, 0x7E00, 0x7FC0), (0xFFC00000, 0xFE00, 0xFFC0),
                               (0x7F800001, 0x7E00, 0x7FC0), (0x7FA00000, 0x7F00, 0x7FE0)]:
        v = np.array([pattern], dtype=np.uint32).view(np.float32)
        a = oracle_mod.decode_shards([S.Shard(32, v, None)], 1, oracle_mod.F16)[0, 0]
        b = oracle_mod.decode_shards([S.Shard(32, v, None)], 1, oracle_mod.BF16)[0, 0]
        assert (int(a), int(b)) == (f16, bf16)


def test_f16_decode_is_rounded_centroid(oracle_mod):
    n = 4096
    sh = S.make_shard(np.random.default_rng(3), n, 5)
    idx = np.array(bigint_indexes(sh.data, 5, n))
    got = oracle_mod.decode_shards([sh], n, oracle_mod.F16)[0]
    assert np.array_equal(got, sh.codebook.astype(np.float16).view(np.uint16)[idx])


def test_size_arithmetic_from_the_paper():
    base, large = S.BERT_BASE, S.BERT_LARGE_SHAPED
    # Table 1: Q,K,V,O slices d x d/M each, FFN1 d_ff/M x d, FFN2 d x d_ff/M
    assert base.weights_per_shard == 4 * 768 * 64 + 2 * 256 * 768 == 589824
    assert base.weights_per_shard * base.n_heads == 4 * 768 * 768 + 2 * 768 * 3072
    assert large.weights_per_shard == 786432
    # k-bit indexes shrink the matrix 32/k times
    for k in (2, 3, 4, 5, 6):
        assert base.packed_bytes(k) * 32 == base.packed_bytes(32) * k
        assert base.packed_bytes(k) == 73728 * k
    # storage of the 12x12 model's {2..6}-bit versions: indexes alone are 212.3 MB,
    # within a few percent below the 215 MB the paper reports with dictionaries and outliers
    idx_bytes = 144 * sum(base.packed_bytes(k) for k in (2, 3, 4, 5, 6))
    assert idx_bytes == 212336640
    assert 0.94 * 215e6 < idx_bytes < 215e6
    # 12 full-precision encoder layers are 339.7 MB of the 418 MB model (rest: embeddings)
    assert 12 * 12 * base.packed_bytes(32) == 339738624 < 418e6
    # decode-only configuration
    counts = S.decode_stream_counts(1 << 30, base.weights_per_shard)
    assert counts == {2: 1456, 3: 970, 4: 728, 5: 582, 6: 485}
    assert sum(c * base.packed_bytes(k) for k, c in counts.items()) == 1073037312
    assert sum(counts.values()) * base.weights_per_shard == 2489647104


def test_codebook_recipe():
    for k in (2, 3, 4, 5, 6):
        cb = S.make_codebook(k, 0.016)
        assert cb.dtype == np.float32 and cb.size == 1 << k
        assert np.all(np.diff(cb) > 0)
        assert np.allclose(cb, -cb[::-1], rtol=1e-6)
        # every centroid is a normal binary16 number after rounding
        assert np.all(np.abs(cb.astype(np.float16).astype(np.float32)) >= 6.1e-5)


# ---------------------------------------------------------------- outlier dictionary

@pytest.mark.parametrize("k", [2, 4, 5])
def test_outliers_replace_exactly_their_offsets(oracle_mod, k):
    n = 6000
    rng = np.random.default_rng(40 + k)
    sh = S.add_outliers(rng, S.make_shard(rng, n, k), n, fraction=0.01)
    assert sh.outlier_pos.size == 60 and np.all(np.diff(sh.outlier_pos.astype(np.int64)) > 0)
    plain = S.Shard(k, sh.data, sh.codebook)
    base = oracle_mod.decode_shards([plain], n)[0]
    got = oracle_mod.decode_shards([sh], n)[0]
    mask = np.zeros(n, bool); mask[sh.outlier_pos] = True
    assert np.array_equal(got[~mask].view(np.uint32), base[~mask].view(np.uint32))
    assert np.array_equal(got[mask].view(np.uint32), sh.outlier_val.view(np.uint32))
    # the substituted part is still pure codebook lookup of the big-integer indexes
    want = sh.codebook[np.array(bigint_indexes(sh.data, k, n))]
    want[sh.outlier_pos] = sh.outlier_val
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    # outliers are outside the centroid range, as in the paper's Gaussian outlier test
    assert np.all(np.abs(sh.outlier_val) > np.max(np.abs(sh.codebook)))
    # rounding applies to outliers too
    h = oracle_mod.decode_shards([sh], n, oracle_mod.F16)[0]
    assert np.array_equal(h[mask], sh.outlier_val.astype(np.float16).view(np.uint16))


def test_outlier_edge_positions_and_errors(oracle_mod):
    n = 100
    sh = S.make_shard(np.random.default_rng(1), n, 3)
    sh.outlier_pos = np.array([0, n - 1], np.uint32); sh.outlier_val = np.array([7.0, -9.0], np.float32)
    got = oracle_mod.decode_shards([sh], n)[0]
    assert got[0] == 7.0 and got[-1] == -9.0
    sh.outlier_pos = np.array([n], np.uint32); sh.outlier_val = np.array([1.0], np.float32)
    with pytest.raises(RuntimeError):
        oracle_mod.decode_shards([sh], n)
