"""GPU parity: sti_decode_shards (through the C ABI) against the CPU oracle, bit for bit."""
import numpy as np
import pytest

import sti_synth as S

pytestmark = pytest.mark.gpu

DT = {"f32": ("float32", 0), "f16": ("float16", 1), "bf16": ("bfloat16", 2)}


@pytest.fixture(scope="module")
def gpu():
    import torch
    import paper_2207_05022_amd as P
    from paper_2207_05022_amd import device as D
    assert torch.cuda.is_available(), "needs a GPU"
    return torch, P, D


def run_decode(gpu, shards, n, dtype):
    torch, P, D = gpu
    dev = [D.upload_shard(s) for s in shards]
    out = torch.full((len(shards) * n,), 7, dtype=getattr(torch, DT[dtype][0]), device="cuda")
    ws_bytes = P.sti_decode_workspace_bytes(len(shards))
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")
    P.sti_decode_shards(dev, n, out, ws)
    torch.cuda.synchronize()
    if dtype == "f32":
        return out.view(torch.int32).cpu().numpy().view(np.uint32).reshape(len(shards), n)
    return out.view(torch.int16).cpu().numpy().view(np.uint16).reshape(len(shards), n)


def oracle_bits(oracle_mod, shards, n, dtype):
    out = oracle_mod.decode_shards(shards, n, DT[dtype][1])
    return out.view(np.uint32) if dtype == "f32" else out


@pytest.mark.parametrize("dtype", ["f16", "f32", "bf16"])
@pytest.mark.parametrize("n", [589824, 16384 * 3 + 8 * 5, 8 * 2048 + 24])
def test_each_bitwidth_whole_units(gpu, oracle_mod, dtype, n):
    rng = np.random.default_rng(n % 1000 + len(dtype))
    shards = [S.make_shard(rng, n, k) for k in (2, 3, 4, 5, 6, 32)]
    got = run_decode(gpu, shards, n, dtype)
    want = oracle_bits(oracle_mod, shards, n, dtype)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("dtype", ["f16", "f32"])
@pytest.mark.parametrize("n", [1, 3, 7, 9, 31, 1001, 16384 + 5, 40003])
def test_ragged_sizes(gpu, oracle_mod, dtype, n):
    rng = np.random.default_rng(n)
    shards = [S.make_shard(rng, n, k) for k in (2, 3, 4, 5, 6, 32, 5, 3)]
    got = run_decode(gpu, shards, n, dtype)
    want = oracle_bits(oracle_mod, shards, n, dtype)
    assert np.array_equal(got, want)


def test_many_shards_use_the_device_table(gpu, oracle_mod):
    n = 4096 + 64
    rng = np.random.default_rng(77)
    ks = rng.choice([2, 3, 4, 5, 6, 32], size=150)
    shards = [S.make_shard(rng, n, int(k)) for k in ks]
    got = run_decode(gpu, shards, n, "f16")
    want = oracle_bits(oracle_mod, shards, n, "f16")
    assert np.array_equal(got, want)


def test_bert_large_shaped_shard(gpu, oracle_mod):
    n = S.BERT_LARGE_SHAPED.weights_per_shard
    rng = np.random.default_rng(3)
    shards = [S.make_shard(rng, n, k) for k in (3, 6)]
    got = run_decode(gpu, shards, n, "f16")
    assert np.array_equal(got, oracle_bits(oracle_mod, shards, n, "f16"))


def test_special_values_round_like_the_oracle(gpu, oracle_mod):
    vals = np.array([0.0, -0.0, np.inf, -np.inf, 65504.0, 65519.9, 65520.0, 1e10, 2.0 ** -14,
                     2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.0001, 2.0 ** -26, 1e-30, 1e-45,
                     1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 3.3895314e38, 0.1, -1 / 3,
                     6.0e-5, 5.96e-8, 2.98e-8, 1.0009765625, 1.00048828125], dtype=np.float32)
    nan_bits = np.array([0x7FC00000, 0xFFC00000, 0x7F800001, 0x7FA00000], dtype=np.uint32)
    vals = np.concatenate([vals, nan_bits.view(np.float32)])
    # as a raw 32-bit shard and as the codebook of a 5-bit shard (32 entries)
    n = vals.size
    raw = S.Shard(32, vals, None)
    cb = np.resize(vals, 32).astype(np.float32)
    idx_stream = np.random.default_rng(1).integers(0, 256, size=5 * 64, dtype=np.uint8)
    packed = S.Shard(5, idx_stream, cb)
    for dtype in ("f16", "bf16", "f32"):
        got = run_decode(gpu, [raw], n, dtype)
        assert np.array_equal(got, oracle_bits(oracle_mod, [raw], n, dtype)), dtype
        got = run_decode(gpu, [packed], 512, dtype)
        assert np.array_equal(got, oracle_bits(oracle_mod, [packed], 512, dtype)), dtype


def test_empty_inputs(gpu):
    torch, P, D = gpu
    out = torch.zeros(8, dtype=torch.float16, device="cuda")
    P.sti_decode_shards([], 100, out, None)
    sh = D.upload_shard(S.make_shard(np.random.default_rng(0), 64, 4))
    P.sti_decode_shards([sh], 0, out, None)
    torch.cuda.synchronize()
    assert float(out.abs().sum()) == 0.0


@pytest.mark.parametrize("dtype", ["f16", "f32", "bf16"])
def test_outlier_dictionary(gpu, oracle_mod, dtype):
    n = 16384 * 2 + 8 * 11
    rng = np.random.default_rng(91)
    shards = []
    for k in (2, 3, 4, 5, 6):
        shards.append(S.add_outliers(rng, S.make_shard(rng, n, k), n, fraction=0.0015))
    shards.append(S.make_shard(rng, n, 32))
    shards.append(S.make_shard(rng, n, 4))          # no dictionary
    edge = S.make_shard(rng, n, 3)
    edge.outlier_pos = np.array([0, 7, 8, n - 1], np.uint32)
    edge.outlier_val = np.array([1.5, -2.5, 65520.0, 1e-8], np.float32)
    shards.append(edge)
    got = run_decode(gpu, shards, n, dtype)
    want = oracle_bits(oracle_mod, shards, n, dtype)
    assert np.array_equal(got, want)


def test_outliers_with_device_table(gpu, oracle_mod):
    n = 4096
    rng = np.random.default_rng(92)
    shards = [S.add_outliers(rng, S.make_shard(rng, n, int(k)), n, 0.01)
              for k in rng.choice([2, 3, 4, 5, 6], size=70)]
    got = run_decode(gpu, shards, n, "f16")
    assert np.array_equal(got, oracle_bits(oracle_mod, shards, n, "f16"))


def test_random_sizes_bitwidths_and_dictionaries(gpu, oracle_mod):
    """Sixty seeded random calls: 1-90 shards of random bitwidths, 1-150,000 weights per shard,
    any of the three output types, outlier dictionaries on a random subset."""
    rng = np.random.default_rng(20240608)
    for case in range(60):
        n = int(rng.choice([int(rng.integers(1, 300)), int(rng.integers(300, 20000)), int(rng.integers(20000, 150000))]))
        n_shards = int(rng.choice([1, 2, 5, 17, 64, 65, 90])) if n < 20000 else int(rng.integers(1, 9))
        dtype = str(rng.choice(["f16", "f32", "bf16"]))
        shards = []
        for _ in range(n_shards):
            k = int(rng.choice([2, 3, 4, 5, 6, 32]))
            sh = S.make_shard(rng, n, k)
            if k != 32 and rng.random() < 0.4 and n >= 8:
                sh = S.add_outliers(rng, sh, n, fraction=float(rng.choice([0.001, 0.01, 0.1])))
            shards.append(sh)
        got = run_decode(gpu, shards, n, dtype)
        want = oracle_bits(oracle_mod, shards, n, dtype)
        assert np.array_equal(got, want), (case, n, n_shards, dtype)


def test_config1_full_size_sampled_shards(gpu, oracle_mod):
    """The whole decode stream of configuration 1 (4221 BERT-base shards, 1 GiB of packed indexes
    split evenly over 2-6 bits, 5 GB of binary16 out) in one call, set up as bench.py sets it
    up (one device buffer, shard streams back to back, device-side table).  The reference decodes
    sampled shards -- the first and last of every bitwidth group and a few inside -- bit for bit;
    over the whole output, every value of a sampled 1 % of positions is a member of its shard's
    rounded codebook."""
    from types import SimpleNamespace
    torch, P, D = gpu
    ds = S.config1()
    n = ds.weights_per_shard
    assert ds.n_shards == 4221 and ds.packed.nbytes == 1073037312
    packed = torch.from_numpy(ds.packed).cuda()
    cb_host = np.zeros((ds.n_shards, 64), dtype=np.float32)
    for s, c in enumerate(ds.codebooks):
        cb_host[s, :c.size] = c
    cbs = torch.from_numpy(cb_host).cuda()
    shards = [SimpleNamespace(bitwidth=int(ds.bitwidths[s]), data=packed[int(ds.offsets[s]):], codebook=cbs[s])
              for s in range(ds.n_shards)]
    out = torch.full((ds.n_shards * n,), 7, dtype=torch.float16, device="cuda")
    ws = torch.empty(max(16, P.sti_decode_workspace_bytes(ds.n_shards)), dtype=torch.uint8, device="cuda")
    P.sti_decode_shards(P.shard_array(shards), n, out, ws)
    torch.cuda.synchronize()
    out = out.view(ds.n_shards, n)
    sample = set()
    for k in (2, 3, 4, 5, 6):
        idx = np.nonzero(ds.bitwidths == k)[0]
        sample.update([int(idx[0]), int(idx[len(idx) // 3]), int(idx[-1])])
    for s in sorted(sample):
        want = oracle_mod.decode_shards([ds.shard(s)], n, oracle_mod.F16)[0]
        got = out[s].view(torch.int16).cpu().numpy().view(np.uint16)
        assert np.array_equal(got, want), s
    # membership over a strided sample of all shards
    rng = np.random.default_rng(5)
    cols = torch.from_numpy(np.sort(rng.choice(n, size=n // 100, replace=False))).cuda()
    sub = out[:, cols].view(torch.int16).cpu().numpy().view(np.uint16)
    for s in range(0, ds.n_shards, 37):
        table = oracle_mod.decode_shards(
            [S.Shard(32, ds.codebooks[s].astype(np.float32), None)], ds.codebooks[s].size, oracle_mod.F16)[0]
        assert np.isin(sub[s], table).all(), s


def test_more_than_2_to_the_32_weights_in_one_shard(gpu, oracle_mod):
    """One 2-bit shard of 2^32 + 24 weights (1 GiB packed, 8.6 GB of binary16 out): positions need
    64 bits.  Compared block by block so that host copies stay small."""
    torch, P, D = gpu
    n = (1 << 32) + 24
    sh = S.make_shard(np.random.default_rng(320), n, 2)
    out = torch.full((n,), 7, dtype=torch.float16, device="cuda")
    P.sti_decode_shards([D.upload_shard(sh)], n, out, None)
    torch.cuda.synchronize()
    want = oracle_mod.decode_shards([sh], n, oracle_mod.F16)[0]
    step = 1 << 28
    for a in range(0, n, step):
        b = min(n, a + step)
        got = out[a:b].view(torch.int16).cpu().numpy().view(np.uint16)
        assert np.array_equal(got, want[a:b]), a


def test_more_shards_than_a_grid_dimension_with_dictionaries(gpu, oracle_mod):
    """70,000 small shards, each with an outlier dictionary: the shard count passes the limit of
    a grid's second and third dimension (the scatter pass once refused such a call after the
    substitution pass had already run)."""
    from types import SimpleNamespace
    torch, P, D = gpu
    n_shards, n, k, n_out = 70000, 64, 4, 2
    rng = np.random.default_rng(70000)
    packed = rng.integers(0, 256, size=(n_shards, n * k // 8), dtype=np.uint8)
    codebooks = np.sort(rng.normal(0, 0.02, size=(n_shards, 1 << k)).astype(np.float32), axis=1)
    pos = np.sort(np.stack([rng.choice(n, size=n_out, replace=False) for _ in range(n_shards)]), axis=1).astype(np.uint32)
    val = rng.normal(0, 0.3, size=(n_shards, n_out)).astype(np.float32)
    host = [S.Shard(k, packed[s], codebooks[s], pos[s], val[s]) for s in range(n_shards)]
    want = oracle_mod.decode_shards(host, n, oracle_mod.F16)
    dp, dc = torch.from_numpy(packed).cuda(), torch.from_numpy(codebooks).cuda()
    dpos, dval = torch.from_numpy(pos.view(np.int32)).cuda(), torch.from_numpy(val).cuda()
    dev = [SimpleNamespace(bitwidth=k, data=dp[s], codebook=dc[s], outlier_pos=dpos[s], outlier_val=dval[s])
           for s in range(n_shards)]
    out = torch.full((n_shards * n,), 7, dtype=torch.float16, device="cuda")
    ws = torch.empty(P.sti_decode_workspace_bytes(n_shards), dtype=torch.uint8, device="cuda")
    P.sti_decode_shards(dev, n, out, ws)
    torch.cuda.synchronize()
    got = out.view(torch.int16).cpu().numpy().view(np.uint16).reshape(n_shards, n)
    assert np.array_equal(got, want)


# ------------------------------------------------------------------ working buffer of the matrix-core path

def untile(image, dims):
    """Logical order of one shard's binary16 image, from the layout the header documents (test-local:
    sub-block, 32-row strip, 64-column tile, 8-column piece, lane = half-tile * 32 + row % 32)."""
    d, dh, f = dims.d_model, dims.d_head, dims.ffn_per_shard
    out = np.empty(dims.weights_per_shard, dtype=image.dtype)
    sub = 0
    for rows, cols in ((3 * dh, d), (d, dh), (f, d), (d, f)):
        r, c = np.meshgrid(np.arange(rows), np.arange(cols), indexing="ij")
        off = (sub + ((r // 32) * (cols // 64) + c // 64) * 2048 + ((c % 32) // 8) * 512
               + (((c % 64) // 32) * 32 + r % 32) * 8 + c % 8)
        out[sub:sub + rows * cols] = image[off.ravel()]
        sub += rows * cols
    return out


@pytest.mark.parametrize("dims", [S.Dims(128, 7, 64, 64, 1e-12), S.BERT_BASE], ids=["small", "bert_base"])
def test_working_buffer_is_the_reference_decode_bit_for_bit(gpu, oracle_mod, dims):
    """The binary16 working buffer that every layer with many tokens multiplies from (and whose
    per-lane loader the few-token projections share): every bitwidth incl. the 3- and 5-bit streams
    whose indexes straddle dwords, an absent slot, outlier dictionaries."""
    torch, P, D = gpu
    rng = np.random.default_rng(97)
    n = dims.weights_per_shard
    bits = [2, 3, 4, 5, 6, 32, 0] + [int(b) for b in rng.choice([2, 3, 4, 5, 6, 32], dims.n_heads - 7)]
    host = [None if b == 0 else S.make_shard(rng, n, b) for b in bits]
    for s in host:
        if s is not None and s.bitwidth != 32:
            S.add_outliers(rng, s, n, 0.002)
    present = [s for s in host if s is not None]
    out = torch.full((len(present) * n,), float("nan"), dtype=torch.float16, device="cuda")
    assert P.sti_working_buffer_bytes(dims) == dims.n_heads * n * 2
    P.sti_decode_working_buffer(dims, [D.upload_shard(s) for s in host], out)
    torch.cuda.synchronize()
    got = out.view(torch.int16).cpu().numpy().view(np.uint16).reshape(len(present), n)
    want = oracle_mod.decode_shards(present, n, oracle_mod.F16)
    for p in range(len(present)):
        assert np.array_equal(untile(got[p], dims), want[p]), (p, present[p].bitwidth)
    # the library's own statement of the layout agrees with the header's formula
    probe = np.concatenate([np.arange(0, n, 4099), [n - 1]])
    image_index = np.array([P.sti_working_buffer_offset(dims, int(j)) for j in probe])
    assert np.array_equal(got[0][image_index], want[0][probe])
    assert P.sti_working_buffer_offset(dims, n) == -1


def test_working_buffer_rejections(gpu):
    torch, P, D = gpu
    dims = S.Dims(128, 2, 64, 64, 1e-12)
    n = dims.weights_per_shard
    sh = [D.upload_shard(S.make_shard(np.random.default_rng(1), n, 4)), None]
    out = torch.zeros(n, dtype=torch.float16, device="cuda")
    with pytest.raises(P.StiError) as e:
        P.sti_decode_working_buffer(dims, sh, out[: n - 8])
    assert e.value.status == 6
    with pytest.raises(P.StiError) as e:
        P.sti_decode_working_buffer(S.Dims(96, 2, 64, 64, 1e-12), sh, out)
    assert e.value.status == 2
    torch.cuda.synchronize()
    assert not out.any()
    P.sti_decode_working_buffer(dims, [None, None], out)   # nothing present: nothing written
    torch.cuda.synchronize()
    assert not out.any()
