"""Pins for the oracle's layer and model forward.

Nothing here recomputes the oracle with its own routine: the checks are a
hand-derived tiny layer (tests/golden/tiny_layer.json), an independently
computed dense post-LayerNorm BERT layer (torch.nn.TransformerEncoderLayer in
float64, fed dense matrices assembled from the shards by numpy code local to
this file), and identities the paper states for shards (independence of the
vertical slices, any subset executes, mixed bitwidths are compatible).
"""
import copy
import json
import math
import os

import numpy as np
import pytest

import sti_synth as S

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
SMALL = S.Dims(48, 3, 16, 32, 1e-12)


# ---------------------------------------------------------------- helpers (test-local)

def np_decode(sh: S.Shard, n: int) -> np.ndarray:
    """Independent decode via numpy bit unpacking (float32 values)."""
    if sh.bitwidth == 32:
        return np.asarray(sh.data, dtype=np.float32)[:n]
    k = sh.bitwidth
    bits = np.unpackbits(sh.data, bitorder="little")[: n * k].reshape(n, k)
    idx = (bits.astype(np.int64) << np.arange(k)).sum(axis=1)
    return sh.codebook[idx]


def split_blocks(dims: S.Dims, w: np.ndarray):
    d, dh, f = dims.d_model, dims.d_head, dims.ffn_per_shard
    o = dims.offsets()
    return {
        "q": w[o["q"]:o["k"]].reshape(dh, d),
        "k": w[o["k"]:o["v"]].reshape(dh, d),
        "v": w[o["v"]:o["o"]].reshape(dh, d),
        "o": w[o["o"]:o["ffn1"]].reshape(d, dh),
        "ffn1": w[o["ffn1"]:o["ffn2"]].reshape(f, d),
        "ffn2": w[o["ffn2"]:].reshape(d, f),
    }


def shard32_from_blocks(blocks) -> S.Shard:
    flat = np.concatenate([np.asarray(blocks[n], dtype=np.float32).ravel()
                           for n in ("q", "k", "v", "o", "ffn1", "ffn2")])
    return S.Shard(32, flat, None)


def dense_torch_layer(dims: S.Dims, shards, params: S.LayerParams, x: np.ndarray,
                      key_lengths=None) -> np.ndarray:
    """Full layer as a stock dense post-LN encoder layer in float64 (key_lengths: padding mask)."""
    import torch
    d, M, dh, f = dims.d_model, dims.n_heads, dims.d_head, dims.ffn_per_shard
    blocks = [split_blocks(dims, np_decode(s, dims.weights_per_shard).astype(np.float64))
              for s in shards]
    Wq = np.concatenate([b["q"] for b in blocks], axis=0)       # [d, d] rows = head-major outputs
    Wk = np.concatenate([b["k"] for b in blocks], axis=0)
    Wv = np.concatenate([b["v"] for b in blocks], axis=0)
    Wo = np.concatenate([b["o"] for b in blocks], axis=1)       # [d, M*dh]
    W1 = np.concatenate([b["ffn1"] for b in blocks], axis=0)    # [M*f, d]
    W2 = np.concatenate([b["ffn2"] for b in blocks], axis=1)    # [d, M*f]
    layer = torch.nn.TransformerEncoderLayer(
        d_model=d, nhead=M, dim_feedforward=M * f, dropout=0.0, activation="gelu",
        layer_norm_eps=dims.ln_eps, batch_first=True, norm_first=False, dtype=torch.float64)
    layer.eval()
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float64))
    with torch.no_grad():
        layer.self_attn.in_proj_weight.copy_(t(np.concatenate([Wq, Wk, Wv], axis=0)))
        layer.self_attn.in_proj_bias.copy_(t(np.concatenate([params.bq, params.bk, params.bv])))
        layer.self_attn.out_proj.weight.copy_(t(Wo))
        layer.self_attn.out_proj.bias.copy_(t(params.bo))
        layer.linear1.weight.copy_(t(W1)); layer.linear1.bias.copy_(t(params.b1))
        layer.linear2.weight.copy_(t(W2)); layer.linear2.bias.copy_(t(params.b2))
        layer.norm1.weight.copy_(t(params.ln1_g)); layer.norm1.bias.copy_(t(params.ln1_b))
        layer.norm2.weight.copy_(t(params.ln2_g)); layer.norm2.bias.copy_(t(params.ln2_b))
        # the python path (no fused fast path) so that eps and ordering are the stock ones
        torch.backends.mha.set_fastpath_enabled(False)
        pad = None
        if key_lengths is not None:
            pad = torch.arange(x.shape[1])[None, :] >= torch.as_tensor(np.asarray(key_lengths))[:, None]
        y = layer(t(x), src_key_padding_mask=pad)
    return y.numpy()


def random_params(rng, dims, gains=True) -> S.LayerParams:
    p = S.make_layer_params(rng, dims)
    if gains:  # non-trivial LayerNorm gains so that gain/shift mix-ups show
        p.ln1_g = rng.normal(1.0, 0.3, dims.d_model).astype(np.float32)
        p.ln2_g = rng.normal(1.0, 0.3, dims.d_model).astype(np.float32)
    return p


# ---------------------------------------------------------------- P6 hand-derived tiny layer

def test_tiny_layer_by_hand(oracle_mod):
    fx = json.load(open(os.path.join(GOLDEN, "tiny_layer.json")))
    dims = S.Dims(**fx["dims"])
    s = math.sqrt(math.sqrt(2.0) * math.log(3.0))

    def mat(m):
        return np.array([[s if v == "s" else v for v in row] for row in m], dtype=np.float64)

    shards = []
    for name in ("shard0", "shard1"):
        b = fx[name]
        shards.append(shard32_from_blocks({"q": mat(b["Wq"]), "k": mat(b["Wk"]), "v": mat(b["Wv"]),
                                           "o": mat(b["Wo"]), "ffn1": mat(b["W1"]),
                                           "ffn2": mat(b["W2"])}))
    params = S.LayerParams(**{k: np.array(v, dtype=np.float32) for k, v in fx["params"].items()})
    x = np.array(fx["x"], dtype=np.float64)
    y, taps = oracle_mod.layer_forward(dims, shards, params, x, taps=True)
    exp = fx["expected"]
    # s and 0.1 are rounded to float32 when stored in a 32-bit shard: 1e-6 covers that
    assert np.allclose(taps["attn"], np.array(exp["attn"]), rtol=0, atol=2e-6)
    assert np.allclose(taps["h"], np.array(exp["h"]), rtol=0, atol=2e-6)
    assert np.allclose(taps["ffn"], np.array(exp["ffn"]), rtol=0, atol=2e-6)
    assert np.allclose(y, np.array(exp["y"]), rtol=0, atol=2e-6)


# ---------------------------------------------------------------- P4 dense equivalence

@pytest.mark.parametrize("bits", [(32, 32, 32), (2, 5, 32), (3, 4, 6)])
@pytest.mark.parametrize("B,L", [(1, 7), (2, 5)])
def test_full_shard_set_equals_dense_bert_layer(oracle_mod, bits, B, L):
    wl = S.small_workload(11 + sum(bits), SMALL, 1, B, L, plan=np.array([bits]))
    # spread the weights so that attention is far from uniform and GELU is exercised
    for sh in wl.shards[0]:
        if sh.bitwidth == 32:
            sh.data *= np.float32(12.0)
        else:
            sh.codebook *= np.float32(12.0)
    params = random_params(np.random.default_rng(99), SMALL)
    y = oracle_mod.layer_forward(SMALL, wl.shards[0], params, wl.x)
    want = dense_torch_layer(SMALL, wl.shards[0], params, wl.x.astype(np.float64))
    assert np.max(np.abs(y - want)) <= 1e-12 * max(1.0, np.max(np.abs(want)))


def test_bert_base_shape_equals_dense(oracle_mod):
    wl = S.small_workload(5, S.BERT_BASE, 1, 1, 16, plan=np.full((1, 12), 4))
    y = oracle_mod.layer_forward(wl.dims, wl.shards[0], wl.params[0], wl.x)
    want = dense_torch_layer(wl.dims, wl.shards[0], wl.params[0], wl.x.astype(np.float64))
    assert np.max(np.abs(y - want)) <= 1e-12 * np.max(np.abs(want))


# ---------------------------------------------------------------- P5 / P8 / P9 / P11 shard identities

def _wl(seed=21, plan=None, **kw):
    return S.small_workload(seed, SMALL, 1, 2, 6, plan=plan, **kw)


def test_absent_equals_zero_weights(oracle_mod):
    wl = _wl(plan=np.array([[4, 32, 3]]))
    params = random_params(np.random.default_rng(1), SMALL)
    for gone in range(3):
        dropped = list(wl.shards[0]); dropped[gone] = None
        zeroed = list(wl.shards[0])
        zeroed[gone] = S.Shard(32, np.zeros(SMALL.weights_per_shard, np.float32), None)
        ya = oracle_mod.layer_forward(SMALL, dropped, params, wl.x)
        yz = oracle_mod.layer_forward(SMALL, zeroed, params, wl.x)
        full = oracle_mod.layer_forward(SMALL, wl.shards[0], params, wl.x)
        assert np.max(np.abs(ya - yz)) <= 1e-13
        assert np.max(np.abs(ya - full)) > 1e-3  # the shard did matter


def test_all_absent_layer(oracle_mod):
    wl = _wl()
    p = random_params(np.random.default_rng(2), SMALL)
    x = wl.x.astype(np.float64)
    y = oracle_mod.layer_forward(SMALL, [None, None, None], p, x)

    def ln(v, g, b):
        m = v.mean(-1, keepdims=True); var = v.var(-1, keepdims=True)
        return (v - m) / np.sqrt(var + SMALL.ln_eps) * g + b

    h = ln(x + p.bo.astype(np.float64), p.ln1_g.astype(np.float64), p.ln1_b.astype(np.float64))
    want = ln(h + p.b2.astype(np.float64), p.ln2_g.astype(np.float64), p.ln2_b.astype(np.float64))
    assert np.max(np.abs(y - want)) <= 1e-12


def test_shard_permutation(oracle_mod):
    wl = _wl(plan=np.array([[2, 6, 32]]))
    p = random_params(np.random.default_rng(3), SMALL)
    y = oracle_mod.layer_forward(SMALL, wl.shards[0], p, wl.x)
    perm = [2, 0, 1]
    dh, f = SMALL.d_head, SMALL.ffn_per_shard
    q = S.LayerParams(**{n: getattr(p, n).copy() for n in S.LayerParams.NAMES})
    for name, w in (("bq", dh), ("bk", dh), ("bv", dh), ("b1", f)):
        src = getattr(p, name).reshape(3, w)
        setattr(q, name, src[perm].reshape(-1).copy())
    y2 = oracle_mod.layer_forward(SMALL, [wl.shards[0][i] for i in perm], q, wl.x)
    assert np.max(np.abs(y - y2)) <= 1e-13


def test_additivity_of_shard_contributions(oracle_mod):
    wl = _wl(plan=np.array([[3, 5, 32]]))
    p = random_params(np.random.default_rng(4), SMALL)
    sh = wl.shards[0]

    def taps(present):
        sel = [s if i in present else None for i, s in enumerate(sh)]
        return oracle_mod.layer_forward(SMALL, sel, p, wl.x, taps=True)[1]

    bo = p.bo.astype(np.float64)
    a01, a0, a1, a2, a012 = taps({0, 1}), taps({0}), taps({1}), taps({2}), taps({0, 1, 2})
    assert np.max(np.abs((a01["attn"] - bo) - ((a0["attn"] - bo) + (a1["attn"] - bo)))) <= 1e-13
    assert np.max(np.abs((a012["attn"] - bo) - ((a01["attn"] - bo) + (a2["attn"] - bo)))) <= 1e-13
    assert np.max(np.abs(a0["attn"] - bo)) > 1e-3


def test_mixed_bitwidth_compatibility(oracle_mod):
    """A k-bit shard and a 32-bit shard holding its decoded values are interchangeable."""
    wl = _wl(plan=np.array([[2, 4, 6]]))
    p = random_params(np.random.default_rng(5), SMALL)
    y = oracle_mod.layer_forward(SMALL, wl.shards[0], p, wl.x)
    swapped = [S.Shard(32, np_decode(s, SMALL.weights_per_shard).copy(), None) for s in wl.shards[0]]
    mixed = [swapped[0], wl.shards[0][1], swapped[2]]
    y2 = oracle_mod.layer_forward(SMALL, mixed, p, wl.x)
    assert np.array_equal(y, y2)


# ---------------------------------------------------------------- P7 internal invariants

def test_layernorm_and_softmax_invariants(oracle_mod):
    dims = S.Dims(48, 3, 16, 32, 1e-5)
    wl = S.small_workload(31, dims, 1, 1, 9, plan=np.array([[32, 32, 32]]))
    p = S.make_layer_params(np.random.default_rng(6), dims)
    for n in ("ln1_b", "ln2_b"):
        setattr(p, n, np.zeros(dims.d_model, np.float32))
    y, taps = oracle_mod.layer_forward(dims, wl.shards[0], p, wl.x, taps=True)
    for out, pre in ((taps["h"], wl.x + taps["attn"]), (y, taps["h"] + taps["ffn"])):
        var = pre.var(-1)
        assert np.max(np.abs(out.mean(-1))) <= 1e-13
        assert np.allclose(out.var(-1), var / (var + dims.ln_eps), rtol=1e-12, atol=0)
    # zero weights: attention output is b_o for every token, whatever x is -> scaling x
    # by a constant leaves LayerNorm1(x + b_o) unchanged when b_o = 0 and eps = 0
    dims0 = S.Dims(48, 3, 16, 32, 0.0)
    zero = [S.Shard(32, np.zeros(dims0.weights_per_shard, np.float32), None)] * 3
    p0 = S.make_layer_params(np.random.default_rng(7), dims0)
    p0.bo = np.zeros(dims0.d_model, np.float32)
    _, t1 = oracle_mod.layer_forward(dims0, zero, p0, wl.x, taps=True)
    _, t2 = oracle_mod.layer_forward(dims0, zero, p0, 8.0 * wl.x, taps=True)
    assert np.max(np.abs(t1["h"] - t2["h"])) <= 1e-12
    assert np.max(np.abs(t1["attn"])) == 0.0


def test_uniform_attention_when_scores_are_equal(oracle_mod):
    """Zero Q weights and biases give uniform attention: every token's context is the
    mean of the values, so the attention output is the same for all tokens."""
    wl = _wl(plan=np.array([[32, 32, 32]]))
    p = random_params(np.random.default_rng(8), SMALL)
    p.bq = np.zeros_like(p.bq)
    shards = []
    for s in wl.shards[0]:
        w = s.data.copy(); w[: SMALL.d_head * SMALL.d_model] = 0
        shards.append(S.Shard(32, w, None))
    _, taps = oracle_mod.layer_forward(SMALL, shards, p, wl.x, taps=True)
    a = taps["attn"]
    assert np.max(np.abs(a - a[:, :1, :])) <= 1e-13
    # and equals b_o + Wo . (Wv . mean(x) + bv)
    xm = wl.x.astype(np.float64).mean(axis=1)
    want = np.tile(p.bo.astype(np.float64), (2, 1))
    for i, s in enumerate(shards):
        b = split_blocks(SMALL, s.data.astype(np.float64))
        v = xm @ b["v"].T + p.bv[i * 16:(i + 1) * 16].astype(np.float64)
        want += v @ b["o"].T
    assert np.max(np.abs(a[:, 0, :] - want)) <= 1e-12


# ---------------------------------------------------------------- P10 model composition

def test_model_is_layer_composition(oracle_mod):
    wl = S.small_workload(41, SMALL, 3, 2, 5, n_absent=1)
    y = oracle_mod.model_forward(SMALL, wl.shards, wl.params, wl.x)
    cur = wl.x.astype(np.float64)
    for l in range(3):
        cur = oracle_mod.layer_forward(SMALL, wl.shards[l], wl.params[l], cur)
    assert np.array_equal(y, cur)
    # batch elements are independent sequences
    y0 = oracle_mod.model_forward(SMALL, wl.shards, wl.params, wl.x[:1])
    assert np.max(np.abs(y0 - y[:1])) <= 1e-13


def test_model_with_dense_reference_two_layers(oracle_mod):
    wl = S.small_workload(42, SMALL, 2, 1, 6, plan=np.array([[2, 3, 32], [6, 32, 5]]))
    y = oracle_mod.model_forward(SMALL, wl.shards, wl.params, wl.x)
    cur = wl.x.astype(np.float64)
    for l in range(2):
        cur = dense_torch_layer(SMALL, wl.shards[l], wl.params[l], cur)
    assert np.max(np.abs(y - cur)) <= 1e-12 * max(1.0, np.max(np.abs(cur)))


def test_outlier_shard_equals_patched_full_precision_shard(oracle_mod):
    """A k-bit shard with an outlier dictionary behaves like the float32 shard holding its
    decoded weights with the outliers written in (decode computed by test-local numpy code)."""
    wl = _wl(seed=23, plan=np.array([[3, 6, 4]]))
    p = random_params(np.random.default_rng(9), SMALL)
    rng = np.random.default_rng(10)
    shards = [S.add_outliers(rng, s, SMALL.weights_per_shard, 0.01) for s in wl.shards[0]]
    y = oracle_mod.layer_forward(SMALL, shards, p, wl.x)
    patched = []
    for s in shards:
        w = np_decode(S.Shard(s.bitwidth, s.data, s.codebook), SMALL.weights_per_shard).copy()
        w[s.outlier_pos] = s.outlier_val
        patched.append(S.Shard(32, w, None))
    y2 = oracle_mod.layer_forward(SMALL, patched, p, wl.x)
    assert np.array_equal(y, y2)
    plain = [S.Shard(s.bitwidth, s.data, s.codebook) for s in shards]
    assert np.max(np.abs(y - oracle_mod.layer_forward(SMALL, plain, p, wl.x))) > 1e-4


# ---------------------------------------------------------------- power of the binary16 parity cases

def test_planted_mistakes_show_only_when_every_term_matters(oracle_mod):
    """How much of a mistake the binary16 tolerance (2e-2) can see.  Mistakes are planted in the
    reference's inputs: no score scale (Wq and bq times sqrt(dh) -- float32 shards only, so the
    plan is all 32-bit), bq left out, b1 left out, a LayerNorm gain taken as 1.  With the
    configurations' recipe the first three change the output by less than the tolerance, so
    parity cases on that recipe alone could not tell; after S.make_every_term_matter every
    one of them costs several times the tolerance.  (bk is absent on purpose: adding q.bk to
    every score of a row leaves its softmax unchanged.)"""
    dims = S.Dims(128, 4, 64, 64, 1e-12)
    TOL16 = 2e-2

    def effects(wl):
        good = oracle_mod.layer_forward(dims, wl.shards[0], wl.params[0], wl.x)
        rel = lambda y: float(np.max(np.abs(y - good)) / np.max(np.abs(good)))
        out = {}
        w2 = copy.deepcopy(wl)
        n = dims.d_head * dims.d_model
        for sh in w2.shards[0]:
            sh.data[:n] *= np.float32(math.sqrt(dims.d_head))
        w2.params[0].bq *= np.float32(math.sqrt(dims.d_head))
        out["scale"] = rel(oracle_mod.layer_forward(dims, w2.shards[0], w2.params[0], w2.x))
        for name, value in (("bq", 0.0), ("b1", 0.0), ("ln1_g", 1.0), ("ln2_g", 1.0)):
            w2 = copy.deepcopy(wl)
            getattr(w2.params[0], name)[:] = value
            out[name] = rel(oracle_mod.layer_forward(dims, w2.shards[0], w2.params[0], w2.x))
        return out

    plan = np.array([[32, 32, 32, 32]])
    recipe = effects(S.small_workload(5, dims, 1, 2, 100, plan=plan))
    assert recipe["scale"] < TOL16 and recipe["bq"] < TOL16 and recipe["b1"] < TOL16
    assert recipe["ln1_g"] == 0.0 and recipe["ln2_g"] == 0.0      # the recipe's gains are 1
    wl = S.small_workload(5, dims, 1, 2, 100, plan=plan)
    S.make_every_term_matter(wl, 3)
    strong = effects(wl)
    for name, e in strong.items():
        assert e > 3 * TOL16, (name, e)


# ---------------------------------------------------------------- padded sequences

def _padded_case(seed, B=4, L=19):
    rng = np.random.default_rng(seed)
    shards = [S.make_shard(rng, SMALL.weights_per_shard, k) for k in (4, 32, 6)]
    params = random_params(rng, SMALL)
    x = rng.normal(0, 1, (B, L, SMALL.d_model))
    lens = np.array([L, 1, 7, L - 1][:B], dtype=np.int32)
    return shards, params, x, lens


def test_padding_mask_matches_the_stock_layer(oracle_mod):
    """Keys beyond a sequence's length get no attention weight: torch's key-padding mask
    (float64, dense matrices assembled above) gives the same rows, padded ones included."""
    shards, params, x, lens = _padded_case(21)
    for s in shards:                                  # weights large enough for attention to matter
        if s.bitwidth == 32:
            s.data = (np.asarray(s.data) * 8).astype(np.float32)
        else:
            s.codebook = (s.codebook * 8).astype(np.float32)
    got = oracle_mod.layer_forward(SMALL, shards, params, x, key_lengths=lens)
    want = dense_torch_layer(SMALL, shards, params, x, key_lengths=lens)
    unmasked = dense_torch_layer(SMALL, shards, params, x)
    assert np.max(np.abs(got - want)) < 1e-10
    assert np.max(np.abs(unmasked - want)) > 1e-2     # the mask changes the result at this scale


def test_padded_rows_do_not_reach_real_rows(oracle_mod):
    """The real positions of a padded sequence come out as if the sequence had been run alone at
    its own length, whatever the padding holds; full lengths reproduce the unmasked layer bit for
    bit."""
    shards, params, x, lens = _padded_case(22)
    rows = [[s for s in shards], [shards[0], None, shards[2]]]
    prm = [params, random_params(np.random.default_rng(5), SMALL)]
    got = oracle_mod.model_forward(SMALL, rows, prm, x, key_lengths=lens)
    for b, n in enumerate(lens):
        alone = oracle_mod.model_forward(SMALL, rows, prm, x[b:b + 1, :n])
        assert np.max(np.abs(got[b, :n] - alone[0])) < 1e-12
    x2 = x.copy()
    for b, n in enumerate(lens):
        x2[b, n:] = 1e3 * np.random.default_rng(b).normal(size=x2[b, n:].shape)
    again = oracle_mod.model_forward(SMALL, rows, prm, x2, key_lengths=lens)
    for b, n in enumerate(lens):
        assert np.array_equal(again[b, :n], got[b, :n])
    full = np.full(len(lens), x.shape[1], dtype=np.int32)
    assert np.array_equal(oracle_mod.model_forward(SMALL, rows, prm, x, key_lengths=full),
                          oracle_mod.model_forward(SMALL, rows, prm, x))


def test_key_lengths_outside_the_sequence_are_refused(oracle_mod):
    shards, params, x, lens = _padded_case(23)
    for bad in (0, x.shape[1] + 1, -3):
        lens2 = lens.copy()
        lens2[2] = bad
        with pytest.raises(Exception):
            oracle_mod.layer_forward(SMALL, shards, params, x, key_lengths=lens2)
