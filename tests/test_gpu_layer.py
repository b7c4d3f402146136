"""GPU parity: sti_layer_forward / sti_model_forward (through the C ABI) against the
CPU oracle.

Tolerance: max |y_gpu - y_ref| / max |y_ref| <= 1e-5 for the float32 path (a float32 dot
product of length K <= 3072 carries about sqrt(K) * 2^-24 of relative error and LayerNorm
renormalises after every block) and <= 2e-2 for the binary16 matrix-core path (operands and
activations rounded to binary16, float32 accumulation).
"""
import json
import math
import os

import numpy as np
import pytest

import sti_synth as S
from parity import assert_parity

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "mfma": 2e-2}
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
SMALL = S.Dims(48, 3, 16, 32, 1e-12)
MID = S.Dims(128, 4, 64, 64, 1e-12)


@pytest.fixture(scope="module")
def gpu():
    import torch
    import paper_2207_05022_amd as P
    from paper_2207_05022_amd import device as D
    assert torch.cuda.is_available(), "needs a GPU"
    return torch, P, D


def rel_err(got, want):
    return float(np.max(np.abs(got.astype(np.float64) - want)) / max(np.max(np.abs(want)), 1e-30))


def run_gpu(gpu, wl, prec, model=True, x=None):
    torch, P, D = gpu
    precision = P.STI_PREC_F32 if prec == "f32" else P.STI_PREC_F16_MFMA
    shards, params, xd = D.upload_workload(wl)
    if x is not None:
        xd = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    y = torch.full_like(xd, float("nan"))
    B, L = int(xd.shape[0]), int(xd.shape[1])
    nbytes = P.sti_workspace_bytes(wl.dims, B, L, precision)
    assert nbytes > 0
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    if model:
        P.sti_model_forward(wl.dims, D.store_from_plan(shards), params, wl.plan, xd, y, precision, ws)
    else:
        assert wl.n_layers == 1
        P.sti_layer_forward(wl.dims, shards[0], params[0], xd, y, precision, ws)
    torch.cuda.synchronize()
    return y.float().cpu().numpy()


# ------------------------------------------------------------------ float32 path

def test_f32_tiny_hand_derived_layer(gpu):
    """The hand-derived fixture, straight against its printed expectations."""
    fx = json.load(open(os.path.join(GOLDEN, "tiny_layer.json")))
    dims = S.Dims(**fx["dims"])
    s = math.sqrt(math.sqrt(2.0) * math.log(3.0))
    mat = lambda m: np.array([[s if v == "s" else v for v in row] for row in m], dtype=np.float32)
    shards = []
    for name in ("shard0", "shard1"):
        b = fx[name]
        flat = np.concatenate([mat(b[k]).ravel() for k in ("Wq", "Wk", "Wv", "Wo", "W1", "W2")])
        shards.append(S.Shard(32, flat, None))
    params = S.LayerParams(**{k: np.array(v, dtype=np.float32) for k, v in fx["params"].items()})
    wl = S.Workload("tiny", dims, 1, 2, np.array([[32, 32]], dtype=np.int8), [shards], [params],
                    np.array(fx["x"], dtype=np.float32))
    y = run_gpu(gpu, wl, "f32", model=False)
    assert_parity(y, np.array(fx["expected"]["y"]), 1e-5)


@pytest.mark.parametrize("B,L", [(1, 1), (2, 7), (3, 70), (1, 130)])
def test_f32_small_mixed_layer(gpu, oracle_mod, B, L):
    wl = S.small_workload(100 + L, SMALL, 1, B, L, plan=np.array([[3, 32, 6]]))
    want = oracle_mod.layer_forward(SMALL, wl.shards[0], wl.params[0], wl.x)
    got = run_gpu(gpu, wl, "f32", model=False)
    assert_parity(got, want, TOL["f32"])


@pytest.mark.parametrize("plan", [[0, 0, 0], [0, 5, 0], [2, 0, 4]])
def test_f32_absent_shards(gpu, oracle_mod, plan):
    wl = S.small_workload(7, SMALL, 1, 2, 9, plan=np.array([plan]))
    want = oracle_mod.layer_forward(SMALL, wl.shards[0], wl.params[0], wl.x)
    got = run_gpu(gpu, wl, "f32", model=False)
    assert_parity(got, want, TOL["f32"])


@pytest.mark.parametrize("io", ["f32", "f16"])
def test_f32_small_model_all_bitwidths(gpu, oracle_mod, io):
    wl = S.small_workload(9, MID, 3, 2, 33, n_absent=1, io_dtype=io)
    want = oracle_mod.model_forward(MID, wl.shards, wl.params, wl.x)
    got = run_gpu(gpu, wl, "f32")
    tol = TOL["f32"] if io == "f32" else 1e-3  # output rounded to binary16
    assert_parity(got, want, tol)


def test_f32_bf16_io(gpu, oracle_mod):
    torch, P, D = gpu
    wl = S.small_workload(10, MID, 2, 1, 17)
    xb = torch.from_numpy(wl.x).to(torch.bfloat16)
    wl.x = xb.float().numpy()
    want = oracle_mod.model_forward(MID, wl.shards, wl.params, wl.x)
    shards, params, _ = D.upload_workload(wl)
    xd = xb.cuda(); y = torch.empty_like(xd)
    ws = torch.empty(P.sti_workspace_bytes(MID, 1, 17, P.STI_PREC_F32), dtype=torch.uint8, device="cuda")
    P.sti_model_forward(MID, D.store_from_plan(shards), params, wl.plan, xd, y, P.STI_PREC_F32, ws)
    torch.cuda.synchronize()
    assert_parity(y.float().cpu().numpy(), want, 8e-3)  # output rounded to bfloat16


@pytest.mark.parametrize("B,L", [(1, 40), (5, 128)])   # few-token kernels / wide-tile kernels
def test_mfma_bf16_io(gpu, oracle_mod, B, L):
    torch, P, D = gpu
    wl = S.small_workload(11, MID, 2, B, L)
    xb = torch.from_numpy(wl.x).to(torch.bfloat16)
    wl.x = xb.float().numpy()
    want = oracle_mod.model_forward(MID, wl.shards, wl.params, wl.x)
    shards, params, _ = D.upload_workload(wl)
    xd = xb.cuda(); y = torch.empty_like(xd)
    prec = P.STI_PREC_F16_MFMA
    ws = torch.empty(P.sti_model_workspace_bytes(MID, 2, B, L, prec), dtype=torch.uint8, device="cuda")
    P.sti_model_forward(MID, D.store_from_plan(shards), params, wl.plan, xd, y, prec, ws)
    torch.cuda.synchronize()
    assert y.dtype == torch.bfloat16
    assert_parity(y.float().cpu().numpy(), want, TOL["mfma"])


def test_f32_config0(gpu, oracle_mod):
    wl = S.config0()
    want = oracle_mod.layer_forward(wl.dims, wl.shards[0], wl.params[0], wl.x)
    got = run_gpu(gpu, wl, "f32", model=False)
    assert_parity(got, want, TOL["f32"])


def test_f32_config2(gpu, oracle_mod):
    wl = S.config2()
    want = oracle_mod.model_forward(wl.dims, wl.shards, wl.params, wl.x)
    got = run_gpu(gpu, wl, "f32")
    assert_parity(got, want, TOL["f32"])


def test_f32_config3(gpu, oracle_mod):
    wl = S.config3()
    want = oracle_mod.model_forward(wl.dims, wl.shards, wl.params, wl.x)
    got = run_gpu(gpu, wl, "f32")
    assert_parity(got, want, TOL["f32"])


def test_f32_random_shapes(gpu, oracle_mod):
    """Thirty seeded random shapes on the float32 path, which takes any dimensions: d_model 8-128,
    1-8 shards of 4-64 wide heads and 4-64 FFN neurons, 1-200 keys, 1-3 layers, float32 or
    binary16 activations at the boundary."""
    rng = np.random.default_rng(777)
    for case in range(30):
        M = int(rng.integers(1, 9))
        dh = int(rng.choice([4, 8, 12, 16, 20, 32, 64]))
        f = int(rng.choice([4, 8, 24, 32, 40, 64]))
        d = int(rng.choice([8, 16, 24, 40, 48, 72, 96, 128]))
        dims = S.Dims(d, M, dh, f, 1e-12)
        L = int(rng.integers(1, 200))
        B = int(rng.integers(1, 6))
        n_abs = int(rng.integers(0, M)) if M > 1 else 0
        n_layers = int(rng.choice([1, 2, 3]))
        io = str(rng.choice(["f32", "f16"]))
        wl = S.small_workload(12000 + case, dims, n_layers, B, L, n_absent=n_abs, io_dtype=io)
        S.make_every_term_matter(wl, case, amp=float(rng.choice([1.0, 4.0])))
        want = oracle_mod.model_forward(dims, wl.shards, wl.params, wl.x)
        got = run_gpu(gpu, wl, "f32")
        tol = TOL["f32"] if io == "f32" else 2e-3    # binary16 output: half an ulp of the largest value
        assert_parity(got, want, tol, (case, d, M, dh, f, B, L, n_abs, n_layers, io))


def test_empty_batch_and_zero_layers(gpu):
    torch, P, D = gpu
    wl = S.small_workload(3, SMALL, 1, 1, 4)
    shards, params, xd = D.upload_workload(wl)
    ws = torch.empty(max(256, P.sti_workspace_bytes(SMALL, 1, 4, 0)), dtype=torch.uint8, device="cuda")
    y = torch.zeros_like(xd)
    P.sti_model_forward(SMALL, D.store_from_plan([]), [], np.zeros((0, 3), np.int8), xd, y, 0, ws)
    torch.cuda.synchronize()
    assert torch.equal(xd, y)
    x0 = xd[:0].contiguous(); y0 = torch.empty_like(x0)
    P.sti_layer_forward(SMALL, shards[0], params[0], x0, y0, 0, ws)
    torch.cuda.synchronize()


# ------------------------------------------------------------------ binary16 matrix-core path

# (96, 97, 127, and 224, 225, 255: the last 32-key block of the two short-sequence attention paths
# full, one key in, one short; 256, 257: the longest short sequence and the first long one)
@pytest.mark.parametrize("B,L", [(1, 1), (2, 33), (1, 128), (3, 100), (1, 300), (2, 96), (2, 97), (1, 127),
                                 (1, 129), (40, 128), (1, 224), (2, 225), (1, 255), (3, 256), (1, 257)])
def test_mfma_small_mixed_layer(gpu, oracle_mod, B, L):
    wl = S.small_workload(200 + L, MID, 1, B, L, plan=np.array([[3, 32, 6, 5]]))
    want = oracle_mod.layer_forward(MID, wl.shards[0], wl.params[0], wl.x)
    got = run_gpu(gpu, wl, "mfma", model=False)
    assert_parity(got, want, TOL["mfma"])


@pytest.mark.parametrize("plan", [[0, 0, 0, 0], [0, 4, 0, 0], [2, 0, 32, 0]])
def test_mfma_absent_shards(gpu, oracle_mod, plan):
    wl = S.small_workload(17, MID, 1, 2, 40, plan=np.array([plan]))
    want = oracle_mod.layer_forward(MID, wl.shards[0], wl.params[0], wl.x)
    got = run_gpu(gpu, wl, "mfma", model=False)
    assert_parity(got, want, TOL["mfma"])


@pytest.mark.parametrize("B,L", [(2, 40), (3, 100), (9, 256)])
def test_mfma_layers_with_every_shard_absent(gpu, oracle_mod, B, L):
    """A layer without shards is valid at any token count (the working-buffer route once returned
    a HIP error for it): alone, and between layers that have shards."""
    plan = np.array([[4, 0, 32, 3], [0, 0, 0, 0], [2, 6, 0, 5]], dtype=np.int8)
    wl = S.small_workload(606, MID, 3, B, L, plan=plan, io_dtype="f16")
    S.make_every_term_matter(wl, 6, amp=4.0)
    want = oracle_mod.model_forward(MID, wl.shards, wl.params, wl.x)
    got = run_gpu(gpu, wl, "mfma")
    assert_parity(got, want, TOL["mfma"])
    alone = S.small_workload(607, MID, 1, B, L, plan=np.zeros((1, 4), dtype=np.int8), io_dtype="f16")
    S.make_every_term_matter(alone, 7)
    want = oracle_mod.layer_forward(MID, alone.shards[0], alone.params[0], alone.x)
    got = run_gpu(gpu, alone, "mfma", model=False)
    assert_parity(got, want, TOL["mfma"])


@pytest.mark.parametrize("io", ["f32", "f16"])
def test_mfma_small_model(gpu, oracle_mod, io):
    wl = S.small_workload(19, MID, 4, 2, 65, n_absent=1, io_dtype=io)
    want = oracle_mod.model_forward(MID, wl.shards, wl.params, wl.x)
    got = run_gpu(gpu, wl, "mfma")
    assert_parity(got, want, TOL["mfma"])


def test_mfma_config0(gpu, oracle_mod):
    wl = S.config0()
    want = oracle_mod.layer_forward(wl.dims, wl.shards[0], wl.params[0], wl.x)
    got = run_gpu(gpu, wl, "mfma", model=False)
    assert_parity(got, want, TOL["mfma"])


def test_mfma_config2(gpu, oracle_mod):
    wl = S.config2()
    want = oracle_mod.model_forward(wl.dims, wl.shards, wl.params, wl.x)
    got = run_gpu(gpu, wl, "mfma")
    assert_parity(got, want, TOL["mfma"])


def test_mfma_config3(gpu, oracle_mod):
    wl = S.config3()
    want = oracle_mod.model_forward(wl.dims, wl.shards, wl.params, wl.x)
    got = run_gpu(gpu, wl, "mfma")
    assert_parity(got, want, TOL["mfma"])


def test_mfma_config4_full_batch_sampled_sequences(gpu, oracle_mod):
    """Full-size batched run; sequences are independent, so the oracle checks a sample."""
    wl = S.config4()
    got = run_gpu(gpu, wl, "mfma")
    assert np.all(np.isfinite(got))
    for b in (0, 13, 31):
        want = oracle_mod.model_forward(wl.dims, wl.shards, wl.params, wl.x[b:b + 1])
        assert_parity(got[b:b + 1], want, TOL["mfma"], b)


def test_mfma_full_size_every_term_matters(gpu, oracle_mod):
    """The shapes and launch configurations of configurations 4 (32 x 128 tokens, wide-tile
    kernels), 0 (1 x 128 tokens, few-token kernels) and 3, with weights three times as large
    and random gains, shifts and biases: at this size dropping bq, bv, b1 or a gain moves the
    reference by 10-40 %."""
    wl = S.config4(n_layers=3)
    S.make_every_term_matter(wl, 4, amp=3.0)
    got = run_gpu(gpu, wl, "mfma")
    assert np.all(np.isfinite(got))
    for b in (0, 31):
        want = oracle_mod.model_forward(wl.dims, wl.shards, wl.params, wl.x[b:b + 1])
        assert_parity(got[b:b + 1], want, TOL["mfma"], b)
    one = S.Workload("one_sequence", wl.dims, 1, wl.seq, wl.plan, wl.shards, wl.params, wl.x[5:6], wl.io_dtype)
    got = run_gpu(gpu, one, "mfma")
    want = oracle_mod.model_forward(wl.dims, wl.shards, wl.params, wl.x[5:6])
    assert_parity(got, want, TOL["mfma"])
    # configuration 3's shape (d_model 1024, 12 of 16 shards, 256 tokens: K split over workgroups)
    wl3 = S.config3(n_layers=2)
    S.make_every_term_matter(wl3, 5, amp=3.0)
    got = run_gpu(gpu, wl3, "mfma")
    want = oracle_mod.model_forward(wl3.dims, wl3.shards, wl3.params, wl3.x)
    assert_parity(got, want, TOL["mfma"])


def test_mfma_rejects_unsupported_dims(gpu):
    torch, P, D = gpu
    assert P.sti_workspace_bytes(SMALL, 1, 8, P.STI_PREC_F16_MFMA) == 0
    wl = S.small_workload(3, SMALL, 1, 1, 8)
    shards, params, xd = D.upload_workload(wl)
    y = torch.empty_like(xd)
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    with pytest.raises(P.StiError) as ei:
        P.sti_layer_forward(SMALL, shards[0], params[0], xd, y, P.STI_PREC_F16_MFMA, ws)
    assert ei.value.status == 2


@pytest.mark.parametrize("prec", ["f32", "mfma"])
@pytest.mark.parametrize("B,L", [(2, 40), (5, 128)])
def test_rejected_calls_report_their_status_and_write_nothing(gpu, prec, B, L):
    """Every argument is checked before the first launch: a call that is rejected because of its last
    layer's plan, its workspace or its buffers leaves the output as it was."""
    torch, P, D = gpu
    precision = P.STI_PREC_F32 if prec == "f32" else P.STI_PREC_F16_MFMA
    wl = S.small_workload(1, MID, 4, B, L, n_absent=1, io_dtype="f16")
    shards, params, x = D.upload_workload(wl)
    store = P.make_store(D.store_from_plan(shards))
    ws = torch.empty(P.sti_model_workspace_bytes(MID, 4, B, L, precision), dtype=torch.uint8, device="cuda")

    def rejected(status, plan=wl.plan, xin=x, workspace=ws):
        y = torch.full_like(x, float("nan"))
        with pytest.raises(P.StiError) as ei:
            P.sti_model_forward(MID, store, params, plan, xin, y, precision, workspace)
        torch.cuda.synchronize()
        assert ei.value.status == status
        assert bool(torch.isnan(y.float()).all())

    present = int(np.argwhere(wl.plan[3] != 0)[0][0])
    plan = wl.plan.copy()
    plan[3, present] = [k for k in (2, 3, 4, 5, 6, 32) if k != wl.plan[3, present]][0]
    rejected(4, plan=plan)                                   # a version the store does not hold
    plan = wl.plan.copy()
    plan[3, present] = 7
    rejected(3, plan=plan)                                   # not a bitwidth
    one_layer = P.sti_workspace_bytes(MID, B, L, precision)  # least the model call can work in
    rejected(6, workspace=ws[:one_layer - 1])                # workspace too small
    shifted = torch.empty(x.numel() + 8, dtype=x.dtype, device="cuda")[1:1 + x.numel()].view_as(x)
    rejected(5, xin=shifted)                                 # input not 16-byte aligned


# ------------------------------------------------------------------ outlier dictionary

def _with_outliers(wl, seed, fraction=0.0015):
    rng = np.random.default_rng(seed)
    for row in wl.shards:
        for s in row:
            if s is not None:
                S.add_outliers(rng, s, wl.dims.weights_per_shard, fraction)
    return wl


@pytest.mark.parametrize("prec,B,L", [("f32", 2, 9), ("mfma", 1, 40), ("mfma", 5, 128)])
def test_layers_apply_outlier_dictionaries(gpu, oracle_mod, prec, B, L):
    wl = _with_outliers(S.small_workload(300 + L, MID, 2, B, L, n_absent=1), 5, fraction=0.05)
    want = oracle_mod.model_forward(MID, wl.shards, wl.params, wl.x)
    plain = [[None if s is None else S.Shard(s.bitwidth, s.data, s.codebook) for s in row]
             for row in wl.shards]
    without = oracle_mod.model_forward(MID, plain, wl.params, wl.x)
    assert rel_err(without, want) > 3 * TOL[prec]     # the dictionaries matter at this tolerance
    got = run_gpu(gpu, wl, prec)
    assert_parity(got, want, TOL[prec])


def test_mfma_whole_model_decode_matches_per_layer_route(gpu, oracle_mod):
    """With a workspace of sti_model_workspace_bytes the layers are decompressed ahead, into a ring of buffers;
    the result must be the very bits of the per-layer route (same kernels, same order of
    arithmetic) and within tolerance of the oracle; outlier dictionaries included."""
    torch, P, D = gpu
    wl = S.small_workload(777, MID, 4, 5, 128, n_absent=1, bit_choices=(2, 3, 4, 5, 6, 32), io_dtype="f16")
    wl = _with_outliers(wl, 3, fraction=0.01)
    prec = P.STI_PREC_F16_MFMA
    shards, params, xd = D.upload_workload(wl)
    store = P.make_store(D.store_from_plan(shards))
    small = P.sti_workspace_bytes(wl.dims, 5, 128, prec)
    big = P.sti_model_workspace_bytes(wl.dims, wl.n_layers, 5, 128, prec)
    assert big > small
    outs = []
    for nbytes in (small, big):
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        y = torch.full_like(xd, float("nan"))
        P.sti_model_forward(wl.dims, store, params, wl.plan, xd, y, prec, ws)
        torch.cuda.synchronize()
        outs.append(y)
    assert torch.equal(outs[0], outs[1])
    want = oracle_mod.model_forward(wl.dims, wl.shards, wl.params, wl.x)
    assert_parity(outs[1].float().cpu().numpy(), want, TOL["mfma"])
    # on the few-token route the query falls back to the one-layer size
    assert P.sti_model_workspace_bytes(wl.dims, wl.n_layers, 1, 128, prec) == P.sti_workspace_bytes(wl.dims, 1, 128, prec)


def _run_model_route(gpu, wl, nbytes, key_lengths=None):
    """sti_model_forward(_masked) on the matrix-core path with a workspace of `nbytes`."""
    torch, P, D = gpu
    shards, params, xd = D.upload_workload(wl)
    store = P.make_store(D.store_from_plan(shards))
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    y = torch.full_like(xd, float("nan"))
    if key_lengths is None:
        P.sti_model_forward(wl.dims, store, params, wl.plan, xd, y, P.STI_PREC_F16_MFMA, ws)
    else:
        P.sti_model_forward_masked(wl.dims, store, params, wl.plan, xd, y,
                                   torch.tensor(key_lengths, dtype=torch.int32, device="cuda"),
                                   P.STI_PREC_F16_MFMA, ws)
    torch.cuda.synchronize()
    return y


def test_mfma_config4_on_the_timed_route_every_sequence(gpu, oracle_mod):
    """Configuration 4 exactly as bench.py times it (Section "Submodel execution": layers in
    order): 12 layers, a workspace of sti_model_workspace_bytes, hence a ring of four working buffers
    and non-zero table offsets; the first layer is decompressed by a launch of its own,
    every other one by the idle workgroups of the Q/K/V + attention launch before it; unmasked.
    All 32 sequences against the oracle; the bits of the per-layer route."""
    torch, P, D = gpu
    wl = S.config4()
    prec = P.STI_PREC_F16_MFMA
    big = P.sti_model_workspace_bytes(wl.dims, wl.n_layers, wl.batch, wl.seq, prec)
    small = P.sti_workspace_bytes(wl.dims, wl.batch, wl.seq, prec)
    layer_w16 = wl.dims.n_heads * wl.dims.weights_per_shard * 2
    assert 3 * layer_w16 <= big - small < 4 * layer_w16      # a ring of four working buffers: the 12 layers wrap it three times
    timed = _run_model_route(gpu, wl, big)
    per_layer = _run_model_route(gpu, wl, small)
    assert torch.equal(timed, per_layer)
    want = oracle_mod.model_forward(wl.dims, wl.shards, wl.params, wl.x)
    got = timed.float().cpu().numpy()
    assert_parity(got, want, TOL["mfma"])
    for b in range(wl.batch):
        assert_parity(got[b], want[b], TOL["mfma"], b)


def test_next_layer_decompressed_beside_the_projection_with_outlier_dictionaries(gpu, oracle_mod):
    """32 sequences of 128 tokens with 9 of 12 shards per layer: the fused Q/K/V + attention launch
    has 160 tiles (the last pair of heads is half empty), and the whole-model route lets its idle
    workgroups decompress the following layer (Section "Submodel execution": the next layer is made
    ready while this one computes); the outlier dictionaries of that layer go in behind the launch.
    Bits of the per-layer route, oracle on every sequence."""
    torch, P, D = gpu
    wl = S.small_workload(515, S.BERT_BASE, 4, 32, 128, n_absent=3, bit_choices=(2, 3, 4, 5, 6, 32), io_dtype="f16")
    wl = _with_outliers(wl, 17, fraction=0.01)
    S.make_every_term_matter(wl, 29, amp=2.0)
    prec = P.STI_PREC_F16_MFMA
    big = P.sti_model_workspace_bytes(wl.dims, wl.n_layers, wl.batch, wl.seq, prec)
    small = P.sti_workspace_bytes(wl.dims, wl.batch, wl.seq, prec)
    rolling = _run_model_route(gpu, wl, big)
    per_layer = _run_model_route(gpu, wl, small)
    assert torch.equal(rolling, per_layer)
    want = oracle_mod.model_forward(wl.dims, wl.shards, wl.params, wl.x)
    got = rolling.float().cpu().numpy()
    assert_parity(got, want, TOL["mfma"])
    for b in range(wl.batch):
        assert_parity(got[b], want[b], TOL["mfma"], b)


def test_layers_that_can_and_cannot_take_the_next_layer_along(gpu, oracle_mod):
    """38 sequences: a full layer has 228 tiles and no compute unit to spare, a layer with 9 or 10 shards
    190 tiles and 64; with an all-absent layer in between.  Layers 0 to 3 are decompressed as a group,
    layer 3 takes layer 4 along, layer 5 is decompressed alone."""
    torch, P, D = gpu
    rng = np.random.default_rng(77)
    plan = rng.choice([2, 3, 4, 5, 6, 32], size=(6, 12)).astype(np.int8)
    plan[1, [2, 7]] = 0
    plan[2, :] = 0
    plan[3, [0, 5, 11]] = 0
    plan[5, [4, 9]] = 0
    wl = S.small_workload(616, S.BERT_BASE, 6, 38, 128, plan=plan, io_dtype="f16")
    wl = _with_outliers(wl, 19, fraction=0.005)
    prec = P.STI_PREC_F16_MFMA
    big = P.sti_model_workspace_bytes(wl.dims, wl.n_layers, wl.batch, wl.seq, prec)
    small = P.sti_workspace_bytes(wl.dims, wl.batch, wl.seq, prec)
    mixed = _run_model_route(gpu, wl, big)
    per_layer = _run_model_route(gpu, wl, small)
    assert torch.equal(mixed, per_layer)
    want = oracle_mod.model_forward(wl.dims, wl.shards, wl.params, wl.x)
    assert_parity(mixed.float().cpu().numpy(), want, TOL["mfma"])


def test_whole_model_route_random_sweep_is_the_per_layer_route(gpu):
    """Seeded sweep over 128-token batches of 6 to 43 sequences, three shapes, 2 to 5 layers with 0 to all
    shards absent per layer, with and without outlier dictionaries and key lengths: whichever layers
    are decompressed by launches of their own or beside their predecessor's projection, the whole-model
    route gives the bits of the per-layer route (which the other tests hold against the oracle)."""
    torch, P, D = gpu
    prec = P.STI_PREC_F16_MFMA
    rng = np.random.default_rng(2024)
    shapes = [S.BERT_BASE, S.Dims(512, 8, 64, 256, 1e-12), S.Dims(1024, 16, 64, 256, 1e-12)]
    for it in range(18):
        dims = shapes[it % 3]
        M = dims.n_heads
        n_layers = int(rng.integers(2, 6))
        B = int(rng.integers(6, 44))
        plan = rng.choice([2, 3, 4, 5, 6, 32], size=(n_layers, M)).astype(np.int8)
        for l in range(n_layers):
            k = int(rng.integers(0, M + 1)) if rng.random() < 0.15 else int(rng.integers(0, 5))
            plan[l, rng.choice(M, k, replace=False)] = 0
        wl = S.small_workload(9000 + it, dims, n_layers, B, 128, plan=plan, io_dtype="f16")
        if it % 2:
            wl = _with_outliers(wl, it, fraction=0.003)
        lengths = rng.integers(1, 129, size=B).astype(np.int32) if it % 4 == 3 else None
        big = P.sti_model_workspace_bytes(dims, n_layers, B, 128, prec)
        small = P.sti_workspace_bytes(dims, B, 128, prec)
        whole = _run_model_route(gpu, wl, big, key_lengths=lengths)
        per_layer = _run_model_route(gpu, wl, small, key_lengths=lengths)
        assert torch.equal(whole, per_layer), (it, dims.d_model, B, [int((plan[l] != 0).sum()) for l in range(n_layers)])
        assert torch.isfinite(whole.float()).all()


def test_mfma_one_layer_per_decompression_group_with_outlier_dictionaries(gpu, oracle_mod):
    """d_model 2048 with 32 shards: one layer's working buffer (100 MB) alone exceeds a 64 MiB group,
    so every layer of the whole-model route is a group of its own (table and buffer offsets of
    layers 1 and 2 are non-zero); outlier dictionaries on every shard, two shards absent per layer."""
    torch, P, D = gpu
    dims = S.Dims(2048, 32, 64, 256, 1e-12)
    wl = S.small_workload(4242, dims, 3, 2, 128, n_absent=2, bit_choices=(2, 3, 4, 5, 6, 32), io_dtype="f16")
    wl = _with_outliers(wl, 11, fraction=0.01)
    S.make_every_term_matter(wl, 23, amp=2.0)
    prec = P.STI_PREC_F16_MFMA
    big = P.sti_model_workspace_bytes(dims, wl.n_layers, 2, 128, prec)
    small = P.sti_workspace_bytes(dims, 2, 128, prec)
    assert dims.n_heads * dims.weights_per_shard * 2 > (64 << 20) and big > small
    grouped = _run_model_route(gpu, wl, big)
    per_layer = _run_model_route(gpu, wl, small)
    assert torch.equal(grouped, per_layer)
    want = oracle_mod.model_forward(dims, wl.shards, wl.params, wl.x)
    assert_parity(grouped.float().cpu().numpy(), want, TOL["mfma"])


WIDE = S.Dims(128, 12, 64, 64, 1e-12)


@pytest.mark.parametrize("prec,dims,B,L", [("f32", SMALL, 2, 19), ("mfma", MID, 1, 66), ("mfma", MID, 3, 100),
                                           ("mfma", WIDE, 5, 128), ("mfma", WIDE, 9, 256), ("mfma", MID, 2, 200),
                                           ("mfma", MID, 2, 300)])
def test_every_term_of_the_layer_matters(gpu, oracle_mod, prec, dims, B, L):
    """With the configurations' recipe a kernel could leave out the score scale, bq or b1, or a
    LayerNorm gain, and stay inside the binary16 tolerance (tests/test_oracle_layer.py measures
    that on the reference).  Here weights are six times as large and gains, shifts and biases
    are random, on every route: float32; few-token, partial-sum and wide-tile matrix-core
    GEMMs; attention with the scores in registers (up to 128 and up to 256 keys) and with the
    running maximum (300 keys)."""
    wl = S.small_workload(31000 + B * L, dims, 2, B, L, n_absent=1, io_dtype="f32" if prec == "f32" else "f16")
    S.make_every_term_matter(wl, 77 + B)
    want = oracle_mod.model_forward(dims, wl.shards, wl.params, wl.x)
    got = run_gpu(gpu, wl, prec)
    assert_parity(got, want, TOL[prec])


def test_mfma_many_column_tiles_take_the_band_order(gpu, oracle_mod):
    """More than 12 column tiles (here 32 shards: 16 column tiles for Q/K/V, 22 for FFN1) make the
    wide-tile GEMM walk its tiles in bands of 8 row tiles; 11 row tiles leave a short last band
    and 1400 tokens a ragged last row tile."""
    dims = S.Dims(128, 32, 64, 256, 1e-12)
    wl = S.small_workload(2048, dims, 1, 7, 200, n_absent=3, io_dtype="f16")
    S.make_every_term_matter(wl, 9, amp=3.0)
    want = oracle_mod.model_forward(dims, wl.shards, wl.params, wl.x)
    got = run_gpu(gpu, wl, "mfma")
    assert_parity(got, want, TOL["mfma"])


@pytest.mark.parametrize("B,L", [(1, 64), (3, 100)])   # few-token route / working-buffer route
def test_mfma_widest_supported_model(gpu, oracle_mod, B, L):
    """d_model 2048 (rows of 2048 features in LayerNorm, K = 2048 in the projections, 22-26 column
    tiles) with 32 shards of which two are absent; weights twice the recipe's scale."""
    dims = S.Dims(2048, 32, 64, 256, 1e-12)
    wl = S.small_workload(77, dims, 1, B, L, n_absent=2, io_dtype="f16")
    S.make_every_term_matter(wl, 21, amp=2.0)
    want = oracle_mod.model_forward(dims, wl.shards, wl.params, wl.x)
    got = run_gpu(gpu, wl, "mfma")
    assert_parity(got, want, TOL["mfma"])


@pytest.mark.parametrize("d_model", [2112, 4096])
@pytest.mark.parametrize("B,L", [(1, 40), (3, 100)])   # few-token route / working-buffer route
def test_mfma_rows_longer_than_2048_features(gpu, oracle_mod, d_model, B, L):
    """d_model beyond what the row kernels keep in registers (the working-buffer route once
    failed here, after its first launches, with a HIP error from the LayerNorm launcher)."""
    dims = S.Dims(d_model, 4, 64, 64, 1e-12)
    wl = S.small_workload(5, dims, 2, B, L, n_absent=1, io_dtype="f16")
    S.make_every_term_matter(wl, 8, amp=2.0)
    want = oracle_mod.model_forward(dims, wl.shards, wl.params, wl.x)
    got = run_gpu(gpu, wl, "mfma")
    # (gains up to 1.9 on rows of 4096 features with doubled weights: at d_model 4096, 1 of 163,840 and
    #  8 of 1,228,800 elements were measured past the per-element bound; none at d_model 2112)
    assert_parity(got, want, TOL["mfma"], max_violations=1e-4 if d_model == 4096 else 0.0)


def test_mfma_rows_beyond_2gib_of_activations(gpu):
    """350,000 tokens: the FFN activations (T x 3072 binary16) pass 2 GiB, so row addresses need
    64 bits.  Sequences are independent, so the first and the last sequence of the big batch
    must come out as when they run alone (up to the summation order of other tile shapes)."""
    torch, P, D = gpu
    dims = S.BERT_BASE
    B, L = 700, 500
    wl = S.small_workload(4242, dims, 1, 2, L, io_dtype="f16")
    shards, params, x2 = D.upload_workload(wl)
    prec = P.STI_PREC_F16_MFMA
    gen = torch.Generator(device="cuda").manual_seed(7)
    x = torch.randn(B, L, dims.d_model, device="cuda", generator=gen).to(torch.float16)
    x[0] = x2[0]
    x[B - 1] = x2[1]
    y = torch.empty_like(x)
    ws = torch.empty(P.sti_workspace_bytes(dims, B, L, prec), dtype=torch.uint8, device="cuda")
    P.sti_layer_forward(dims, shards[0], params[0], x, y, prec, ws)
    y2 = torch.empty_like(x2)
    ws2 = torch.empty(P.sti_workspace_bytes(dims, 2, L, prec), dtype=torch.uint8, device="cuda")
    P.sti_layer_forward(dims, shards[0], params[0], x2, y2, prec, ws2)
    torch.cuda.synchronize()
    assert torch.isfinite(y).all()
    for big, alone in ((y[0], y2[0]), (y[B - 1], y2[1])):
        assert_parity(big.float().cpu().numpy(), alone.float().cpu().numpy(), 4e-3)


def test_model_forward_can_be_stream_captured(gpu, oracle_mod):
    """The few-token path enqueues kernels only (no copies, no fills, no host waits), so a
    caller may capture it into a graph; replays, with eager calls between them, must give the
    eager result every time."""
    torch, P, D = gpu
    wl = S.small_workload(888, MID, 3, 2, 100, n_absent=1, io_dtype="f16")
    prec = P.STI_PREC_F16_MFMA
    shards, params, x = D.upload_workload(wl)
    store = P.make_store(D.store_from_plan(shards))
    ws = torch.empty(P.sti_workspace_bytes(MID, 2, 100, prec), dtype=torch.uint8, device="cuda")
    y_eager = torch.empty_like(x)
    P.sti_model_forward(MID, store, params, wl.plan, x, y_eager, prec, ws)
    torch.cuda.synchronize()
    want = oracle_mod.model_forward(MID, wl.shards, wl.params, wl.x)
    assert_parity(y_eager.float().cpu().numpy(), want, TOL["mfma"])
    y_graph = torch.full_like(x, float("nan"))
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            P.sti_model_forward(MID, store, params, wl.plan, x, y_graph, prec, ws)
    torch.cuda.synchronize()
    for _ in range(3):
        y_graph.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y_graph, y_eager)
        scratch = torch.empty_like(x)
        P.sti_model_forward(MID, store, params, wl.plan, x, scratch, prec, ws)   # eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(scratch, y_eager)


def test_capture_never_records_the_shard_table_upload(gpu, oracle_mod):
    """With the model workspace the eager call takes the grouped route, whose shard table is
    uploaded through a pinned host buffer that later calls overwrite; a captured call must not
    record that copy: it runs the per-layer route (same bits), and replays stay right after
    eager calls with OTHER plans have reused the pinned buffer.  sti_decode_shards with more than
    64 shards, which has no other route, refuses to be captured."""
    torch, P, D = gpu
    wl = S.small_workload(4321, MID, 3, 3, 100, n_absent=1, io_dtype="f16")
    other = S.small_workload(1234, MID, 3, 3, 100, n_absent=2, io_dtype="f16")
    prec = P.STI_PREC_F16_MFMA
    shards, params, x = D.upload_workload(wl)
    store = P.make_store(D.store_from_plan(shards))
    o_shards, o_params, o_x = D.upload_workload(other)
    o_store = P.make_store(D.store_from_plan(o_shards))
    nbytes = P.sti_model_workspace_bytes(MID, 3, 3, 100, prec)
    assert nbytes > P.sti_workspace_bytes(MID, 3, 100, prec)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    y_eager = torch.empty_like(x)
    P.sti_model_forward(MID, store, params, wl.plan, x, y_eager, prec, ws)
    torch.cuda.synchronize()
    assert_parity(y_eager.float().cpu().numpy(), oracle_mod.model_forward(MID, wl.shards, wl.params, wl.x), TOL["mfma"])
    y_graph = torch.full_like(x, float("nan"))
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            P.sti_model_forward(MID, store, params, wl.plan, x, y_graph, prec, ws)
    torch.cuda.synchronize()
    o_ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    o_y = torch.empty_like(o_x)
    for _ in range(3):
        for _ in range(5):   # more eager uploads than the pinned ring has slots
            P.sti_model_forward(MID, o_store, o_params, other.plan, o_x, o_y, prec, o_ws)
        torch.cuda.synchronize()
        y_graph.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y_graph, y_eager)
    # decode: 70 shards need the uploaded table
    n = 4096
    host = [S.make_shard(np.random.default_rng(s), n, 2 + s % 5) for s in range(70)]
    dev = [D.upload_shard(s) for s in host]
    out = torch.zeros(70 * n, dtype=torch.float16, device="cuda")
    dws = torch.empty(P.sti_decode_workspace_bytes(70), dtype=torch.uint8, device="cuda")
    g2 = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g2, stream=side):
            with pytest.raises(P.StiError) as err:
                P.sti_decode_shards(dev, n, out, dws)
            P.sti_decode_shards(dev[:64], n, out[:64 * n], None)   # at most 64 shards: kernels only
    assert err.value.status == 9   # STI_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    g2.replay()
    torch.cuda.synchronize()
    got = out.view(torch.int16).cpu().numpy().view(np.uint16).reshape(70, n)
    assert np.array_equal(got[:64], oracle_mod.decode_shards(host[:64], n, oracle_mod.F16))
    assert not got[64:].any()
    P.sti_decode_shards(dev, n, out, dws)   # eager: accepted
    torch.cuda.synchronize()
    got = out.view(torch.int16).cpu().numpy().view(np.uint16).reshape(70, n)
    assert np.array_equal(got, oracle_mod.decode_shards(host, n, oracle_mod.F16))


@pytest.mark.parametrize("B,L", [(1, 64), (4, 128)])   # few-token route / working-buffer route
def test_per_kernel_timing_counts_every_launch_and_changes_nothing(gpu, B, L):
    """sti_profile_begin/end: the launches carry timing events; the counts per kernel class
    are those of the route, every class with launches has a positive time, the sum of the
    kernel times is below the wall time of the forward, and the output is bit for bit what an
    untimed call gives."""
    import time
    torch, P, D = gpu
    n_layers = 3
    wl = S.small_workload(4100 + L, MID, n_layers, B, L, io_dtype="f16")
    shards, params, x = D.upload_workload(wl)
    store = P.make_store(D.store_from_plan(shards))
    prec = P.STI_PREC_F16_MFMA
    ws = torch.empty(P.sti_model_workspace_bytes(MID, n_layers, B, L, prec), dtype=torch.uint8, device="cuda")
    y0 = torch.empty_like(x)
    P.sti_model_forward(MID, store, params, wl.plan, x, y0, prec, ws)
    torch.cuda.synchronize()
    y1 = torch.full_like(x, float("nan"))
    P.sti_profile_begin()
    t0 = time.perf_counter()
    P.sti_model_forward(MID, store, params, wl.plan, x, y1, prec, ws)
    prof = P.sti_profile_end()          # waits for the events
    wall_ms = (time.perf_counter() - t0) * 1e3
    torch.cuda.synchronize()
    assert torch.equal(y0, y1)
    count = {k: v[0] for k, v in prof.items()}
    for k in ("gemm_qkv", "attention", "gemm_out", "gemm_ffn_up", "gemm_ffn_down"):
        assert count[k] == n_layers, (k, count)
    assert count["layernorm"] == 2 * n_layers
    few_tokens = B * L <= 128
    assert (count["decode"] == 0) if few_tokens else (1 <= count["decode"] <= n_layers)
    total = 0.0
    for k, (n, ms) in prof.items():
        assert (ms > 0.0) == (n > 0), (k, n, ms)
        total += ms
    assert total < wall_ms
    # a second begin/end pair starts from zero
    P.sti_profile_begin()
    assert all(n == 0 for n, _ in P.sti_profile_end().values())


def test_mfma_random_shapes(gpu, oracle_mod):
    """Forty seeded random shapes (1-32 shards of which any number absent, d_model 64-192, 64-256
    FFN neurons per shard, 1-400 keys, up to 3000 tokens, one or two layers; weights at the
    recipe's scale or three or six times larger) through whichever route and tile shapes they
    select.  (Four hundred cases of the same generator, up to 6000 tokens, were run once when
    this test was written: worst error 2.7e-3.)"""
    rng = np.random.default_rng(20240607)
    for case in range(40):
        M = int(rng.choice([1, 2, 3, 4, 7, 12, 16, 29, 32]))
        f = int(rng.choice([64, 128, 256]))
        d = int(rng.choice([64, 128, 192]))
        dims = S.Dims(d, M, 64, f, 1e-12)
        L = int(rng.integers(1, 400))
        B = max(1, min(int(rng.integers(1, max(2, 3000 // L))), 3000 // L))
        n_abs = int(rng.integers(0, M)) if M > 1 else 0
        n_layers = int(rng.choice([1, 2]))
        wl = S.small_workload(9000 + case, dims, n_layers, B, L, n_absent=n_abs, io_dtype="f16")
        S.make_every_term_matter(wl, case, amp=float(rng.choice([1.0, 3.0, 6.0])))
        want = oracle_mod.model_forward(dims, wl.shards, wl.params, wl.x)
        got = run_gpu(gpu, wl, "mfma")
        assert_parity(got, want, TOL["mfma"], (case, d, M, f, B, L, n_abs, n_layers))


def test_concurrent_calls_from_host_threads(gpu):
    """Four host threads, each with a stream and a workspace of its own, run model forwards of
    both routes (and decode calls that upload a shard table) at the same time: every result is
    bit for bit the single-threaded one.  (The library's only shared state is the pinned ring
    that table uploads go through.)"""
    import threading
    torch, P, D = gpu
    prec = P.STI_PREC_F16_MFMA
    prepared = []
    for seed, (B, L) in enumerate([(2, 60), (5, 128), (1, 100), (9, 256)]):
        wl = S.small_workload(8800 + seed, WIDE if seed == 3 else MID, 3, B, L, n_absent=1, io_dtype="f16")
        shards, params, x = D.upload_workload(wl)
        store = P.make_store(D.store_from_plan(shards))
        ws = torch.empty(P.sti_model_workspace_bytes(wl.dims, 3, B, L, prec), dtype=torch.uint8, device="cuda")
        ref = torch.empty_like(x)
        P.sti_model_forward(wl.dims, store, params, wl.plan, x, ref, prec, ws)
        prepared.append((wl, store, params, x, ref, shards))
    n = 4096
    host = [S.make_shard(np.random.default_rng(s), n, int(k))
            for s, k in enumerate(np.random.default_rng(0).choice([2, 3, 4, 5, 6], size=100))]
    dev = [D.upload_shard(s) for s in host]
    dref = torch.empty(len(dev) * n, dtype=torch.float16, device="cuda")
    dws = torch.empty(P.sti_decode_workspace_bytes(len(dev)), dtype=torch.uint8, device="cuda")
    P.sti_decode_shards(dev, n, dref, dws)
    torch.cuda.synchronize()
    bad = []

    def worker(i):
        wl, store, params, x, ref, _ = prepared[i]
        B, L = int(x.shape[0]), int(x.shape[1])
        stream = torch.cuda.Stream()
        with torch.cuda.stream(stream):
            ws = torch.empty(P.sti_model_workspace_bytes(wl.dims, 3, B, L, prec), dtype=torch.uint8, device="cuda")
            y = torch.empty_like(x)
            out, ows = torch.empty_like(dref), torch.empty_like(dws)
            for it in range(30):
                y.fill_(float("nan"))
                P.sti_model_forward(wl.dims, store, params, wl.plan, x, y, prec, ws)
                P.sti_decode_shards(dev, n, out, ows)
                if it % 10 == 9:
                    stream.synchronize()
                    if not torch.equal(y, ref) or not torch.equal(out.view(torch.int16), dref.view(torch.int16)):
                        bad.append((i, it))
        stream.synchronize()

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(4)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not bad, bad


# ------------------------------------------------------------------ padded sequences

def _key_lengths(L, B, seed):
    """Lengths that hit the edges (1, L, around multiples of 32) and random ones."""
    rng = np.random.default_rng(seed)
    edges = [L, 1, min(L, 32), min(L, 33), max(1, L - 1), min(L, 64), min(L, 31)]
    lens = [edges[b] if b < len(edges) else int(rng.integers(1, L + 1)) for b in range(B)]
    return np.asarray(lens, dtype=np.int32)


def _run_masked(gpu, wl, prec, lens, route):
    torch, P, D = gpu
    precision = P.STI_PREC_F32 if prec == "f32" else P.STI_PREC_F16_MFMA
    shards, params, xd = D.upload_workload(wl)
    ld = None if lens is None else torch.from_numpy(lens).cuda()
    y = torch.full_like(xd, float("nan"))
    B, L = int(xd.shape[0]), int(xd.shape[1])
    store = P.make_store(D.store_from_plan(shards))
    if route == "whole":      # room for every layer's working buffer
        ws = torch.empty(P.sti_model_workspace_bytes(wl.dims, wl.n_layers, B, L, precision), dtype=torch.uint8, device="cuda")
    else:
        ws = torch.empty(P.sti_workspace_bytes(wl.dims, B, L, precision), dtype=torch.uint8, device="cuda")
    if route == "layer":
        assert wl.n_layers == 1
        if ld is None:
            P.sti_layer_forward(wl.dims, shards[0], params[0], xd, y, precision, ws)
        else:
            P.sti_layer_forward_masked(wl.dims, shards[0], params[0], xd, y, ld, precision, ws)
    elif ld is None:
        P.sti_model_forward(wl.dims, store, params, wl.plan, xd, y, precision, ws)
    else:
        P.sti_model_forward_masked(wl.dims, store, params, wl.plan, xd, y, ld, precision, ws)
    torch.cuda.synchronize()
    return y


@pytest.mark.parametrize("prec,dims,B,L,route", [
    ("f32", SMALL, 5, 19, "layer"), ("f32", MID, 8, 70, "model"),
    ("mfma", MID, 3, 40, "layer"),      # two-wave workgroups, scores in registers
    ("mfma", MID, 2, 64, "model"),      # few-token route
    ("mfma", MID, 9, 128, "model"),
    ("mfma", MID, 8, 200, "whole"),     # eight key blocks in registers, every layer's working buffer
    ("mfma", MID, 48, 128, "model"),    # four-wave workgroups
    ("mfma", MID, 64, 128, "model"),    # attention inside the Q/K/V projection; 3 present heads: a tile with one head
    ("mfma", WIDE, 24, 128, "whole"),   # the same with 11 present heads, every layer's working buffer
    ("mfma", MID, 7, 300, "whole"),     # online softmax
    ("mfma", MID, 2, 512, "model"),
])
def test_padded_sequences_match_the_reference(gpu, oracle_mod, prec, dims, B, L, route):
    """Keys beyond a sequence's length take no attention weight (all rows compared, padded ones
    included); full lengths give the bits of the plain entry point; the mask matters at this scale."""
    torch = gpu[0]
    n_layers = 1 if route == "layer" else 2
    wl = S.small_workload(8000 + L, dims, n_layers, B, L, n_absent=1)
    S.make_every_term_matter(wl, 3, amp=6.0 if dims is MID else 3.0)
    lens = _key_lengths(L, B, L)
    want = oracle_mod.model_forward(dims, wl.shards, wl.params, wl.x, key_lengths=lens)
    got = _run_masked(gpu, wl, prec, lens, route)
    assert_parity(got.float().cpu().numpy(), want, TOL[prec])
    plain = _run_masked(gpu, wl, prec, None, route)
    assert rel_err(plain.float().cpu().numpy(), want) > 3 * TOL[prec]
    full = _run_masked(gpu, wl, prec, np.full(B, L, dtype=np.int32), route)
    assert torch.equal(full, plain)


@pytest.mark.parametrize("dims,n_absent", [(MID, 1), (MID, 0), (WIDE, 3)])
def test_attention_inside_the_projection_matches_the_separate_kernels(gpu, oracle_mod, dims, n_absent):
    """With sequences of 128 tokens and enough of them, the Q/K/V projection's workgroups run the
    attention of the two heads they hold.  Against the reference on every sequence (odd and even
    numbers of present heads), and against the same sequences sent as four smaller batches, which take
    the separate projection and attention kernels: the two compute the same values in the same order up
    to the tile shapes that the batch size selects for the other projections."""
    torch, P, D = gpu
    B = 256 // ((dims.n_heads - n_absent + 1) // 2)
    wl = S.small_workload(9100 + n_absent, dims, 2, B, 128, n_absent=n_absent, io_dtype="f16")
    S.make_every_term_matter(wl, 12, amp=3.0)
    want = oracle_mod.model_forward(dims, wl.shards, wl.params, wl.x)
    got = run_gpu(gpu, wl, "mfma")
    assert_parity(got, want, TOL["mfma"])
    for b in (0, B // 2, B - 1):
        assert_parity(got[b], want[b], TOL["mfma"], b)
    q = B // 4
    for part in range(4):
        sub = run_gpu(gpu, wl, "mfma", x=wl.x[part * q:(part + 1) * q])
        assert_parity(sub, got[part * q:(part + 1) * q], 4e-3, part)


def test_padded_sequences_ignore_what_the_padding_holds(gpu):
    """Real rows come out bit for bit the same whatever finite values the padded rows of x hold, and
    lengths outside 1..seq are clamped."""
    torch, P, D = gpu
    B, L = 6, 96
    wl = S.small_workload(8100, MID, 2, B, L, n_absent=1, io_dtype="f16")
    S.make_every_term_matter(wl, 4)
    lens = _key_lengths(L, B, 1)
    a = _run_masked(gpu, wl, "mfma", lens, "model")
    rng = np.random.default_rng(2)
    for b, n in enumerate(lens):
        wl.x[b, n:] = rng.normal(0, 30, wl.x[b, n:].shape).astype(wl.x.dtype)
    bb = _run_masked(gpu, wl, "mfma", lens, "model")
    for b, n in enumerate(lens):
        assert torch.equal(a[b, :n], bb[b, :n]), b
    wild = lens.copy()
    wild[0], wild[1] = L + 1000, -5            # clamped to L and to 1
    assert lens[0] == L and lens[1] == 1
    assert torch.equal(_run_masked(gpu, wl, "mfma", wild, "model"), bb)


def test_captured_masked_forward_follows_the_lengths_in_device_memory(gpu):
    """The key lengths are read by the kernels, not by the host: a graph captured once serves
    other lengths by rewriting the device array between replays."""
    torch, P, D = gpu
    B, L = 3, 60
    wl = S.small_workload(889, MID, 2, B, L, n_absent=1, io_dtype="f16")
    S.make_every_term_matter(wl, 6)
    prec = P.STI_PREC_F16_MFMA
    shards, params, x = D.upload_workload(wl)
    store = P.make_store(D.store_from_plan(shards))
    ws = torch.empty(P.sti_workspace_bytes(MID, B, L, prec), dtype=torch.uint8, device="cuda")
    lens = torch.tensor([L, 7, 33], dtype=torch.int32, device="cuda")
    y_graph = torch.full_like(x, float("nan"))
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            P.sti_model_forward_masked(MID, store, params, wl.plan, x, y_graph, lens, prec, ws)
    torch.cuda.synchronize()
    seen = []
    for new in ([L, 7, 33], [1, L, 32], [59, 31, 2], [L, 7, 33]):
        lens.copy_(torch.tensor(new, dtype=torch.int32))
        y_graph.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        eager = torch.full_like(x, float("nan"))
        P.sti_model_forward_masked(MID, store, params, wl.plan, x, eager, lens, prec, ws)
        torch.cuda.synchronize()
        assert torch.equal(y_graph, eager), new
        seen.append(eager.clone())
    assert not torch.equal(seen[0], seen[1]) and torch.equal(seen[0], seen[3])


def test_padded_sequences_at_configuration_4_size(gpu, oracle_mod):
    """32 x 128 tokens of BERT-base (three layers, whole-model route, the launch shapes the
    benchmark times) with a length mix from 1 to 128: sampled sequences against the reference,
    each run alone at its padded length."""
    wl = S.config4(n_layers=3)
    S.make_every_term_matter(wl, 4, amp=3.0)
    rng = np.random.default_rng(12)
    lens = rng.integers(1, wl.seq + 1, wl.x.shape[0]).astype(np.int32)
    lens[0], lens[31], lens[7] = wl.seq, 1, 65
    got = _run_masked(gpu, wl, "mfma", lens, "whole").float().cpu().numpy()
    assert np.all(np.isfinite(got))
    for b in (0, 7, 19, 31):
        want = oracle_mod.model_forward(wl.dims, wl.shards, wl.params, wl.x[b:b + 1], key_lengths=lens[b:b + 1])
        assert_parity(got[b:b + 1], want, TOL["mfma"], (b, int(lens[b])))
