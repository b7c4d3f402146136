"""GPU parity of the load || compute pipeline (Section "Elastic pipelining"; the preload
buffer's content after an inference follows Section "Submodel execution").

sti_pipeline_forward runs the same kernels on the same bits as sti_model_forward, so the two
must agree bit for bit; against the CPU oracle the usual tolerances apply.  The byte counts
it reports are checked against the packed sizes of the selected shards (Table "shard
versions": Wsh * k / 8 bytes per k-bit shard, 4 * Wsh at full precision).
"""
import numpy as np
import pytest

import sti_synth as S
from parity import assert_parity

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "mfma": 2e-2}
SMALL = S.Dims(48, 3, 16, 32, 1e-12)
MID = S.Dims(128, 4, 64, 64, 1e-12)


@pytest.fixture(scope="module")
def gpu():
    import torch
    import paper_2207_05022_amd as P
    from paper_2207_05022_amd import device as D
    assert torch.cuda.is_available(), "needs a GPU"
    return torch, P, D



def shard_bytes(dims, k):
    return dims.weights_per_shard * 4 if k == 32 else dims.weights_per_shard * k // 8


def plan_bytes(dims, plan):
    return [shard_bytes(dims, int(k)) for k in np.asarray(plan).ravel() if k != 0]


def expected_resident(dims, plan, preload_bytes):
    """Longest prefix of the selected shards, in (layer, shard) order, that fits the buffer
    when every shard starts on a 256-byte boundary."""
    cum, n, total = 0, 0, 0
    for b in plan_bytes(dims, plan):
        if cum + b > preload_bytes:
            break
        n, total = n + 1, total + b
        cum = (cum + b + 255) // 256 * 256
    return n, total


class Rig:
    """Device-resident store for sti_model_forward and a pinned-host twin for the pipeline."""

    def __init__(self, gpu, wl, prec, preload_bytes, host_data=True, slots=2):
        torch, P, D = gpu
        self.torch, self.P, self.wl = torch, P, wl
        self.precision = P.STI_PREC_F32 if prec == "f32" else P.STI_PREC_F16_MFMA
        self.dev_shards, self.params, self.x = D.upload_workload(wl)
        self.host_shards, _, _ = D.upload_workload(wl, host_data=host_data)
        self.dev_store = P.make_store(D.store_from_plan(self.dev_shards))
        self.host_store = P.make_store(D.store_from_plan(self.host_shards))
        B, L = int(self.x.shape[0]), int(self.x.shape[1])
        self.ws = torch.empty(P.sti_workspace_bytes(wl.dims, B, L, self.precision), dtype=torch.uint8,
                              device="cuda")
        self.staging = torch.empty(P.sti_pipeline_staging_bytes(wl.dims) // 2 * slots, dtype=torch.uint8,
                                   device="cuda")
        self.preload = (torch.empty(preload_bytes, dtype=torch.uint8, device="cuda")
                        if preload_bytes else None)
        self.pipe = P.StiPipeline(wl.dims, self.preload, self.staging)

    def reference(self, x=None, plan=None, store=None):
        x = self.x if x is None else x
        y = self.torch.full_like(x, float("nan"))
        self.P.sti_model_forward(self.wl.dims, self.dev_store if store is None else store, self.params,
                                 self.wl.plan if plan is None else plan, x, y, self.precision, self.ws)
        self.torch.cuda.synchronize()
        return y

    def run(self, x=None, plan=None, store=None, sync=True):
        x = self.x if x is None else x
        y = self.torch.full_like(x, float("nan"))
        stats = self.pipe.forward(self.host_store if store is None else store, self.params,
                                  self.wl.plan if plan is None else plan, x, y, self.precision, self.ws)
        if sync:
            self.torch.cuda.synchronize()
        return y, stats


@pytest.mark.parametrize("prec,dims,B,L", [("f32", SMALL, 2, 37), ("mfma", MID, 3, 70), ("mfma", MID, 8, 128)])
def test_pipeline_matches_model_forward_and_oracle(gpu, oracle_mod, prec, dims, B, L):
    torch = gpu[0]
    wl = S.small_workload(900 + L, dims, 5, B, L, n_absent=1)
    total = sum(plan_bytes(dims, wl.plan))
    rig = Rig(gpu, wl, prec, preload_bytes=total // 3)
    want = oracle_mod.model_forward(dims, wl.shards, wl.params, wl.x)
    ref = rig.reference()
    n_res, b_res = expected_resident(dims, wl.plan, total // 3)
    assert 0 < n_res < len(plan_bytes(dims, wl.plan))

    y, st = rig.run()                      # cold: everything crosses the host link
    assert torch.equal(y, ref)
    assert_parity(y.float().cpu().numpy(), want, TOL[prec])
    assert st["bytes_copied"] == total and st["shards_copied"] == len(plan_bytes(dims, wl.plan))
    assert st["shards_hit"] == 0
    assert st["shards_preloaded"] == n_res and st["bytes_resident"] == b_res

    y, st = rig.run()                      # warm: the preloaded prefix is not copied again
    assert torch.equal(y, ref)
    assert st["shards_hit"] == n_res and st["bytes_copied"] == total - b_res
    assert st["shards_copied"] == len(plan_bytes(dims, wl.plan)) - n_res
    rig.pipe.close()


def test_pipeline_without_preload_buffer(gpu, oracle_mod):
    torch = gpu[0]
    wl = S.small_workload(931, MID, 3, 2, 64)
    rig = Rig(gpu, wl, "mfma", preload_bytes=0)
    ref = rig.reference()
    for _ in range(2):
        y, st = rig.run()
        assert torch.equal(y, ref)
        assert st["shards_hit"] == 0 and st["shards_preloaded"] == 0
        assert st["bytes_copied"] == sum(plan_bytes(MID, wl.plan))
    assert_parity(y.float().cpu().numpy(), oracle_mod.model_forward(MID, wl.shards, wl.params, wl.x), TOL["mfma"])
    rig.pipe.close()


def test_pipeline_reads_ordinary_host_memory(gpu):
    """Streams in pageable memory cannot be read by a kernel; the runtime's copies move them."""
    torch = gpu[0]
    wl = S.small_workload(933, MID, 4, 2, 33, n_absent=1)
    rig = Rig(gpu, wl, "mfma", preload_bytes=sum(plan_bytes(MID, wl.plan)) // 2, host_data="pageable")
    ref = rig.reference()
    y, st = rig.run()
    assert torch.equal(y, ref) and st["bytes_copied"] == sum(plan_bytes(MID, wl.plan))
    y, st = rig.run()
    assert torch.equal(y, ref) and 0 < st["shards_hit"] == st["shards_preloaded"]
    rig.pipe.close()


def test_pipeline_preload_holds_everything(gpu):
    torch = gpu[0]
    wl = S.small_workload(932, SMALL, 4, 1, 19)
    total_padded = sum((b + 255) // 256 * 256 for b in plan_bytes(SMALL, wl.plan))
    rig = Rig(gpu, wl, "f32", preload_bytes=total_padded)
    ref = rig.reference()
    y, st = rig.run()
    assert torch.equal(y, ref) and st["shards_preloaded"] == len(plan_bytes(SMALL, wl.plan))
    y, st = rig.run()
    assert torch.equal(y, ref) and st["bytes_copied"] == 0 and st["shards_copied"] == 0
    rig.pipe.close()


def test_pipeline_plan_change_invalidates_from_the_changed_shard(gpu, oracle_mod):
    """Two versions of every shard; the second plan switches shard (1, 0) to the other
    version: layer 0 stays resident, everything placed after the switch is loaded again."""
    torch, P, D = gpu
    dims = MID
    plan_a = np.array([[3, 4, 2, 6], [5, 0, 4, 3], [2, 2, 6, 0]], dtype=np.int8)
    plan_b = plan_a.copy()
    plan_b[1, 0] = 2
    wl_a = S.small_workload(940, dims, 3, 2, 50, plan=plan_a)
    wl_b = S.small_workload(941, dims, 3, 2, 50, plan=plan_b)
    # one store holding, per shard, version a and (where it differs) version b; parameters of a
    dev_a, params, x = D.upload_workload(wl_a)
    host_a, _, _ = D.upload_workload(wl_a, host_data=True)
    dev_b1 = D.upload_shard(wl_b.shards[1][0])
    host_b1 = D.upload_shard(wl_b.shards[1][0], host_data=True)
    dev_rows, host_rows = D.store_from_plan(dev_a), D.store_from_plan(host_a)
    dev_rows[1][0][2] = dev_b1
    host_rows[1][0][2] = host_b1
    rig = Rig(gpu, wl_a, "mfma", preload_bytes=sum(plan_bytes(dims, plan_a)) + 16 * 256)
    dev_store, host_store = P.make_store(dev_rows), P.make_store(host_rows)

    y, st = rig.run(store=host_store)
    assert torch.equal(y, rig.reference(store=dev_store))
    y, st = rig.run(store=host_store)
    assert st["bytes_copied"] == 0

    ref_b = rig.reference(plan=plan_b, store=dev_store)
    y, st = rig.run(plan=plan_b, store=host_store)
    assert torch.equal(y, ref_b)
    assert st["shards_hit"] == 4                       # layer 0 only
    assert st["bytes_copied"] == sum(plan_bytes(dims, plan_b[1:]))
    # against the oracle: the model of plan b is wl_a with shard (1, 0) replaced
    shards = [list(r) for r in wl_a.shards]
    shards[1][0] = wl_b.shards[1][0]
    want = oracle_mod.model_forward(dims, shards, wl_a.params, wl_a.x)
    assert_parity(y.float().cpu().numpy(), want, TOL["mfma"])
    y, st = rig.run(plan=plan_b, store=host_store)
    assert torch.equal(y, ref_b) and st["bytes_copied"] == 0
    rig.pipe.close()


@pytest.mark.parametrize("slots", [2, 3, 11])
def test_pipeline_back_to_back_calls_without_host_sync(gpu, slots):
    """Calls enqueued one behind the other reuse the staging slots (a ring of 2, of 3, and one
    deeper than the model); each must still see its own layers' weights."""
    torch = gpu[0]
    wl = S.small_workload(950, MID, 7, 4, 96, n_absent=1)
    rig = Rig(gpu, wl, "mfma", preload_bytes=0, slots=slots)
    xs = [rig.x, rig.x * 0.5, -rig.x]
    refs = [rig.reference(x=x) for x in xs]
    outs = [rig.run(x=x, sync=False)[0] for x in xs]
    torch.cuda.synchronize()
    for y, ref in zip(outs, refs):
        assert torch.equal(y, ref)
    rig.pipe.close()


def test_pipeline_outliers_and_io_dtypes(gpu, oracle_mod):
    torch = gpu[0]
    wl = S.small_workload(960, MID, 2, 2, 40, bit_choices=(2, 3, 4), io_dtype="f16")
    rng = np.random.default_rng(5)
    for row in wl.shards:
        for sh in row:
            S.add_outliers(rng, sh, MID.weights_per_shard, fraction=0.01)
    rig = Rig(gpu, wl, "mfma", preload_bytes=1 << 16)
    y, _ = rig.run()
    assert torch.equal(y, rig.reference())
    want = oracle_mod.model_forward(MID, wl.shards, wl.params, wl.x)
    assert_parity(y.float().cpu().numpy(), want, TOL["mfma"])
    rig.pipe.close()


def test_pipeline_config2_full_size(gpu, oracle_mod):
    """BERT-base, mixed 2..6 / 32-bit versions, 3 of 12 shards absent per layer, with a
    preload buffer of about one layer."""
    torch = gpu[0]
    wl = S.config2()
    rig = Rig(gpu, wl, "mfma", preload_bytes=8 << 20)
    ref = rig.reference()
    y, st = rig.run()
    assert torch.equal(y, ref)
    assert st["bytes_copied"] == sum(plan_bytes(wl.dims, wl.plan))
    y, st2 = rig.run()
    assert torch.equal(y, ref)
    n_res, b_res = expected_resident(wl.dims, wl.plan, 8 << 20)
    assert st2["shards_hit"] == n_res > 0 and st2["bytes_copied"] == st["bytes_copied"] - b_res
    want = oracle_mod.model_forward(wl.dims, wl.shards, wl.params, wl.x)
    assert_parity(y.float().cpu().numpy(), want, TOL["mfma"])
    rig.pipe.close()


def test_pipeline_empty_batch_and_zero_layers(gpu):
    torch, P, D = gpu
    wl = S.small_workload(970, SMALL, 2, 1, 5)
    rig = Rig(gpu, wl, "f32", preload_bytes=4096)
    x0 = torch.empty(0, 5, SMALL.d_model, device="cuda")
    y0 = torch.empty_like(x0)
    st = rig.pipe.forward(rig.host_store, rig.params, wl.plan, x0, y0, rig.precision, rig.ws)
    assert st["bytes_copied"] == 0
    y = torch.full_like(rig.x, float("nan"))
    st = rig.pipe.forward(rig.host_store, [], np.zeros((0, SMALL.n_heads), dtype=np.int8), rig.x, y,
                          rig.precision, rig.ws)
    torch.cuda.synchronize()
    assert torch.equal(y, rig.x) and st["bytes_copied"] == 0
    rig.pipe.close()


def test_pipeline_random_models_buffers_and_slots(gpu):
    """Twenty seeded random set-ups (precision, 1-6 layers, tokens, absent shards, preload buffer
    from none to more than everything, 2-8 staging slots, pinned or ordinary host memory): cold,
    warm and unsynchronised back-to-back calls give the bits of sti_model_forward, and the byte
    counts are those of the longest prefix that fits the buffer."""
    torch = gpu[0]
    rng = np.random.default_rng(4711)
    for case in range(20):
        prec = str(rng.choice(["f32", "mfma"]))
        dims = SMALL if prec == "f32" else MID
        n_layers = int(rng.integers(1, 7))
        B, L = int(rng.integers(1, 6)), int(rng.integers(1, 200))
        wl = S.small_workload(5000 + case, dims, n_layers, B, L, n_absent=int(rng.integers(0, dims.n_heads)))
        total = sum(plan_bytes(dims, wl.plan))
        preload = int(rng.choice([0, total // 7, total // 2, total, total + 4096]))
        rig = Rig(gpu, wl, prec, preload_bytes=preload, host_data=bool(rng.random() < 0.8),
                  slots=int(rng.integers(2, 9)))
        ref = rig.reference()
        n_res, b_res = expected_resident(dims, wl.plan, preload)
        y, st = rig.run()
        assert torch.equal(y, ref), case
        assert st["bytes_copied"] == total and st["shards_hit"] == 0, case
        assert st["shards_preloaded"] == n_res and st["bytes_resident"] == b_res, case
        y, st = rig.run()
        assert torch.equal(y, ref), case
        assert st["shards_hit"] == n_res and st["bytes_copied"] == total - b_res, case
        y3, _ = rig.run(sync=False)
        y4, _ = rig.run()
        assert torch.equal(y3, ref) and torch.equal(y4, ref), case
        rig.pipe.close()


@pytest.mark.parametrize("prec", ["f32", "mfma"])
def test_pipeline_rejected_calls_write_nothing_and_keep_the_preload_buffer(gpu, prec):
    """A call rejected for its last layer's plan or for its workspace leaves the output and the
    pipeline's resident shards as they were: the next good call still hits them all."""
    torch, P, D = gpu
    wl = S.small_workload(77, MID, 4, 2, 60, n_absent=1)
    total = sum(plan_bytes(MID, wl.plan))
    rig = Rig(gpu, wl, prec, preload_bytes=total // 2)
    ref = rig.reference()
    n_res, b_res = expected_resident(MID, wl.plan, total // 2)
    y, _ = rig.run()
    assert torch.equal(y, ref)

    def rejected(status, plan=wl.plan, workspace=rig.ws):
        y = torch.full_like(rig.x, float("nan"))
        with pytest.raises(P.StiError) as ei:
            rig.pipe.forward(rig.host_store, rig.params, plan, rig.x, y, rig.precision, workspace)
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
    rejected(6, workspace=rig.ws[:rig.ws.numel() // 2])      # workspace too small
    y, st = rig.run()
    assert torch.equal(y, ref)
    assert st["shards_hit"] == n_res and st["bytes_copied"] == total - b_res
    rig.pipe.close()


@pytest.mark.parametrize("prec", ["f32", "mfma"])
def test_pipeline_padded_sequences(gpu, oracle_mod, prec):
    """sti_pipeline_forward_masked gives the bits of sti_model_forward_masked (and the oracle's
    values), cold and warm."""
    torch, P, D = gpu
    dims = SMALL if prec == "f32" else MID
    B, L = 5, 70
    wl = S.small_workload(91, dims, 3, B, L, n_absent=1)
    S.make_every_term_matter(wl, 9, amp=3.0)
    total = sum(plan_bytes(dims, wl.plan))
    rig = Rig(gpu, wl, prec, preload_bytes=total // 3)
    lens = np.array([L, 1, 33, 64, 17], dtype=np.int32)
    ld = torch.from_numpy(lens).cuda()
    ref = torch.full_like(rig.x, float("nan"))
    P.sti_model_forward_masked(dims, rig.dev_store, rig.params, wl.plan, rig.x, ref, ld, rig.precision, rig.ws)
    torch.cuda.synchronize()
    want = oracle_mod.model_forward(dims, wl.shards, wl.params, wl.x, key_lengths=lens)
    assert_parity(ref.float().cpu().numpy(), want, TOL[prec])
    for _ in range(2):
        y = torch.full_like(rig.x, float("nan"))
        rig.pipe.forward(rig.host_store, rig.params, wl.plan, rig.x, y, rig.precision, rig.ws, key_lengths=ld)
        torch.cuda.synchronize()
        assert torch.equal(y, ref)
    assert not torch.equal(rig.run()[0], ref)      # the plain call differs
    rig.pipe.close()
