"""GPU: profile the delays (Section "Prerequisite: Offline Profiling"), plan a submodel for a
deadline (Sections "Compute Planning", "IO Planning"), and execute the plan through the
load || compute pipeline; the result must match the CPU oracle's forward of the same plan."""
import numpy as np
import pytest

import sti_synth as S

pytestmark = pytest.mark.gpu

MID = S.Dims(128, 4, 64, 64, 1e-12)


def test_profile_plan_execute(oracle_mod):
    import torch
    import paper_2207_05022_amd as P
    from paper_2207_05022_amd import device as D, profiling
    from oracle import sti_planner_oracle as O
    prec = P.STI_PREC_F16_MFMA
    N, M, B, L = 6, MID.n_heads, 4, 64
    t_io = profiling.measure_t_io(MID)
    t_comp = profiling.measure_t_comp(MID, B, L, prec)
    assert len(t_io) == 6 and len(t_comp) == M and min(t_io) > 0 and min(t_comp) > 0
    assert t_io[5] > t_io[0]                                   # 32-bit shards take longer to move than 2-bit ones
    deadline = 4.5 * t_comp[-1]                                 # room for four full layers, not for six
    n, m = P.sti_plan_submodel(t_io, t_comp, N, deadline)
    assert (n, m) == O.plan_submodel(t_comp, N, deadline) and 0 < n < N
    pre = np.zeros((N, M), dtype=np.int8)
    pre[0, :] = 2                                               # the preload buffer holds layer 0 at 2 bits
    importance = np.random.default_rng(3).permutation(N * M).astype(np.int32)
    plan, aib = P.sti_plan_bitwidths(t_io, t_comp, N, n, m, pre, importance)
    want_plan, _ = O.plan_bitwidths(t_io, t_comp, N, M, n, m, pre.ravel().tolist(), importance.tolist())
    assert plan.ravel().tolist() == want_plan and (aib >= -1e-9).all()

    # execute layers 0..n-1 of the plan with the shard streams in pinned host memory
    sub = plan[:n]
    wl = S.small_workload(4242, MID, n, B, L, plan=sub, io_dtype="f16")
    host, params, x = D.upload_workload(wl, host_data=True)
    store = P.make_store(D.store_from_plan(host))
    ws = torch.empty(P.sti_workspace_bytes(MID, B, L, prec), dtype=torch.uint8, device="cuda")
    staging = torch.empty(P.sti_pipeline_staging_bytes(MID), dtype=torch.uint8, device="cuda")
    preload = torch.empty(M * MID.weights_per_shard, dtype=torch.uint8, device="cuda")   # > layer 0 at 2 bits
    pipe = P.StiPipeline(MID, preload, staging)
    y = torch.full_like(x, float("nan"))
    pipe.forward(store, params, sub, x, y, prec, ws)            # fills the preload buffer
    st = pipe.forward(store, params, sub, x, y, prec, ws)
    torch.cuda.synchronize()
    assert st["shards_hit"] >= int((sub[0] != 0).sum())         # layer 0 is served from the preload buffer
    want = oracle_mod.model_forward(MID, wl.shards, wl.params, wl.x)
    got = y.float().cpu().numpy()
    assert float(np.max(np.abs(got - want)) / np.max(np.abs(want))) <= 2e-2
    pipe.close()
