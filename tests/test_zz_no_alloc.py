"""GPU test of sti_layer_forward_static: the layer for callers that cannot allocate, whose workspace is
a fixed array inside the library's device image.  Through the C ABI (raw ctypes), against
sti_layer_forward with a caller workspace (same kernels: the very bits) and against the CPU oracle, on
two calls in a row of which the second is smaller, so that what the first call left in the array
is there when the second runs."""
import ctypes as C

import numpy as np
import pytest

import sti_synth as S
from parity import assert_parity

pytestmark = pytest.mark.gpu

TOL = {0: 1e-5, 1: 2e-2}


@pytest.fixture(scope="module")
def gpu():
    import torch
    import paper_2207_05022_amd as P
    from paper_2207_05022_amd import device as D
    assert torch.cuda.is_available(), "needs a GPU"
    return torch, P, D


def _call_both(gpu, wl, prec):
    """(static entry point's y, sti_layer_forward's y) for a one-layer workload."""
    torch, P, D = gpu
    shards, params, x = D.upload_workload(wl)
    d = P.binding.make_dims(wl.dims)
    arr = P.shard_array(shards[0])
    prm = P.binding.make_params(params[0])
    B, L = int(x.shape[0]), int(x.shape[1])
    io = {torch.float32: 0, torch.float16: 1}[x.dtype]
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    y_static = torch.full_like(x, float("nan"))
    st = P.lib.sti_layer_forward_static(C.byref(d), arr, C.byref(prm), x.data_ptr(), y_static.data_ptr(), io, B, L,
                                        prec, stream)
    assert st == 0, P.status_string(st)
    nbytes = P.lib.sti_workspace_bytes(C.byref(d), B, L, prec)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    y_ws = torch.full_like(x, float("nan"))
    st = P.lib.sti_layer_forward(C.byref(d), arr, C.byref(prm), x.data_ptr(), y_ws.data_ptr(), io, B, L, prec,
                                 ws.data_ptr(), nbytes, stream)
    assert st == 0, P.status_string(st)
    torch.cuda.synchronize()
    return y_static, y_ws


@pytest.mark.parametrize("prec", [1, 0], ids=["mfma", "f32"])
def test_two_calls_in_a_row_the_second_smaller(gpu, oracle_mod, prec):
    torch, P, D = gpu
    io = "f16" if prec == 1 else "f32"
    # first: configuration 0's dimensions with five sequences (working-buffer route on the matrix cores),
    # mixed bitwidths with one shard absent and outlier dictionaries; second: one short sequence
    # (few-token route) of a smaller model, which reuses the front of the array
    big = S.small_workload(51, S.BERT_BASE, 1, 5, 128, n_absent=1, io_dtype=io)
    rng = np.random.default_rng(8)
    for s in big.shards[0]:
        if s is not None and s.bitwidth != 32:
            S.add_outliers(rng, s, big.dims.weights_per_shard, 0.002)
    small = S.small_workload(52, S.Dims(128, 4, 64, 64, 1e-12), 1, 1, 40, n_absent=1, io_dtype=io)
    S.make_every_term_matter(small, 3)
    for wl in (big, small):
        y_static, y_ws = _call_both(gpu, wl, prec)
        assert torch.equal(y_static, y_ws)
        want = oracle_mod.layer_forward(wl.dims, wl.shards[0], wl.params[0], wl.x)
        assert_parity(y_static.float().cpu().numpy(), want, TOL[prec])


def test_sizes_beyond_the_array_are_refused_and_nothing_is_written(gpu):
    torch, P, D = gpu
    assert P.lib.sti_static_scratch_bytes() == 64 << 20
    dims = S.Dims(2048, 32, 64, 256, 1e-12)
    d = P.binding.make_dims(dims)
    assert P.lib.sti_workspace_bytes(C.byref(d), 1, 64, 1) > P.lib.sti_static_scratch_bytes()
    wl = S.small_workload(5, dims, 1, 1, 64, io_dtype="f16")
    shards, params, x = D.upload_workload(wl)
    y = torch.zeros_like(x)
    prm = P.binding.make_params(params[0])
    st = P.lib.sti_layer_forward_static(C.byref(d), P.shard_array(shards[0]), C.byref(prm), x.data_ptr(),
                                        y.data_ptr(), 1, 1, 64, 1, C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert st == 6   # STI_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert not y.any()
