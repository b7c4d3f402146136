"""Host-side checks of the C ABI: the shared library loads, exports every entry point that
include/sti.h declares, and rejects bad arguments before touching the device.  No kernel runs."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def P():
    lib = os.path.join(ROOT, "paper_2207_05022_amd", "libsti.so")
    if not os.path.exists(lib):
        import importlib.util
        spec = importlib.util.spec_from_file_location(
            "_sti_build", os.path.join(ROOT, "paper_2207_05022_amd", "build.py"))
        mod = importlib.util.module_from_spec(spec)
        spec.loader.exec_module(mod)
        mod.build()
    import paper_2207_05022_amd as pkg
    return pkg


def declared_functions():
    text = open(os.path.join(ROOT, "include", "sti.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sti_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(P):
    names = declared_functions()
    assert {"sti_decode_shards", "sti_layer_forward", "sti_model_forward", "sti_workspace_bytes",
            "sti_decode_workspace_bytes", "sti_status_string"} <= set(names)
    for n in names:
        assert hasattr(P.lib, n), n


def test_phase_stamp_build_exports_the_same_boundary(P):
    """libsti_phases.so (bench.py --phase-budget loads it through STI_LIBRARY) is the library with
    clock stamps compiled into one kernel: same boundary, plus the call that reads the stamps,
    which the product library does not have."""
    import ctypes as C
    L = C.CDLL(os.path.join(ROOT, "paper_2207_05022_amd", "libsti_phases.so"))
    for n in declared_functions():
        assert hasattr(L, n), n
    assert hasattr(L, "sti_phase_stamps_read") and not hasattr(P.lib, "sti_phase_stamps_read")


def test_status_strings(P):
    seen = {P.status_string(i) for i in range(10)}
    assert len(seen) == 10 and "ok" in seen
    assert P.status_string(99) == "unknown status"


FAKE = 0x1000  # aligned, never dereferenced: all checks below fail before any launch


def shard(P, bits, data=FAKE, cb=FAKE, nout=0):
    return P.StiShard(bits, data, cb, nout, None, None)


def decode(P, shards, n=8, out=FAKE, dtype=1, ws=None, ws_bytes=0):
    arr = (P.StiShard * max(1, len(shards)))(*shards)
    return P.lib.sti_decode_shards(arr, len(shards), n, out, dtype, ws, ws_bytes, None)


def test_decode_argument_errors(P):
    assert decode(P, [shard(P, 7)]) == 3                      # bitwidth
    assert decode(P, [shard(P, 0)]) == 3                      # absent is not decodable
    assert decode(P, [shard(P, 1)]) == 3
    assert decode(P, [shard(P, 4, data=None)]) == 4           # missing data
    assert decode(P, [shard(P, 4, cb=None)]) == 4             # missing codebook
    assert decode(P, [shard(P, 4, data=FAKE + 8)]) == 5       # stream alignment
    assert decode(P, [shard(P, 4, cb=FAKE + 2)]) == 5
    assert decode(P, [shard(P, 4)], out=FAKE + 4) == 5
    assert decode(P, [shard(P, 4)], out=None) == 1
    assert decode(P, [shard(P, 4)], dtype=5) == 7
    assert decode(P, [shard(P, 4, nout=3)]) == 1              # outlier arrays missing
    assert decode(P, [P.StiShard(32, FAKE, None, 3, FAKE, FAKE)]) == 9   # raw shards have no dictionary
    assert decode(P, [P.StiShard(4, FAKE, FAKE, 3, FAKE + 2, FAKE)]) == 5
    assert P.lib.sti_decode_shards(None, 3, 8, FAKE, 1, None, 0, None) == 1
    assert P.lib.sti_decode_shards(None, -1, 8, FAKE, 1, None, 0, None) == 2
    assert P.lib.sti_decode_shards(None, 0, 8, FAKE, 1, None, 0, None) == 0
    many = [shard(P, 3)] * 100
    assert P.sti_decode_workspace_bytes(100) > 0 and P.sti_decode_workspace_bytes(64) == 0
    assert decode(P, many) == 6                               # workspace missing
    assert decode(P, many, ws=FAKE, ws_bytes=8) == 6          # workspace too small
    assert decode(P, [shard(P, 32, cb=None)], n=0) == 0       # nothing to do


class Dims:
    def __init__(self, d=768, M=12, dh=64, f=256, eps=1e-12):
        self.d_model, self.n_heads, self.d_head, self.ffn_per_shard, self.ln_eps = d, M, dh, f, eps


def test_model_workspace_query(P):
    one = P.sti_workspace_bytes(Dims(), 32, 128, P.STI_PREC_F16_MFMA)
    whole = P.sti_model_workspace_bytes(Dims(), 12, 32, 128, P.STI_PREC_F16_MFMA)
    layer = 12 * 589824 * 2
    # a ring of four binary16 working buffers (64 MiB worth of layers) + the model's shard table
    assert one + 3 * layer + 12 * 12 * 48 <= whole < one + 4 * layer
    # never fewer than two buffers: a layer is decompressed while the one before it computes
    big = Dims(d=2048, M=32)
    assert (P.sti_model_workspace_bytes(big, 3, 2, 128, P.STI_PREC_F16_MFMA) - P.sti_workspace_bytes(big, 2, 128, P.STI_PREC_F16_MFMA)
            >= 32 * 2048 * 768 * 2)
    assert P.sti_model_workspace_bytes(Dims(), 1, 32, 128, P.STI_PREC_F16_MFMA) == one
    assert P.sti_model_workspace_bytes(Dims(), 12, 32, 128, P.STI_PREC_F32) == P.sti_workspace_bytes(Dims(), 32, 128, P.STI_PREC_F32)
    assert P.sti_model_workspace_bytes(Dims(), -1, 32, 128, P.STI_PREC_F16_MFMA) == 0


def test_workspace_query(P):
    assert P.sti_workspace_bytes(Dims(), 1, 128, P.STI_PREC_F32) > 12 * 589824 * 4
    assert P.sti_workspace_bytes(Dims(), 32, 128, P.STI_PREC_F16_MFMA) > 0
    assert P.sti_workspace_bytes(Dims(), 0, 128, P.STI_PREC_F32) >= 256
    assert P.sti_workspace_bytes(Dims(d=0), 1, 8, 0) == 0
    assert P.sti_workspace_bytes(Dims(M=65), 1, 8, 0) == 0
    assert P.sti_workspace_bytes(Dims(), -1, 8, 0) == 0
    assert P.sti_workspace_bytes(Dims(), 1, 8, 3) == 0
    assert P.sti_workspace_bytes(Dims(dh=32), 1, 8, P.STI_PREC_F16_MFMA) == 0     # needs d_head 64
    assert P.sti_workspace_bytes(Dims(d=100), 1, 8, P.STI_PREC_F16_MFMA) == 0
    assert P.sti_workspace_bytes(Dims(), 1, 513, P.STI_PREC_F16_MFMA) == 0
    assert P.sti_workspace_bytes(Dims(d=100, dh=10, f=7), 2, 9, P.STI_PREC_F32) > 0


def layer(P, dims=None, shards=None, params="ok", x=FAKE, y=FAKE + 0x100000, io=0, batch=1, seq=8,
          prec=0, ws=FAKE + 0x200000, ws_bytes=1 << 40):
    d = P.binding.make_dims(dims or Dims(d=64, M=2, dh=64, f=64))
    shards = shards if shards is not None else [shard(P, 4), shard(P, 0, None, None)]
    arr = (P.StiShard * len(shards))(*shards)
    prm = P.StiLayerParams(*([FAKE] * 10)) if params == "ok" else params
    return P.lib.sti_layer_forward(C.byref(d), arr, C.byref(prm) if prm is not None else None, x, y, io,
                                   batch, seq, prec, ws, ws_bytes, None)


def test_layer_argument_errors(P):
    assert layer(P, shards=[shard(P, 9), shard(P, 4)]) == 3
    assert layer(P, shards=[shard(P, 4, data=None), shard(P, 4)]) == 4
    assert layer(P, params=None) == 1
    bad = P.StiLayerParams(*([FAKE] * 9 + [None]))
    assert layer(P, params=bad) == 1
    assert layer(P, x=None) == 1
    assert layer(P, x=FAKE + 4) == 5
    assert layer(P, y=FAKE) == 2                    # x and y alias
    assert layer(P, io=7) == 7
    assert layer(P, prec=2) == 7
    assert layer(P, batch=-1) == 2
    assert layer(P, ws=None) == 6
    assert layer(P, ws_bytes=16) == 6
    assert layer(P, ws=FAKE + 0x200010) == 5
    assert layer(P, dims=Dims(d=64, M=2, dh=32, f=64), prec=1) == 2
    assert layer(P, batch=0) == 0                   # empty batch: nothing to do


def test_masked_layer_argument_errors(P):
    d = P.binding.make_dims(Dims(d=64, M=2, dh=64, f=64))
    arr = (P.StiShard * 2)(shard(P, 4), shard(P, 0, None, None))
    prm = P.StiLayerParams(*([FAKE] * 10))

    def call(lengths, batch=1, x=FAKE):
        return P.lib.sti_layer_forward_masked(C.byref(d), arr, C.byref(prm), x, FAKE + 0x100000, 0, batch, 8,
                                              lengths, 0, None, 0, None)

    assert call(None) == 1                          # key lengths are required ...
    assert call(None, batch=0) == 6                 # ... unless there are no tokens (then: workspace)
    assert call(FAKE + 2) == 5                      # 4-byte alignment
    assert call(FAKE + 4) == 6                      # accepted; the missing workspace is next
    assert call(FAKE + 4, x=None) == 1              # the checks of the plain entry point still apply


def test_model_argument_errors(P):
    d = P.binding.make_dims(Dims(d=64, M=2, dh=64, f=64))
    store = (P.StiShard * 12)(*[shard(P, k) for k in (2, 3, 4, 5, 6, 32)] * 2)
    prm = (P.StiLayerParams * 1)(P.StiLayerParams(*([FAKE] * 10)))

    def call(plan, store=store, n_layers=1):
        pl = np.asarray(plan, dtype=np.int8)
        return P.lib.sti_model_forward(C.byref(d), n_layers, store, prm,
                                       pl.ctypes.data_as(C.POINTER(C.c_int8)), FAKE, FAKE + 0x100000, 0,
                                       1, 8, 0, None, 0, None)

    assert call([4, 7]) == 3                        # plan bitwidth
    assert call([4, 0]) == 6                        # valid plan, then workspace is missing
    missing = (P.StiShard * 12)(*[shard(P, k, data=None) for k in (2, 3, 4, 5, 6, 32)] * 2)
    assert call([4, 0], store=missing) == 4         # selected version not stored
    wrong = (P.StiShard * 12)(*[shard(P, 5) for _ in range(12)])
    assert call([4, 0], store=wrong) == 3           # slot holds another bitwidth
    assert call([4, 0], n_layers=-1) == 2


def test_pipeline_argument_errors(P):
    """Everything sti_pipeline_create rejects is rejected before a stream is created."""
    d = P.binding.make_dims(Dims(d=768, M=12, dh=64, f=256))
    need = P.lib.sti_pipeline_staging_bytes(C.byref(d))
    assert need == 2 * 12 * 768 * (4 * 64 + 2 * 256) * 4      # two slots of one full-precision layer
    assert P.lib.sti_pipeline_staging_bytes(None) == 0
    bad = P.binding.make_dims(Dims(d=768, M=0, dh=64, f=256))
    assert P.lib.sti_pipeline_staging_bytes(C.byref(bad)) == 0
    h = C.c_void_p()
    create = P.lib.sti_pipeline_create
    assert create(None, None, 0, FAKE, need, C.byref(h)) == 1
    assert create(C.byref(d), None, 0, FAKE, need, None) == 1
    assert create(C.byref(bad), None, 0, FAKE, need, C.byref(h)) == 2
    assert create(C.byref(d), None, 0, FAKE, need - 1, C.byref(h)) == 6
    assert create(C.byref(d), None, 0, None, need, C.byref(h)) == 6
    assert create(C.byref(d), None, 4096, FAKE, need, C.byref(h)) == 1     # bytes without a buffer
    assert create(C.byref(d), FAKE + 8, 4096, FAKE, need, C.byref(h)) == 5
    assert create(C.byref(d), None, 0, FAKE + 16, need, C.byref(h)) == 5
    assert not h.value
    assert P.lib.sti_pipeline_forward(None, 0, None, None, None, None, None, 0, 0, 0, 0, None, 0, None,
                                      None) == 1
    assert P.lib.sti_pipeline_destroy(None) == 0


def test_quantizer_argument_errors(P):
    d = P.binding.make_dims(Dims(d=768, M=12, dh=64, f=256))
    assert P.lib.sti_quantize_workspace_bytes(C.byref(d)) > 62 * 65536 * 4
    odd = P.binding.make_dims(Dims(d=24, M=2, dh=8, f=8))       # Wsh = 1152: not a multiple of 1024
    assert P.lib.sti_quantize_workspace_bytes(C.byref(odd)) == 0
    q = P.lib.sti_quantize_layer
    args = lambda dims=d, w=FAKE, k=4, thr=-4.0, reg=1e-6, packed=FAKE, cb=FAKE, pos=FAKE, val=FAKE, mx=8, cnt=FAKE, ws=FAKE, wsb=1 << 40: \
        (C.byref(dims), w, k, thr, reg, packed, cb, pos, val, mx, cnt, None, ws, wsb, None)
    assert q(*args(w=None)) == 1
    assert q(*args(cnt=None)) == 1
    assert q(*args(pos=None)) == 1
    assert q(*args(k=7)) == 3 and q(*args(k=32)) == 3
    assert q(*args(dims=odd)) == 9
    assert q(*args(reg=-1.0)) == 2 and q(*args(thr=float("nan"))) == 2
    assert q(*args(w=FAKE + 4)) == 5
    assert q(*args(ws=None)) == 6 and q(*args(wsb=1024)) == 6


def test_working_buffer_layout_is_a_permutation_of_the_shard(P):
    """Host arithmetic only: every weight of a shard has a place of its own inside the shard's image,
    sub-blocks stay inside their own range, and 8 consecutive columns stay consecutive."""
    import sti_synth as S
    dims = S.Dims(128, 3, 64, 192, 1e-12)
    n = dims.weights_per_shard
    d = P.binding.make_dims(dims)
    off = np.array([P.lib.sti_working_buffer_offset(C.byref(d), j) for j in range(n)])
    assert np.array_equal(np.sort(off), np.arange(n))
    bounds = [0, 3 * 64 * 128, 4 * 64 * 128, 4 * 64 * 128 + 192 * 128, n]
    for a, b in zip(bounds[:-1], bounds[1:]):
        assert off[a:b].min() == a and off[a:b].max() == b - 1
    assert np.all(np.diff(off.reshape(-1, 8), axis=1) == 1)
    assert P.lib.sti_working_buffer_offset(C.byref(d), n) == -1
    bad = P.binding.make_dims(S.Dims(100, 3, 64, 192, 1e-12))
    assert P.lib.sti_working_buffer_offset(C.byref(bad), 0) == -1
    assert P.lib.sti_working_buffer_bytes(C.byref(bad)) == 0
    assert P.lib.sti_working_buffer_bytes(C.byref(d)) == 3 * n * 2
    arr = (P.StiShard * 3)(shard(P, 4), shard(P, 0), shard(P, 9))
    assert P.lib.sti_decode_working_buffer(C.byref(d), arr, FAKE, 1 << 30, None) == 3
    arr = (P.StiShard * 3)(shard(P, 4), shard(P, 0), shard(P, 2))
    assert P.lib.sti_decode_working_buffer(C.byref(d), arr, FAKE, 8, None) == 6
    assert P.lib.sti_decode_working_buffer(C.byref(d), arr, None, 1 << 30, None) == 1
    assert P.lib.sti_decode_working_buffer(C.byref(d), None, FAKE, 1 << 30, None) == 1
