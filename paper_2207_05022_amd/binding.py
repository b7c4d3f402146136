"""ctypes marshalling for the C ABI declared in include/sti.h.

Device buffers are ``torch`` CUDA tensors (PyTorch-ROCm is used only to own
device memory and streams); their ``data_ptr()`` and the current stream's
handle are what crosses the boundary.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
# STI_LIBRARY names another build of the same sources to load instead (the build with phase time
# stamps that bench.py --phase-budget measures with); unset, the product library beside this file
LIB_PATH = os.environ.get("STI_LIBRARY") or os.path.join(HERE, "libsti.so")

STI_F32, STI_F16, STI_BF16 = 0, 1, 2
STI_PREC_F32, STI_PREC_F16_MFMA = 0, 1
VERSION_SLOTS = (2, 3, 4, 5, 6, 32)


class StiDims(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("n_heads", C.c_int32), ("d_head", C.c_int32),
                ("ffn_per_shard", C.c_int32), ("ln_eps", C.c_float)]


class StiShard(C.Structure):
    _fields_ = [("bitwidth", C.c_int8), ("data", C.c_void_p), ("codebook", C.c_void_p),
                ("n_outliers", C.c_uint32), ("outlier_pos", C.c_void_p),
                ("outlier_val", C.c_void_p)]


class StiLayerParams(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("bq", "bk", "bv", "bo", "b1", "b2", "ln1_g", "ln1_b", "ln2_g", "ln2_b")]


KERNEL_CLASSES = ("decode", "gemm_qkv", "attention", "gemm_out", "layernorm", "gemm_ffn_up",
                  "gemm_ffn_down", "convert")


class StiProfile(C.Structure):
    _fields_ = [("launches", C.c_uint64 * 8), ("ms", C.c_double * 8)]


class StiPipelineStats(C.Structure):
    _fields_ = [("bytes_copied", C.c_uint64), ("bytes_resident", C.c_uint64),
                ("shards_copied", C.c_uint32), ("shards_hit", C.c_uint32),
                ("shards_preloaded", C.c_uint32)]


class StiPlanTables(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_shards", C.c_int32), ("t_io", C.c_double * 6),
                ("t_comp", C.POINTER(C.c_double))]


class StiQuantStats(C.Structure):
    _fields_ = [("mean", C.c_double), ("variance", C.c_double), ("n_outliers", C.c_uint64), ("status", C.c_uint32)]


class StiError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({status_string(status)})")


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build the HIP library first "
            "(python paper_2207_05022_amd/build.py); there is no CPU fallback")
    L = C.CDLL(LIB_PATH)
    L.sti_status_string.restype = C.c_char_p
    L.sti_status_string.argtypes = [C.c_int]
    L.sti_decode_workspace_bytes.restype = C.c_size_t
    L.sti_decode_workspace_bytes.argtypes = [C.c_int]
    L.sti_decode_shards.restype = C.c_int
    L.sti_decode_shards.argtypes = [C.POINTER(StiShard), C.c_int, C.c_uint64, C.c_void_p, C.c_int,
                                    C.c_void_p, C.c_size_t, C.c_void_p]
    L.sti_workspace_bytes.restype = C.c_size_t
    L.sti_workspace_bytes.argtypes = [C.POINTER(StiDims), C.c_int, C.c_int, C.c_int]
    L.sti_layer_forward.restype = C.c_int
    L.sti_layer_forward.argtypes = [
        C.POINTER(StiDims), C.POINTER(StiShard), C.POINTER(StiLayerParams), C.c_void_p,
        C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]
    L.sti_layer_forward_masked.restype = C.c_int
    L.sti_layer_forward_masked.argtypes = [
        C.POINTER(StiDims), C.POINTER(StiShard), C.POINTER(StiLayerParams), C.c_void_p,
        C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]
    L.sti_model_forward_masked.restype = C.c_int
    L.sti_model_forward_masked.argtypes = [
        C.POINTER(StiDims), C.c_int, C.POINTER(StiShard), C.POINTER(StiLayerParams),
        C.POINTER(C.c_int8), C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_int,
        C.c_void_p, C.c_size_t, C.c_void_p]
    L.sti_model_forward.restype = C.c_int
    L.sti_model_forward.argtypes = [
        C.POINTER(StiDims), C.c_int, C.POINTER(StiShard), C.POINTER(StiLayerParams),
        C.POINTER(C.c_int8), C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int,
        C.c_void_p, C.c_size_t, C.c_void_p]
    L.sti_static_scratch_bytes.restype = C.c_size_t
    L.sti_static_scratch_bytes.argtypes = []
    L.sti_layer_forward_static.restype = C.c_int
    L.sti_layer_forward_static.argtypes = [
        C.POINTER(StiDims), C.POINTER(StiShard), C.POINTER(StiLayerParams), C.c_void_p,
        C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p]
    L.sti_working_buffer_bytes.restype = C.c_size_t
    L.sti_working_buffer_bytes.argtypes = [C.POINTER(StiDims)]
    L.sti_working_buffer_offset.restype = C.c_int64
    L.sti_working_buffer_offset.argtypes = [C.POINTER(StiDims), C.c_uint64]
    L.sti_decode_working_buffer.restype = C.c_int
    L.sti_decode_working_buffer.argtypes = [C.POINTER(StiDims), C.POINTER(StiShard), C.c_void_p, C.c_size_t,
                                            C.c_void_p]
    L.sti_quantize_workspace_bytes.restype = C.c_size_t
    L.sti_quantize_workspace_bytes.argtypes = [C.POINTER(StiDims)]
    L.sti_quantize_layer.restype = C.c_int
    L.sti_quantize_layer.argtypes = [C.POINTER(StiDims), C.c_void_p, C.c_int, C.c_double, C.c_double, C.c_void_p,
                                     C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_size_t, C.c_void_p]
    L.sti_plan_submodel.restype = C.c_int
    L.sti_plan_submodel.argtypes = [C.POINTER(StiPlanTables), C.c_double, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    L.sti_plan_bitwidths.restype = C.c_int
    L.sti_plan_bitwidths.argtypes = [C.POINTER(StiPlanTables), C.c_int32, C.c_int32, C.POINTER(C.c_int8),
                                     C.POINTER(C.c_int32), C.POINTER(C.c_int8), C.POINTER(C.c_double)]
    L.sti_model_workspace_bytes.restype = C.c_size_t
    L.sti_model_workspace_bytes.argtypes = [C.POINTER(StiDims), C.c_int, C.c_int, C.c_int, C.c_int]
    L.sti_pipeline_staging_bytes.restype = C.c_size_t
    L.sti_pipeline_staging_bytes.argtypes = [C.POINTER(StiDims)]
    L.sti_pipeline_create.restype = C.c_int
    L.sti_pipeline_create.argtypes = [C.POINTER(StiDims), C.c_void_p, C.c_size_t, C.c_void_p,
                                      C.c_size_t, C.POINTER(C.c_void_p)]
    L.sti_pipeline_forward_masked.restype = C.c_int
    L.sti_pipeline_forward_masked.argtypes = [
        C.c_void_p, C.c_int, C.POINTER(StiShard), C.POINTER(StiLayerParams), C.POINTER(C.c_int8),
        C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_int, C.c_void_p, C.c_size_t,
        C.c_void_p, C.POINTER(StiPipelineStats)]
    L.sti_pipeline_forward.restype = C.c_int
    L.sti_pipeline_forward.argtypes = [
        C.c_void_p, C.c_int, C.POINTER(StiShard), C.POINTER(StiLayerParams), C.POINTER(C.c_int8),
        C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_size_t,
        C.c_void_p, C.POINTER(StiPipelineStats)]
    L.sti_pipeline_destroy.restype = C.c_int
    L.sti_pipeline_destroy.argtypes = [C.c_void_p]
    L.sti_profile_begin.restype = C.c_int
    L.sti_profile_begin.argtypes = []
    L.sti_profile_end.restype = C.c_int
    L.sti_profile_end.argtypes = [C.POINTER(StiProfile)]
    return L


lib = _load()


def status_string(status: int) -> str:
    return lib.sti_status_string(int(status)).decode()


def _dtype_code(t) -> int:
    import torch
    return {torch.float32: STI_F32, torch.float16: STI_F16, torch.bfloat16: STI_BF16}[t.dtype]


def _stream_handle(stream) -> Optional[int]:
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def make_dims(dims) -> StiDims:
    """dims: any object with d_model, n_heads, d_head, ffn_per_shard, ln_eps."""
    if isinstance(dims, StiDims):
        return dims
    return StiDims(dims.d_model, dims.n_heads, dims.d_head, dims.ffn_per_shard, dims.ln_eps)


def make_shard(bitwidth: int, data=None, codebook=None, outlier_pos=None, outlier_val=None) -> StiShard:
    """data / codebook: CUDA tensors (uint8 stream or float32 weights; float32 centroids);
    outlier_pos / outlier_val: optional CUDA int32 offsets and float32 weights."""
    n_out = 0 if outlier_pos is None else int(outlier_pos.numel())
    return StiShard(int(bitwidth), _ptr(data), _ptr(codebook), n_out,
                    _ptr(outlier_pos) if n_out else None, _ptr(outlier_val) if n_out else None)


def make_params(p) -> StiLayerParams:
    """p: object with CUDA float32 tensors bq, bk, bv, bo, b1, b2, ln1_g, ln1_b, ln2_g, ln2_b."""
    if isinstance(p, StiLayerParams):
        return p
    return StiLayerParams(*[_ptr(getattr(p, n)) for n, _ in StiLayerParams._fields_])


def shard_array(shards: Sequence) -> "C.Array":
    """HOST array of sti_shard from shard objects (.bitwidth/.data/.codebook CUDA tensors, optional
    .outlier_pos/.outlier_val; None = absent).  Building it once saves the marshalling per call."""
    if isinstance(shards, C.Array):
        return shards
    arr = (StiShard * max(1, len(shards)))()
    for i, s in enumerate(shards):
        if s is None:
            arr[i] = StiShard(0, None, None, 0, None, None)
        elif isinstance(s, StiShard):
            arr[i] = s
        else:
            arr[i] = make_shard(s.bitwidth, s.data, s.codebook, getattr(s, "outlier_pos", None),
                                getattr(s, "outlier_val", None))
    return arr


def sti_decode_workspace_bytes(n_shards: int) -> int:
    return int(lib.sti_decode_workspace_bytes(int(n_shards)))


def sti_decode_shards(shards: Sequence, weights_per_shard: int, out, workspace=None,
                      stream=None) -> None:
    """Decode ``shards`` into ``out`` (CUDA tensor of float32/float16/bfloat16 with
    len(shards) * weights_per_shard elements)."""
    arr = shard_array(shards)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = lib.sti_decode_shards(arr, len(shards), int(weights_per_shard), _ptr(out),
                               _dtype_code(out), _ptr(workspace), ws_bytes, _stream_handle(stream))
    if st != 0:
        raise StiError(st, "sti_decode_shards")


def sti_working_buffer_bytes(dims) -> int:
    d = make_dims(dims)
    return int(lib.sti_working_buffer_bytes(C.byref(d)))


def sti_working_buffer_offset(dims, j: int) -> int:
    d = make_dims(dims)
    return int(lib.sti_working_buffer_offset(C.byref(d), int(j)))


def sti_decode_working_buffer(dims, shards: Sequence, out, stream=None) -> None:
    """shards: M entries, None = absent; out: CUDA float16 tensor for the present shards' images."""
    d = make_dims(dims)
    arr = shard_array(shards)
    st = lib.sti_decode_working_buffer(C.byref(d), arr, _ptr(out), out.numel() * out.element_size(),
                                       _stream_handle(stream))
    if st != 0:
        raise StiError(st, "sti_decode_working_buffer")


def sti_workspace_bytes(dims, batch: int, seq: int, precision: int) -> int:
    d = make_dims(dims)
    return int(lib.sti_workspace_bytes(C.byref(d), int(batch), int(seq), int(precision)))


def sti_model_workspace_bytes(dims, n_layers: int, batch: int, seq: int, precision: int) -> int:
    d = make_dims(dims)
    return int(lib.sti_model_workspace_bytes(C.byref(d), int(n_layers), int(batch), int(seq), int(precision)))


def _key_lengths_ptr(key_lengths, batch: int):
    """key_lengths: CUDA int32 tensor [batch] (None passes a null pointer through)."""
    if key_lengths is None:
        return None
    import torch
    if key_lengths.dtype != torch.int32 or tuple(key_lengths.shape) != (batch,):
        raise ValueError("key_lengths must be an int32 tensor with one entry per sequence")
    return _ptr(key_lengths)


def sti_layer_forward(dims, shards: Sequence, params, x, y, precision: int, workspace,
                      stream=None) -> None:
    """x, y: CUDA tensors [batch, seq, d_model] of one dtype; shards: M entries, None = absent."""
    d = make_dims(dims)
    arr = shard_array(shards)
    p = make_params(params)
    batch, seq = int(x.shape[0]), int(x.shape[1])
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = lib.sti_layer_forward(C.byref(d), arr, C.byref(p), _ptr(x), _ptr(y), _dtype_code(x),
                               batch, seq, int(precision), _ptr(workspace), ws_bytes,
                               _stream_handle(stream))
    if st != 0:
        raise StiError(st, "sti_layer_forward")


def sti_layer_forward_static(dims, shards: Sequence, params, x, y, precision: int, stream=None) -> None:
    """sti_layer_forward with the library's own fixed scratch array as workspace (no allocation)."""
    d = make_dims(dims)
    arr = shard_array(shards)
    p = make_params(params)
    st = lib.sti_layer_forward_static(C.byref(d), arr, C.byref(p), _ptr(x), _ptr(y), _dtype_code(x),
                                      int(x.shape[0]), int(x.shape[1]), int(precision), _stream_handle(stream))
    if st != 0:
        raise StiError(st, "sti_layer_forward_static")


def sti_layer_forward_masked(dims, shards: Sequence, params, x, y, key_lengths, precision: int,
                             workspace, stream=None) -> None:
    """As sti_layer_forward; key_lengths: CUDA int32 tensor [batch], real positions per sequence."""
    d = make_dims(dims)
    arr = shard_array(shards)
    p = make_params(params)
    batch, seq = int(x.shape[0]), int(x.shape[1])
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = lib.sti_layer_forward_masked(C.byref(d), arr, C.byref(p), _ptr(x), _ptr(y), _dtype_code(x),
                                      batch, seq, _key_lengths_ptr(key_lengths, batch), int(precision),
                                      _ptr(workspace), ws_bytes, _stream_handle(stream))
    if st != 0:
        raise StiError(st, "sti_layer_forward_masked")


def make_store(store_rows: Sequence[Sequence[dict]]) -> "C.Array":
    """store_rows[l][i]: dict bitwidth -> shard object (.bitwidth/.data/.codebook CUDA tensors)."""
    n_layers = len(store_rows)
    M = len(store_rows[0]) if n_layers else 0
    arr = (StiShard * max(1, n_layers * M * 6))()
    for l, row in enumerate(store_rows):
        for i, versions in enumerate(row):
            for v, k in enumerate(VERSION_SLOTS):
                s = versions.get(k) if versions else None
                idx = (l * M + i) * 6 + v
                arr[idx] = (make_shard(k, s.data, s.codebook, getattr(s, "outlier_pos", None),
                                       getattr(s, "outlier_val", None)) if s is not None
                            else StiShard(k, None, None, 0, None, None))
    return arr


def sti_model_forward(dims, store, params: Sequence, plan, x, y, precision: int, workspace,
                      stream=None) -> None:
    """store: result of make_store (or a ctypes StiShard array [n_layers][M][6]);
    plan: int8 numpy array [n_layers][M]."""
    import numpy as np
    d = make_dims(dims)
    plan = np.ascontiguousarray(plan, dtype=np.int8)
    n_layers = int(plan.shape[0]) if plan.ndim == 2 else 0
    if not isinstance(store, C.Array):
        store = make_store(store)
    ps = (StiLayerParams * max(1, n_layers))()
    for l in range(n_layers):
        ps[l] = make_params(params[l])
    batch, seq = int(x.shape[0]), int(x.shape[1])
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = lib.sti_model_forward(C.byref(d), n_layers, store, ps,
                               plan.ctypes.data_as(C.POINTER(C.c_int8)), _ptr(x), _ptr(y),
                               _dtype_code(x), batch, seq, int(precision), _ptr(workspace),
                               ws_bytes, _stream_handle(stream))
    if st != 0:
        raise StiError(st, "sti_model_forward")


def sti_model_forward_masked(dims, store, params: Sequence, plan, x, y, key_lengths, precision: int,
                             workspace, stream=None) -> None:
    """As sti_model_forward; key_lengths: CUDA int32 tensor [batch], the same in every layer."""
    import numpy as np
    d = make_dims(dims)
    plan = np.ascontiguousarray(plan, dtype=np.int8)
    n_layers = int(plan.shape[0]) if plan.ndim == 2 else 0
    if not isinstance(store, C.Array):
        store = make_store(store)
    ps = (StiLayerParams * max(1, n_layers))()
    for l in range(n_layers):
        ps[l] = make_params(params[l])
    batch, seq = int(x.shape[0]), int(x.shape[1])
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = lib.sti_model_forward_masked(C.byref(d), n_layers, store, ps,
                                      plan.ctypes.data_as(C.POINTER(C.c_int8)), _ptr(x), _ptr(y),
                                      _dtype_code(x), batch, seq, _key_lengths_ptr(key_lengths, batch),
                                      int(precision), _ptr(workspace), ws_bytes, _stream_handle(stream))
    if st != 0:
        raise StiError(st, "sti_model_forward_masked")


def sti_profile_begin() -> None:
    st = lib.sti_profile_begin()
    if st != 0:
        raise StiError(st, "sti_profile_begin")


def sti_profile_end() -> dict:
    """Returns {kernel class: (launches, total milliseconds)}."""
    prof = StiProfile()
    st = lib.sti_profile_end(C.byref(prof))
    if st != 0:
        raise StiError(st, "sti_profile_end")
    return {name: (int(prof.launches[i]), float(prof.ms[i])) for i, name in enumerate(KERNEL_CLASSES)}


def sti_pipeline_staging_bytes(dims) -> int:
    d = make_dims(dims)
    return int(lib.sti_pipeline_staging_bytes(C.byref(d)))


class StiPipeline:
    """Handle of the load || compute pipeline.  ``preload`` and ``staging`` are CUDA uint8
    tensors that must stay alive as long as the handle."""

    def __init__(self, dims, preload, staging):
        self._dims = make_dims(dims)
        self._keep = (preload, staging)
        handle = C.c_void_p()
        pre_bytes = 0 if preload is None else preload.numel() * preload.element_size()
        st = lib.sti_pipeline_create(C.byref(self._dims), _ptr(preload), pre_bytes, _ptr(staging),
                                     staging.numel() * staging.element_size(), C.byref(handle))
        if st != 0:
            raise StiError(st, "sti_pipeline_create")
        self._h = handle

    def forward(self, store, params: Sequence, plan, x, y, precision: int, workspace, stream=None,
                key_lengths=None) -> dict:
        """store: make_store(...) of versions whose ``data`` are pinned host tensors.
        With key_lengths (CUDA int32 tensor [batch]) the call goes to sti_pipeline_forward_masked."""
        import numpy as np
        plan = np.ascontiguousarray(plan, dtype=np.int8)
        n_layers = int(plan.shape[0]) if plan.ndim == 2 else 0
        if not isinstance(store, C.Array):
            store = make_store(store)
        ps = (StiLayerParams * max(1, n_layers))()
        for l in range(n_layers):
            ps[l] = make_params(params[l])
        stats = StiPipelineStats()
        ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        if key_lengths is not None:
            st = lib.sti_pipeline_forward_masked(
                self._h, n_layers, store, ps, plan.ctypes.data_as(C.POINTER(C.c_int8)), _ptr(x), _ptr(y),
                _dtype_code(x), int(x.shape[0]), int(x.shape[1]),
                _key_lengths_ptr(key_lengths, int(x.shape[0])), int(precision), _ptr(workspace), ws_bytes,
                _stream_handle(stream), C.byref(stats))
            if st != 0:
                raise StiError(st, "sti_pipeline_forward_masked")
            return {n: int(getattr(stats, n)) for n, _ in StiPipelineStats._fields_}
        st = lib.sti_pipeline_forward(self._h, n_layers, store, ps,
                                      plan.ctypes.data_as(C.POINTER(C.c_int8)), _ptr(x), _ptr(y),
                                      _dtype_code(x), int(x.shape[0]), int(x.shape[1]), int(precision),
                                      _ptr(workspace), ws_bytes, _stream_handle(stream), C.byref(stats))
        if st != 0:
            raise StiError(st, "sti_pipeline_forward")
        return {n: int(getattr(stats, n)) for n, _ in StiPipelineStats._fields_}

    def close(self):
        if self._h:
            st = lib.sti_pipeline_destroy(self._h)
            self._h = None
            if st != 0:
                raise StiError(st, "sti_pipeline_destroy")

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _plan_tables(t_io, t_comp, n_layers: int):
    tc = (C.c_double * len(t_comp))(*[float(x) for x in t_comp])
    tab = StiPlanTables(int(n_layers), len(t_comp), (C.c_double * 6)(*[float(x) for x in t_io]), tc)
    return tab, tc


def sti_plan_submodel(t_io, t_comp, n_layers: int, deadline_s: float):
    """t_io: 6 delays (bitwidths 2..6, 32); t_comp[m-1]: seconds per layer of m shards -> (n, m)."""
    tab, _keep = _plan_tables(t_io, t_comp, n_layers)
    n, m = C.c_int32(), C.c_int32()
    st = lib.sti_plan_submodel(C.byref(tab), float(deadline_s), C.byref(n), C.byref(m))
    if st != 0:
        raise StiError(st, "sti_plan_submodel")
    return int(n.value), int(m.value)


def sti_plan_bitwidths(t_io, t_comp, n_layers: int, n: int, m: int, preloaded, importance):
    """Returns (plan int8 [n_layers][M], aib float64 [n])."""
    import numpy as np
    tab, _keep = _plan_tables(t_io, t_comp, n_layers)
    M = len(t_comp)
    pre = None if preloaded is None else np.ascontiguousarray(preloaded, dtype=np.int8).ravel()
    imp = np.ascontiguousarray(importance, dtype=np.int32).ravel()
    plan = np.zeros(n_layers * M, dtype=np.int8)
    aib = np.zeros(max(n, 1), dtype=np.float64)
    st = lib.sti_plan_bitwidths(C.byref(tab), int(n), int(m),
                                None if pre is None else pre.ctypes.data_as(C.POINTER(C.c_int8)),
                                imp.ctypes.data_as(C.POINTER(C.c_int32)),
                                plan.ctypes.data_as(C.POINTER(C.c_int8)),
                                aib.ctypes.data_as(C.POINTER(C.c_double)))
    if st != 0:
        raise StiError(st, "sti_plan_bitwidths")
    return plan.reshape(n_layers, M), aib[:n]


def sti_quantize_workspace_bytes(dims) -> int:
    d = make_dims(dims)
    return int(lib.sti_quantize_workspace_bytes(C.byref(d)))


def sti_quantize_layer(dims, weights, bitwidth: int, packed, codebook, outlier_pos, outlier_val, outlier_count,
                       stats, workspace, loglik_threshold: float = -4.0, reg_covar: float = 1e-6, stream=None) -> None:
    """weights: CUDA float32 [M][Wsh]; packed: CUDA uint8 [M][Wsh*k/8]; codebook: CUDA float32 [2^k];
    outlier_pos (int32/uint32 bits) and outlier_val (float32): CUDA [M][max]; outlier_count: CUDA int32 [M];
    stats: CUDA uint8 tensor of 32 bytes or None (layout StiQuantStats)."""
    d = make_dims(dims)
    max_out = 0 if outlier_pos is None else int(outlier_pos.shape[1])
    st = lib.sti_quantize_layer(C.byref(d), _ptr(weights), int(bitwidth), float(loglik_threshold), float(reg_covar),
                                _ptr(packed), _ptr(codebook), _ptr(outlier_pos), _ptr(outlier_val), max_out,
                                _ptr(outlier_count), _ptr(stats), _ptr(workspace),
                                0 if workspace is None else workspace.numel() * workspace.element_size(),
                                _stream_handle(stream))
    if st != 0:
        raise StiError(st, "sti_quantize_layer")
