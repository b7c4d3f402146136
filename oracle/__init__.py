"""ctypes front end of the CPU oracle (TEST INFRASTRUCTURE ONLY).

The arithmetic lives in ``sti_oracle.c``; this file only marshals numpy arrays.
Only tests, the smoke check and the benchmark's CPU-baseline leg may import it;
the product package never does.
"""
from __future__ import annotations

import ctypes as C
from typing import List, Optional, Sequence

import numpy as np

from . import build as _build

F32, F16, BF16 = 0, 1, 2


class _Shard(C.Structure):
    _fields_ = [("bitwidth", C.c_int32), ("data", C.c_void_p), ("codebook", C.c_void_p),
                ("n_outliers", C.c_uint32), ("outlier_pos", C.c_void_p), ("outlier_val", C.c_void_p)]


class _Params(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("bq", "bk", "bv", "bo", "b1", "b2", "ln1_g", "ln1_b", "ln2_g", "ln2_b")]


_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        L.oracle_num_threads.restype = C.c_int
        L.oracle_unpack_index.restype = C.c_uint32
        L.oracle_unpack_index.argtypes = [C.c_void_p, C.c_int, C.c_uint64]
        L.oracle_f32_to_f16.restype = C.c_uint16
        L.oracle_f32_to_f16.argtypes = [C.c_float]
        L.oracle_f32_to_bf16.restype = C.c_uint16
        L.oracle_f32_to_bf16.argtypes = [C.c_float]
        L.oracle_decode_shards.restype = C.c_int
        L.oracle_decode_shards.argtypes = [C.POINTER(_Shard), C.c_int, C.c_uint64, C.c_void_p, C.c_int]
        L.oracle_layer_forward_taps.restype = C.c_int
        L.oracle_layer_forward_taps.argtypes = [
            C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_double, C.POINTER(_Shard),
            C.POINTER(_Params), C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
            C.c_void_p, C.c_void_p, C.c_void_p]
        L.oracle_model_forward.restype = C.c_int
        L.oracle_model_forward.argtypes = [
            C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_double, C.c_int32, C.POINTER(_Shard),
            C.POINTER(_Params), C.c_void_p, C.c_void_p, C.c_int32, C.c_int32]
        L.oracle_layer_forward_masked.restype = C.c_int
        L.oracle_layer_forward_masked.argtypes = [
            C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_double, C.POINTER(_Shard),
            C.POINTER(_Params), C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
        L.oracle_model_forward_masked.restype = C.c_int
        L.oracle_model_forward_masked.argtypes = [
            C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_double, C.c_int32, C.POINTER(_Shard),
            C.POINTER(_Params), C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
        _lib = L
    return _lib


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def _check(rc: int, what: str):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def _shard_array(shards: Sequence, keep: list):
    """shards: objects with .bitwidth/.data/.codebook (numpy), or None for absent."""
    arr = (_Shard * max(1, len(shards)))()
    for i, s in enumerate(shards):
        if s is None or s.bitwidth == 0:
            arr[i].bitwidth = 0
            arr[i].data = None
            arr[i].codebook = None
            continue
        if s.bitwidth == 32:
            data = np.ascontiguousarray(s.data, dtype=np.float32)
            cb = None
        else:
            data = np.ascontiguousarray(s.data, dtype=np.uint8)
            cb = np.ascontiguousarray(s.codebook, dtype=np.float32)
            if cb.size != (1 << s.bitwidth):
                raise ValueError("codebook must hold 2**k entries")
            keep.append(cb)
        keep.append(data)
        arr[i].bitwidth = int(s.bitwidth)
        arr[i].data = data.ctypes.data
        arr[i].codebook = cb.ctypes.data if cb is not None else None
        pos = getattr(s, "outlier_pos", None)
        if pos is not None and len(pos):
            pos = np.ascontiguousarray(pos, dtype=np.uint32)
            val = np.ascontiguousarray(s.outlier_val, dtype=np.float32)
            if pos.size != val.size:
                raise ValueError("outlier_pos and outlier_val differ in length")
            keep += [pos, val]
            arr[i].n_outliers = pos.size
            arr[i].outlier_pos = pos.ctypes.data
            arr[i].outlier_val = val.ctypes.data
    return arr


def _params_struct(p, keep: list) -> _Params:
    st = _Params()
    for name, _ in _Params._fields_:
        a = np.ascontiguousarray(getattr(p, name), dtype=np.float32)
        keep.append(a)
        setattr(st, name, a.ctypes.data)
    return st


def unpack_index(stream: np.ndarray, k: int, j: int) -> int:
    s = np.ascontiguousarray(stream, dtype=np.uint8)
    return int(lib().oracle_unpack_index(s.ctypes.data, k, j))


def f32_to_f16_bits(v: float) -> int:
    return int(lib().oracle_f32_to_f16(np.float32(v)))


def f32_to_bf16_bits(v: float) -> int:
    return int(lib().oracle_f32_to_bf16(np.float32(v)))


def decode_shards(shards: Sequence, n_weights: int, dtype: int = F32) -> np.ndarray:
    """Decode shards to an [n_shards, n_weights] array: float32, or uint16 bit
    patterns of binary16 / bfloat16."""
    keep: list = []
    arr = _shard_array(shards, keep)
    out = np.empty((len(shards), n_weights), dtype=np.float32 if dtype == F32 else np.uint16)
    _check(lib().oracle_decode_shards(arr, len(shards), n_weights, out.ctypes.data, dtype), "decode")
    return out


def _lengths(key_lengths, B: int) -> np.ndarray:
    lens = np.ascontiguousarray(key_lengths, dtype=np.int32)
    if lens.shape != (B,):
        raise ValueError("need one key length per sequence")
    return lens


def layer_forward(dims, shards: Sequence, params, x: np.ndarray, taps: bool = False, key_lengths=None):
    """One layer over the present shards; x [B, L, d] (any float dtype, widened exactly).
    key_lengths [B] (optional): real positions per padded sequence; the rest get no attention."""
    keep: list = []
    arr = _shard_array(shards, keep)
    if len(shards) != dims.n_heads:
        raise ValueError("need one entry per shard of the layer")
    p = _params_struct(params, keep)
    x64 = np.ascontiguousarray(x, dtype=np.float64)
    B, L, d = x64.shape
    if d != dims.d_model:
        raise ValueError("x last dim")
    y = np.empty_like(x64)
    attn = np.empty_like(x64) if taps else None
    h = np.empty_like(x64) if taps else None
    ffn = np.empty_like(x64) if taps else None
    if key_lengths is not None:
        if taps:
            raise ValueError("taps are not offered with key lengths")
        lens = _lengths(key_lengths, B)
        rc = lib().oracle_layer_forward_masked(
            dims.d_model, dims.n_heads, dims.d_head, dims.ffn_per_shard, float(dims.ln_eps), arr,
            C.byref(p), x64.ctypes.data, y.ctypes.data, B, L, lens.ctypes.data)
        _check(rc, "layer_forward_masked")
        return y
    rc = lib().oracle_layer_forward_taps(
        dims.d_model, dims.n_heads, dims.d_head, dims.ffn_per_shard, float(dims.ln_eps), arr,
        C.byref(p), x64.ctypes.data, y.ctypes.data, B, L,
        attn.ctypes.data if taps else None, h.ctypes.data if taps else None,
        ffn.ctypes.data if taps else None)
    _check(rc, "layer_forward")
    if taps:
        return y, {"attn": attn, "h": h, "ffn": ffn}
    return y


def model_forward(dims, shards: Sequence[Sequence], params: Sequence, x: np.ndarray,
                  key_lengths=None) -> np.ndarray:
    """shards [n_layers][M] (None = absent), params [n_layers]; key_lengths as in layer_forward."""
    keep: list = []
    n_layers = len(shards)
    flat = [s for row in shards for s in row]
    if any(len(row) != dims.n_heads for row in shards):
        raise ValueError("need one entry per shard of every layer")
    arr = _shard_array(flat, keep)
    ps = (_Params * max(1, n_layers))()
    for l, p in enumerate(params):
        ps[l] = _params_struct(p, keep)
    x64 = np.ascontiguousarray(x, dtype=np.float64)
    B, L, d = x64.shape
    y = np.empty_like(x64)
    if key_lengths is not None:
        lens = _lengths(key_lengths, B)
        rc = lib().oracle_model_forward_masked(
            dims.d_model, dims.n_heads, dims.d_head, dims.ffn_per_shard, float(dims.ln_eps), n_layers,
            arr, ps, x64.ctypes.data, y.ctypes.data, B, L, lens.ctypes.data)
        _check(rc, "model_forward_masked")
        return y
    rc = lib().oracle_model_forward(
        dims.d_model, dims.n_heads, dims.d_head, dims.ffn_per_shard, float(dims.ln_eps), n_layers,
        arr, ps, x64.ctypes.data, y.ctypes.data, B, L)
    _check(rc, "model_forward")
    return y
