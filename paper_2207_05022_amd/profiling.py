"""One-time measurement of the delays the planner needs (Section "Prerequisite: Offline
Profiling"): T_io(k), the delay of bringing one shard of bitwidth k over the host link, and
T_comp(m), the delay of decompressing and executing one layer of m shards (measured with
6-bit shards, the slowest packed version to decompress, as the paper does).  Plumbing around
the C ABI: every measured step runs in the library's kernels."""
from __future__ import annotations

from types import SimpleNamespace
from typing import List, Sequence

import torch

from . import binding as B

BITWIDTHS = (2, 3, 4, 5, 6, 32)


def _wsh(dims) -> int:
    return dims.d_model * (4 * dims.d_head + 2 * dims.ffn_per_shard)


def _elapsed(fn, reps: int) -> float:
    for _ in range(2):
        fn()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) * 1e-3 / reps


def measure_t_io(dims, reps: int = 20) -> List[float]:
    """Seconds per shard for bitwidths 2, 3, 4, 5, 6, 32: a pinned host buffer of the shard's
    size copied to the device."""
    out = []
    for k in BITWIDTHS:
        nbytes = _wsh(dims) * 4 if k == 32 else _wsh(dims) * k // 8
        src = torch.empty(nbytes, dtype=torch.uint8).pin_memory()
        dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        out.append(_elapsed(lambda: dst.copy_(src, non_blocking=True), reps))
    return out


def measure_t_comp(dims, batch: int, seq: int, precision: int, reps: int = 10) -> List[float]:
    """t_comp[m-1]: seconds for sti_layer_forward over the first m of M shards, all at 6 bits."""
    M, wsh = dims.n_heads, _wsh(dims)
    gen = torch.Generator(device="cuda").manual_seed(2207)
    shards = []
    for _ in range(M):
        data = torch.randint(0, 256, (wsh * 6 // 8,), dtype=torch.uint8, device="cuda", generator=gen)
        cb = torch.randn(64, device="cuda", generator=gen) * 0.02
        shards.append(SimpleNamespace(bitwidth=6, data=data, codebook=cb, outlier_pos=None, outlier_val=None))
    names = ("bq", "bk", "bv", "bo", "b1", "b2", "ln1_g", "ln1_b", "ln2_g", "ln2_b")
    sizes = {"bq": M * dims.d_head, "bk": M * dims.d_head, "bv": M * dims.d_head, "bo": dims.d_model,
             "b1": M * dims.ffn_per_shard, "b2": dims.d_model, "ln1_g": dims.d_model, "ln1_b": dims.d_model,
             "ln2_g": dims.d_model, "ln2_b": dims.d_model}
    params = SimpleNamespace(**{n: (torch.ones(sizes[n], device="cuda") if n.endswith("_g")
                                    else torch.zeros(sizes[n], device="cuda")) for n in names})
    dtype = torch.float32 if precision == B.STI_PREC_F32 else torch.float16
    x = torch.randn(batch, seq, dims.d_model, device="cuda", generator=gen).to(dtype)
    y = torch.empty_like(x)
    ws = torch.empty(B.sti_workspace_bytes(dims, batch, seq, precision), dtype=torch.uint8, device="cuda")
    out = []
    for m in range(1, M + 1):
        sel: Sequence = shards[:m] + [None] * (M - m)
        out.append(_elapsed(lambda: B.sti_layer_forward(dims, sel, params, x, y, precision, ws), reps))
    return out
