"""Upload helpers: host (numpy) shards and parameters -> CUDA tensors.

Plumbing only.  Streams are copied through one pooled allocation per call so
that every shard starts on a 256-byte boundary.
"""
from __future__ import annotations

from types import SimpleNamespace
from typing import List, Optional, Sequence

import numpy as np
import torch


def upload_shard(sh, device="cuda", host_data=False):
    """sh: object with bitwidth, data (numpy uint8 / float32), codebook (numpy float32 or None).
    With ``host_data`` the stream stays in host memory for the load || compute pipeline (pinned,
    or ordinary memory when ``host_data == "pageable"``); dictionaries always go to the device."""
    if sh is None:
        return None
    if host_data == "pageable":
        place = lambda t: t.clone()
    elif host_data:
        place = lambda t: t.pin_memory()
    else:
        place = lambda t: t.to(device)
    if sh.bitwidth == 32:
        data = place(torch.from_numpy(np.ascontiguousarray(sh.data, dtype=np.float32)))
        cb = None
    else:
        data = place(torch.from_numpy(np.ascontiguousarray(sh.data, dtype=np.uint8)))
        cb = torch.from_numpy(np.ascontiguousarray(sh.codebook, dtype=np.float32)).to(device)
    pos = val = None
    if getattr(sh, "outlier_pos", None) is not None and len(sh.outlier_pos):
        pos = torch.from_numpy(np.ascontiguousarray(sh.outlier_pos, dtype=np.uint32).view(np.int32)).to(device)
        val = torch.from_numpy(np.ascontiguousarray(sh.outlier_val, dtype=np.float32)).to(device)
    return SimpleNamespace(bitwidth=int(sh.bitwidth), data=data, codebook=cb, outlier_pos=pos,
                           outlier_val=val)


def upload_params(p, device="cuda"):
    names = ("bq", "bk", "bv", "bo", "b1", "b2", "ln1_g", "ln1_b", "ln2_g", "ln2_b")
    return SimpleNamespace(**{n: torch.from_numpy(np.ascontiguousarray(getattr(p, n), dtype=np.float32)).to(device)
                              for n in names})


def upload_workload(wl, device="cuda", host_data=False):
    """Returns (shards [n_layers][M] with None = absent, params [n_layers], x tensor)."""
    shards = [[upload_shard(s, device, host_data) for s in row] for row in wl.shards]
    params = [upload_params(p, device) for p in wl.params]
    x = torch.from_numpy(np.ascontiguousarray(wl.x)).to(device)
    return shards, params, x


def store_from_plan(shards) -> List[List[dict]]:
    """Version store holding exactly the versions a workload's plan uses."""
    return [[({s.bitwidth: s} if s is not None else {}) for s in row] for row in shards]
