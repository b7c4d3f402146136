#!/usr/bin/env python3
"""Throughput of the shard-decode + encoder-layer path on one MI355X.

One step = one pass of the whole path over one batch: a 12-layer mixed-bitwidth
BERT-base forward over 32 x 128 tokens (per group of layers: shards decompressed
into the binary16 working buffer; per layer: four projections on the matrix
cores, attention, two LayerNorms).  The same run also times the standalone
shard-decode entry point on the 1 GiB packed stream, the three single-sequence
configurations (where the projections decode the packed streams in their weight
loader) and the CPU oracle on a bounded sample, and compares the outputs of the
timed calls with the oracle's.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from types import SimpleNamespace

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (profiles/
# bench_config4_config1_hbm_counters.txt, calibrated against a 1 GiB device copy).  Reported
# only while the kernel sources still hash to the value recorded with the counters.
TRAFFIC = {
    "gemm": {"files": ("gemm_wide.hip", "attention_core.hpp", "weight_loader.hpp", "sti_internal.hpp"),
             "sha256": "8949c4b33f5dd01a86878197acbb80d4d8d1104a7d7ae490a31041f1e3cdd6b4",
             "bytes_per_launch": 58889559},
    "decode": {"files": ("decode.hip", "weight_loader.hpp", "sti_internal.hpp"),
               "sha256": "7c03c917b13cf37b695d0f4f52d3fbdf7feaa160de9b1c72985b0183cafc7896",
               "bytes_per_launch": 6089426482},
}


def sources_sha256(files):
    import hashlib
    h = hashlib.sha256()
    for f in files:
        with open(os.path.join(ROOT, "paper_2207_05022_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def measured_traffic(kernel):
    t = TRAFFIC[kernel]
    if t["bytes_per_launch"] is None or sources_sha256(t["files"]) != t["sha256"]:
        return None
    return t["bytes_per_launch"]


METRIC = "BERT layer fwd tokens/s (mixed-bit shards); shard decode GB/s vs HBM peak"
HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
MFMA_F16_PEAK_TFLOPS = 2500.0  # MI355X dense fp16 MFMA, published


def layer_flops_per_token(dims, seq, present):
    """Algorithmic flops per token of one layer with `present` shards (2 flops per multiply-add)."""
    d, dh, f = dims.d_model, dims.d_head, dims.ffn_per_shard
    proj = 2 * present * (4 * d * dh + 2 * d * f)
    attn = 4 * seq * dh * present
    return proj + attn


def gemm_flops(dims, tokens, present, kind):
    d, dh, f = dims.d_model, dims.d_head, dims.ffn_per_shard
    per_shard = {"gemm_qkv": 3 * dh * d, "gemm_out": d * dh, "gemm_ffn_up": f * d, "gemm_ffn_down": d * f}
    return 2.0 * tokens * present * per_shard[kind]


def bench_model(P, D, torch, S, steps, warmup):
    wl = S.config4()
    dims = wl.dims
    shards, params, x = D.upload_workload(wl)
    store = P.binding.make_store(D.store_from_plan(shards))
    y = torch.empty_like(x)
    prec = P.STI_PREC_F16_MFMA
    ws = torch.empty(P.sti_model_workspace_bytes(dims, wl.n_layers, wl.batch, wl.seq, prec), dtype=torch.uint8,
                     device="cuda")

    def step():
        P.sti_model_forward(dims, store, params, wl.plan, x, y, prec, ws)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall / steps * 1e3
    tokens_per_s = wl.tokens * steps / wall

    # second pass of the same steps in which every launch carries events on the launch stream
    P.sti_profile_begin()
    for _ in range(steps):
        step()
    prof = P.sti_profile_end()
    gemm_kinds = ("gemm_qkv", "gemm_out", "gemm_ffn_up", "gemm_ffn_down")
    present_total = int((wl.plan != 0).sum())
    gemm_launches = sum(prof[k][0] for k in gemm_kinds)
    gemm_ms = sum(prof[k][1] for k in gemm_kinds)
    flops_per_forward_gemm = sum(gemm_flops(dims, wl.tokens, present_total, k) for k in gemm_kinds)
    attention_inside = prof["attention"][0] == 0   # the Q/K/V launches ran the attention as well
    if attention_inside:
        flops_per_forward_gemm += 4.0 * wl.seq * dims.d_head * present_total * wl.tokens
    launches_per_forward = gemm_launches / steps
    flops_per_launch = flops_per_forward_gemm / launches_per_forward
    avg_launch_ms = gemm_ms / gemm_launches
    achieved_tflops = flops_per_launch / (avg_launch_ms * 1e-3) / 1e12
    total_flops = sum(layer_flops_per_token(dims, wl.seq, int((wl.plan[l] != 0).sum())) for l in range(wl.n_layers)) * wl.tokens
    out = {
        "workload": wl,
        "tokens_per_s": tokens_per_s,
        "ms_per_step": ms_per_step,
        "whole_path_tflops": total_flops / (ms_per_step * 1e-3) / 1e12,
        "roofline": {
            "bound": "mfma",
            "kernel": "gemm_wide_kernel (Q/K/V projection" + (" with the two heads' attention" if attention_inside else "")
                      + ", O, FFN1 + GELU, FFN2 projections; weights from the binary16 working buffer)",
            "achieved": round(achieved_tflops, 2), "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": round(achieved_tflops / MFMA_F16_PEAK_TFLOPS, 4), "traffic": measured_traffic("gemm"),
            "avg_launch_us": round(avg_launch_ms * 1e3, 2), "launches_per_step": launches_per_forward,
            "flops_per_launch": flops_per_launch,
        },
        "kernel_ms_per_step": {k: round(v[1] / steps, 4) for k, v in prof.items() if v[0]},
    }
    return out, (wl, y)


def bench_decode(P, torch, S, steps, warmup):
    ds = S.config1()
    n = ds.weights_per_shard
    packed = torch.from_numpy(ds.packed).cuda()
    cb_host = np.zeros((ds.n_shards, 64), dtype=np.float32)
    for s, c in enumerate(ds.codebooks):
        cb_host[s, :c.size] = c
    cbs = torch.from_numpy(cb_host).cuda()
    shards = [SimpleNamespace(bitwidth=int(ds.bitwidths[s]), data=packed[int(ds.offsets[s]):], codebook=cbs[s])
              for s in range(ds.n_shards)]
    arr = P.shard_array(shards)
    out = torch.empty(ds.n_shards * n, dtype=torch.float16, device="cuda")
    ws = torch.empty(max(16, P.sti_decode_workspace_bytes(ds.n_shards)), dtype=torch.uint8, device="cuda")
    for _ in range(warmup):
        P.sti_decode_shards(arr, n, out, ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        P.sti_decode_shards(arr, n, out, ws)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) / steps * 1e3
    P.sti_profile_begin()
    for _ in range(steps):
        P.sti_decode_shards(arr, n, out, ws)
    prof = P.sti_profile_end()
    kern_ms = prof["decode"][1] / prof["decode"][0]
    algo_bytes = ds.packed.nbytes + out.numel() * 2 + sum(c.nbytes for c in ds.codebooks)
    gbs = algo_bytes / (kern_ms * 1e-3) / 1e9
    res = {
        "workload": f"config1: {ds.n_shards} BERT-base shards, {ds.packed.nbytes} packed bytes split evenly over k=2..6, fp16 out",
        "value": round(algo_bytes / (wall_ms * 1e-3) / 1e9, 1), "unit": "GB/s (packed in + fp16 out, whole call)",
        "ms_per_call": round(wall_ms, 4),
        "roofline": {"bound": "hbm", "kernel": "decode_kernel", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": measured_traffic("decode"),
                     "avg_launch_us": round(kern_ms * 1e3, 2), "bytes_per_launch": algo_bytes},
    }
    return res, ds


def bench_host_link(P, D, torch, S, steps, warmup):
    """The same model forward with the shard streams in pinned host memory, through the
    load || compute pipeline: cold (no preload buffer), with a preload buffer of one layer at
    full precision, and with one that holds the whole selection (after its first call)."""
    wl = S.config4()
    dims = wl.dims
    prec = P.STI_PREC_F16_MFMA
    host, params, x = D.upload_workload(wl, host_data=True)
    store = P.make_store(D.store_from_plan(host))
    y = torch.empty_like(x)
    ws = torch.empty(P.sti_workspace_bytes(dims, wl.batch, wl.seq, prec), dtype=torch.uint8, device="cuda")
    slot = P.sti_pipeline_staging_bytes(dims) // 2
    staging = torch.empty(4 * slot, dtype=torch.uint8, device="cuda")
    out = {"workload": "config4 with every shard stream in pinned host memory", "staging_slots": 4}
    for name, preload_bytes in (("cold", 0), ("preload_one_layer", slot), ("preload_all", 1 << 30)):
        preload = torch.empty(preload_bytes, dtype=torch.uint8, device="cuda") if preload_bytes else None
        pipe = P.StiPipeline(dims, preload, staging)
        for _ in range(max(1, warmup)):
            stats = pipe.forward(store, params, wl.plan, x, y, prec, ws)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            stats = pipe.forward(store, params, wl.plan, x, y, prec, ws)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / steps * 1e3
        pipe.close()
        out[name] = {"ms_per_step": round(ms, 4), "tokens_per_s": round(wl.tokens / ms * 1e3, 1),
                     "preload_bytes": preload_bytes, "bytes_copied_per_step": stats["bytes_copied"],
                     "link_GBps": round(stats["bytes_copied"] / ms / 1e6, 2)}
    return out


def parity(got, want, tol):
    """max |y - y_ref| / max |y_ref|, and the fraction of elements with
    |y - y_ref| > tol * |y_ref| + tol * rms(y_ref) (expected 0)."""
    got = np.asarray(got, dtype=np.float64)
    delta = np.abs(got - want)
    rms = float(np.sqrt(np.mean(want * want)))
    bad = (delta > tol * np.abs(want) + tol * rms) | ~np.isfinite(got)
    return {"max_rel_err": float(np.max(delta) / np.max(np.abs(want))), "tolerance": tol,
            "elementwise_violations": float(np.mean(bad))}


def packed_bytes(wl):
    """Bytes of the selected shard versions (index streams or float32 weights) and their codebooks."""
    total = 0
    for row in wl.shards:
        for s in row:
            if s is not None:
                total += s.data.nbytes + (0 if s.codebook is None else s.codebook.nbytes)
    return total


def bench_few_token(P, D, torch, S, steps, warmup, with_oracle):
    """Configurations 0, 2 and 3 (one sequence of 128 / 128 / 256 tokens): the latency-bound
    regime of single-input inference (Section "Submodel execution": one input at a time).
    Resident shards, float32 in and out.  Fractions are of the matrix-core and HBM peaks for the
    algorithmic flops and bytes (selected shards as stored + input + output); a forward is a chain
    of dependent launches of a few microseconds each, so both are small by construction."""
    out = {"regime": "latency-bound: 8 dependent launches per layer; fractions of both rooflines are "
                     "reported for completeness"}
    prec = P.STI_PREC_F16_MFMA
    for name, make in (("config0", S.config0), ("config2", S.config2), ("config3", S.config3)):
        wl = make()
        shards, params, x = D.upload_workload(wl)
        store = P.make_store(D.store_from_plan(shards))
        y = torch.empty_like(x)
        ws = torch.empty(P.sti_model_workspace_bytes(wl.dims, wl.n_layers, wl.batch, wl.seq, prec),
                         dtype=torch.uint8, device="cuda")
        run = lambda: P.sti_model_forward(wl.dims, store, params, wl.plan, x, y, prec, ws)
        for _ in range(max(1, warmup)):
            run()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            run()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / steps * 1e3
        flops = sum(layer_flops_per_token(wl.dims, wl.seq, int((wl.plan[l] != 0).sum()))
                    for l in range(wl.n_layers)) * wl.tokens
        nbytes = packed_bytes(wl) + 2 * x.numel() * x.element_size()
        out[name] = {"tokens": wl.tokens, "layers": wl.n_layers, "ms_per_forward": round(ms, 4),
                     "us_per_layer": round(ms * 1e3 / wl.n_layers, 2),
                     "tokens_per_s": round(wl.tokens / ms * 1e3, 1),
                     "algorithmic_gflop": round(flops / 1e9, 3), "algorithmic_mbytes": round(nbytes / 1e6, 2),
                     "frac_mfma_peak": round(flops / (ms * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS, 5),
                     "frac_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 5)}
        if with_oracle:
            import oracle
            want = oracle.model_forward(wl.dims, wl.shards, wl.params, wl.x)
            out[name]["parity"] = parity(y.float().cpu().numpy(), want, 2e-2)
    return out


def bench_quantizer(P, torch, S, steps, warmup):
    """Outlier-aware quantization of one BERT-base layer (12 shards of float32 weights
    ~ N(0, 0.04^2)) into k-bit indexes + centroids + outlier lists, k = 2, 4, 6."""
    dims = S.BERT_BASE
    M, wsh = dims.n_heads, dims.weights_per_shard
    gen = torch.Generator(device="cuda").manual_seed(220705022)
    w = torch.randn(M, wsh, device="cuda", generator=gen) * 0.04
    ws = torch.empty(P.sti_quantize_workspace_bytes(dims), dtype=torch.uint8, device="cuda")
    out = {"workload": "one BERT-base layer, 12 shards x 589824 float32 weights"}
    for k in (2, 4, 6):
        packed = torch.empty(M, wsh * k // 8, dtype=torch.uint8, device="cuda")
        cb = torch.empty(1 << k, device="cuda")
        pos = torch.empty(M, 4096, dtype=torch.int32, device="cuda")
        val = torch.empty(M, 4096, device="cuda")
        cnt = torch.empty(M, dtype=torch.int32, device="cuda")
        st = torch.zeros(32, dtype=torch.uint8, device="cuda")
        run = lambda: P.sti_quantize_layer(dims, w, k, packed, cb, pos, val, cnt, st, ws)
        for _ in range(max(1, warmup)):
            run()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            run()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / steps * 1e3
        out[f"k{k}"] = {"ms_per_layer": round(ms, 4), "input_GBps": round(M * wsh * 4 / ms / 1e6, 1)}
    return out


def bench_ceilings(torch, steps):
    """What the chip delivers for the two resources this path is bound by, measured with kernels that
    use nothing else (libsti_probes.so), and what the vendor's GEMM library reaches on the four
    projection shapes of configuration 4 (torch.nn.functional.linear on binary16 operands: a plain
    GEMM + bias without GELU or residual; a reference point, not part of the path)."""
    import ctypes as C
    lib = C.CDLL(os.path.join(ROOT, "paper_2207_05022_amd", "libsti_probes.so"))
    lib.sti_probe_mfma.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                   C.POINTER(C.c_double), C.POINTER(C.c_double)]
    lib.sti_probe_stream.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_int, C.c_int, C.c_void_p,
                                     C.POINTER(C.c_double), C.POINTER(C.c_double)]
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    out = {}
    scratch = torch.empty(256 * 768, dtype=torch.float32, device="cuda")
    ms, work = C.c_double(), C.c_double()
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    for waves, varied in ((4, 0), (12, 0), (12, 1)):
        rc = lib.sti_probe_mfma(cus, waves, 3000, 5, varied, scratch.data_ptr(), stream, C.byref(ms), C.byref(work))
        assert rc == 0, rc
        tflops = work.value / (ms.value * 1e-3) / 1e12
        out[f"mfma_only_loop_{waves}_waves_per_cu" + ("_varied_random_operands" if varied else "")] = {
            "TFLOP/s": round(tflops, 1), "frac_of_published_peak": round(tflops / MFMA_F16_PEAK_TFLOPS, 4),
            "implied_clock_GHz": round(tflops * 1e12 / (cus * 4096.0) / 1e9, 3), "ms_per_launch": round(ms.value, 4)}
    n_in = 1 << 26
    src = torch.empty(n_in * 16, dtype=torch.uint8, device="cuda").random_(0, 256)
    dst = torch.empty(n_in * 16 * 5, dtype=torch.uint8, device="cuda")
    for ratio in (1, 4, 5):
        rc = lib.sti_probe_stream(src.data_ptr(), dst.data_ptr(), n_in, ratio, 5, stream, C.byref(ms), C.byref(work))
        assert rc == 0, rc
        gbs = work.value / (ms.value * 1e-3) / 1e9
        out[f"hbm_stream_read_to_write_1_to_{ratio}"] = {"GB/s": round(gbs, 1), "frac_of_published_peak": round(gbs / HBM_PEAK_GBS, 4),
                                                        "bytes_per_launch": int(work.value), "ms_per_launch": round(ms.value, 4)}
    del src, dst
    vendor = {}
    for name, (M, N, K) in (("gemm_qkv", (4096, 2304, 768)), ("gemm_out", (4096, 768, 768)),
                            ("gemm_ffn_up", (4096, 3072, 768)), ("gemm_ffn_down", (4096, 768, 3072))):
        a = torch.randn(M, K, device="cuda", dtype=torch.float16)
        w = torch.randn(N, K, device="cuda", dtype=torch.float16) * 0.02
        b = torch.randn(N, device="cuda", dtype=torch.float16)
        for _ in range(5):
            torch.nn.functional.linear(a, w, b)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = max(20, steps * 5)
        e0.record()
        for _ in range(reps):
            torch.nn.functional.linear(a, w, b)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / reps * 1e3
        vendor[name] = {"us_per_call": round(us, 2), "TFLOP/s": round(2.0 * M * N * K / us / 1e6, 1),
                        "frac_of_published_peak": round(2.0 * M * N * K / us / 1e6 / MFMA_F16_PEAK_TFLOPS, 4)}
    # the same call on all-zero operands: how much of the time is the clock the chip holds under
    # switching activity (its shader clock is data dependent), not the kernel
    a = torch.zeros(4096, 768, device="cuda", dtype=torch.float16)
    w = torch.zeros(3072, 768, device="cuda", dtype=torch.float16)
    b = torch.zeros(3072, device="cuda", dtype=torch.float16)
    for _ in range(5):
        torch.nn.functional.linear(a, w, b)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = max(20, steps * 5)
    e0.record()
    for _ in range(reps):
        torch.nn.functional.linear(a, w, b)
    e1.record()
    torch.cuda.synchronize()
    zero_us = e0.elapsed_time(e1) / reps * 1e3
    flops = sum(2.0 * 4096 * n * k for n, k in ((2304, 768), (768, 768), (3072, 768), (768, 3072)))
    us = sum(v["us_per_call"] for v in vendor.values())
    vendor["mean_of_the_four"] = {"us_per_call": round(us / 4, 2), "TFLOP/s": round(flops / us / 1e6, 1),
                                  "frac_of_published_peak": round(flops / us / 1e6 / MFMA_F16_PEAK_TFLOPS, 4)}
    vendor["gemm_ffn_up_all_zero_operands"] = {"us_per_call": round(zero_us, 2),
                                               "speedup_over_random_operands": round(vendor["gemm_ffn_up"]["us_per_call"] / zero_us, 3)}
    out["vendor_gemm_library_same_shapes"] = vendor
    return out


PHASES = ("start-up: entry -> first two K tiles requested", "start-up: -> first K tile landed", "K loop",
          "epilogue arithmetic (Q/K/V tile into LDS for the fused kind)", "stores acknowledged (attention + stores for the fused kind)")
GEMM_KINDS = {4: "gemm_qkv_attention", 2: "gemm_out", 1: "gemm_ffn_up", 3: "gemm_ffn_down"}


def phase_budget_child():
    """Runs in a process of its own with STI_LIBRARY = libsti_phases.so: configuration 4 through
    sti_model_forward, then the clock stamps that wave 0 of every workgroup of the last launch of
    each projection kind left (see STI_PHASE_STAMPS in csrc/gemm_wide.hip)."""
    import ctypes as C
    import numpy as np
    import torch
    import paper_2207_05022_amd as P
    from paper_2207_05022_amd import device as D
    import sti_synth as S
    wl = S.config4()
    prec = P.STI_PREC_F16_MFMA
    shards, params, x = D.upload_workload(wl)
    store = P.binding.make_store(D.store_from_plan(shards))
    y = torch.empty_like(x)
    ws = torch.empty(P.sti_model_workspace_bytes(wl.dims, wl.n_layers, wl.batch, wl.seq, prec), dtype=torch.uint8, device="cuda")
    for _ in range(3):
        P.sti_model_forward(wl.dims, store, params, wl.plan, x, y, prec, ws)
    torch.cuda.synchronize()
    buf = np.zeros((5, 512, 8), dtype=np.uint64)
    P.lib.sti_phase_stamps_read.argtypes = [C.c_void_p, C.c_int]
    rc = P.lib.sti_phase_stamps_read(buf.ctypes.data, 0)
    assert rc == 0, rc
    out = {}
    for kind, name in GEMM_KINDS.items():
        b = buf[kind].astype(np.int64)
        b = b[b[:, 0] != 0]
        if not len(b):
            continue
        d = np.diff(b[:, :6], axis=1)                     # clocks per phase, per workgroup
        wall_us = (b[:, 7] - b[:, 6]) / 100.0             # the wall clock runs at 100 MHz
        total = b[:, 5] - b[:, 0]
        out[name] = {
            "workgroups": int(len(b)),
            "clocks_per_phase_median": {PHASES[i]: int(np.median(d[:, i])) for i in range(5)},
            "clocks_per_phase_p90": [int(np.percentile(d[:, i], 90)) for i in range(5)],
            "clocks_entry_to_exit_median": int(np.median(total)),
            "clock_ticks_per_us": round(float(np.median(total / np.maximum(wall_us, 1e-9))), 1),
            "us_entry_to_exit_median": round(float(np.median(wall_us)), 2),
            "us_first_entry_to_last_exit": round(float((b[:, 7].max() - b[:, 6].min()) / 100.0), 2),
            "us_entry_after_first_entry_p90": round(float(np.percentile(b[:, 6] - b[:, 6].min(), 90) / 100.0), 2),
        }
    print(json.dumps(out))


def bench_phase_budget():
    import subprocess
    env = dict(os.environ, STI_LIBRARY=os.path.join(ROOT, "paper_2207_05022_amd", "libsti_phases.so"))
    r = subprocess.run([sys.executable, os.path.abspath(__file__), "--phase-budget-child"], env=env,
                       capture_output=True, text=True, timeout=300)
    if r.returncode != 0:
        raise RuntimeError(f"phase budget run failed ({r.returncode}): {r.stderr[-2000:]}")
    return json.loads(r.stdout.strip().split("\n")[-1])


def cpu_baselines(S, wl, y, ds):
    """The oracle as it stands, on a bounded sample of both workloads; its output for the model
    workload is also what the output `y` of the timed calls is compared with."""
    import oracle
    threads = oracle.num_threads()
    nseq = wl.batch          # the whole batch: about 10-15 s on 16 host threads
    t0 = time.perf_counter()
    want = oracle.model_forward(wl.dims, wl.shards, wl.params, wl.x[:nseq])
    dt = time.perf_counter() - t0
    model = {"value": round(nseq * wl.seq / dt, 2), "unit": "tokens/s", "cores": threads, "kind": "oracle",
             "sample": f"{nseq} of {wl.batch} sequences through all {wl.n_layers} layers ({dt:.1f} s)"}
    model_parity = parity(y.float().cpu().numpy()[:nseq], want, 2e-2)
    model_parity["compared"] = f"output of the timed sti_model_forward calls, {nseq} of {wl.batch} sequences"
    # decode: a few shards of every bitwidth
    pick = [ds.shard(i) for i in range(ds.n_shards)]   # the whole stream: a few seconds
    t0 = time.perf_counter()
    out = oracle.decode_shards(pick, ds.weights_per_shard, oracle.F16)
    dt = time.perf_counter() - t0
    nbytes = sum(s.data.nbytes for s in pick) + out.nbytes
    dec = {"value": round(nbytes / dt / 1e9, 3), "unit": "GB/s", "cores": threads, "kind": "oracle",
           "sample": f"{len(pick)} of {ds.n_shards} shards, {dt:.1f} s"}
    return model, dec, model_parity


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--print-source-hashes", action="store_true",
                    help="print the kernel source hashes that TRAFFIC is keyed on and exit")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (reference for HBM byte counters)")
    ap.add_argument("--host-link", action="store_true",
                    help="also time the load || compute pipeline with the shard streams in pinned host "
                         "memory (reported beside the headline value, never as it)")
    ap.add_argument("--no-few-token", action="store_true",
                    help="leave out configurations 0, 2 and 3 (reported beside the headline value)")
    ap.add_argument("--ceilings", action="store_true",
                    help="also run the ceiling probes: an MFMA-only loop, HBM streams with the read : write mix of "
                         "decompression, and the vendor GEMM library on configuration 4's projection shapes")
    ap.add_argument("--phase-budget", action="store_true",
                    help="also run configuration 4 on the build whose many-token GEMM kernel records clock stamps "
                         "(libsti_phases.so, in a process of its own) and report the clocks per kernel phase")
    ap.add_argument("--phase-budget-child", action="store_true", help=argparse.SUPPRESS)
    ap.add_argument("--quantize", action="store_true",
                    help="also time the outlier-aware quantizer on one BERT-base layer")
    args = ap.parse_args()
    if args.print_source_hashes:
        for k, t in TRAFFIC.items():
            print(k, sources_sha256(t["files"]))
        return
    if args.gpus != 1:
        print("bench.py measures one GPU: this path has no multi-GPU code (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU (no CPU fallback exists)", file=sys.stderr)
        sys.exit(2)
    if args.phase_budget_child:
        phase_budget_child()
        return
    import paper_2207_05022_amd as P
    from paper_2207_05022_amd import device as D
    import sti_synth as S

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").random_(0, 256)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    model, (wl, y) = bench_model(P, D, torch, S, args.steps, args.warmup)
    decode, ds = bench_decode(P, torch, S, args.steps, args.warmup)
    line = {
        "metric": METRIC, "value": round(model["tokens_per_s"], 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(model["ms_per_step"], 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": "config4: BERT-base 12 layers, batch 32 x seq 128, bitwidths U{2,3,4,6,32}, full shard set, fp16 activations",
                   "tokens_per_step": wl.tokens, "precision": "STI_PREC_F16_MFMA",
                   "device": torch.cuda.get_device_name(0)},
        "whole_path_tflops": round(model["whole_path_tflops"], 2),
        "roofline": model["roofline"],
        "kernel_ms_per_step": model["kernel_ms_per_step"],
        "decode": decode,
    }
    if args.host_link:
        line["host_link_pipeline"] = bench_host_link(P, D, torch, S, args.steps, args.warmup)
    if not args.no_few_token:
        line["few_token"] = bench_few_token(P, D, torch, S, args.steps, args.warmup, not args.no_cpu_baseline)
    if args.ceilings:
        line["ceilings"] = bench_ceilings(torch, args.steps)
    if args.phase_budget:
        line["phase_budget"] = bench_phase_budget()
    if args.quantize:
        line["quantizer"] = bench_quantizer(P, torch, S, args.steps, args.warmup)
    if not args.no_cpu_baseline:
        cpu_model, cpu_dec, model_parity = cpu_baselines(S, wl, y, ds)
        line["cpu_baseline"] = cpu_model
        line["parity"] = model_parity
        line["decode"]["cpu_baseline"] = cpu_dec
    print(json.dumps(line))


if __name__ == "__main__":
    main()
