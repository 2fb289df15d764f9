#!/usr/bin/env python3
"""Benchmark of the SALR bitmap-sparse + concatenated-LoRA linear on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-extras] [--no-cpu-baseline]
                    [--workload q_proj_M16|gate_up_M2048|down_proj_M4096]

A step is one call of salr_sparse_lowrank_linear (decode stage, contraction, both adapter stages) on
the Llama-3-8B q_proj-shaped layer (W [4096, 4096], 50 % per-row magnitude sparsity, two rank-16
adapters concatenated, X [16, 4096]) with all operands resident in HBM.  Successive steps rotate over
enough distinct encoded copies of the weight that the cycled footprint exceeds twice the 256 MB
Infinity Cache, so the weight stream comes from HBM, not from cache.

Prints ONE JSON line on stdout (everything else goes to stderr):
  value     = algorithmic bytes of one call / wall-clock time per step (whole job, K steps bracketed
              by synchronize), GB/s;
  roofline  = the fused kernel's own duration from a HIP event pair attached to its launch (the
              events take the kernel's begin and end; a second pass of K steps, same rotation),
              against the 8 TB/s HBM peak; `traffic` = measured HBM bytes per launch;
  cpu_baseline = the CPU oracle (fp64, OpenMP) timed on this machine's host cores on the same workload.
Extra keys report the other batch sizes, the prefill-sized gate/up and down layers against the bf16 MFMA peak,
the dense bf16 GEMM (hipBLASLt via torch.matmul) under the same rotation, and mask/encode/decode.
With --workload gate_up_M2048 or down_proj_M4096 the step is that prefill-sized layer instead: value in
TFLOP/s, roofline = the dense MFMA stage of the call against the 2.5 PFLOP/s bf16 peak.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "TFLOP/s & HBM GB/s of bitmap-sparse+LoRA linear vs roofline; speedup vs dense"
HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
ROTATE_BYTES = 640 * 1024 * 1024


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class HipEvents:
    """hipEvent_t pairs through the HIP runtime that torch already loaded."""

    def __init__(self, n):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.pairs = []
        for _ in range(n):
            a, b = ctypes.c_void_p(), ctypes.c_void_p()
            assert self.hip.hipEventCreate(ctypes.byref(a)) == 0
            assert self.hip.hipEventCreate(ctypes.byref(b)) == 0
            self.pairs.append((a, b))

    def elapsed_ms(self):
        out = []
        for a, b in self.pairs:
            self.hip.hipEventSynchronize(b)
            ms = ctypes.c_float()
            rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b)
            assert rc == 0, rc
            out.append(ms.value)
        return out

    def close(self):
        for a, b in self.pairs:
            self.hip.hipEventDestroy(a)
            self.hip.hipEventDestroy(b)
        self.pairs = []


class Layer:
    """Encoded weight copies + adapters of one synthetic layer on the device."""

    def __init__(self, cfg, permille, max_copies=64, nm=None):
        import numpy as np
        import torch
        import paper_2601_16991_amd as salr
        import salr_workloads as wl
        dev = torch.device("cuda:0")
        self.cfg, self.permille = cfg, permille
        w = torch.from_numpy(wl.dense_weight(cfg).view(np.int16)).to(dev)
        if nm is None:   # per-row top-keep (the workloads of the configs)
            self.w_hat = salr.mask_rows(w, cfg.keep(permille))
            expect = cfg.N * cfg.keep(permille)
        else:            # N:M groups (the pattern of the paper's inference-throughput table)
            self.w_hat = salr.mask_nm(w, nm[0], nm[1])
            expect = cfg.N * cfg.K // nm[1] * nm[0]
        del w
        bitmap, values, offsets = salr.encode(self.w_hat)
        torch.cuda.synchronize()
        self.nnz = int(values.numel())
        assert self.nnz == expect, (self.nnz, expect)
        enc_bytes = bitmap.numel() * 4 + self.nnz * 2 + offsets.numel() * 4
        self.ncopies = int(min(max_copies, max(2, -(-ROTATE_BYTES // enc_bytes))))
        self.enc = [(bitmap, values, offsets)]
        for _ in range(self.ncopies - 1):
            v = salr.values_alloc(self.nnz, dev)
            v.copy_(values)
            self.enc.append((bitmap.clone(), v, offsets.clone()))
        As, Bs = wl.adapters(cfg)
        a_cat, b_cat = wl.concat_adapters(As, Bs)
        self.a_cat = torch.from_numpy(a_cat.view(np.int16)).to(dev)
        self.b_cat = torch.from_numpy(b_cat.view(np.int16)).to(dev)
        self.R = cfg.R
        self._tables = None

    def tables(self):
        """The layer's slice table, one per encoded copy (built on first use)."""
        import paper_2601_16991_amd as salr
        if self._tables is None:
            self._tables = [salr.build_slice_table(b, o, self.cfg.K) for (b, v, o) in self.enc]
        return self._tables

    def dense_copies(self):
        import torch
        n = int(min(32, max(2, -(-ROTATE_BYTES // (self.w_hat.numel() * 2)))))
        return [self.w_hat.view(torch.bfloat16).clone() for _ in range(n)]


def time_linear(layer, M, steps, warmup, events=False, two_of_four=False, lean=False, prepared=False):
    """(ms per step by wall clock, list of per-launch kernel ms from HIP events or None).  two_of_four: the call is
    salr_sparse_lowrank_linear_2of4 (the layer must be 2:4-masked).  lean: the call gets the least workspace it accepts
    (large batches then run the fused kernel that keeps no decoded copy of the weight).  prepared: the call is
    salr_sparse_lowrank_linear_prepared with the layer's slice table."""
    import numpy as np
    import torch
    import paper_2601_16991_amd as salr
    import salr_workloads as wl
    cfg = layer.cfg
    dev = torch.device("cuda:0")
    x = torch.from_numpy(wl.activations(cfg, M).view(np.int16)).to(dev)
    y = torch.empty((M, cfg.N), dtype=torch.int16, device=dev)
    ws_fn = salr.salr_linear_2of4_workspace_bytes if two_of_four else salr.salr_linear_workspace_bytes
    if lean:
        ws_fn = salr.salr_linear_workspace_bytes_min
    ws = torch.empty(max(ws_fn(M, cfg.K, cfg.N, layer.R), 256), dtype=torch.uint8, device=dev)[:max(ws_fn(M, cfg.K, cfg.N, layer.R), 1)]

    tables = layer.tables() if prepared else [None] * len(layer.enc)
    calls = [salr.PreparedLinear(x, b, v, o, layer.a_cat, layer.b_cat, y, ws, two_of_four=two_of_four, slice_table=t)
             for (b, v, o), t in zip(layer.enc, tables)]
    stream = torch.cuda.current_stream().cuda_stream or None

    def call(i):
        calls[i % layer.ncopies].run(stream)

    for i in range(warmup):
        call(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        call(i)
    torch.cuda.synchronize()
    ms_wall = (time.perf_counter() - t0) * 1e3 / steps
    kernel_ms = None
    if events:
        ev = HipEvents(steps)
        for i in range(steps):
            a, b = ev.pairs[i]
            salr.salr_set_kernel_timing_events(a, b)
            call(i)
        salr.salr_set_kernel_timing_events(None, None)
        torch.cuda.synchronize()
        kernel_ms = ev.elapsed_ms()
        ev.close()
    return ms_wall, kernel_ms


def time_dense(layer, M, steps, warmup, with_lora):
    import numpy as np
    import torch
    import salr_workloads as wl
    cfg = layer.cfg
    dev = torch.device("cuda:0")
    x = torch.from_numpy(wl.activations(cfg, M).view(np.int16)).to(dev).view(torch.bfloat16)
    ws = layer.dense_copies()
    a = layer.a_cat.view(torch.bfloat16)
    b = layer.b_cat.view(torch.bfloat16)

    def call(i):
        y = torch.matmul(x, ws[i % len(ws)].t())
        if with_lora:
            y = y + torch.matmul(torch.matmul(x, a), b)
        return y

    for i in range(warmup):
        call(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        call(i)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def time_codec(layer, steps):
    import torch
    import paper_2601_16991_amd as salr
    cfg = layer.cfg
    bitmap, values, offsets = layer.enc[0]
    out = torch.empty((cfg.N, cfg.K), dtype=torch.int16, device=bitmap.device)
    res = {}
    keep = cfg.keep(layer.permille)
    for name, fn in (("decode", lambda: salr.salr_decode(bitmap, values, offsets, cfg.N, cfg.K, out)),
                     ("encode", lambda: salr.salr_encode_bitmap(layer.w_hat, bitmap, values, offsets)),
                     ("mask_rows", lambda: salr.salr_magnitude_mask_rows(layer.w_hat, keep, out)),
                     ("mask_2of4", lambda: salr.salr_magnitude_mask_nm(layer.w_hat, 2, 4, out))):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        if name.startswith("mask"):
            nbytes = 4 * cfg.N * cfg.K   # the matrix once in, once out
        else:
            nbytes = 2 * cfg.N * cfg.K + cfg.N * cfg.K // 8 + 2 * layer.nnz + 4 * (cfg.N + 1)
        res[name] = {"ms": round(ms, 4), "GB/s": round(nbytes / ms / 1e6, 1)}
    return res


def time_prepare(layer, steps):
    """Model-preparation steps on the bench layer: residual, adapter concatenation, residual adapter (rank 32, 16
    extra sketch columns, 2 power iterations: 6 passes over E, each 2 N K bytes, plus one transposed copy)."""
    import numpy as np
    import torch
    import paper_2601_16991_amd as salr
    cfg = layer.cfg
    dev = layer.w_hat.device
    import salr_workloads as wl
    w = torch.from_numpy(wl.dense_weight(cfg).view(np.int16)).to(dev)
    e = torch.empty_like(w)
    r, over, iters = 32, 16, 2
    omega = torch.from_numpy(np.random.default_rng(1).standard_normal((cfg.K, r + over)).astype(np.float32)).to(dev)
    ws = torch.empty(salr.salr_residual_adapter_workspace_bytes(cfg.N, cfg.K, r, over), dtype=torch.uint8, device=dev)
    a_res = torch.empty((cfg.K, r), dtype=torch.int16, device=dev)
    b_res = torch.empty((r, cfg.N), dtype=torch.int16, device=dev)
    sigma = torch.empty(r, dtype=torch.float32, device=dev)
    a_cat = torch.empty((cfg.K, layer.R + r), dtype=torch.int16, device=dev)
    b_cat = torch.empty((layer.R + r, cfg.N), dtype=torch.int16, device=dev)
    res = {}
    nk = cfg.N * cfg.K
    for name, nbytes, fn in (
            ("residual", 6 * nk, lambda: salr.salr_residual(w, layer.w_hat, e)),
            ("concat_adapters", 4 * (layer.R + r) * (cfg.K + cfg.N),
             lambda: salr.salr_concat_adapters([layer.a_cat, a_res], [layer.b_cat, b_res], a_cat, b_cat)),
            ("residual_adapter_r32", (2 * iters + 2) * 2 * nk + 4 * nk,
             lambda: salr.salr_residual_adapter(e, r, over, iters, omega, a_res, b_res, sigma, ws))):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        res[name] = {"ms": round(ms, 4), "GB/s": round(nbytes / ms / 1e6, 1)}
    return res


def time_backward(layer, M, steps):
    """Backward pass of the layer (dX, dA, dB) at batch M: wall time per call and TFLOP/s on its algorithmic flops
    2 M N K (dX) + 2 M R (N + K) (dY B^T and its way back through A^T) + 4 M K R (X A, dA) + 2 M R N (dB)."""
    import numpy as np
    import torch
    import paper_2601_16991_amd as salr
    import salr_workloads as wl
    cfg = layer.cfg
    dev = layer.w_hat.device
    x = torch.from_numpy(wl.activations(cfg, M).view(np.int16)).to(dev)
    dy = torch.from_numpy(wl.gaussian_bf16((M, cfg.N), 1.0, 4242).view(np.int16)).to(dev)
    bitmap, values, offsets = layer.enc[0]
    R = layer.R
    dx = torch.empty((M, cfg.K), dtype=torch.int16, device=dev)
    da = torch.empty((cfg.K, R), dtype=torch.int16, device=dev)
    db = torch.empty((R, cfg.N), dtype=torch.int16, device=dev)
    ws = torch.empty(salr.salr_linear_backward_workspace_bytes(M, cfg.K, cfg.N, R, True, True), dtype=torch.uint8, device=dev)
    res = {}
    for name, outs in (("dx", (dx, None, None)), ("dx_da_db", (dx, da, db))):
        def fn():
            salr.salr_sparse_lowrank_linear_backward(x, dy, bitmap, values, offsets, layer.a_cat, layer.b_cat, *outs, ws)
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        flops = 2 * M * cfg.N * cfg.K + 2 * M * R * (cfg.N + cfg.K)
        if outs[1] is not None:
            flops += 4 * M * cfg.K * R + 2 * M * R * cfg.N
        res[name] = {"ms": round(ms, 4), "TFLOP/s": round(flops / ms / 1e9, 1)}
    return res


def cpu_baseline(cfg, permille, M, alg_bytes, budget_s=10.0, max_reps=50):
    import numpy as np
    import oracle
    import salr_workloads as wl
    w_hat = oracle.mask_topk_rows(wl.dense_weight(cfg), cfg.keep(permille))
    x = wl.activations(cfg, M)
    a_cat, b_cat = wl.concat_adapters(*wl.adapters(cfg))
    oracle.linear(x[:1], w_hat, a_cat, b_cat)  # warm the library
    reps, t0 = 0, time.perf_counter()
    while True:
        oracle.linear(x, w_hat, a_cat, b_cat)
        reps += 1
        el = time.perf_counter() - t0
        if el >= budget_s or reps >= max_reps:
            break
    s = el / reps
    return {"value": round(alg_bytes / s / 1e9, 4), "unit": "GB/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": f"{reps} full calls of the fp64 oracle linear on the same workload (M={M}, all {cfg.N} outputs), "
                      f"{s * 1e3:.1f} ms per call"}


def load_traffic(workload_key, field="bytes"):
    """HBM traffic per launch measured with rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE), if a summary was committed;
    `measured_at` names the state of the kernel sources the counters were read on."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as f:
            entry = json.load(f).get(workload_key)
        return None if entry is None else entry.get(field)
    except Exception:
        return None


def config_row(layer, M, steps, warmup, two_of_four=False, lean=False, prepared=False):
    """One row of the table: the call on `layer` at batch M, weights rotated so that they come from HBM.  Both the whole
    call (wall clock per step: every kernel of the call and the gaps between them) and its dominant kernel alone (HIP
    events on its launch) are set against the roofline that bounds the shape: HBM bytes up to 128 tokens, bf16 MFMA
    flops above (2:4 rows: dense-equivalent flops; the sparse instructions execute half of them).  prepared: the call
    with the layer's slice table (64 more bytes per weight row, counted)."""
    import numpy as np
    import paper_2601_16991_amd as salr
    import salr_workloads as wl
    cfg = layer.cfg
    w_ms, k_ms = time_linear(layer, M, steps, warmup, events=True, two_of_four=two_of_four, lean=lean, prepared=prepared)
    d_ms = time_dense(layer, M, steps, warmup, with_lora=False)
    k = float(np.mean(k_ms))
    nbytes = wl.algorithmic_bytes(M, cfg.K, cfg.N, layer.R, layer.nnz) + (64 * cfg.N if prepared else 0)
    fl = wl.algorithmic_flops(M, cfg.K, cfg.N, layer.R)
    ws_fn = salr.salr_linear_2of4_workspace_bytes if two_of_four else salr.salr_linear_workspace_bytes
    if lean:
        ws_fn = salr.salr_linear_workspace_bytes_min
    row = {"ms_per_step": round(w_ms, 6), "kernel_avg_us": round(k * 1e3, 2), "dense_gemm_ms": round(d_ms, 6),
           "speedup_vs_dense_gemm": round(d_ms / w_ms, 3), "workspace_bytes": int(ws_fn(M, cfg.K, cfg.N, layer.R))}
    if M <= 128:
        row.update({"bound": "hbm", "GB/s": round(nbytes / w_ms / 1e6, 1),
                    "frac_call": round(nbytes / w_ms / 1e6 / HBM_PEAK_GBS, 4),
                    "frac_kernel": round(nbytes / k / 1e6 / HBM_PEAK_GBS, 4)})
    else:
        row.update({"bound": "mfma", "TFLOP/s": round(fl / w_ms / 1e9, 1),
                    "frac_call": round(fl / w_ms / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4),
                    "frac_kernel": round(fl / k / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4),
                    "dense_gemm_TFLOP/s": round(2 * M * cfg.N * cfg.K / d_ms / 1e9, 1)})
        if two_of_four:
            row["TFLOP/s_executed"] = round(fl / 2 / w_ms / 1e9, 1)   # the sparse MFMA multiplies the stored half only
            row["frac_kernel_vs_sparse_mfma_peak"] = round(fl / k / 1e9 / (2 * MFMA_BF16_PEAK_TFLOPS), 4)
    return row


def measure_ceilings():
    """What this machine's memory system and vendor GEMM reach in this very run, beside the nominal peaks: a device copy of
    1 GiB (read + write, four sources rotated), a cold read stream (hipBLASLt's bf16 product of one token with a dense
    [28672, 8192] weight, 470 MB read once per call, two weights rotated), and hipBLASLt's bf16 GEMM on two prefill shapes."""
    import torch
    dev = torch.device("cuda:0")
    out = {}
    bufs = [torch.ones(1 << 28, dtype=torch.int32, device=dev) for _ in range(4)]
    dst = torch.empty_like(bufs[0])

    def timed(fn, n):
        for i in range(2):
            fn(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n):
            fn(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n

    t = timed(lambda i: dst.copy_(bufs[i % 4]), 12)
    out["copy_read_plus_write_GB/s"] = round(2 * (1 << 30) / t / 1e9, 1)
    del bufs, dst
    torch.cuda.empty_cache()
    wbig = [torch.randn((28672, 8192), device=dev, dtype=torch.bfloat16) for _ in range(2)]
    x1 = torch.randn((1, 8192), device=dev, dtype=torch.bfloat16)
    t = timed(lambda i: torch.matmul(x1, wbig[i % 2].t()), 20)
    out["read_stream_GB/s"] = round(wbig[0].numel() * 2 / t / 1e9, 1)
    del wbig, x1
    torch.cuda.empty_cache()
    for (m, n, k) in ((2048, 14336, 4096), (4096, 4096, 14336)):
        a = torch.randn((m, k), device=dev, dtype=torch.bfloat16)
        ws = [torch.randn((n, k), device=dev, dtype=torch.bfloat16) for _ in range(3)]
        t = timed(lambda i: torch.matmul(a, ws[i % 3].t()), 10)
        out[f"hipblaslt_bf16_M{m}_N{n}_K{k}_TFLOP/s"] = round(2 * m * n * k / t / 1e12, 1)
        del a, ws
    torch.cuda.empty_cache()
    out["nominal"] = {"hbm_GB/s": HBM_PEAK_GBS, "mfma_bf16_TFLOP/s": MFMA_BF16_PEAK_TFLOPS}
    return out


def time_qsalr(cfg, Ms, steps):
    """QSALR on one layer shape: 20 % per-row magnitude sparsity, packed values as NF4 codes with one bf16 scale per 64
    values.  Times the coding and decoding passes and salr_qsalr_linear (dequantisation + the layer) against the
    format's own algorithmic bytes: bitmap + codes + scales + row offsets (+ the layer's other operands)."""
    import numpy as np
    import torch
    import paper_2601_16991_amd as salr
    import salr_workloads as wl
    layer = Layer(cfg, 200, max_copies=2)
    dev = layer.w_hat.device
    bitmap, values, offsets = layer.enc[0]
    nnz = layer.nnz
    codes, scales = salr.nf4_quantize(values)
    out = salr.values_alloc(nnz, dev)
    torch.cuda.synchronize()
    fmt_bytes = bitmap.numel() * 4 + codes.numel() + scales.numel() * 2 + offsets.numel() * 4
    res = {"sparsity": 0.2, "nnz": nnz, "bits_per_weight": round(8 * fmt_bytes / (cfg.N * cfg.K), 3),
           "compression_vs_bf16": round(2 * cfg.N * cfg.K / fmt_bytes, 3)}
    for name, nbytes, fn in (("quantize", 2 * nnz + codes.numel() + scales.numel() * 2, lambda: salr.salr_nf4_quantize_values(values, codes, scales)),
                             ("dequantize", 2 * nnz + codes.numel() + scales.numel() * 2, lambda: salr.salr_nf4_dequantize_values(codes, scales, nnz, out))):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        res[name] = {"ms": round(ms, 4), "GB/s": round(nbytes / ms / 1e6, 1)}
    # the layer: encoded copies at different addresses are rotated so that no call finds its weight in a cache
    ncopies = int(min(64, max(2, -(-ROTATE_BYTES // fmt_bytes))))
    copies = []
    for _ in range(ncopies):
        c = salr.codes_alloc(nnz, dev)
        c.copy_(codes)
        copies.append((bitmap.clone(), c, scales.clone(), offsets.clone()))
    res["weight_copies_rotated"] = ncopies
    stream = torch.cuda.current_stream().cuda_stream or None
    for M in Ms:
        x = torch.from_numpy(wl.activations(cfg, M).view(np.int16)).to(dev)
        y = torch.empty((M, cfg.N), dtype=torch.int16, device=dev)
        ws_bytes = salr.salr_qsalr_linear_workspace_bytes(M, cfg.K, cfg.N, layer.R, nnz)
        ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)
        calls = [salr.PreparedQsalrLinear(x, b, c, sc, o, nnz, layer.a_cat, layer.b_cat, y, ws) for (b, c, sc, o) in copies]
        n_steps = steps if M > 64 else 10 * steps
        for i in range(5):
            calls[i % ncopies].run(stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n_steps):
            calls[i % ncopies].run(stream)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / n_steps
        ev = HipEvents(n_steps)
        for i in range(n_steps):
            e0, e1 = ev.pairs[i]
            salr.salr_set_kernel_timing_events(e0, e1)
            calls[i % ncopies].run(stream)
        salr.salr_set_kernel_timing_events(None, None)
        torch.cuda.synchronize()
        k_us = float(np.mean(ev.elapsed_ms())) * 1e3
        ev.close()
        dense_ms = time_dense(layer, M, max(n_steps // 2, 10), 5, with_lora=False)
        nbytes = fmt_bytes + 2 * M * cfg.K + 2 * cfg.K * layer.R + 2 * layer.R * cfg.N + 2 * M * cfg.N
        res[f"linear_M{M}"] = {"ms": round(ms, 4), "kernel_avg_us": round(k_us, 2), "GB/s": round(nbytes / ms / 1e6, 1),
                               "frac_call": round(nbytes / ms / 1e6 / HBM_PEAK_GBS, 4),
                               "frac_kernel": round(nbytes / k_us / 1e3 / HBM_PEAK_GBS, 4),
                               "TFLOP/s": round(wl.algorithmic_flops(M, cfg.K, cfg.N, layer.R) / ms / 1e9, 1),
                               "dense_gemm_ms": round(dense_ms, 4), "speedup_vs_dense_gemm": round(dense_ms / ms, 3),
                               "workspace_bytes": int(ws_bytes),
                               "path": "one kernel on the 4-bit codes" if (M <= 64 and cfg.K % 128 == 0) else
                                       "decode stage on the 4-bit codes, then the dense MFMA stage" if (M > 128 and cfg.K % 64 == 0)
                                       else "dequantise, then the layer"}
        del calls, ws
    return res


WORKLOADS = {"q_proj_M16": ("llama3_8b_q_proj", 16), "gate_up_M2048": ("llama3_8b_gate_up_proj", 2048),
             "down_proj_M4096": ("llama3_8b_down_proj", 4096), "gate_up_70b_M1": ("llama3_70b_gate_up_proj", 1),
             "gate_up_70b_M16": ("llama3_70b_gate_up_proj", 16), "gate_up_M16": ("llama3_8b_gate_up_proj", 16),
             "gate_up_M64": ("llama3_8b_gate_up_proj", 64), "down_proj_M128": ("llama3_8b_down_proj", 128),
             "down_proj_M8": ("llama3_8b_down_proj", 8), "down_proj_70b_M1": ("llama3_70b_down_proj", 1),
             # QSALR (20 % sparsity, NF4 values) through salr_qsalr_linear: the whole sweep of batch sizes of one layer
             "qsalr_q_proj": ("llama3_8b_q_proj", 0), "qsalr_gate_up": ("llama3_8b_gate_up_proj", 0),
             "qsalr_70b_gate_up": ("llama3_70b_gate_up_proj", 0),
             # 2:4-masked layers through salr_sparse_lowrank_linear_2of4
             "q_proj_M16_2of4": ("llama3_8b_q_proj", 16), "gate_up_M16_2of4": ("llama3_8b_gate_up_proj", 16),
             "gate_up_70b_M1_2of4": ("llama3_70b_gate_up_proj", 1), "gate_up_70b_M16_2of4": ("llama3_70b_gate_up_proj", 16),
             "gate_up_M2048_2of4": ("llama3_8b_gate_up_proj", 2048), "down_proj_M4096_2of4": ("llama3_8b_down_proj", 4096)}


def decode_result(args, name, M, two_of_four=False, prepared=False):
    """One memory-bound layer other than the headline one as the step (the largest layer: 264 MB per call, so the
    stream reaches steady state and the launch no longer matters).  two_of_four: the layer is 2:4-masked and the call
    is salr_sparse_lowrank_linear_2of4.  prepared: the call is salr_sparse_lowrank_linear_prepared (slice table)."""
    import numpy as np
    import paper_2601_16991_amd as salr
    import salr_workloads as wl
    cfg = wl.CONFIGS[name]
    layer = Layer(cfg, 500, max_copies=4, nm=(2, 4) if two_of_four else None)
    if two_of_four:
        assert salr.bitmap_is_2of4(layer.enc[0][0])
    steps, warmup = max(5, min(args.steps, 60)), max(2, min(args.warmup, 6))
    w_ms, k_ms = time_linear(layer, M, steps, warmup, events=True, two_of_four=two_of_four, prepared=prepared)
    nbytes = wl.algorithmic_bytes(M, cfg.K, cfg.N, layer.R, layer.nnz) + (64 * cfg.N if prepared else 0)
    d_ms = time_dense(layer, M, steps, warmup, with_lora=False)
    k = float(np.mean(k_ms))
    log(f"{name} M={M}: wall {w_ms * 1e3:.1f} us, fused kernel {k * 1e3:.1f} us, dense GEMM {d_ms * 1e3:.1f} us")
    achieved = nbytes / (k * 1e-3) / 1e9
    return {
        "metric": METRIC, "value": round(nbytes / (w_ms * 1e-3) / 1e9, 2), "unit": "GB/s", "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": round(w_ms, 6), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name} W[{cfg.N},{cfg.K}] {'2:4 mask' if two_of_four else 'p=0.5'} R={layer.R} M={M}"
                               + (" (prepared layer: slice table)" if prepared else ""),
                   "weight_copies_rotated": layer.ncopies,
                   "algorithmic_bytes": nbytes},
        "speedup_vs_dense_gemm": round(d_ms / w_ms, 3), "dense_gemm_ms": round(d_ms, 6),
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
                     "frac_call": round(nbytes / (w_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                     "kernel": ("sparse-MFMA kernel of salr_sparse_lowrank_linear_2of4" if two_of_four
                                else "fused decode+GEMM kernel of salr_sparse_lowrank_linear_prepared" if prepared
                                else "fused decode+GEMM kernel of salr_sparse_lowrank_linear"),
                     "kernel_avg_us": round(k * 1e3, 2)},
        "cpu_baseline": None,
    }


def prefill_result(args, name, M, two_of_four=False):
    """One MFMA-bound layer as the step: decode stage + adapter stage + dense MFMA stage per call; with two_of_four the
    layer is 2:4-masked and the call is salr_sparse_lowrank_linear_2of4 (adapter stage + GEMM on the sparse MFMA)."""
    import numpy as np
    import paper_2601_16991_amd as salr
    import salr_workloads as wl
    cfg = wl.CONFIGS[name]
    layer = Layer(cfg, 500, max_copies=4, nm=(2, 4) if two_of_four else None)
    if two_of_four:
        assert salr.bitmap_is_2of4(layer.enc[0][0])
    steps, warmup = max(5, min(args.steps, 50)), max(2, min(args.warmup, 5))
    w_ms, k_ms = time_linear(layer, M, steps, warmup, events=True, two_of_four=two_of_four)
    fl = wl.algorithmic_flops(M, cfg.K, cfg.N, layer.R)
    d_ms = time_dense(layer, M, steps, warmup, with_lora=False)
    k = float(np.mean(k_ms))
    log(f"{name} M={M}: wall {w_ms * 1e3:.1f} us, MFMA stage {k * 1e3:.1f} us, dense GEMM {d_ms * 1e3:.1f} us")
    achieved = fl / (k * 1e-3) / 1e12
    return {
        "metric": METRIC, "value": round(fl / (w_ms * 1e-3) / 1e12, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": round(w_ms, 6), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name} W[{cfg.N},{cfg.K}] {'2:4 mask' if two_of_four else 'p=0.5'} R={layer.R} M={M}",
                   "weight_copies_rotated": layer.ncopies,
                   "algorithmic_flops": fl},
        "speedup_vs_dense_gemm": round(d_ms / w_ms, 3), "dense_gemm_ms": round(d_ms, 6),
        "dense_gemm_TFLOP/s": round(2 * M * cfg.N * cfg.K / d_ms / 1e9, 1),
        "roofline": {"bound": "mfma", "achieved": round(achieved, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4),
                     "traffic": None if two_of_four else load_traffic(f"{name}_M{M}"),
                     "traffic_measured_at": None if two_of_four else load_traffic(f"{name}_M{M}", "measured_at"),
                     "frac_call": round(fl / (w_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                     "kernel": ("GEMM on the sparse MFMA (gemm_2of4_kernel) of salr_sparse_lowrank_linear_2of4, in "
                                "dense-equivalent flops; the adapter stage of the call is in `value` but not in this figure"
                                if two_of_four else
                                "dense MFMA stage (dense_gemm_kernel) of salr_sparse_lowrank_linear; the decode and "
                                "adapter stages of the call are in `value` but not in this figure"),
                     "kernel_avg_us": round(k * 1e3, 2)},
        "cpu_baseline": None,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", default="q_proj_M16", choices=sorted(WORKLOADS),
                    help="q_proj_M16 (default) is the memory-bound headline; the M2048 / M4096 ones time one prefill-sized, "
                         "MFMA-bound layer as the step instead (unit TFLOP/s, roofline against the bf16 MFMA peak), the "
                         "70b ones the largest layer at decode batch sizes and the M16 / M64 / M128 ones the 8B MLP layers at "
                         "batch sizes in between, the _2of4 ones 2:4-masked layers on the sparse matrix-core path (GB/s "
                         "against the HBM peak)")
    ap.add_argument("--prepared", action="store_true",
                    help="with a --workload of up to 128 tokens: call salr_sparse_lowrank_linear_prepared (the layer's slice table)")
    ap.add_argument("--no-extras", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="run three plain copies of 64 MiB (torch copy_, int32) before the workload: under rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE they give the factor between the counters and bytes moved")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(no collectives, no sharding in this library)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2601_16991_amd as salr
    import salr_workloads as wl
    salr.lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    log("device:", torch.cuda.get_device_name(0))
    if args.pmc_calibration:
        src = torch.arange(16 << 20, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if args.workload != "q_proj_M16":
        name, m = WORKLOADS[args.workload]
        if args.workload.startswith("qsalr_"):
            res = time_qsalr(wl.CONFIGS[name], (1, 16, 32, 64, 2048), 20)
            print(json.dumps({"workload": args.workload, "qsalr": res}), flush=True)
            return
        if args.workload.endswith("_2of4"):
            result = (decode_result if m <= 128 else prefill_result)(args, name, m, two_of_four=True)
        else:
            result = decode_result(args, name, m, prepared=args.prepared) if m <= 128 else prefill_result(args, name, m)
        print(json.dumps(result), flush=True)
        return

    cfg = wl.CONFIGS["llama3_8b_q_proj"]
    permille, M = 500, 16
    t_prep = time.perf_counter()
    layer = Layer(cfg, permille)
    log(f"prepared {cfg.name}: nnz={layer.nnz} copies={layer.ncopies} ({time.perf_counter() - t_prep:.1f}s)")

    alg_bytes = wl.algorithmic_bytes(M, cfg.K, cfg.N, layer.R, layer.nnz)
    alg_flops = wl.algorithmic_flops(M, cfg.K, cfg.N, layer.R)
    ms_wall, kernel_ms = time_linear(layer, M, args.steps, args.warmup, events=True)
    k_avg = float(np.mean(kernel_ms))
    k_med = float(np.median(kernel_ms))
    log(f"M={M}: wall {ms_wall * 1e3:.2f} us/step, kernel avg {k_avg * 1e3:.2f} us (median {k_med * 1e3:.2f})")
    dense_ms = time_dense(layer, M, args.steps, args.warmup, with_lora=False)
    dense_lora_ms = time_dense(layer, M, args.steps, args.warmup, with_lora=True)
    log(f"dense bf16 GEMM {dense_ms * 1e3:.2f} us, dense + unfused LoRA {dense_lora_ms * 1e3:.2f} us")

    achieved = alg_bytes / (k_avg * 1e-3) / 1e9
    result = {
        "metric": METRIC,
        "value": round(alg_bytes / (ms_wall * 1e-3) / 1e9, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_wall, 6),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name} W[{cfg.N},{cfg.K}] p=0.{permille // 100} R={layer.R} M={M}",
                   "weight_copies_rotated": layer.ncopies, "algorithmic_bytes": alg_bytes,
                   "algorithmic_flops": alg_flops,   # executed: the method multiplies the decoded zeros too
                   "useful_flops": 2 * M * layer.nnz + 2 * M * layer.R * (cfg.K + cfg.N)},
        "tflops": round(alg_flops / (ms_wall * 1e-3) / 1e12, 3),
        "speedup_vs_dense_gemm": round(dense_ms / ms_wall, 3),
        "speedup_vs_dense_gemm_plus_lora": round(dense_lora_ms / ms_wall, 3),
        "dense_gemm_ms": round(dense_ms, 6),
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": load_traffic(f"{cfg.name}_M{M}"),
                     "traffic_measured_at": load_traffic(f"{cfg.name}_M{M}", "measured_at"),
                     "frac_call": round(alg_bytes / (ms_wall * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                     "kernel": "fused decode+GEMM kernel of salr_sparse_lowrank_linear",
                     "kernel_avg_us": round(k_avg * 1e3, 3), "kernel_median_us": round(k_med * 1e3, 3),
                     "kernel_p10_us": round(float(np.percentile(kernel_ms, 10)) * 1e3, 3),
                     "kernel_p90_us": round(float(np.percentile(kernel_ms, 90)) * 1e3, 3)},
    }

    if not args.no_extras:
        extras = {}
        result["ceilings"] = measure_ceilings()
        log("ceilings:", result["ceilings"])
        # every layer shape / sparsity / batch size of the workload list (the headline row is measured above with the
        # driver's own step count; here it appears again with the short protocol, for comparison within the table)
        extras["configs"] = {}
        # second workload: the headline layer under a 2:4 mask (constant popcount per nibble), general call and sparse-MFMA call
        layer24 = Layer(cfg, permille, nm=(2, 4))
        assert salr.bitmap_is_2of4(layer24.enc[0][0])
        for key, sparse_mfma in ((f"{cfg.name}_M{M}_mask2of4", False), (f"{cfg.name}_M{M}_mask2of4_sparse_mfma", True)):
            extras[key] = config_row(layer24, M, min(args.steps, 100), min(args.warmup, 10), two_of_four=sparse_mfma)
            log(f"2:4 mask, M={M}, sparse MFMA path {sparse_mfma}: {extras[key]}")
        del layer24
        extras["codec_" + cfg.name] = time_codec(layer, 20)
        log("codec:", extras["codec_" + cfg.name])
        extras["prepare_" + cfg.name] = time_prepare(layer, 10)
        log("prepare:", extras["prepare_" + cfg.name])
        extras["backward_" + cfg.name + "_M2048"] = time_backward(layer, 2048, 10)
        log("backward:", extras["backward_" + cfg.name + "_M2048"])
        extras["qsalr_" + cfg.name] = time_qsalr(cfg, (1, 16, 64, 2048), 20)
        log("qsalr:", extras["qsalr_" + cfg.name])
        for m in cfg.Ms:
            extras["configs"][f"{cfg.name}_p{permille}_M{m}"] = config_row(layer, m, min(args.steps, 100), min(args.warmup, 10))
            log(f"{cfg.name} p={permille} M={m}: {extras['configs'][f'{cfg.name}_p{permille}_M{m}']}")
            # the same call on the prepared layer (salr_sparse_lowrank_linear_prepared: cursors from the slice table)
            key = f"{cfg.name}_p{permille}_M{m}_prepared"
            extras["configs"][key] = config_row(layer, m, min(args.steps, 100), min(args.warmup, 10), prepared=True)
            log(f"{key}: {extras['configs'][key]}")
        del layer
        torch.cuda.empty_cache()
        for name2 in ("llama3_8b_gate_up_proj", "llama3_8b_down_proj", "llama3_70b_attn", "llama3_70b_gate_up_proj",
                      "llama3_70b_down_proj"):
            cfg2 = wl.CONFIGS[name2]
            for pm in cfg2.sparsity_permille:
                layer2 = Layer(cfg2, pm, max_copies=4)
                ms_list = list(cfg2.Ms)
                if name2 == "llama3_8b_gate_up_proj":
                    ms_list = [1, 8, 16, 64, 128] + ms_list      # decode sizes and the batch sizes up to prefill as well
                if name2 == "llama3_8b_down_proj" and pm == 500:
                    ms_list = sorted(set(ms_list + [16, 128]))
                for m2 in ms_list:
                    steps2 = max(5, min(args.steps, 30))
                    warm2 = 3 if m2 <= 512 else 8   # the long kernels need a few more calls before clocks settle
                    key = f"{cfg2.name}_p{pm}_M{m2}"
                    extras["configs"][key] = config_row(layer2, m2, steps2, warm2)
                    log(f"{key}: {extras['configs'][key]}")
                    if name2 in ("llama3_8b_gate_up_proj", "llama3_8b_down_proj") and pm == 500 and m2 >= 2048:
                        # the same call with the least workspace: decode stage and MFMA stage in one kernel (LDS double
                        # buffer), no decoded copy of the weight in memory
                        key = f"{cfg2.name}_p{pm}_M{m2}_no_decoded_copy"
                        extras["configs"][key] = config_row(layer2, m2, steps2, warm2, lean=True)
                        log(f"{key}: {extras['configs'][key]}")
                    if pm == 500 and m2 <= 128:
                        # up to 128 tokens the kernels can take their cursors from the layer's slice table: the same call
                        # on the prepared layer
                        key = f"{cfg2.name}_p{pm}_M{m2}_prepared"
                        extras["configs"][key] = config_row(layer2, m2, steps2, warm2, prepared=True)
                        log(f"{key}: {extras['configs'][key]}")
                del layer2
                torch.cuda.empty_cache()
        # 2:4-masked layers through salr_sparse_lowrank_linear_2of4 (sparse MFMA on bitmap and values as they are)
        for name3, m3 in (("llama3_8b_gate_up_proj", 16), ("llama3_8b_gate_up_proj", 2048), ("llama3_70b_gate_up_proj", 1)):
            cfg3 = wl.CONFIGS[name3]
            layer3 = Layer(cfg3, 500, max_copies=4, nm=(2, 4))
            key = f"{cfg3.name}_M{m3}_mask2of4_sparse_mfma"
            extras[key] = config_row(layer3, m3, max(5, min(args.steps, 30)), 3, two_of_four=True)
            log(f"{key}: {extras[key]}")
            del layer3
            torch.cuda.empty_cache()
        result["extras"] = extras

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, permille, M, alg_bytes)
        log("cpu_baseline:", result["cpu_baseline"])
    else:
        result["cpu_baseline"] = None

    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
