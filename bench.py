#!/usr/bin/env python3
"""Throughput of the fused GEMM hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

A step is one pass of the whole path (tile dispatch, global->LDS staging, MFMA
main loop, fused epilogue, and the split-K reduction when the plan has one) over
one synthetic batch already resident in HBM.  The default workload is the
8192^3 bf16 GEMM + bias + tanh-GELU the headline metric is quoted on.  Prints one
JSON line with the whole-job rate, the roofline fraction of the dominant kernel
(algorithmic FLOP or bytes per launch over the launch time measured with HIP
events on the launch stream) and the CPU oracle timed on a sample of the same
workload (`--oracle-rows`; the default is every row of C at 8192^3, about 15 s on the 16
host cores; the widened operator's oracle takes 512 rows).
fp32 workloads (c1_f32_256, c13_f32_8192x8192x2048) are measured against the fp32 matrix peak.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6   # MI355X dense bf16 matrix peak (datasheet)
PEAK_F32_TFLOPS = 157.3     # MI355X fp32 matrix peak (datasheet)
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E bandwidth (datasheet)
DEFAULT_WORKLOAD = "c3_bf16_8192_bias_gelu"
# which roofline bounds the dominant kernel of each workload
BOUND = {
    "c2_bf16_4096": "mfma",
    "c3_bf16_8192_bias_gelu": "mfma",
    "c4_bf16_batched_512x512x64": "hbm",
    "c5_bf16_splitk_1024x1024x65536": "mfma",
    "c6_fused_nt_8192_bias_gelu_bf16out": "mfma",
    "c7_fused_tn_8192_chain": "mfma",
    "c8_fused_batched_512x512x64_bf16out": "hbm",
    "c11_fused_lower_8192_bias_relu": "mfma",
    "c1_f32_256": "mfma",
    "c13_f32_8192x8192x2048": "mfma",
}
# 16-byte pieces read : written by the HBM-bound workloads, for the stream probe of the same mix
# (c4: 33.5 MB in, 268 MB out; c8: 33.5 in, 134 out; c9: 134 in, 268 out; c12: reads only)
STREAM_MIX = {
    "c4_bf16_batched_512x512x64": (1, 8),
    "c8_fused_batched_512x512x64_bf16out": (1, 4),
    "c9_diag_bf16_8192": (1, 2),
    "c12_rowsum_linear_8192": (1, 0),
    "c14_symm_lower_16384_n16": (1, 0),
}


# HBM-side traffic per launch of the dominant kernel, from rocprofv3 --pmc runs of this file
# (profiles/): FETCH_SIZE and WRITE_SIZE in KiB per dispatch, each scaled by what the same counter
# reads for a plain 1 GiB device-to-device copy (FETCH_SIZE reads 0.5 KiB per KiB copied there,
# WRITE_SIZE 1.0).  An entry is valid only for the kernel it was taken on: it names the kernel
# configuration and carries a hash of the source files that kernel is compiled from, and is dropped
# (reported as null) as soon as either changes.
FETCH_SCALE, WRITE_SCALE = 2.0, 1.0
_MAIN_W4 = ("bf16_layout.h", "ge_device.h", "gemm_bf16_w4.h")
_MAIN_W8 = ("bf16_layout.h", "ge_device.h", "gemm_bf16_fast.h")
_F32 = ("bf16_layout.h", "ge_device.h", "gemm_f32_fast.h")
# workload -> (kernel configuration, FETCH_SIZE KiB, WRITE_SIZE KiB, source files, their hash)
# TRAFFIC-BEGIN (rows written from the counter runs; see profiles/)
TRAFFIC = {
    "c1_f32_256": ("f32_small_32x32_k4", 1234, 256, ('ge_device.h', 'gemm_f32_small.h'), "1637c34d4b8c3bd3"),
    "c2_bf16_4096": ("bf16_256x256x64_w4", 98449, 65536, _MAIN_W4, "f4cba42cb2332e07"),
    "c3_bf16_8192_bias_gelu": ("bf16_256x256x64_w4", 799742, 262147, _MAIN_W4, "f4cba42cb2332e07"),
    "c4_bf16_batched_512x512x64": ("bf16_256x256x32_w8", 16479, 262157, _MAIN_W8, "eee542088afa5b72"),
    "c5_bf16_splitk_1024x1024x65536": ("bf16_256x256x64_w4_splitk", 131500, 65536, _MAIN_W4, "f4cba42cb2332e07"),
    "c6_fused_nt_8192_bias_gelu_bf16out": ("bf16_fused_256x256x64_w4_nt", 792367, 131149, _MAIN_W4, "f4cba42cb2332e07"),
    "c7_fused_tn_8192_chain": ("bf16_fused_256x256x32_w8_tn", 860439, 131072, _MAIN_W8, "eee542088afa5b72"),
    "c8_fused_batched_512x512x64_bf16out": ("bf16_fused_256x256x32_w8_nn", 16542, 131072, _MAIN_W8, "eee542088afa5b72"),
    "c9_diag_bf16_8192": ("diag_rows_vec4", 65970, 262594, ('gemm_diag.hip',), "95489dc912964713"),
    "c10_conv3x3_256_bf16out": ("conv_bf16_halo_3x3_w4_14_11", 60945, 50176, ('bf16_layout.h', 'conv_halo.h', 'conv_halo_launch.h', 'conv_halo_layout.h', 'ge_device.h', 'gemm_bf16_fast.h'), "8ba5a9b1fd08f19c"),
    "c11_fused_lower_8192_bias_relu": ("bf16_fused_256x256x64_w4_nn", 670998, 262144, _MAIN_W4, "f4cba42cb2332e07"),
    "c12_rowsum_linear_8192": ("rowsum_rows_wide", 133354, 4374, ('gemm_rowsum.hip',), "ccd59ba6279a089a"),
    "c13_f32_8192x8192x2048": ("f32_128x128x16_w4", 783979, 262144, _F32, "994f5e7506b6a876"),
    "c15_conv7x7_first_layer_bf16out": ("conv_bf16_rows_k32", 16594, 50176, ('conv_rows.h', 'conv_rows_layout.h', 'ge_device.h'), "92d0096482844c2c"),
    "c14_symm_lower_16384_n16": ("bf16_symm_lower_768x768_n16", 146167, 23552, ('ge_device.h', 'gemm_fused.h', 'gemm_symm.h', 'symm_layout.h'), "a15e2616694f0443"),
}
# TRAFFIC-END


def kernel_source_hash(files) -> str:
    import hashlib
    h = hashlib.sha256()
    for f in files:
        with open(os.path.join(ROOT, "paper_2604_01489_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def measured_ceilings(torch, binding, dA, stream, mix=None, mfma=True):
    """What the device itself sustains, measured in this run with HIP events: a register-resident
    bf16 MFMA loop fed with the workload's own operand values (the clock is power-managed and
    depends on them), a streaming fp32 store of 256 MiB, and -- for an HBM-bound workload -- a
    stream with the workload's own ratio of bytes read to bytes written (`mix` = 16-byte pieces
    read, written per step; about 256 MiB moved per launch)."""
    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps

    out, how = {}, []
    if mfma:
        blocks, iters = 512, 40000
        sink = torch.empty(blocks * 512, dtype=torch.float32, device=dA.device)
        operands = dA.reshape(-1).view(torch.int16)[:32768]
        t = timed(lambda: binding.probe_mfma_bf16(operands, sink, blocks, iters, stream=stream), 3)
        out["mfma_bf16_tflops"] = round(blocks * 8 * iters * 16 * (2.0 * 16 * 16 * 32) / t / 1e12, 1)
        how.append("v_mfma_f32_16x16x32_bf16 loop, 512 blocks x 8 waves, operands = first 64 KiB of A")
    buf = torch.empty(64 << 20, dtype=torch.float32, device=dA.device)
    t = timed(lambda: binding.probe_store_f32(buf, 1.0, stream=stream), 20)
    out["store_gbs"] = round(buf.numel() * 4 / t / 1e9, 1)
    how.append("fp32 store of 256 MiB, 16 B per lane")
    if mix is not None:
        reads, writes = mix
        trips = (256 << 20) // (16 * (reads + writes))
        src = torch.ones(trips * reads * 4, dtype=torch.int32, device=dA.device)
        dst = torch.empty(max(trips * writes * 4, 4), dtype=torch.int32, device=dA.device)
        t = timed(lambda: binding.probe_stream_mix(src, dst, trips, reads, writes, stream=stream), 20)
        out["stream_mix_gbs"] = round(trips * 16.0 * (reads + writes) / t / 1e9, 1)
        out["stream_mix"] = {"reads": reads, "writes": writes}
        how.append(f"stream of {reads} read : {writes} written 16-byte pieces, 256 MiB per launch")
    out["how"] = "; ".join(how)
    return out


def blas_yardstick(torch, dA, dB, transA: bool, transB: bool, flops: float, warmup: int, steps: int):
    """The same product through the BLAS that ships with PyTorch-ROCm, on the operands as they are stored
    (a transposed operand is passed as a transposed view, not copied), bf16 output, no bias or activation:
    less work than the timed operator does, so a yardstick for the box, not a like-for-like baseline."""
    a = dA.view(torch.bfloat16)
    b = dB.view(torch.bfloat16)
    a = a.transpose(-1, -2) if transA else a
    b = b.transpose(-1, -2) if transB else b
    fn = torch.bmm if a.shape[0] > 1 else (lambda x, y: torch.matmul(x[0], y[0]))
    for _ in range(warmup):
        fn(a, b)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        fn(a, b)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    return {"call": "torch.bmm" if a.shape[0] > 1 else "torch.matmul", "out_dtype": "bf16", "epilogue": None,
            "ms_per_launch": round(ms, 4), "tflops": round(flops / (ms * 1e-3) / 1e12, 2)}


def measured_traffic(workload: str, config_name: str):
    """HBM-side bytes per launch from the stored counters, or None when the kernel chosen for the
    workload or its source files are no longer the ones the counters were taken on."""
    v = TRAFFIC.get(workload)
    if v is None or v[0] != config_name or kernel_source_hash(v[3]) != v[4]:
        return None
    return float((v[1] * FETCH_SCALE + v[2] * WRITE_SCALE) * 1024)


def sample_rows(M: int, count: int) -> np.ndarray:
    """`count` rows in blocks of 32 spread evenly over M, always including the
    first and the last block (so first/last tiles and wave sub-tiles are hit)."""
    count = min(count, M)
    blocks = max(1, count // 32)
    if blocks * 32 >= M:
        return np.arange(M)
    starts = np.unique(np.round(np.linspace(0, M - 32, blocks)).astype(np.int64))
    starts = starts + (np.arange(starts.size) % 7)      # not always tile aligned
    starts = np.clip(starts, 0, M - 32)
    return np.unique((starts[:, None] + np.arange(32)[None, :]).ravel())


def bench_diag(args, torch, binding, gen) -> int:
    """The structured-operand entry point (A = diag(d)): HBM-bound scaled copy of B, with the same
    product through the dense GEMM beside it for scale."""
    import oracle
    w = gen.DIAG_WORKLOADS[args.workload]
    dev = torch.device("cuda:0")
    M, N, batch = w.M, w.N, w.batch
    d, B, bias = gen.make_diag_inputs(w)
    dd, dbias = torch.from_numpy(d).to(dev), torch.from_numpy(bias).to(dev)
    dB = torch.from_numpy(B.view(np.int16)).to(dev)
    dC = torch.empty(batch, M, N, dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()

    def timed(fn, warmup, steps):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record(stream)
        for _ in range(steps):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps, e0.elapsed_time(e1) / steps

    ms_wall, ms_dev = timed(lambda: binding.gemm_epilogue_diag_bf16(M, N, dd, dB, N, dbias, w.alpha, w.act, dC, N,
                                                                   batch, stream=stream), args.warmup, args.steps)
    config_name = binding.last_config()
    nbytes = gen.diag_algorithmic_bytes(w)
    achieved = nbytes / (ms_dev * 1e-3) / 1e9
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": round(achieved / PEAK_HBM_GBS, 4), "traffic": measured_traffic(args.workload, config_name),
                "kernel": config_name,
                "ms_per_launch": round(ms_dev, 4)}
    ceilings = None
    if not args.no_ceilings:
        ceilings = measured_ceilings(torch, binding, dB, stream, mix=STREAM_MIX.get(args.workload), mfma=False)
        roofline["frac_of_measured"] = round(achieved / ceilings["stream_mix_gbs"], 4)
    # the same product as a dense GEMM: A = diag(d) rounded to bf16 (context only; d is fp32 in the entry point)
    dense = None
    if batch == 1:
        dAd = torch.zeros(M, M, dtype=torch.bfloat16, device=dev)
        dAd.diagonal().copy_(dd.to(torch.bfloat16))
        dC2 = torch.empty(M, N, dtype=torch.float32, device=dev)
        _, ms_gemm = timed(lambda: binding.gemm_epilogue_bf16(M, N, M, dAd.view(torch.int16), M, dB, N, dbias, w.alpha,
                                                              w.act, dC2, N, 1, stream=stream), 3, 10)
        dense = {"ms_per_launch": round(ms_gemm, 4), "kernel": binding.last_config(),
                 "speedup_of_structured": round(ms_gemm / ms_dev, 2)}
        del dAd, dC2
    cpu_baseline = parity = None
    if args.oracle_rows > 0:
        rows = sample_rows(M, min(args.oracle_rows, 64))
        got = dC[0][torch.from_numpy(rows).to(dev)].cpu().numpy().astype(np.float64)
        eye_rows = np.zeros((len(rows), M), dtype=np.float32)
        eye_rows[np.arange(len(rows)), rows] = 1.0
        c0 = time.perf_counter()
        ref = oracle.gemm_fused(len(rows), N, M, gen.to_bf16_bits(eye_rows), B[0], alpha=w.alpha, row_scale=d[rows],
                                bias=bias, act=w.act)[0]
        c1 = time.perf_counter()
        cpu_baseline = {"value": round(len(rows) * N * 6.0 / (c1 - c0) / 1e9, 6), "unit": "GB/s",
                        "cores": oracle.num_threads(), "kind": "oracle",
                        "sample": f"{len(rows)} of {M} rows of C by the dense definition (A = the matching rows of "
                                  f"diag(d)), full N={N}, K={M}; {c1 - c0:.1f} s"}
        err = np.abs(got - ref)
        rel = float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))
        parity = {"rows_checked": int(len(rows)), "rel_frobenius": rel, "max_abs_err": float(err.max()),
                  "ok": bool(rel <= 1e-3 and np.all(err <= 1e-2 * np.maximum(1.0, np.abs(ref))))}
    out = {"metric": "HBM GB/s of the structured-operand (diagonal) product", "value": round(nbytes / (ms_wall * 1e-3) / 1e9, 1),
           "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_wall, 4),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": args.workload, "M": M, "N": N, "batch": batch, "alpha": w.alpha, "act": w.act,
                      "bias": True, "out_dtype": "f32", "kernel": config_name},
           "roofline": roofline, "ceilings": ceilings, "dense_gemm": dense, "cpu_baseline": cpu_baseline, "parity": parity}
    print(json.dumps(out))
    return 0 if parity is None or parity["ok"] else 1


def bench_symm(args, torch, binding, gen) -> int:
    """A symmetric operand given by its lower triangle, few output columns: the call that fetches every
    stored element once, with the general call on the same array (as a dense matrix) beside it."""
    import oracle
    w = gen.SYMM_WORKLOADS[args.workload]
    dev = torch.device("cuda:0")
    M, N = w.M, w.N
    A, B, bias = gen.make_symm_inputs(w)
    dA = torch.from_numpy(A.view(np.int16)).to(dev)
    dB = torch.from_numpy(B.view(np.int16)).to(dev)
    dbias = torch.from_numpy(bias).to(dev)
    dC = torch.empty(M, N, dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()

    def timed(fn, warmup, steps):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record(stream)
        for _ in range(steps):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps, e0.elapsed_time(e1) / steps

    def step(structure="sym_lower"):
        binding.gemm_epilogue_bf16_fused(M, N, M, dA, M, dB, N, dC, N, alpha=w.alpha, bias=dbias, act=w.act,
                                         stream=stream, a_structure=structure)

    ms_wall, ms_dev = timed(step, args.warmup, args.steps)
    config_name = binding.last_config()
    nbytes = gen.symm_algorithmic_bytes(w)
    achieved = nbytes / (ms_dev * 1e-3) / 1e9
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": round(achieved / PEAK_HBM_GBS, 4), "traffic": measured_traffic(args.workload, config_name),
                "kernel": config_name, "ms_per_launch": round(ms_dev, 4)}
    ceilings = None
    if not args.no_ceilings:
        ceilings = measured_ceilings(torch, binding, dA, stream, mix=(1, 0), mfma=False)
        roofline["frac_of_measured"] = round(achieved / ceilings["stream_mix_gbs"], 4)
    # the same array read as a dense matrix by the general call (a different product unless A is symmetric: for scale)
    _, ms_general = timed(lambda: step("general"), 3, 10)
    general = {"ms_per_launch": round(ms_general, 4), "kernel": binding.last_config(),
               "speedup_of_the_structure": round(ms_general / ms_dev, 2)}
    step()
    torch.cuda.synchronize()
    cpu_baseline = parity = None
    if args.oracle_rows > 0:
        got = dC.cpu().numpy().astype(np.float64)
        c0 = time.perf_counter()
        ref = oracle.gemm_symm(M, N, A, B, uplo="lower", alpha=w.alpha, bias=bias, act=w.act)[0]
        c1 = time.perf_counter()
        cpu_baseline = {"value": round(nbytes / (c1 - c0) / 1e9, 6), "unit": "GB/s", "cores": oracle.num_threads(),
                        "kind": "oracle", "sample": f"all {M} rows of C; {c1 - c0:.1f} s"}
        err = np.abs(got - ref)
        rel = float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))
        parity = {"rows_checked": M, "rel_frobenius": rel, "max_abs_err": float(err.max()),
                  "ok": bool(rel <= 1e-3 and np.all(err <= 1e-2 * np.maximum(1.0, np.abs(ref))))}
    out = {"metric": "HBM GB/s of the product with a symmetric operand given by one triangle", "value": round(nbytes / (ms_wall * 1e-3) / 1e9, 1),
           "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_wall, 4),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": args.workload, "M": M, "N": N, "K": M, "alpha": w.alpha, "act": w.act, "bias": True,
                      "a_structure": "sym_lower", "out_dtype": "f32", "kernel": config_name},
           "roofline": roofline, "ceilings": ceilings, "general_call": general, "cpu_baseline": cpu_baseline, "parity": parity}
    print(json.dumps(out))
    return 0 if parity is None or parity["ok"] else 1


def bench_rowsum(args, torch, binding, gen) -> int:
    """The row sum of a linear layer by its collapsed form: a step is the parameter reduction plus the
    reduction over the input (nothing cached); the input-only call and the long way round (the layer
    through the fused GEMM, then a sum over its output) are timed beside it."""
    import oracle
    w = gen.ROWSUM_WORKLOADS[args.workload]
    dev = torch.device("cuda:0")
    M, N, K = w.M, w.N, w.K
    A, Wt, bias = gen.make_rowsum_inputs(w)
    dA = torch.from_numpy(A.view(np.int16)).to(dev)
    dW = torch.from_numpy(Wt.view(np.int16)).to(dev)
    dbias = torch.from_numpy(bias).to(dev)
    params = torch.empty(K + 1, dtype=torch.float32, device=dev)
    y = torch.empty(M, dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()

    def timed(fn, warmup, steps):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record(stream)
        for _ in range(steps):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps, e0.elapsed_time(e1) / steps

    def step():
        binding.gemm_rowsum_params_bf16(N, K, dW, K, True, dbias, params, stream=stream)
        binding.gemm_rowsum_bf16(M, K, dA, K, params, w.alpha, y, stream=stream)

    ms_wall, ms_dev = timed(step, args.warmup, args.steps)
    _, ms_params = timed(lambda: binding.gemm_rowsum_params_bf16(N, K, dW, K, True, dbias, params, stream=stream),
                         args.warmup, args.steps)
    cfg_params = binding.last_config()
    _, ms_apply = timed(lambda: binding.gemm_rowsum_bf16(M, K, dA, K, params, w.alpha, y, stream=stream),
                        args.warmup, args.steps)
    config_name = binding.last_config()
    nbytes = gen.rowsum_algorithmic_bytes(w)
    achieved = nbytes / (ms_dev * 1e-3) / 1e9
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": round(achieved / PEAK_HBM_GBS, 4), "traffic": measured_traffic(args.workload, config_name),
                "kernel": config_name, "ms_per_launch": round(ms_dev, 4),
                "ms_parameter_pass": round(ms_params, 4), "kernel_parameter_pass": cfg_params,
                "ms_input_pass": round(ms_apply, 4)}
    ceilings = None
    if not args.no_ceilings:
        ceilings = measured_ceilings(torch, binding, dA, stream, mix=STREAM_MIX.get(args.workload), mfma=False)
        roofline["frac_of_measured"] = round(achieved / ceilings["stream_mix_gbs"], 4)
    # the long way round: the layer's output through the fused GEMM (fp32), then its sum over n
    dC = torch.empty(M, N, dtype=torch.float32, device=dev)
    _, ms_long = timed(lambda: (binding.gemm_epilogue_bf16_fused(M, N, K, dA, K, dW, K, dC, N, transB=True, alpha=w.alpha,
                                                                bias=dbias, stream=stream), dC.sum(dim=1)),
                       3, 10)
    long_way = {"ms_per_launch": round(ms_long, 4), "what": "gemm_epilogue_bf16_fused (fp32 out) + torch sum over n",
                "speedup_of_the_collapse": round(ms_long / ms_dev, 1)}
    cpu_baseline = parity = None
    if args.oracle_rows > 0:
        rows = sample_rows(M, min(args.oracle_rows, 2048))
        got = y[torch.from_numpy(rows).to(dev)].cpu().numpy().astype(np.float64)
        c0 = time.perf_counter()
        ref = oracle.gemm_rowsum(np.ascontiguousarray(A[rows]), np.ascontiguousarray(Wt.T), bias, w.alpha)
        c1 = time.perf_counter()
        cpu_baseline = {"value": round(len(rows) / M * nbytes / (c1 - c0) / 1e9, 6), "unit": "GB/s",
                        "cores": oracle.num_threads(), "kind": "oracle",
                        "sample": f"{len(rows)} of {M} rows of y, by the definition (full product, then the sum); "
                                  f"{c1 - c0:.1f} s"}
        err = np.abs(got - ref)
        rel = float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))
        parity = {"rows_checked": int(len(rows)), "rel_frobenius": rel, "max_abs_err": float(err.max()),
                  "ok": bool(rel <= 1e-3 and np.all(err <= 1e-2 * np.maximum(1.0, np.abs(ref))))}
    out = {"metric": "GB/s of the row sum of a linear layer (collapsed form)", "value": round(nbytes / (ms_wall * 1e-3) / 1e9, 1),
           "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_wall, 4),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": args.workload, "M": M, "N": N, "K": K, "alpha": w.alpha, "bias": True,
                      "weights": "N x K", "kernel": config_name},
           "roofline": roofline, "ceilings": ceilings, "long_way": long_way, "cpu_baseline": cpu_baseline, "parity": parity}
    print(json.dumps(out))
    return 0 if parity is None or parity["ok"] else 1


def bench_conv(args, torch, binding, gen) -> int:
    """The convolution front-end (implicit GEMM on the main kernel, fused consumer chain)."""
    import oracle
    cw = gen.CONV_WORKLOADS[args.workload]
    dev = torch.device("cuda:0")
    host = gen.make_conv_inputs(cw)
    oh, ow = cw.out_hw()

    def dev_bits(x):
        return None if x is None else torch.from_numpy(x.view(np.int16) if x.dtype == np.uint16 else x).to(dev)

    dX, dW, dbias, dR = dev_bits(host["X"]), dev_bits(host["Wt"]), dev_bits(host["bias"]), dev_bits(host["residual"])
    if dR is not None and cw.residual == "bf16":
        dR = dR.view(torch.bfloat16)
    dY = torch.empty(cw.N, oh, ow, cw.Cout, dtype=torch.float32 if cw.out == "f32" else torch.bfloat16, device=dev)
    stream = torch.cuda.current_stream()

    def step():
        binding.conv2d_epilogue_bf16(dX, dW, dY, stride=cw.stride, pad=cw.pad, dil=cw.dil, alpha=cw.alpha, bias=dbias,
                                     residual=dR, beta=cw.beta, act=cw.act, clamp=cw.clamp, stream=stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(args.steps):
        step()
    e1.record(stream)
    torch.cuda.synchronize()
    ms_wall = (time.perf_counter() - t0) * 1e3 / args.steps
    ms_dev = e0.elapsed_time(e1) / args.steps
    config_name = binding.last_config()
    hbm = gen.CONV_BOUND[args.workload] == "hbm"
    if hbm:
        achieved = cw.algorithmic_bytes / (ms_dev * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": round(achieved / PEAK_HBM_GBS, 4), "traffic": measured_traffic(args.workload, config_name),
                    "kernel": config_name, "ms_per_launch": round(ms_dev, 4),
                    "tflops": round(cw.flops / (ms_dev * 1e-3) / 1e12, 2)}
    else:
        achieved = cw.flops / (ms_dev * 1e-3) / 1e12
        roofline = {"bound": "mfma", "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": measured_traffic(args.workload, config_name),
                    "kernel": config_name, "ms_per_launch": round(ms_dev, 4)}
    ceilings = None
    if not args.no_ceilings:
        # bytes in to bytes out of the few-channel layer: 9.6 MB to 51.4 MB; the nearest mix the probe has is one
        # 16-byte piece read to four written
        ceilings = measured_ceilings(torch, binding, dX, stream, mix=(1, 4) if hbm else None, mfma=not hbm)
        roofline["frac_of_measured"] = round(achieved / (ceilings["stream_mix_gbs"] if hbm else ceilings["mfma_bf16_tflops"]), 4)
    lib = None
    if not args.no_blas:
        # yardstick: the convolution that ships with PyTorch-ROCm on the same tensors (channels-last views,
        # bf16 output, no bias, residual or activation: less work than the timed operator does)
        try:
            x = dX.view(torch.bfloat16).permute(0, 3, 1, 2)                     # NHWC storage seen as NCHW
            wt = dW.view(torch.bfloat16).permute(0, 3, 1, 2)
            conv = lambda: torch.nn.functional.conv2d(x, wt, stride=cw.stride, padding=cw.pad, dilation=cw.dil)
            for _ in range(args.warmup):
                conv()
            torch.cuda.synchronize()
            l0, l1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            l0.record()
            for _ in range(args.steps):
                conv()
            l1.record()
            torch.cuda.synchronize()
            lms = l0.elapsed_time(l1) / args.steps
            lib = {"call": "torch.nn.functional.conv2d (channels_last)", "out_dtype": "bf16", "epilogue": None,
                   "ms_per_launch": round(lms, 4), "tflops": round(cw.flops / (lms * 1e-3) / 1e12, 2)}
        except Exception as exc:
            lib = {"error": f"{type(exc).__name__}: {exc}"[:200]}
    cpu_baseline = parity = None
    if args.oracle_rows > 0:
        imgs = sorted({0, cw.N - 1})                    # first and last image: first and last tiles of the GEMM
        sub = gen.make_conv_inputs(cw, imgs)
        got = dY[torch.tensor(imgs, device=dev)].to(torch.float32).cpu().numpy().astype(np.float64)
        c0 = time.perf_counter()
        ref = oracle.conv2d_nhwc(sub["X"], sub["Wt"], stride=cw.stride, pad=cw.pad, dil=cw.dil, alpha=cw.alpha,
                                 bias=sub["bias"], residual=sub["residual"], beta=cw.beta, act=cw.act, clamp=cw.clamp,
                                 out=cw.out)
        c1 = time.perf_counter()
        cpu_baseline = {"value": round((cw.algorithmic_bytes / 1e9 if hbm else cw.flops / 1e12) * len(imgs) / cw.N / (c1 - c0), 6),
                        "unit": "GB/s" if hbm else "TFLOP/s",
                        "cores": oracle.num_threads(), "kind": "oracle",
                        "sample": f"images {imgs} of {cw.N}, all positions and channels; {c1 - c0:.1f} s"}
        err = np.abs(got - ref)
        rel = float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))
        parity = {"outputs_checked": int(ref.size), "rel_frobenius": rel, "max_abs_err": float(err.max()),
                  "ok": bool(rel <= 1e-3 and np.all(err <= 1e-2 * np.maximum(1.0, np.abs(ref))))}
    out = {"metric": ("HBM GB/s" if hbm else "TFLOP/s") + " of the implicit-GEMM convolution with fused epilogue",
           "value": round(cw.algorithmic_bytes / (ms_wall * 1e-3) / 1e9, 1) if hbm else round(cw.flops / (ms_wall * 1e-3) / 1e12, 2),
           "unit": "GB/s" if hbm else "TFLOP/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": round(ms_wall, 4), "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": args.workload, "N": cw.N, "H": cw.H, "W": cw.W, "Cin": cw.Cin, "Cout": cw.Cout,
                      "KH": cw.KH, "KW": cw.KW, "stride": cw.stride, "pad": cw.pad, "dil": cw.dil, "act": cw.act,
                      "residual": cw.residual, "out_dtype": cw.out, "layout": "NHWC", "kernel": config_name},
           "roofline": roofline, "ceilings": ceilings, "blas_yardstick": lib, "cpu_baseline": cpu_baseline,
           "parity": parity}
    print(json.dumps(out))
    return 0 if parity is None or parity["ok"] else 1


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD)
    ap.add_argument("--oracle-rows", type=int, default=8192,
                    help="rows of C the CPU oracle computes (bounded sample); 0 skips the oracle")
    ap.add_argument("--rotate", type=int, default=1, metavar="R",
                    help="cycle through R copies of A, B and C (R x the footprint) so that no launch finds "
                         "its inputs in the 256 MB memory-side cache")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the measured-ceiling probes")
    ap.add_argument("--no-blas", action="store_true",
                    help="skip the yardstick: the BLAS that ships with PyTorch-ROCm (torch.matmul / torch.bmm, bf16 "
                         "output, no epilogue) timed on the same operands in the same run")
    ap.add_argument("--blas-probe", action="store_true",
                    help="only run the yardstick's BLAS call on this workload's operands, six times (for hardware "
                         "counters of that kernel under rocprofv3)")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="MiB",
                    help="only run a plain device-to-device copy of this many MiB five times "
                         "(calibrates the FETCH_SIZE / WRITE_SIZE counters under rocprofv3)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this library has no multi-GPU path (--gpus must be 1)",
              file=sys.stderr)
        return 2

    import torch
    from paper_2604_01489_amd import binding, inputs as gen

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    if args.copy_probe > 0:
        n = args.copy_probe * (1 << 20)
        src = torch.ones(n, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes": n, "launches": 5}))
        return 0
    binding.load()
    if args.workload in gen.DIAG_WORKLOADS:
        return bench_diag(args, torch, binding, gen)
    if args.workload in gen.CONV_WORKLOADS:
        return bench_conv(args, torch, binding, gen)
    if args.workload in gen.ROWSUM_WORKLOADS:
        return bench_rowsum(args, torch, binding, gen)
    if args.workload in gen.SYMM_WORKLOADS:
        return bench_symm(args, torch, binding, gen)
    fused = args.workload in gen.FUSED_WORKLOADS
    fw = gen.FUSED_WORKLOADS[args.workload] if fused else None
    w = fw.base if fused else gen.WORKLOADS[args.workload]
    job = fw if fused else w                       # flops and algorithmic bytes
    f32 = w.dtype == "f32"
    peak_mfma = PEAK_F32_TFLOPS if f32 else PEAK_BF16_TFLOPS
    dev = torch.device("cuda:0")
    M, N, K, batch = w.M, w.N, w.K, w.batch
    stream = torch.cuda.current_stream()

    def dev_bits(x):
        return None if x is None else torch.from_numpy(x.view(np.int16) if x.dtype == np.uint16 else x).to(dev)

    # ---- seeded synthetic inputs, generated on the host, resident in HBM before timing
    if fused:
        host = gen.make_fused_inputs(fw)
        A, B, bias = host["A"], host["B"], host["bias"]
        lda, ldb = A.shape[2], B.shape[2]
        dA, dB, dbias = dev_bits(A), dev_bits(B), dev_bits(bias)
        drs, dR = dev_bits(host["row_scale"]), dev_bits(host["residual"])
        if dR is not None and fw.residual == "bf16":
            dR = dR.view(torch.bfloat16)
        dC = torch.empty(batch, M, N, dtype=torch.float32 if fw.out == "f32" else torch.bfloat16, device=dev)
    else:
        A = gen.make_operand(w, "A")
        B = gen.make_operand(w, "B")
        bias = gen.make_bias(w)
        dA, dB, dbias = dev_bits(A), dev_bits(B), dev_bits(bias)
        dC = torch.empty(batch, M, N, dtype=torch.float32, device=dev)
    if args.blas_probe:
        y = blas_yardstick(torch, dA, dB, bool(fused and fw.transA), bool(fused and fw.transB), job.flops, 1, 5)
        print(json.dumps({"blas_probe": args.workload, "launches": 6, **y}))
        return 0
    sets = [(dA, dB, dC)]
    for _ in range(1, max(1, args.rotate)):
        sets.append((dA.clone(), dB.clone(), torch.empty_like(dC)))
    calls = [0]
    structure = [fw.a_structure if fused else "general"]       # what step() promises about A

    def step():
        a, b, c = sets[calls[0] % len(sets)]
        calls[0] += 1
        if fused:
            binding.gemm_epilogue_bf16_fused(M, N, K, a, lda, b, ldb, c, N, batch=batch, transA=fw.transA,
                                             transB=fw.transB, alpha=w.alpha, row_scale=drs, bias=dbias,
                                             residual=dR, ldr=N, beta=fw.beta, act=w.act, clamp=fw.clamp,
                                             stream=stream, a_structure=structure[0])
        elif f32:
            binding.gemm_epilogue_f32(M, N, K, a, K, b, N, dbias, w.alpha, w.act, c, N, batch, stream=stream)
        else:
            binding.gemm_epilogue_bf16(M, N, K, a, K, b, N, dbias, w.alpha, w.act, c, N, batch, stream=stream)

    for _ in range(args.warmup):
        step()
    calls[0] = 0
    torch.cuda.synchronize()
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record(stream)
    for _ in range(args.steps):
        step()
    ev1.record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_wall = (t1 - t0) * 1e3 / args.steps
    ms_dev = ev0.elapsed_time(ev1) / args.steps     # HIP events on the launch stream
    config_name = binding.last_config()
    # spread of single launches (outside the timed region): an event pair around each of 20 launches
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(20)]
    for a, b in pairs:
        a.record(stream)
        step()
        b.record(stream)
    torch.cuda.synchronize()
    singles = sorted(a.elapsed_time(b) for a, b in pairs)

    tflops = job.flops / (ms_wall * 1e-3) / 1e12
    bound = BOUND[args.workload]
    if bound == "mfma":
        achieved = job.flops / (ms_dev * 1e-3) / 1e12
        roofline = {"bound": "mfma", "achieved": round(achieved, 2), "peak": peak_mfma,
                    "unit": "TFLOP/s", "frac": round(achieved / peak_mfma, 4), "traffic": None}
    else:
        achieved = job.algorithmic_bytes / (ms_dev * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": round(achieved / PEAK_HBM_GBS, 4), "traffic": None}
    roofline["traffic"] = measured_traffic(args.workload, config_name)     # HBM-side bytes per launch, or null
    roofline["kernel"] = config_name
    roofline["ms_per_launch"] = round(ms_dev, 4)
    roofline["ms_single_launch"] = {"median": round(singles[len(singles) // 2], 4), "min": round(singles[0], 4)}
    ceilings = None
    if not args.no_ceilings:
        # fp32 operands: no probe of the fp32 matrix pipe exists, the datasheet fraction stands alone
        ceilings = measured_ceilings(torch, binding, dA, stream, mix=STREAM_MIX.get(args.workload), mfma=not f32)
        if bound == "hbm":
            roofline["frac_of_measured"] = round(achieved / ceilings["stream_mix_gbs"], 4)
        elif not f32:
            roofline["frac_of_measured"] = round(achieved / ceilings["mfma_bf16_tflops"], 4)

    # a structured A: the same call without the promise (every multiply-add of the full product), for scale
    general = None
    if structure[0] != "general":
        structure[0] = "general"
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        g0.record(stream)
        for _ in range(args.steps):
            step()
        g1.record(stream)
        torch.cuda.synchronize()
        general = {"ms_per_launch": round(g0.elapsed_time(g1) / args.steps, 4), "kernel": binding.last_config(),
                   "speedup_of_the_promise": round(g0.elapsed_time(g1) / args.steps / ms_dev, 3)}
        structure[0] = fw.a_structure
        step()                                                  # leave the promised call's result in C
        torch.cuda.synchronize()
    blas = None
    if not args.no_blas and not f32:
        try:
            blas = blas_yardstick(torch, dA, dB, bool(fused and fw.transA), bool(fused and fw.transB), job.flops,
                                  args.warmup, args.steps)
        except Exception as exc:        # a yardstick only: its failure is reported, not fatal
            blas = {"error": f"{type(exc).__name__}: {exc}"[:200]}

    # ---- CPU oracle on a bounded sample of the same workload, and parity on that sample
    cpu_baseline = None
    parity = None
    if args.oracle_rows > 0:
        import oracle
        # the widened operator's oracle walks every output with its own k loop: a smaller sample
        rows = sample_rows(M, min(args.oracle_rows, 512) if fused else args.oracle_rows)
        nb = 1 if batch == 1 else min(batch, max(1, args.oracle_rows // len(rows)))
        bsel = np.unique(np.round(np.linspace(0, batch - 1, nb)).astype(np.int64))
        got = dC[torch.from_numpy(bsel).to(dev)][:, torch.from_numpy(rows).to(dev)].to(torch.float32)
        got = got.cpu().numpy().astype(np.float64)
        B_s = np.ascontiguousarray(B[bsel])
        if fused:
            # the sampled rows of A in A's own storage (columns of it when A is stored K x M)
            A_s = np.ascontiguousarray(A[bsel][:, :, rows] if fw.transA else A[bsel][:, rows])
            rs_s = None if host["row_scale"] is None else host["row_scale"][rows]
            R_s = None if host["residual"] is None else np.ascontiguousarray(host["residual"][bsel][:, rows])
            c0 = time.perf_counter()
            ref = oracle.gemm_fused(len(rows), N, K, A_s, B_s, batch=len(bsel), transA=fw.transA, transB=fw.transB,
                                    alpha=w.alpha, row_scale=rs_s, bias=bias, residual=R_s, beta=fw.beta,
                                    act=w.act, clamp=fw.clamp, out=fw.out)
            c1 = time.perf_counter()
        else:
            A_s = np.ascontiguousarray(A[bsel][:, rows])
            c0 = time.perf_counter()
            ref = oracle.gemm_epilogue(A_s, B_s, bias, w.alpha, w.act)
            c1 = time.perf_counter()
        sample_flops = 2.0 * len(bsel) * len(rows) * N * K
        cpu_baseline = {"value": round(sample_flops / (c1 - c0) / 1e12, 6), "unit": "TFLOP/s",
                        "cores": oracle.num_threads(), "kind": "oracle",
                        "sample": f"{len(rows)} of {M} rows of C in {len(bsel)} of {batch} batch(es), "
                                  f"full N={N}, K={K}; {c1 - c0:.1f} s"}
        err = np.abs(got - ref)
        rel = float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))
        ok = bool(rel <= 1e-3 and np.all(err <= 1e-2 * np.maximum(1.0, np.abs(ref))))
        parity = {"rows_checked": int(len(rows) * len(bsel)), "rel_frobenius": rel,
                  "max_abs_err": float(err.max()), "ok": ok}

    out = {
        "metric": ("TFLOP/s and % of MI355X fp32 MFMA peak, fp32 GEMM" if f32 else
                   "TFLOP/s and % of MI355X bf16 MFMA peak, GEMM+bias+GELU at 8192^3"),
        "value": round(tflops, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_wall, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if f32 else "bf16",
        "data": "synthetic",
        "config": {"workload": args.workload, "M": M, "N": N, "K": K, "batch": batch,
                   "alpha": w.alpha, "act": w.act, "bias": w.bias is not None,
                   "out_dtype": fw.out if fused else "f32",
                   "layout": ("t" if fused and fw.transA else "n") + ("t" if fused and fw.transB else "n"),
                   "row_scale": bool(fused and fw.row_scale), "residual": fw.residual if fused else None,
                   "clamp": fw.clamp if fused else None, "a_structure": fw.a_structure if fused else "general",
                   "kernel": config_name},
        ("pct_of_f32_mfma_peak" if f32 else "pct_of_bf16_mfma_peak"): round(100.0 * tflops / peak_mfma, 2),
        "roofline": roofline,
        "ceilings": ceilings,
        "general_call": general,
        "blas_yardstick": blas,
        "cpu_baseline": cpu_baseline,
        "parity": parity,
    }
    print(json.dumps(out))
    if parity is not None and not parity["ok"]:
        print("parity check against the oracle FAILED", file=sys.stderr)
        return 1
    return 0


if __name__ == "__main__":
    sys.exit(main())
