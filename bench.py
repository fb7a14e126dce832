#!/usr/bin/env python3
"""Benchmark of the format-customization hot path on one MI355X.

One step = one pass of the whole path over the headline workload (BASELINE config 2:
1,048,576^2 power-law matrix, ~16.8 M nnz, unsorted COO resident in HBM):
COO->CSR, COO->DCSR, SpMV over each.  The other four workloads are run as well and
reported under "workloads" (DIA+CSR and ELL+COO decompositions, BCSR, SpMM).

Prints ONE JSON line.  `value` = matrix non-zeros pushed through the whole step per second.
Per-kernel figures come from HIP events recorded by the library around every kernel launch
on its own stream during the timed steps (us_profile_*).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
FP32_MFMA_PEAK_TFLOPS = 157.3  # MI355X dense fp32 matrix peak, published
# HBM bytes per launch (fetched + written) of the dominant kernel on the headline workload, from the
# two rocprofv3 --pmc runs summarised in profiles/config2_hbm_traffic_pmc.txt (mean over all
# scatter launches; FETCH_SIZE x2.00, WRITE_SIZE x1.00 after calibration with a plain copy)
PMC_TRAFFIC_BYTES = {"radix_scatter": 435.1e6}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--only-headline", action="store_true", help="skip the four other workloads")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pmc", nargs="?", const="headline", default=None, choices=["headline", "config4", "config5"],
                    help="counter-collection workload for rocprofv3 --pmc: 3 plain copies of 256 MiB (calibration), "
                         "then 3 headline steps (default), or 3 products of config 4 (BCSR SpMM) / config 5 (ELL+COO SpMM)")
    return ap.parse_args()


def timed(torch, fn, steps, warmup):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps * 1e3


def kernel_table(report):
    rows = []
    for e in report:
        avg_ms = e["total_ms"] / e["launches"]
        per_launch = e["alg_bytes"] / e["launches"]
        rows.append({"kernel": e["kernel"], "launches": e["launches"], "total_ms": round(e["total_ms"], 4),
                     "avg_us": round(avg_ms * 1e3, 2), "alg_bytes_per_launch": per_launch,
                     "gbps": round(per_launch / (avg_ms * 1e-3) / 1e9, 1) if avg_ms > 0 else None})
    rows.sort(key=lambda r: -r["total_ms"])
    return rows


def profile_of(B, torch, ctx, fn, steps):
    ctx.enable_profile()
    ctx.profile_reset()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    rep = ctx.profile_report()
    ctx.disable_profile()
    for e in rep:
        e["launches_per_step"] = e["launches"] / steps
    return rep


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2403_05802_amd import binding as B
    from paper_2403_05802_amd import workloads as W
    B.lib()  # fails loudly if the HIP library is missing
    dev = torch.device("cuda:0")
    ctx = B.Context("cuda:0")
    up = lambda a: torch.from_numpy(a).to(dev)
    K, Wm = args.steps, args.warmup
    CSR, DCSR = B.us_desc_preset(B.US_F_CSR), B.us_desc_preset(B.US_F_DCSR)
    out = {}

    # ------------------------------------------------------------------ headline: config 2
    m = W.cfg2_powerlaw()
    r, c, v = up(m.row), up(m.col), up(m.val)
    x = up(W.dense_operand(2, m.ncols))
    y = torch.empty(m.nrows, device=dev)
    nnz = m.nnz

    def step():
        # each layout is multiplied right after it is built (its arrays are then still in the memory-side cache)
        # and released without waiting for the product: torch's allocator orders the reuse of the memory with the
        # stream, so the frees and the next conversion's set-up overlap the product
        a = B.us_convert(ctx, m.nrows, m.ncols, r, c, v, CSR)
        B.us_spmv(ctx, a, x, y)
        a.free(wait=False)
        b = B.us_convert(ctx, m.nrows, m.ncols, r, c, v, DCSR)
        B.us_spmv(ctx, b, x, y)
        b.free(wait=False)

    if args.pmc:
        a = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device=dev).fill_(1.0)
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        del a, b
        if args.pmc == "headline":
            for _ in range(3):
                step()
            torch.cuda.synchronize()
            what = "3 headline steps"
        else:
            del r, c, v
            what = pmc_products(B, W, torch, ctx, up, args.pmc)
        print(json.dumps({"pmc_workload": "3 copies of 268435456 B, then " + what}))
        return

    # the timed steps: W warm-up, then exactly K, with a HIP event pair around every launch of the
    # dominant kernel only (launches moving at least 300 MB: the ten scatter passes of a step); the
    # other ~90 launches per step are left alone so that event recording costs the timed region a
    # few per cent, not 20 %.  The full per-kernel table comes from a separate loop below.
    ctx.enable_profile(); ctx.profile_min_bytes(3e8); ctx.profile_reset()
    for _ in range(Wm):
        step()
    torch.cuda.synchronize(); ctx.profile_reset()
    t0 = time.perf_counter()
    for _ in range(K):
        step()
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) / K * 1e3
    rep = ctx.profile_report()
    ctx.disable_profile()
    ms_plain = timed(torch, step, K, 1)          # the same K steps without event recording
    per = []
    for _ in range(K):                           # per-step spread (each step ends with a synchronize)
        torch.cuda.synchronize(); t1 = time.perf_counter(); step(); torch.cuda.synchronize()
        per.append((time.perf_counter() - t1) * 1e3)
    ms_std = float(np.std(per))
    dom = kernel_table(rep)[0]
    ctx.profile_min_bytes(0.0)
    table = kernel_table(profile_of(B, torch, ctx, step, K))   # every launch, for the full per-kernel table
    roofline = {"bound": "hbm", "kernel": dom["kernel"], "achieved": dom["gbps"], "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(dom["gbps"] / HBM_PEAK_GBS, 4),
                "avg_launch_us": dom["avg_us"], "alg_bytes_per_launch": dom["alg_bytes_per_launch"],
                "traffic": PMC_TRAFFIC_BYTES.get(dom["kernel"])}
    # practical ceiling: a plain device-to-device copy of 256 MiB timed in the same run
    ca = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device=dev).fill_(1.0)
    cb = torch.empty_like(ca)
    ms_copy = timed(torch, lambda: cb.copy_(ca), 20, 3)
    copy_gbps = 2 * ca.numel() * 4 / ms_copy / 1e6
    del ca, cb

    # separate timings of the pieces (each its own timed loop)
    fa = B.us_convert(ctx, m.nrows, m.ncols, r, c, v, CSR)
    fb = B.us_convert(ctx, m.nrows, m.ncols, r, c, v, DCSR)
    ms_csr = timed(torch, lambda: B.us_convert(ctx, m.nrows, m.ncols, r, c, v, CSR).free(), K, 1)
    ms_dcsr = timed(torch, lambda: B.us_convert(ctx, m.nrows, m.ncols, r, c, v, DCSR).free(), K, 1)
    ms_spmv = timed(torch, lambda: B.us_spmv(ctx, fa, x, y), K * 5, 3)
    ms_spmv_d = timed(torch, lambda: B.us_spmv(ctx, fb, x, y), K * 5, 3)
    conv_bytes = 20.0 * nnz + 4.0 * (m.nrows + 1)
    spmv_bytes = 8.0 * nnz + 4.0 * (m.nrows + 1) + 8.0 * m.nrows
    headline = {
        "nnz": nnz, "nrows": m.nrows,
        "coo_to_csr": {"ms": round(ms_csr, 4), "mnnz_s": round(nnz / ms_csr / 1e3, 1),
                       "useful_gbps": round(conv_bytes / ms_csr / 1e6, 1),
                       "useful_frac_of_hbm": round(conv_bytes / ms_csr / 1e6 / HBM_PEAK_GBS, 4)},
        "coo_to_dcsr": {"ms": round(ms_dcsr, 4), "mnnz_s": round(nnz / ms_dcsr / 1e3, 1)},
        "spmv_csr": {"ms": round(ms_spmv, 4), "gflop_s": round(2.0 * nnz / ms_spmv / 1e6, 1),
                     "useful_gbps": round(spmv_bytes / ms_spmv / 1e6, 1),
                     "useful_frac_of_hbm": round(spmv_bytes / ms_spmv / 1e6 / HBM_PEAK_GBS, 4)},
        "spmv_dcsr": {"ms": round(ms_spmv_d, 4), "gflop_s": round(2.0 * nnz / ms_spmv_d / 1e6, 1)},
        "ms_per_step_without_event_recording": round(ms_plain, 4),
        "ms_per_step_std": round(ms_std, 4),
        "mnnz_s_without_event_recording": round(nnz / ms_plain / 1e3, 1),
        "device_copy_gbps": round(copy_gbps, 1),
        "kernels": table,
    }
    fa.free(); fb.free()

    # ------------------------------------------------------------------ CPU baseline: the oracle, bounded sample
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import unisparse_oracle as O
        ns = nnz   # the whole headline workload: ~10 s of single-core numpy on the GPU machine's host
        sr, sc, sv = m.row[:ns], m.col[:ns], m.val[:ns]
        xs = W.dense_operand(2, m.ncols)
        t0 = time.perf_counter()
        oa = O.convert(m.nrows, m.ncols, sr, sc, sv, O.CSR())
        ob = O.convert(m.nrows, m.ncols, sr, sc, sv, O.DCSR())
        O.spmv(oa, xs); O.spmv(ob, xs)
        dt = time.perf_counter() - t0
        cpu = {"value": round(ns / dt / 1e6, 3), "unit": "Mnnz/s", "cores": 1, "kind": "oracle",
               "sample": f"all {ns} entries of config 2, one step (COO->CSR, COO->DCSR, SpMV over each), "
                         f"numpy single thread; {dt:.1f} s"}
        del oa, ob
    del r, c, v, m
    torch.cuda.empty_cache()

    # ------------------------------------------------------------------ the other workloads
    if not args.only_headline:
        try:
            out["workloads"] = other_workloads(B, W, torch, ctx, up, max(3, K // 2), 2)
        except Exception as e:   # the headline line is still printed; the failure is in it and on stderr
            out["workloads_error"] = repr(e)
            print("bench.py: a workload beside the headline failed: " + repr(e), file=sys.stderr)

    line = {
        "metric": "conversion Mnnz/s + SpMV GFLOP/s; achieved HBM GB/s as % of MI355X peak",
        "value": round(nnz / ms_step / 1e3, 1), "unit": "Mnnz/s",
        "n_gpus": 1, "steps": K, "warmup": Wm, "ms_per_step": round(ms_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u64",
        "dtype_note": "sort keys u64 (40-bit packed (row,col)), indices int32, values and products f32 (f32 accumulate)",
        "data": "synthetic",
        "config": {"workload": "config 2: 1,048,576^2 fp32, Zipf(1.8) row lengths 1..20000, uniform columns, "
                               f"{nnz} nnz, unsorted COO in HBM; step = COO->CSR + COO->DCSR + SpMV over each"},
        "conversion_mnnz_s": headline["coo_to_csr"]["mnnz_s"],
        "spmv_gflop_s": headline["spmv_csr"]["gflop_s"],
        "roofline": roofline,
        "cpu_baseline": cpu,
        "headline": headline,
    }
    line.update(out)
    print(json.dumps(line))


def pmc_products(B, W, torch, ctx, up, which):
    """Three products of config 4 (COO->BCSR once, then SpMM N=64) or config 5 (decompose once, then the
    hybrid SpMM N=128), for a rocprofv3 --pmc run."""
    dev = torch.device("cuda:0")
    if which == "config4":
        m = W.cfg4_blockfem()
        parts = [B.us_convert(ctx, m.nrows, m.ncols, up(m.row), up(m.col), up(m.val), B.us_desc_preset(B.US_F_BCSR, 4, 4))]
        N = 64
    else:
        m = W.cfg5_powerlaw_local()
        pr = B.make_predicate([B.expr(B.US_E_AFFINE, 1, 0)], B.US_P_RANK_LT_PERCENTILE, 9, 10)
        parts = list(B.us_decompose(ctx, m.nrows, m.ncols, up(m.row), up(m.col), up(m.val),
                                    B.us_desc_preset(B.US_F_ELL), B.us_desc_preset(B.US_F_COO), pr))
        N = 128
    X = up(W.dense_operand(int(which[-1]), (m.ncols, N))); Y = torch.empty(m.nrows, N, device=dev)
    for _ in range(3):
        for k, p in enumerate(parts):
            B.us_spmm(ctx, p, X, Y, accumulate=k > 0)
        torch.cuda.synchronize()
    return f"3 products of {which} (N = {N}, {m.nnz} nnz)"


def other_workloads(B, W, torch, ctx, up, K, Wm):
    """Configs 1, 3, 4, 5: conversion / decomposition and the product each names."""
    dev = torch.device("cuda:0")
    res = {}
    E = B.expr

    def run(name, m, conv, prod, flops, conv_bytes):
        r, c, v = up(m.row), up(m.col), up(m.val)
        parts = conv(r, c, v)
        ms_conv = timed(torch, lambda: [p.free() for p in conv(r, c, v)], K, Wm)
        ms_prod = timed(torch, lambda: prod(parts), K * 2, Wm)
        rep = profile_of(B, torch, ctx, lambda: ([p.free() for p in conv(r, c, v)], prod(parts)), 3)
        res[name] = {"nnz": m.nnz, "convert_ms": round(ms_conv, 4), "convert_mnnz_s": round(m.nnz / ms_conv / 1e3, 1),
                     "convert_useful_gbps": round(conv_bytes(parts) / ms_conv / 1e6, 1),
                     "product_ms": round(ms_prod, 4), "product_gflop_s": round(flops / ms_prod / 1e6, 1),
                     "kernels": kernel_table(rep)[:8]}
        for p in parts:
            p.free()
        del r, c, v
        torch.cuda.empty_cache()

    CSR, COO = B.us_desc_preset(B.US_F_CSR), B.us_desc_preset(B.US_F_COO)
    # config 1
    m = W.cfg1_uniform()
    x = up(W.dense_operand(1, m.ncols)); y = torch.empty(m.nrows, device=dev)
    run("config1_csr_spmv", m, lambda r, c, v: [B.us_convert(ctx, m.nrows, m.ncols, r, c, v, CSR)],
        lambda p: B.us_spmv(ctx, p[0], x, y), 2.0 * m.nnz, lambda p: 20.0 * m.nnz + 4.0 * m.nrows)
    # config 2 once more, into the scheduled layout of Section 7.2.4 (1024 partitions, its core count) + SpMV
    m = W.cfg2_powerlaw()
    x = up(W.dense_operand(2, m.ncols)); y = torch.empty(m.nrows, device=dev)
    CP = B.us_desc_preset(B.US_F_CISR_PLUS, 1024)
    run("config2_cisr_plus_spmv", m, lambda r, c, v: [B.us_convert(ctx, m.nrows, m.ncols, r, c, v, CP)],
        lambda p: B.us_spmv(ctx, p[0], x, y), 2.0 * m.nnz, lambda p: 20.0 * m.nnz + 8.0 * m.nrows)
    # config 2 with half of its rows emptied, so that the doubly compressed layout has rows to drop
    m = W.cfg2_powerlaw(empty_frac=0.5)
    x = up(W.dense_operand(2, m.ncols)); y = torch.empty(m.nrows, device=dev)
    DCSR = B.us_desc_preset(B.US_F_DCSR)
    run("config2_half_empty_rows_dcsr_spmv", m, lambda r, c, v: [B.us_convert(ctx, m.nrows, m.ncols, r, c, v, DCSR)],
        lambda p: B.us_spmv(ctx, p[0], x, y), 2.0 * m.nnz, lambda p: 20.0 * m.nnz + 8.0 * p[0].idx(0).numel())
    # config 3
    m = W.cfg3_banded()
    x = up(W.dense_operand(3, m.ncols)); y = torch.empty(m.nrows, device=dev)
    DIA = B.us_desc_preset(B.US_F_DIA)
    pd = B.make_predicate([E(B.US_E_AFFINE, -1, 1)], B.US_P_SUM_GE_FRAC_OF_CAPACITY, 9, 10)

    def prod3(p):
        B.us_spmv(ctx, p[0], x, y); B.us_spmv(ctx, p[1], x, y, accumulate=True)
    run("config3_dia_csr_spmv", m, lambda r, c, v: list(B.us_decompose(ctx, m.nrows, m.ncols, r, c, v, DIA, CSR, pd)),
        prod3, 2.0 * m.nnz,
        lambda p: 12.0 * m.nnz + 4.0 * p[0].val().numel() + 8.0 * p[1].nnz + 4.0 * m.nrows)
    # the same matrix through the program of Figure 3c: blocked DIA (block 4) + CSR, #sum over (d0/4, d1-d0) >= 4
    BDIA = B.us_desc_preset(B.US_F_BDIA, 4)
    pb = B.make_predicate([E(B.US_E_DIV, 1, 0, 0, 4), E(B.US_E_AFFINE, -1, 1)], B.US_P_SUM_GE_ABS, abs_=4)
    run("config3_bdia_csr_spmv", m, lambda r, c, v: list(B.us_decompose(ctx, m.nrows, m.ncols, r, c, v, BDIA, CSR, pb)),
        prod3, 2.0 * m.nnz,
        lambda p: 12.0 * m.nnz + 4.0 * p[0].val().numel() + 4.0 * p[0].idx(1).numel() + 8.0 * p[1].nnz + 4.0 * m.nrows)
    # config 4
    m = W.cfg4_blockfem()
    X = up(W.dense_operand(4, (m.ncols, 64))); Y = torch.empty(m.nrows, 64, device=dev)
    BC = B.us_desc_preset(B.US_F_BCSR, 4, 4)
    run("config4_bcsr_spmm64", m, lambda r, c, v: [B.us_convert(ctx, m.nrows, m.ncols, r, c, v, BC)],
        lambda p: B.us_spmm(ctx, p[0], X, Y), 2.0 * m.nnz * 64,
        lambda p: 12.0 * m.nnz + 4.0 * p[0].val().numel() + 4.0 * p[0].idx(1).numel())
    # the same conversion with whole-array digit passes only (blocked tuples finish inside LDS by default)
    ctx.set_sort_lds_finish(False)
    try:
        r, c, v = up(m.row), up(m.col), up(m.val)
        ms = timed(torch, lambda: B.us_convert(ctx, m.nrows, m.ncols, r, c, v, BC).free(), K, Wm)
        res["config4_bcsr_spmm64"]["convert_ms_whole_array_passes_only"] = round(ms, 4)
        res["config4_bcsr_spmm64"]["convert_mnnz_s_whole_array_passes_only"] = round(m.nnz / ms / 1e3, 1)
        del r, c, v
    finally:
        ctx.set_sort_lds_finish(None)
    del X, Y
    # config 5
    m = W.cfg5_powerlaw_local()
    X = up(W.dense_operand(5, (m.ncols, 128))); Y = torch.empty(m.nrows, 128, device=dev)
    ELL = B.us_desc_preset(B.US_F_ELL)
    pr = B.make_predicate([E(B.US_E_AFFINE, 1, 0)], B.US_P_RANK_LT_PERCENTILE, 9, 10)

    def prod5(p):
        B.us_spmm(ctx, p[0], X, Y); B.us_spmm(ctx, p[1], X, Y, accumulate=True)
    run("config5_ell_coo_spmm128", m,
        lambda r, c, v: list(B.us_decompose(ctx, m.nrows, m.ncols, r, c, v, ELL, COO, pr)), prod5,
        2.0 * m.nnz * 128, lambda p: 12.0 * m.nnz + 8.0 * p[0].val().numel() + 12.0 * p[1].nnz)
    res["label_propagation"] = label_propagation(B, W, torch, ctx, up)
    res["format_to_format"] = format_to_format(B, W, torch, ctx, up, K, Wm)
    return res


def format_to_format(B, W, torch, ctx, up, K, Wm):
    """The conversion cases of Table 5 on the benchmark matrices: COO -> ELL (config 4), COO -> DIA (config 3's
    diagonals), and through the COO hub CSR -> CSC (config 2), DCSC -> BCSR 4x4 (config 4), CSB -> DIA variant
    (config 3's diagonals)."""
    out = {}

    def one(name, m, src_desc, dst_desc):
        r, c, v = up(m.row), up(m.col), up(m.val)
        src = B.us_convert(ctx, m.nrows, m.ncols, r, c, v, src_desc)
        del r, c, v
        ms = timed(torch, lambda: B.us_convert_formatted(ctx, src, dst_desc).free(), K, Wm)
        out[name] = {"nnz": m.nnz, "convert_ms": round(ms, 4), "convert_mnnz_s": round(m.nnz / ms / 1e3, 1)}
        src.free()
        torch.cuda.empty_cache()

    def from_coo(name, m, dst_desc, also_with_lds_finish=False):
        r, c, v = up(m.row), up(m.col), up(m.val)
        ms = timed(torch, lambda: B.us_convert(ctx, m.nrows, m.ncols, r, c, v, dst_desc).free(), K, Wm)
        out[name] = {"nnz": m.nnz, "convert_ms": round(ms, 4), "convert_mnnz_s": round(m.nnz / ms / 1e3, 1)}
        if also_with_lds_finish:
            # (row, col) tuples keep whole-array digit passes by default (rows of a power-law matrix overflow the
            # buckets of the in-LDS finish); a caller who knows its rows are even can ask for the finish
            ctx.set_sort_lds_finish(True)
            try:
                ms = timed(torch, lambda: B.us_convert(ctx, m.nrows, m.ncols, r, c, v, dst_desc).free(), K, Wm)
                out[name]["convert_ms_with_lds_finish"] = round(ms, 4)
                out[name]["convert_mnnz_s_with_lds_finish"] = round(m.nnz / ms / 1e3, 1)
            finally:
                ctx.set_sort_lds_finish(None)
        del r, c, v
        torch.cuda.empty_cache()

    P = B.us_desc_preset
    from_coo("config4_coo_to_ell", W.cfg4_blockfem(), P(B.US_F_ELL), also_with_lds_finish=True)   # 96 entries in every row
    from_coo("config3_diagonals_coo_to_dia", W.cfg3_banded(extra_frac=0.0), P(B.US_F_DIA))
    one("config2_csr_to_csc", W.cfg2_powerlaw(), P(B.US_F_CSR), P(B.US_F_CSC))
    one("config4_dcsc_to_bcsr", W.cfg4_blockfem(), P(B.US_F_DCSC), P(B.US_F_BCSR, 4, 4))
    one("config3_diagonals_csb_to_dia_variant", W.cfg3_banded(extra_frac=0.0), P(B.US_F_CSB, 512, 512),
        P(B.US_F_DIA_VARIANT))
    return out


def label_propagation(B, W, torch, ctx, up, iters=20, N=1000):
    """The paper's label-propagation case study (Section 7.2.5): `iters` products Y <- A_hat Y with a
    row-normalised power-law graph and N = 1000 labels, over CSR and over the ELL+COO hybrid,
    with the conversion (pre-processing) time beside the kernel time."""
    import numpy as np
    dev = torch.device("cuda:0")
    m = W.cfg5_powerlaw_local(n=1 << 18, target_nnz=5_200_000, max_len=20000, index=6)
    deg = np.bincount(m.row, minlength=m.nrows)
    val = (1.0 / deg[m.row]).astype(np.float32)
    r, c, v = up(m.row), up(m.col), up(val)
    Y0 = up(W.dense_operand(6, (m.ncols, N)))
    bufs = [Y0.clone(), torch.empty_like(Y0)]
    CSR, COO, ELL = B.us_desc_preset(B.US_F_CSR), B.us_desc_preset(B.US_F_COO), B.us_desc_preset(B.US_F_ELL)
    pr = B.make_predicate([B.expr(B.US_E_AFFINE, 1, 0)], B.US_P_RANK_LT_PERCENTILE, 9, 10)

    def loop(parts):
        for t in range(iters):
            src, dst = bufs[t & 1], bufs[(t + 1) & 1]
            for k, p in enumerate(parts):
                B.us_spmm(ctx, p, src, dst, accumulate=k > 0)

    out = {"nrows": m.nrows, "nnz": m.nnz, "N": N, "iterations": iters}
    for name, conv in (("csr", lambda: [B.us_convert(ctx, m.nrows, m.ncols, r, c, v, CSR)]),
                       ("ell_coo", lambda: list(B.us_decompose(ctx, m.nrows, m.ncols, r, c, v, ELL, COO, pr)))):
        ms_conv = timed(torch, lambda: [p.free() for p in conv()], 5, 2)
        parts = conv()
        ms_loop = timed(torch, lambda: loop(parts), 3, 1)
        out[name] = {"preprocess_ms": round(ms_conv, 3), "kernels_ms": round(ms_loop, 3),
                     "total_ms": round(ms_conv + ms_loop, 3),
                     "gflop_s": round(2.0 * m.nnz * N * iters / ms_loop / 1e6, 1)}
        for p in parts:
            p.free()
    return out


if __name__ == "__main__":
    main()
