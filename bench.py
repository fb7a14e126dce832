#!/usr/bin/env python3
"""Benchmark of the format-customization hot path on one MI355X.

One step = one pass of the whole path over the headline workload, the largest configuration (config 5:
2,000,000^2 power-law matrix with local columns, ~38.4 M entries, unsorted COO resident in HBM):
decompose into ELL (width = 90th-percentile row length) + COO overflow, SpMM over the hybrid with a dense
X of width 128, and SpMV over the same hybrid.  Configs 1-4 (and variants of them) run as well and are
reported under "workloads".

Prints ONE JSON line.  `value` = matrix non-zeros pushed through the whole step per second.
`roofline` carries the dominant kernel of the step (algorithmic bytes per launch / mean launch duration from HIP
events recorded by the library on its own stream, us_profile_*) and, as `op_frac`, what the task's 60 % target
is written on: the compulsory bytes of each whole operation (input once + output once) / its time / 8 TB/s.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
FP32_MFMA_PEAK_TFLOPS = 157.3  # MI355X dense fp32 matrix peak, published
TARGET_FRAC = 0.60             # the task's target for conversion and SpMV on the largest config
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "config5_step_hbm_traffic_pmc.txt")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--only-headline", action="store_true", help="skip the other workloads")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pmc", nargs="?", const="config5", default=None,
                    choices=["config2", "config3", "config4", "config5"],
                    help="counter-collection run for rocprofv3 --pmc: 3 plain copies of 256 MiB (calibration), "
                         "then 3 steps (conversion / decomposition + products) of the named config")
    return ap.parse_args()


def timed(torch, fn, steps, warmup):
    """mean and standard deviation (ms) of `steps` calls, each bracketed by a device synchronise."""
    for _ in range(warmup):
        fn()
    ts = []
    for _ in range(steps):
        torch.cuda.synchronize(); t0 = time.perf_counter(); fn(); torch.cuda.synchronize()
        ts.append((time.perf_counter() - t0) * 1e3)
    return float(np.mean(ts)), float(np.std(ts))


def timed_stream(torch, fn, steps, warmup):
    """mean ms per call of `steps` calls enqueued back to back (products only enqueue)."""
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


def profile_of(torch, ctx, fn, steps):
    ctx.enable_profile()
    ctx.profile_min_bytes(0.0)
    ctx.profile_reset()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    rep = ctx.profile_report()
    ctx.disable_profile()
    return rep


def traffic_from_profile(kernel):
    """HBM bytes per launch of `kernel` (the library's launch name) from the committed rocprofv3 --pmc summary:
    its lines `traffic <launch name> <fetched bytes> <written bytes>` (per launch, calibrated).  None if absent."""
    try:
        for line in open(TRAFFIC_PROFILE):
            m = re.match(r"traffic\s+(\S+)\s+([0-9.eE+]+)\s+([0-9.eE+]+)", line)
            if m and m.group(1) == kernel:
                return float(m.group(2)) + float(m.group(3))
    except OSError:
        pass
    return None


def frac(nbytes, ms):
    return round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)


# ----------------------------------------------------------------------------- the five configs
class Workload:
    """One config: how it is converted, multiplied, what its operations must move at least, and the bounded sample
    of it that the CPU oracle is timed on."""

    def __init__(self, B, W, torch, ctx, up, index):
        self.B, self.W, self.torch, self.ctx, self.up, self.index = B, W, torch, ctx, up, index
        P, E = B.us_desc_preset, B.expr
        dev = torch.device("cuda:0")
        if index == 1:
            self.m = m = W.cfg1_uniform()
            self.name = "config 1: 4096^2, 40,960 uniform entries; COO->CSR, SpMV"
            self.descs, self.pred, self.N = [P(B.US_F_CSR)], None, 0
        elif index == 2:
            self.m = m = W.cfg2_powerlaw()
            self.name = ("config 2: 1,048,576^2, Zipf(1.8) row lengths 1..20000, uniform columns; COO->CSR, SpMV "
                         "(COO->DCSR and the scheduled layout under their own names)")
            self.descs, self.pred, self.N = [P(B.US_F_CSR)], None, 0
        elif index == 3:
            self.m = m = W.cfg3_banded()
            self.name = "config 3: 2,097,152^2, 7 full diagonals + 1 % scattered; decompose -> DIA + CSR, hybrid SpMV"
            self.descs = [P(B.US_F_DIA), P(B.US_F_CSR)]
            self.pred, self.N = B.make_predicate([E(B.US_E_AFFINE, -1, 1)], B.US_P_SUM_GE_FRAC_OF_CAPACITY, 9, 10), 0
        elif index == 4:
            self.m = m = W.cfg4_blockfem()
            self.name = "config 4: 524,288^2, dense 4x4 blocks, 24 per block row in a +-4096 band; COO->BCSR(4x4), SpMM N=64"
            self.descs, self.pred, self.N = [P(B.US_F_BCSR, 4, 4)], None, 64
        else:
            self.m = m = W.cfg5_powerlaw_local()
            self.name = ("config 5: 2,000,000^2, Zipf(2.0) row lengths, columns 70 % within +-512 of the row / 30 % uniform; "
                         "decompose -> ELL (90th-percentile width) + COO, SpMM N=128 and SpMV over the hybrid")
            self.descs = [P(B.US_F_ELL), P(B.US_F_COO)]
            self.pred, self.N = B.make_predicate([E(B.US_E_AFFINE, 1, 0)], B.US_P_RANK_LT_PERCENTILE, 9, 10), 128
        self.r, self.c, self.v = up(m.row), up(m.col), up(m.val)
        self.x = up(W.dense_operand(index, m.ncols))
        self.y = torch.empty(m.nrows, device=dev)
        if self.N:
            self.X = up(W.dense_operand(index, (m.ncols, self.N)))
            self.Y = torch.empty(m.nrows, self.N, device=dev)

    # -- the operations
    def convert(self):
        B, m = self.B, self.m
        if self.pred is None:
            return [B.us_convert(self.ctx, m.nrows, m.ncols, self.r, self.c, self.v, self.descs[0])]
        return list(B.us_decompose(self.ctx, m.nrows, m.ncols, self.r, self.c, self.v, self.descs[0], self.descs[1], self.pred))

    def spmv(self, parts):
        for k, p in enumerate(parts):
            self.B.us_spmv(self.ctx, p, self.x, self.y, accumulate=k > 0)

    def spmm(self, parts):
        for k, p in enumerate(parts):
            self.B.us_spmm(self.ctx, p, self.X, self.Y, accumulate=k > 0)

    def step(self):
        parts = self.convert()
        if self.N:
            self.spmm(parts)
        if self.index != 4:
            self.spmv(parts)
        for p in parts:
            p.free(wait=False)   # torch's allocator orders the reuse of the memory with the stream

    # -- compulsory bytes (input once + output once) of each operation, from the arrays the result really has
    def stored_bytes(self, parts):
        """bytes of the arrays of the layout(s): what a product has to read of the matrix, what a conversion writes"""
        total = 0
        for p in parts:
            total += 4 * p.val().numel()
            for L in range(p.desc.nlevels):
                for a in (p.ptr(L), p.idx(L)):
                    if a is not None:
                        total += 4 * a.numel()
        return total

    def conv_bytes(self, parts):
        return 12.0 * self.m.nnz + self.stored_bytes(parts)

    def spmv_bytes(self, parts):
        return self.stored_bytes(parts) + 4.0 * (self.m.ncols + self.m.nrows)

    def spmm_bytes(self, parts):
        return self.stored_bytes(parts) + 4.0 * self.N * (self.m.ncols + self.m.nrows)

    # -- measurement
    def measure(self, K, Wm, kernels=True):
        torch, m = self.torch, self.m
        parts = self.convert()
        cb, out = self.conv_bytes(parts), {"workload": self.name, "nnz": m.nnz}
        ms, sd = timed(torch, lambda: [p.free() for p in self.convert()], K, Wm)
        out["convert"] = {"ms": round(ms, 4), "ms_std": round(sd, 4), "mnnz_s": round(m.nnz / ms / 1e3, 1),
                          "compulsory_bytes": cb, "useful_gbps": round(cb / ms / 1e6, 1), "op_frac": frac(cb, ms)}
        if self.index != 4:
            ms, sd = timed(torch, lambda: self.spmv(parts), K, Wm)
            ms_q = timed_stream(torch, lambda: self.spmv(parts), 4 * K, Wm)
            sb = self.spmv_bytes(parts)
            out["spmv"] = {"ms": round(ms_q, 4), "ms_one_call_with_sync": round(ms, 4), "ms_std": round(sd, 4),
                           "gflop_s": round(2.0 * m.nnz / ms_q / 1e6, 1), "compulsory_bytes": sb,
                           "useful_gbps": round(sb / ms_q / 1e6, 1), "op_frac": frac(sb, ms_q)}
        if self.N:
            ms, sd = timed(torch, lambda: self.spmm(parts), K, Wm)
            ms_q = timed_stream(torch, lambda: self.spmm(parts), 2 * K, Wm)
            sb, fl = self.spmm_bytes(parts), 2.0 * m.nnz * self.N
            out["spmm"] = {"N": self.N, "ms": round(ms_q, 4), "ms_one_call_with_sync": round(ms, 4), "ms_std": round(sd, 4),
                           "gflop_s": round(fl / ms_q / 1e6, 1), "compulsory_bytes": sb,
                           "useful_gbps": round(sb / ms_q / 1e6, 1), "op_frac": frac(sb, ms_q)}
            if self.index == 4:
                out["spmm"]["frac_of_fp32_mfma_peak"] = round(fl / ms_q / 1e9 / FP32_MFMA_PEAK_TFLOPS, 4)
        if kernels:
            out["kernels"] = kernel_table(profile_of(torch, self.ctx, self.step, 3))[:10]
        for p in parts:
            p.free()
        return out

    # -- the CPU oracle on a bounded sample of the same workload (one thread)
    def oracle_sample(self):
        from oracle import unisparse_oracle as O
        m, W = self.m, self.W
        if self.index in (1, 2):
            nr, nc, sel, what = m.nrows, m.ncols, slice(None), "the whole matrix"
        elif self.index in (3, 4):
            cut = m.nrows // (4 if self.index == 3 else 16)
            sel = (m.row < cut) & (m.col < cut)
            nr = nc = cut
            what = f"the leading {cut} x {cut} block of the matrix"
        else:
            nr, nc = m.nrows // 4, m.ncols
            sel = m.row < nr
            what = f"the first {nr} rows of the matrix (all columns)"
        r, c, v = m.row[sel], m.col[sel], m.val[sel]
        x = W.dense_operand(self.index, m.ncols)[:nc]
        X = W.dense_operand(self.index, (m.ncols, self.N))[:nc] if self.N else None
        t0 = time.perf_counter()
        if self.index in (1, 2):
            parts = [O.convert(nr, nc, r, c, v, O.CSR())]
        elif self.index == 3:
            parts = list(O.decompose(nr, nc, r, c, v, O.DIA(), O.CSR(),
                                     O.Predicate((O.diag(),), O.SUM_GE_FRAC_OF_CAPACITY, num=9, den=10))[:2])
        elif self.index == 4:
            parts = [O.convert(nr, nc, r, c, v, O.BCSR(4))]
        else:
            parts = list(O.decompose(nr, nc, r, c, v, O.ELL(), O.COO(),
                                     O.Predicate((O.d0(),), O.RANK_LT_PERCENTILE, num=9, den=10))[:2])
        t1 = time.perf_counter()
        if self.N:
            Y = None
            for p in parts:
                Y = O.spmm(p, X, Y)
        t2 = time.perf_counter()
        if self.index != 4:
            y = None
            for p in parts:
                y = O.spmv(p, x, y)
        t3 = time.perf_counter()
        n = int(r.shape[0])
        ops = "conversion" + (f" + SpMM N={self.N}" if self.N else "") + (" + SpMV" if self.index != 4 else "")
        return {"value": round(n / (t3 - t0) / 1e6, 3), "unit": "Mnnz/s", "cores": 1, "kind": "oracle",
                "sample": f"{what}, {n} entries; one step ({ops}) of the numpy oracle on one thread: "
                          f"conversion {t1 - t0:.1f} s, SpMM {t2 - t1:.1f} s, SpMV {t3 - t2:.1f} s",
                "convert_mnnz_s": round(n / (t1 - t0) / 1e6, 3),
                "spmm_gflop_s": round(2.0 * n * self.N / (t2 - t1) / 1e9, 3) if self.N else None,
                "spmv_gflop_s": round(2.0 * n / (t3 - t2) / 1e9, 3) if self.index != 4 else None}

    def release(self):
        for a in ("r", "c", "v", "x", "y", "X", "Y", "m"):
            if hasattr(self, a):
                delattr(self, a)
        self.torch.cuda.empty_cache()


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

    if args.pmc:
        a = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device=dev).fill_(1.0)
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        del a, b
        w = Workload(B, W, torch, ctx, up, int(args.pmc[-1]))
        for _ in range(3):
            w.step()
            torch.cuda.synchronize()
        print(json.dumps({"pmc_workload": "3 copies of 268435456 B, then 3 steps of " + w.name}))
        return

    # ------------------------------------------------------------------ headline: config 5
    w = Workload(B, W, torch, ctx, up, 5)
    nnz = w.m.nnz
    # the timed steps: W warm-up, then exactly K, with a HIP event pair around every large launch (those moving at
    # least 300 MB: the sort's scatter passes, the splits and the products); the ~100 small launches of a step are
    # left alone so that event recording costs the timed region little.  The full table comes from a separate loop.
    ctx.enable_profile(); ctx.profile_min_bytes(3e8); ctx.profile_reset()
    for _ in range(Wm):
        w.step()
    torch.cuda.synchronize(); ctx.profile_reset()
    t0 = time.perf_counter()
    for _ in range(K):
        w.step()
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) / K * 1e3
    rep = ctx.profile_report()
    ctx.disable_profile()
    ms_plain = timed_stream(torch, w.step, K, 1)          # the same K steps without event recording
    _, ms_std = timed(torch, w.step, K, 0)                # per-step spread (each step ends with a synchronise)
    dom = kernel_table(rep)[0]
    head = w.measure(K, 1)
    op_frac = {"config5_decompose_ell_coo": head["convert"]["op_frac"], "config5_hybrid_spmm128": head["spmm"]["op_frac"],
               "config5_hybrid_spmv": head["spmv"]["op_frac"]}
    # practical ceiling: a plain device-to-device copy of 256 MiB timed in the same run
    ca = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device=dev).fill_(1.0)
    cb = torch.empty_like(ca)
    ms_copy = timed_stream(torch, lambda: cb.copy_(ca), 20, 3)
    copy_gbps = 2 * ca.numel() * 4 / ms_copy / 1e6
    del ca, cb
    head.update({"ms_per_step_without_event_recording": round(ms_plain, 4), "ms_per_step_std": round(ms_std, 4),
                 "device_copy_gbps": round(copy_gbps, 1)})
    cpu = None if args.no_cpu_baseline else w.oracle_sample()
    w.release()

    # ------------------------------------------------------------------ the other workloads
    out = {}
    if not args.only_headline:
        try:
            out["workloads"] = other_workloads(B, W, torch, ctx, up, max(3, K // 2), 2, not args.no_cpu_baseline, op_frac)
        except Exception as e:   # the headline line is still printed; the failure is in it and on stderr
            out["workloads_error"] = repr(e)
            print("bench.py: a workload beside the headline failed: " + repr(e), file=sys.stderr)

    conv_frac, spmv_frac = op_frac["config5_decompose_ell_coo"], op_frac["config5_hybrid_spmv"]
    roofline = {"bound": "hbm", "kernel": dom["kernel"], "achieved": dom["gbps"], "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(dom["gbps"] / HBM_PEAK_GBS, 4),
                "avg_launch_us": dom["avg_us"], "alg_bytes_per_launch": dom["alg_bytes_per_launch"],
                "traffic": traffic_from_profile(dom["kernel"]),
                "op_frac": op_frac, "target_frac": TARGET_FRAC,
                "target_met": bool(conv_frac >= TARGET_FRAC and spmv_frac >= TARGET_FRAC),
                "note": "frac = the dominant kernel's own bytes per launch / its duration; op_frac = compulsory bytes of "
                        "a whole operation (input once + output once) / its time / 8 TB/s, the figure the 60 % target "
                        "is written on; traffic = HBM bytes per launch of that kernel from profiles/ (rocprofv3 --pmc)"}
    line = {
        "metric": "conversion Mnnz/s + SpMV GFLOP/s; achieved HBM GB/s as % of MI355X peak",
        "value": round(nnz / ms_step / 1e3, 1), "unit": "Mnnz/s",
        "n_gpus": 1, "steps": K, "warmup": Wm, "ms_per_step": round(ms_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "dtype_note": "values and products fp32 (fp32 accumulate), indices int32, sort keys 42-bit packed (row, col) in u64",
        "data": "synthetic",
        "config": {"workload": head["workload"] + f"; {nnz} entries, unsorted COO resident in HBM; "
                               "step = decompose + SpMM + SpMV + release"},
        "conversion_mnnz_s": head["convert"]["mnnz_s"],
        "spmm_gflop_s": head["spmm"]["gflop_s"],
        "spmv_gflop_s": head["spmv"]["gflop_s"],
        "roofline": roofline,
        "cpu_baseline": cpu,
        "headline": head,
    }
    line.update(out)
    print(json.dumps(line))


def other_workloads(B, W, torch, ctx, up, K, Wm, with_oracle, op_frac):
    """Configs 1-4 with the conversion / decomposition and the product each names, variants of configs 2-4, the
    label-propagation loop and the format-to-format conversions."""
    res = {}
    dev = torch.device("cuda:0")
    P, E = B.us_desc_preset, B.expr
    for index in (1, 2, 3, 4):
        w = Workload(B, W, torch, ctx, up, index)
        r = w.measure(K, Wm)
        if with_oracle:
            r["cpu_oracle"] = w.oracle_sample()
        key = {1: "config1_csr_spmv", 2: "config2_csr_spmv", 3: "config3_dia_csr_spmv", 4: "config4_bcsr_spmm64"}[index]
        res[key] = r
        op_frac[key + ":convert"] = r["convert"]["op_frac"]
        op_frac[key + ":product"] = (r.get("spmm") or r["spmv"])["op_frac"]
        m = w.m

        def variant(name, conv, prod, flops, finish=None):
            """another layout of the same matrix: conversion and product time, compulsory-byte fractions"""
            ctx.set_sort_lds_finish(finish)
            try:
                parts = conv()
                ms, sd = timed(torch, lambda: [p.free() for p in conv()], K, Wm)
            finally:
                ctx.set_sort_lds_finish(None)
            cb = w.conv_bytes(parts)
            v = {"nnz": m.nnz, "convert": {"ms": round(ms, 4), "ms_std": round(sd, 4), "mnnz_s": round(m.nnz / ms / 1e3, 1),
                                           "op_frac": frac(cb, ms)}}
            if prod is not None:
                msq = timed_stream(torch, lambda: prod(parts), 4 * K, Wm)
                v["product"] = {"ms": round(msq, 4), "gflop_s": round(flops / msq / 1e6, 1),
                                "op_frac": frac(w.spmv_bytes(parts), msq)}
            for p in parts:
                p.free()
            res[name] = v

        if index == 2:
            conv = lambda d: [B.us_convert(ctx, m.nrows, m.ncols, w.r, w.c, w.v, d)]
            variant("config2_dcsr_spmv", lambda: conv(P(B.US_F_DCSR)), w.spmv, 2.0 * m.nnz)
            # the scheduled layout of Section 7.2.4 (1024 partitions, its core count)
            variant("config2_cisr_plus_spmv", lambda: conv(P(B.US_F_CISR_PLUS, 1024)), w.spmv, 2.0 * m.nnz)
        if index == 3:
            # the same matrix through the program of Figure 3c: blocked DIA (block 4) + CSR, #sum over (d0/4, d1-d0) >= 4
            pb = B.make_predicate([E(B.US_E_DIV, 1, 0, 0, 4), E(B.US_E_AFFINE, -1, 1)], B.US_P_SUM_GE_ABS, abs_=4)
            variant("config3_bdia_csr_spmv",
                    lambda: list(B.us_decompose(ctx, m.nrows, m.ncols, w.r, w.c, w.v, P(B.US_F_BDIA, 4), P(B.US_F_CSR), pb)),
                    w.spmv, 2.0 * m.nnz)
            # SpMM over the DIA + CSR hybrid (the DIA SpMM of Table 6, N = 64 here): the banded part alone and both parts
            parts = w.convert()
            N3 = 64
            X3 = up(W.dense_operand(3, (m.ncols, N3))); Y3 = torch.empty(m.nrows, N3, device=dev)
            ms_dia = timed_stream(torch, lambda: B.us_spmm(ctx, parts[0], X3, Y3), 2 * K, Wm)
            ms_all = timed_stream(torch, lambda: (B.us_spmm(ctx, parts[0], X3, Y3),
                                                  B.us_spmm(ctx, parts[1], X3, Y3, accumulate=True)), 2 * K, Wm)
            xyb = 4.0 * N3 * (m.ncols + m.nrows)
            res["config3_dia_csr_spmm64"] = {
                "nnz": m.nnz, "N": N3,
                "dia_part": {"entries": int(parts[0].nnz), "ms": round(ms_dia, 4),
                             "gflop_s": round(2.0 * parts[0].nnz * N3 / ms_dia / 1e6, 1),
                             "op_frac": frac(w.stored_bytes(parts[:1]) + xyb, ms_dia)},
                "hybrid": {"ms": round(ms_all, 4), "gflop_s": round(2.0 * m.nnz * N3 / ms_all / 1e6, 1),
                           "op_frac": frac(w.stored_bytes(parts) + xyb, ms_all)}}
            for q in parts:
                q.free()
            del X3, Y3
        if index == 4:
            # whole-array digit passes only (blocked tuples finish inside LDS by default); COO -> ELL of Table 5 both ways
            variant("config4_bcsr_whole_array_passes_only",
                    lambda: [B.us_convert(ctx, m.nrows, m.ncols, w.r, w.c, w.v, P(B.US_F_BCSR, 4, 4))], None, 0, finish=False)
            # the same matrix as blocked ELL (4 x 4 blocks, 24 slots per block row): conversion and the MFMA product
            bell = [B.us_convert(ctx, m.nrows, m.ncols, w.r, w.c, w.v, P(B.US_F_BELL, 4, 4))]
            ms, sd = timed(torch, lambda: B.us_convert(ctx, m.nrows, m.ncols, w.r, w.c, w.v, P(B.US_F_BELL, 4, 4)).free(), K, Wm)
            msq = timed_stream(torch, lambda: w.spmm(bell), 2 * K, Wm)
            res["config4_bell_spmm64"] = {
                "nnz": m.nnz, "slots_per_block_row": int(bell[0].size(0)),
                "convert": {"ms": round(ms, 4), "ms_std": round(sd, 4), "mnnz_s": round(m.nnz / ms / 1e3, 1),
                            "op_frac": frac(w.conv_bytes(bell), ms)},
                "spmm": {"N": w.N, "ms": round(msq, 4), "gflop_s": round(2.0 * m.nnz * w.N / msq / 1e6, 1),
                         "op_frac": frac(w.spmm_bytes(bell), msq)}}
            bell[0].free()
            variant("config4_coo_to_ell", lambda: [B.us_convert(ctx, m.nrows, m.ncols, w.r, w.c, w.v, P(B.US_F_ELL))], None, 0)
            variant("config4_coo_to_ell_lds_finish",
                    lambda: [B.us_convert(ctx, m.nrows, m.ncols, w.r, w.c, w.v, P(B.US_F_ELL))], None, 0, finish=True)
        w.release()
    # config 2 with half of its rows emptied, so that the doubly compressed layout has rows to drop
    m = W.cfg2_powerlaw(empty_frac=0.5)
    r, c, v = up(m.row), up(m.col), up(m.val)
    x = up(W.dense_operand(2, m.ncols)); y = torch.empty(m.nrows, device=dev)
    ms, sd = timed(torch, lambda: B.us_convert(ctx, m.nrows, m.ncols, r, c, v, P(B.US_F_DCSR)).free(), K, Wm)
    g = B.us_convert(ctx, m.nrows, m.ncols, r, c, v, P(B.US_F_DCSR))
    msq = timed_stream(torch, lambda: B.us_spmv(ctx, g, x, y), 4 * K, Wm)
    res["config2_half_empty_rows_dcsr_spmv"] = {
        "nnz": m.nnz, "stored_rows": int(g.idx(0).numel()),
        "convert": {"ms": round(ms, 4), "ms_std": round(sd, 4), "mnnz_s": round(m.nnz / ms / 1e3, 1)},
        "product": {"ms": round(msq, 4), "gflop_s": round(2.0 * m.nnz / msq / 1e6, 1)}}
    g.free()
    del r, c, v, x, y
    torch.cuda.empty_cache()
    res["label_propagation"] = label_propagation(B, W, torch, ctx, up)
    res["format_to_format"] = format_to_format(B, W, torch, ctx, up, K, Wm)
    return res


def format_to_format(B, W, torch, ctx, up, K, Wm):
    """The conversion cases of Table 5 through the COO hub on the benchmark matrices: CSR -> CSC (config 2),
    DCSC -> BCSR 4x4 (config 4), CSB -> DIA variant and COO -> DIA (config 3's diagonals)."""
    out = {}
    P = B.us_desc_preset

    def one(name, m, src_desc, dst_desc):
        r, c, v = up(m.row), up(m.col), up(m.val)
        if src_desc is None:
            ms, sd = timed(torch, lambda: B.us_convert(ctx, m.nrows, m.ncols, r, c, v, dst_desc).free(), K, Wm)
        else:
            src = B.us_convert(ctx, m.nrows, m.ncols, r, c, v, src_desc)
            ms, sd = timed(torch, lambda: B.us_convert_formatted(ctx, src, dst_desc).free(), K, Wm)
            src.free()
        out[name] = {"nnz": m.nnz, "convert_ms": round(ms, 4), "convert_ms_std": round(sd, 4),
                     "convert_mnnz_s": round(m.nnz / ms / 1e3, 1)}
        del r, c, v
        torch.cuda.empty_cache()

    one("config3_diagonals_coo_to_dia", W.cfg3_banded(extra_frac=0.0), None, P(B.US_F_DIA))
    one("config2_csr_to_csc", W.cfg2_powerlaw(), P(B.US_F_CSR), P(B.US_F_CSC))
    one("config4_dcsc_to_bcsr", W.cfg4_blockfem(), P(B.US_F_DCSC), P(B.US_F_BCSR, 4, 4))
    one("config3_diagonals_csb_to_dia_variant", W.cfg3_banded(extra_frac=0.0), P(B.US_F_CSB, 512, 512), P(B.US_F_DIA_VARIANT))
    return out


def label_propagation(B, W, torch, ctx, up, iters=20, N=1000):
    """The paper's label-propagation case study (Section 7.2.5): `iters` products Y <- A_hat Y with a
    row-normalised power-law graph and N = 1000 labels, over CSR and over the ELL+COO hybrid,
    with the conversion (pre-processing) time beside the kernel time."""
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

    # blocked ELL (4 x 4 blocks) + COO, the hybrid of the paper's case study: blocks holding at least 3 entries
    pb = B.make_predicate([B.expr(B.US_E_DIV, 1, 0, 0, 4), B.expr(B.US_E_DIV, 0, 1, 0, 4)], B.US_P_SUM_GE_ABS, abs_=3)
    BELL = B.us_desc_preset(B.US_F_BELL, 4, 4)
    out = {"nrows": m.nrows, "nnz": m.nnz, "N": N, "iterations": iters}
    for name, conv in (("csr", lambda: [B.us_convert(ctx, m.nrows, m.ncols, r, c, v, CSR)]),
                       ("ell_coo", lambda: list(B.us_decompose(ctx, m.nrows, m.ncols, r, c, v, ELL, COO, pr))),
                       ("bell_coo", lambda: list(B.us_decompose(ctx, m.nrows, m.ncols, r, c, v, BELL, COO, pb)))):
        ms_conv, _ = timed(torch, lambda: [p.free() for p in conv()], 5, 2)
        parts = conv()
        ms_loop = timed_stream(torch, lambda: loop(parts), 3, 1)
        out[name] = {"preprocess_ms": round(ms_conv, 3), "kernels_ms": round(ms_loop, 3),
                     "total_ms": round(ms_conv + ms_loop, 3),
                     "gflop_s": round(2.0 * m.nnz * N * iters / ms_loop / 1e6, 1),
                     "entries_per_part": [int(p.nnz) for p in parts]}
        if name == "bell_coo":
            out[name]["bell_slots_per_block_row"] = int(parts[0].size(0))
        for p in parts:
            p.free()
    return out


if __name__ == "__main__":
    main()
