#!/usr/bin/env python3
"""Benchmark of libspdl on one MI355X.

One step = one pass of the whole hot path over the weight-sparse LSTM workload: for each
sparsity in {70,80,90,95,98} % one SpMM (forward, A 8192x10240, B 10240x128) and one SDDMM
(weight gradient, L 8192x128, R 10240x128) on the same topology: ten kernel launches through
the C ABI, inputs resident in HBM, row orders built beforehand (a per-topology one-off).

Prints ONE JSON line.  value = useful GFLOP/s = sum(2*nnz*n) / time.  Extra fields give the
per-case times, the roofline of the dominant kernel (HIP events around every launch inside
the timed region) and the CPU oracle timed on this machine's host cores.
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

FP32_VECTOR_PEAK_TFLOPS = 157.3      # 256 CUs x 2.4 GHz x 256 flop/clk/CU (published)
MFMA_F16_PEAK_TFLOPS = 2500.0
HBM_PEAK_GBS = 8000.0


TRAFFIC_PROFILE = os.path.join("profiles", "lstm_sweep_hbm_traffic.md")


def measured_hbm_traffic():
    """HBM bytes per launch (read + written) of each kernel family on the LSTM sweep, from the two
    rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE) summarised in profiles/lstm_sweep_hbm_traffic.md
    (already scaled by the copy-kernel factors given there).  Hardware counters cannot be read
    from inside this process, so the figure reported as roofline.traffic is the one of that
    summary, refreshed whenever the kernels change; the JSON says where it comes from."""
    out = {}
    path = os.path.join(ROOT, TRAFFIC_PROFILE)
    if not os.path.exists(path):
        return out
    for line in open(path):
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) >= 7 and cells[0] and cells[0] != "kernel" and not set(cells[0]) <= set("-: "):
            try:
                out[cells[0]] = (float(cells[4]) + float(cells[5])) * 1e6
            except ValueError:
                pass
    return out


def spmm_bytes(m, k, n, nnz, eb=4):
    return nnz * (eb + 4) + (m + 1) * 4 + m * 4 + k * n * eb + m * n * eb


def sddmm_bytes(m, k, n, nnz, eb=4):
    return nnz * 4 + (m + 1) * 4 + m * n * eb + k * n * eb + nnz * eb


def log(msg):
    print(msg, file=sys.stderr, flush=True)


class Case:
    """One (operation, problem) pair with its device buffers and a launch closure."""

    def __init__(self, name, op, A, n, dense_ops, spdl, torch, f16=False):
        dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
        self.name, self.op, self.n = name, op, n
        self.m, self.k, self.nnz = A.m, A.k, A.nnz
        self.flops = 2.0 * A.nnz * n
        eb = 2 if f16 else 4
        self.bytes = (spmm_bytes if op == "spmm" else sddmm_bytes)(A.m, A.k, n, A.nnz, eb)
        ro, ci = dev(A.row_offsets), dev(A.column_indices)
        dt = torch.float16 if f16 else torch.float32
        if op == "spmm":
            val = dev(A.values)
            order = dev(spdl.spdl_build_row_order(A.m, A.row_offsets))
            B = dev(dense_ops[0])
            C = torch.empty((A.m, n), dtype=dt, device="cuda")
            fn = spdl.spdl_spmm_f16 if f16 else spdl.spdl_spmm
            self.launch = lambda: fn(A.m, A.k, n, A.nnz, ro, ci, val, order, B, C)
            self.info = spdl.spdl_select_spmm(A.m, A.k, n, A.nnz, eb, B, C)
        else:
            L, R = dev(dense_ops[0]), dev(dense_ops[1])
            out = torch.empty(A.nnz, dtype=dt, device="cuda")
            fn = spdl.spdl_sddmm_f16 if f16 else spdl.spdl_sddmm
            self.launch = lambda: fn(A.m, A.k, n, A.nnz, ro, ci, L, R, out)
            self.info = spdl.spdl_select_sddmm(A.m, A.k, n, A.nnz, eb, L, R)
        self.kernel = spdl.spdl_variant_name(0 if op == "spmm" else 1, self.info["variant"])
        self.ms = []

    def report(self):
        t = float(np.mean(self.ms)) * 1e-3
        extra = {}
        if self.kernel == "mfma":
            # the matrix-core kernels do the dense block products: report that rate as well
            dense = 2.0 * self.m * self.k * self.n
            extra = {"dense_equiv_tflops": round(dense / t / 1e12, 1),
                     "frac_mfma_f16_peak": round(dense / t / 1e12 / MFMA_F16_PEAK_TFLOPS, 4)}
        return {**extra, 
            "case": self.name, "op": self.op, "kernel": self.kernel, "nnz": self.nnz,
            "us": round(t * 1e6, 2), "us_median": round(float(np.median(self.ms)) * 1e3, 2),
            "us_min": round(float(np.min(self.ms)) * 1e3, 2),
            **({"us_warm": round(self.warm_us, 2)} if getattr(self, "warm_us", None) else {}),
            "gflops": round(self.flops / t / 1e9, 1), "eff_GBs": round(self.bytes / t / 1e9, 1),
            "frac_fp32_peak": round(self.flops / t / 1e12 / FP32_VECTOR_PEAK_TFLOPS, 4),
            "frac_hbm_peak": round(self.bytes / t / 1e9 / HBM_PEAK_GBS, 4),
        }


class WidenedCase:
    """An operation around the two kernels (softmax, fused epilogue, transposed SpMM): a launch
    closure with its algorithmic bytes and, where it multiplies, useful flops."""

    def __init__(self, name, op, kernel, nnz, launch, nbytes, flops=0.0, dims=(0, 0, 0)):
        self.name, self.op, self.kernel, self.nnz = name, op, kernel, nnz
        self.launch, self.bytes, self.flops, self.ms = launch, nbytes, flops, []
        self.m, self.k, self.n = dims

    report = Case.report


def widened_cases(wl, spdl, torch):
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    out = []
    # softmax of one attention head's scores (4096 x 4096 banded topology, 10 % dense)
    A = wl.attention(0)["A"]
    ro = dev(A.row_offsets)
    x = torch.randn(A.nnz, device="cuda")
    p = torch.empty_like(x)
    out.append(WidenedCase("attention_head", "csr_softmax", "wave_per_row", A.nnz,
                           lambda: spdl.spdl_csr_softmax(A.m, A.nnz, ro, x, 0.125, p),
                           8 * A.nnz + 4 * (A.m + 1)))
    # the same for the eight heads of a layer stacked into one CSR matrix (32768 rows)
    ro8 = np.concatenate([[0]] + [A.row_offsets[1:].astype(np.int64) + h * A.nnz for h in range(8)]).astype(np.int32)
    dro8 = dev(ro8)
    x8 = torch.randn(8 * A.nnz, device="cuda")
    p8 = torch.empty_like(x8)
    out.append(WidenedCase("attention_8_heads", "csr_softmax", "wave_per_row", 8 * A.nnz,
                           lambda: spdl.spdl_csr_softmax(8 * A.m, 8 * A.nnz, dro8, x8, 0.125, p8),
                           8 * 8 * A.nnz + 4 * (8 * A.m + 1)))
    # 1x1 convolution with bias and ReLU fused (fp16, 1024 x 1024 weights at 90 % sparsity, 56x56 pixels)
    w = wl.conv1x1(False)
    C1 = w["A"]
    cro, cci, cval = dev(C1.row_offsets), dev(C1.column_indices), dev(C1.values)
    corder = dev(spdl.spdl_build_row_order(C1.m, C1.row_offsets))
    cB = dev(w["B"])
    cbias = torch.randn(C1.m, device="cuda").half()
    cC = torch.empty((C1.m, 3136), dtype=torch.float16, device="cuda")
    info = spdl.spdl_select_spmm(C1.m, C1.k, 3136, C1.nnz, 2, cB, cC)
    out.append(WidenedCase("conv1x1_f16", "spmm_bias_relu", spdl.spdl_variant_name(0, info["variant"]), C1.nnz,
                           lambda: spdl.spdl_spmm_bias_relu_f16(C1.m, C1.k, 3136, C1.nnz, cro, cci, cval, corder, cB,
                                                                cbias, 1, cC),
                           spmm_bytes(C1.m, C1.k, 3136, C1.nnz, 2) + 2 * C1.m, 2.0 * C1.nnz * 3136,
                           dims=(C1.m, C1.k, 3136)))
    # A^T B for the first Transformer feed-forward weight (the data gradient of that layer):
    # cached transposed topology, values permuted on the device, then the ordinary SpMM
    w = wl.transformer_ffn(1, with_dense=False)
    F = w["A"]
    tro_h, tci_h, perm_h = spdl.spdl_build_transpose_host(F.m, F.k, F.nnz, F.row_offsets, F.column_indices)
    tro, tci, perm, fval = dev(tro_h), dev(tci_h), dev(perm_h), dev(F.values)
    tval = torch.empty_like(fval)
    torder = dev(spdl.spdl_build_row_order(F.k, tro_h))
    tB = torch.randn((F.m, 4096), device="cuda")
    tC = torch.empty((F.k, 4096), device="cuda")
    info = spdl.spdl_select_spmm(F.k, F.m, 4096, F.nnz, 4, tB, tC)

    def transposed():
        spdl.spdl_permute_values(F.nnz, 4, perm, fval, tval)
        spdl.spdl_spmm(F.k, F.m, 4096, F.nnz, tro, tci, tval, torder, tB, tC)
    out.append(WidenedCase("ffn_W1_transposed", "permute+spmm", spdl.spdl_variant_name(0, info["variant"]), F.nnz,
                           transposed, spmm_bytes(F.k, F.m, 4096, F.nnz) + 12 * F.nnz, 2.0 * F.nnz * 4096))
    # SDDMM with the right-hand operand not transposed (n x k), on the LSTM topology at 90 %
    w = wl.lstm(90, with_dense=False)
    N = w["A"]
    nro, nci = dev(N.row_offsets), dev(N.column_indices)
    nL = torch.randn((N.m, 128), device="cuda")
    nRn = torch.randn((128, N.k), device="cuda")
    nout = torch.empty(N.nnz, device="cuda")
    out.append(WidenedCase("lstm90_rhs_not_transposed", "sddmm_nt", "lane_nt", N.nnz,
                           lambda: spdl.spdl_sddmm_nt(N.m, N.k, 128, N.nnz, nro, nci, None, nL, nRn, nout),
                           sddmm_bytes(N.m, N.k, 128, N.nnz), 2.0 * N.nnz * 128, dims=(N.m, N.k, 128)))
    return out


EXTRA_GROUPS = ("ffn", "attention", "attention_n128", "conv_f16", "conv_f32", "imbalance", "widened")


def extra_cases(groups, wl, spdl, torch):
    """The configurations outside the timed step, by group name (also selectable with --only for
    profiling runs)."""
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    extra = []
    if "ffn" in groups:                     # Transformer feed-forward layer, 4096 tokens
        for which in (1, 2):
            w = wl.transformer_ffn(which)
            extra.append(Case(f"ffn_W{which}", "spmm", w["A"], 4096, (w["B"],), spdl, torch))
            extra.append(Case(f"ffn_W{which}", "sddmm", w["A"], 4096, (w["L"], w["R"]), spdl, torch))
            # the same SDDMM with the row order that SpMM uses (spdl_sddmm_ordered)
            A = w["A"]
            ro, ci = dev(A.row_offsets), dev(A.column_indices)
            order = dev(spdl.spdl_build_row_order(A.m, A.row_offsets))
            L, R, out = dev(w["L"]), dev(w["R"]), torch.empty(A.nnz, device="cuda")
            extra.append(WidenedCase(f"ffn_W{which}", "sddmm_ordered", extra[-1].kernel, A.nnz,
                                     lambda A=A, ro=ro, ci=ci, order=order, L=L, R=R, out=out:
                                     spdl.spdl_sddmm_ordered(A.m, A.k, 4096, A.nnz, ro, ci, order, L, R, out),
                                     sddmm_bytes(A.m, A.k, 4096, A.nnz), 2.0 * A.nnz * 4096, dims=(A.m, A.k, 4096)))
    if "attention" in groups:               # one head of the banded sparse attention
        w = wl.attention(0)
        extra.append(Case("attention_head", "sddmm", w["A"], 64, (w["Q"], w["K"]), spdl, torch))
        extra.append(Case("attention_head", "spmm", w["A"], 64, (w["V"],), spdl, torch))
    if "attention_n128" in groups:
        w = wl.attention(0)
        # The same mask with heads of 128 columns (hidden 1024 over 8 heads, paper Sec. "Application:
        # Sparse Transformer"): what spdl_spmm / spdl_sddmm choose from the shape alone, and the entry
        # points for banded masks, which the caller of an attention layer can name.
        A = w["A"]
        Q2, K2, V2 = wl.dense(A.m, 128, 611), wl.dense(A.k, 128, 612), wl.dense(A.k, 128, 613)
        extra.append(Case("attention_head_n128", "sddmm", A, 128, (Q2, K2), spdl, torch))
        extra.append(Case("attention_head_n128", "spmm", A, 128, (V2,), spdl, torch))
        ro, ci, val = dev(A.row_offsets), dev(A.column_indices), dev(A.values)
        dQ, dK, dV = dev(Q2), dev(K2), dev(V2)
        out2, C2 = torch.empty(A.nnz, device="cuda"), torch.empty((A.m, 128), device="cuda")
        extra.append(WidenedCase("attention_head_n128", "sddmm_banded", "window", A.nnz,
                                 lambda A=A, ro=ro, ci=ci, dQ=dQ, dK=dK, out2=out2:
                                 spdl.spdl_sddmm_banded(A.m, A.k, 128, A.nnz, ro, ci, dQ, dK, out2),
                                 sddmm_bytes(A.m, A.k, 128, A.nnz), 2.0 * A.nnz * 128, dims=(A.m, A.k, 128)))
        extra.append(WidenedCase("attention_head_n128", "spmm_banded", "window", A.nnz,
                                 lambda A=A, ro=ro, ci=ci, val=val, dV=dV, C2=C2:
                                 spdl.spdl_spmm_banded(A.m, A.k, 128, A.nnz, ro, ci, val, dV, C2),
                                 spmm_bytes(A.m, A.k, 128, A.nnz), 2.0 * A.nnz * 128, dims=(A.m, A.k, 128)))
    if "conv_f16" in groups:                # sparse 1x1 convolution, fp16 in / fp32 accumulate
        for skew in (False, True):
            w = wl.conv1x1(skew)
            nm = "conv1x1_f16_skewed" if skew else "conv1x1_f16"
            extra.append(Case(nm, "spmm", w["A"], 3136, (w["B"],), spdl, torch, f16=True))
            extra.append(Case(nm, "sddmm", w["A"], 3136, (w["L"], w["R"]), spdl, torch, f16=True))
    if "conv_f32" in groups:                # the same two topologies in fp32 (row-length skew without matrix cores)
        for skew in (False, True):
            w = wl.conv1x1(skew)
            A = w["A"]
            A32 = wl.Csr(A.m, A.k, A.row_offsets, A.column_indices, A.values.astype(np.float32))
            nm = "conv1x1_f32_skewed" if skew else "conv1x1_f32"
            f32 = lambda a: a.astype(np.float32)
            extra.append(Case(nm, "spmm", A32, 3136, (f32(w["B"]),), spdl, torch))
            extra.append(Case(nm, "sddmm", A32, 3136, (f32(w["L"]), f32(w["R"])), spdl, torch))
            if skew:
                # ... and through the entry points for rows of strongly unequal length
                ro, ci, val = dev(A32.row_offsets), dev(A32.column_indices), dev(A32.values)
                B, L, R = dev(f32(w["B"])), dev(f32(w["L"])), dev(f32(w["R"]))
                C = torch.empty((A32.m, 3136), device="cuda")
                out = torch.empty(A32.nnz, device="cuda")
                extra.append(WidenedCase(nm, "spmm_skewed", "by hint", A32.nnz,
                                         lambda A=A32, ro=ro, ci=ci, val=val, B=B, C=C:
                                         spdl.spdl_spmm_skewed(A.m, A.k, 3136, A.nnz, ro, ci, val, B, C),
                                         spmm_bytes(A32.m, A32.k, 3136, A32.nnz), 2.0 * A32.nnz * 3136,
                                         dims=(A32.m, A32.k, 3136)))
                extra.append(WidenedCase(nm, "sddmm_skewed", "by hint", A32.nnz,
                                         lambda A=A32, ro=ro, ci=ci, L=L, R=R, out=out:
                                         spdl.spdl_sddmm_skewed(A.m, A.k, 3136, A.nnz, ro, ci, L, R, out),
                                         sddmm_bytes(A32.m, A32.k, 3136, A32.nnz), 2.0 * A32.nnz * 3136,
                                         dims=(A32.m, A32.k, 3136)))
    if "imbalance" in groups:
        # Load imbalance (the paper's load-imbalance figure): 8192 x 2048 at 75 % sparsity, n = 128,
        # equal row lengths against gamma-distributed ones (coefficient of variation about 1),
        # each with the row order sorted by length and with no row order.
        for cov in (0.0, 1.0):
            w = wl.imbalance_sweep(cov)
            A = w["A"]
            lens = A.row_lengths
            tag = f"imbalance_cov{lens.std() / max(lens.mean(), 1e-9):.2f}"
            sorted_case = Case(tag + "_sorted_order", "spmm", A, 128, (w["B"],), spdl, torch)
            extra.append(sorted_case)
            ro, ci, val, B = dev(A.row_offsets), dev(A.column_indices), dev(A.values), dev(w["B"])
            C = torch.empty((A.m, 128), device="cuda")
            extra.append(WidenedCase(tag + "_natural_order", "spmm", sorted_case.kernel, A.nnz,
                                     lambda A=A, ro=ro, ci=ci, val=val, B=B, C=C:
                                     spdl.spdl_spmm(A.m, A.k, 128, A.nnz, ro, ci, val, None, B, C),
                                     spmm_bytes(A.m, A.k, 128, A.nnz), 2.0 * A.nnz * 128, dims=(A.m, A.k, 128)))
            # SDDMM on the same topology (its interface has no row order)
            sd = Case(tag + "_natural_order", "sddmm", A, 128, (wl.dense(A.m, 128, 515), wl.dense(A.k, 128, 516)), spdl, torch)
            extra.append(sd)
            # ... and with the sorted order handed to spdl_sddmm_ordered
            order = dev(spdl.spdl_build_row_order(A.m, A.row_offsets))
            L, R = dev(wl.dense(A.m, 128, 515)), dev(wl.dense(A.k, 128, 516))
            out = torch.empty(A.nnz, device="cuda")
            extra.append(WidenedCase(tag + "_sorted_order", "sddmm_ordered", sd.kernel, A.nnz,
                                     lambda A=A, ro=ro, ci=ci, order=order, L=L, R=R, out=out:
                                     spdl.spdl_sddmm_ordered(A.m, A.k, 128, A.nnz, ro, ci, order, L, R, out),
                                     sddmm_bytes(A.m, A.k, 128, A.nnz), 2.0 * A.nnz * 128, dims=(A.m, A.k, 128)))
    if "widened" in groups:
        extra += widened_cases(wl, spdl, torch)
    return extra


def time_cases(cases, steps, warmup, torch):
    """Warm up, then time `steps` passes over `cases`: wall clock around the whole region and a
    HIP event pair (on the launch stream) around every launch."""
    for _ in range(warmup):
        for c in cases:
            c.launch()
    torch.cuda.synchronize()
    events = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in cases] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(steps):
        for c, (e0, e1) in zip(cases, events[s]):
            e0.record()
            c.launch()
            e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    for c in cases:
        c.ms = []
    for s in range(steps):
        for c, (e0, e1) in zip(cases, events[s]):
            c.ms.append(e0.elapsed_time(e1))
    return wall


def time_warm(cases, torch, reps=20):
    """The same launch back to back on the same buffers (operands stay in the 256 MB Infinity
    Cache); the timed step above rotates through all cases and so runs every launch cold."""
    for c in cases:
        for _ in range(3):
            c.launch()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            c.launch()
        e1.record()
        torch.cuda.synchronize()
        c.warm_us = e0.elapsed_time(e1) / reps * 1e3


def one_off_host_costs(wl, spdl, lstm90):
    """Per-topology host work that is not part of a step (the paper amortises it the same way)."""
    out = {}
    A = lstm90["A"]
    t0 = time.perf_counter()
    spdl.spdl_build_row_order(A.m, A.row_offsets)
    out["row_order_build_lstm_ms"] = round((time.perf_counter() - t0) * 1e3, 3)
    F = wl.transformer_ffn(1, with_dense=False)["A"]
    t0 = time.perf_counter()
    spdl.spdl_build_transpose_host(F.m, F.k, F.nnz, F.row_offsets, F.column_indices)
    out["transpose_build_ffn_W1_ms"] = round((time.perf_counter() - t0) * 1e3, 3)
    return out


def cpu_baseline(lstm90, oracle, min_seconds=8.0):
    """The oracle as it stands, on this machine's host cores, on a bounded sample of the
    workload: SpMM + SDDMM of the 90 %-sparse LSTM problem (one of the step's five), repeated
    until about `min_seconds` of CPU work has been timed."""
    A, n = lstm90["A"], lstm90["n"]
    oracle.spmm(64, A.k, n, A.row_offsets[:65], A.column_indices, A.values, lstm90["B"])   # page in
    reps, dt = 0, 0.0
    t0 = time.perf_counter()
    while dt < min_seconds and reps < 200:
        oracle.spmm(A.m, A.k, n, A.row_offsets, A.column_indices, A.values, lstm90["B"])
        oracle.sddmm(A.m, A.k, n, A.row_offsets, A.column_indices, lstm90["L"], lstm90["R"])
        reps += 1
        dt = time.perf_counter() - t0
    threads = oracle.num_threads()
    # one thread, on a 512-row slice of the same SpMM (about a second)
    oracle.set_num_threads(1)
    rows = 512
    t1 = time.perf_counter()
    oracle.spmm(rows, A.k, n, A.row_offsets[:rows + 1], A.column_indices, A.values, lstm90["B"])
    single = 2.0 * int(A.row_offsets[rows]) * n / (time.perf_counter() - t1) / 1e9
    oracle.set_num_threads(threads)
    return {"value": round(reps * 2 * 2.0 * A.nnz * n / dt / 1e9, 2), "unit": "GFLOP/s",
            "cores": threads, "kind": "oracle", "single_thread_value": round(single, 2),
            "sample": f"SpMM + SDDMM of the LSTM problem at 90 % sparsity (nnz={A.nnz}, n=128), fp64 "
                      f"accumulation plus the |product| scale, {reps} repetitions in {dt:.2f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-extra", action="store_true", help="skip the Transformer/attention/conv report")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--only", default="",
                    help="profiling aid: comma list of LSTM sparsities and/or groups of the other configurations ("
                         + ", ".join(EXTRA_GROUPS) + ") to run in the timed loop instead of the full step")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run plain 256 MiB device copies (reference dispatches for rocprofv3 --pmc runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (--gpus 1); no multi-GPU path exists")

    import torch
    import paper_2006_10901_amd as spdl
    import workloads as wl
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    spdl.lib()

    tokens = [t for t in args.only.split(",") if t]
    only_groups = [t for t in tokens if t in EXTRA_GROUPS]
    bad = [t for t in tokens if t not in EXTRA_GROUPS and not t.isdigit()]
    if bad:
        sys.exit(f"bench.py: --only does not know {bad}")
    sparsities = [int(t) for t in tokens if t.isdigit()] if tokens else list(wl.LSTM_SPARSITIES)
    cases, lstm90 = [], None
    for sp in sparsities:
        t0 = time.time()
        w = wl.lstm(sp)
        if sp == 90:
            lstm90 = w
        cases.append(Case(f"lstm{sp}", "spmm", w["A"], 128, (w["B"],), spdl, torch))
        cases.append(Case(f"lstm{sp}", "sddmm", w["A"], 128, (w["L"], w["R"]), spdl, torch))
        log(f"[bench] lstm {sp}%: nnz={w['A'].nnz} generated+uploaded in {time.time() - t0:.1f}s")

    if only_groups:
        cases += extra_cases(only_groups, wl, spdl, torch)
        args.no_extra = True

    if args.copy_calibration:
        # a plain copy kernel of known size: 256 MiB read + 256 MiB written per dispatch
        src = torch.empty(64 << 20, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    wall = time_cases(cases, args.steps, args.warmup, torch)
    ms_per_step = wall / args.steps * 1e3
    step_flops = sum(c.flops for c in cases)
    value = step_flops / (wall / args.steps) / 1e9
    log(f"[bench] {args.steps} steps, {ms_per_step:.3f} ms/step, {value:.0f} GFLOP/s")

    # dominant kernel = the kernel family with the largest share of event time
    by_kernel = {}
    for c in cases:
        d = by_kernel.setdefault((c.op, c.kernel), {"ms": 0.0, "flops": 0.0, "bytes": 0.0, "launches": 0})
        d["ms"] += float(np.sum(c.ms)); d["flops"] += c.flops * len(c.ms)
        d["bytes"] += c.bytes * len(c.ms); d["launches"] += len(c.ms)
    (dom_op, dom_kernel), dom = max(by_kernel.items(), key=lambda kv: kv[1]["ms"])
    achieved = dom["flops"] / (dom["ms"] * 1e-3) / 1e12
    roofline = {
        "bound": "alu", "achieved": round(achieved, 3), "peak": FP32_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
        "frac": round(achieved / FP32_VECTOR_PEAK_TFLOPS, 4),
        "traffic": measured_hbm_traffic().get(f"{dom_op}_{dom_kernel}"),
        "traffic_source": TRAFFIC_PROFILE + " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, per dispatch)",
        "traffic_measured_in_run": False,
        "algorithmic_bytes_per_launch": dom["bytes"] / dom["launches"],
        "kernel": f"{dom_op}_{dom_kernel}", "avg_launch_us": round(dom["ms"] / dom["launches"] * 1e3, 2),
        "flops_per_launch": dom["flops"] / dom["launches"],
        "eff_GBs": round(dom["bytes"] / (dom["ms"] * 1e-3) / 1e9, 1),
        "frac_hbm_peak": round(dom["bytes"] / (dom["ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
    }

    result = {
        "metric": "SpMM & SDDMM useful GFLOP/s (2*nnz*n), 1 MI355X", "value": round(value, 1),
        "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "weight-sparse LSTM SpMM + SDDMM fp32, A 8192x10240, n=128, "
                               "sparsity sweep " + "/".join(str(s) for s in sparsities) + " %, uniform mask"},
        "roofline": roofline,
        "cases": [c.report() for c in cases],
    }

    time_warm(cases, torch)
    result["cases"] = [c.report() for c in cases]
    if lstm90 is not None:
        result["one_off_host_costs"] = one_off_host_costs(wl, spdl, lstm90)

    if not args.no_extra:
        extra = extra_cases(EXTRA_GROUPS, wl, spdl, torch)
        time_cases(extra, max(5, args.steps // 2), 2, torch)
        result["other_configs"] = [c.report() for c in extra]
        ffn = [c for c in extra if c.name.startswith("ffn_W") and c.op in ("spmm", "sddmm")]
        t = sum(float(np.mean(c.ms)) for c in ffn) * 1e-3
        result["transformer_ffn_gflops"] = round(sum(c.flops for c in ffn) / t / 1e9, 1)
        # the same four products with the SDDMMs given the row order too
        ffo = [c for c in extra if c.name.startswith("ffn_W") and c.op in ("spmm", "sddmm_ordered")]
        to = sum(float(np.mean(c.ms)) for c in ffo) * 1e-3
        result["transformer_ffn_gflops_sddmm_with_row_order"] = round(sum(c.flops for c in ffo) / to / 1e9, 1)

    if not args.no_cpu:
        import oracle
        if lstm90 is None:
            lstm90 = wl.lstm(90)
        result["cpu_baseline"] = cpu_baseline(lstm90, oracle)

    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
