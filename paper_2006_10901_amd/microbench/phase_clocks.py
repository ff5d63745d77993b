"""Where a wave's time goes in the slab kernels on the LSTM problem (8192 x 10240, n = 128) and in the
window SpMM kernel on the attention head (4096 x 4096 banded mask, n = 64).

Loads the copy of the library that is built with clocks inside the kernels
(paper_2006_10901_amd.build.build_phase_clocks(), also built by __graft_entry__.build()), runs
the fp32 SpMM (slab kernel) and SDDMM (lane kernel) at three sparsities and prints, per kernel, the
share of a wave's resident time spent in each phase: set-up before the first slab, issuing the
slab copies, counting the look-ahead and fetching the next one, the multiply-add steps, the full
wait that ends a stage, the barrier, the rest (stores, loop overhead, the clocks themselves), and,
in the window kernel, the gathers of the entries outside the window with their multiply-adds.  The
last column is the slowest wave's total over the mean total.

Run from the repository root on the GPU:  python3 paper_2006_10901_amd/microbench/phase_clocks.py
"""
import ctypes
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2006_10901_amd import binding, build  # noqa: E402

PHASES = ("set-up", "copy issue", "count+fetch", "steps", "full wait", "barrier", "rest", "gathers")
STRIDE = 10


def main():
    if not os.path.exists(build.CLOCKS_LIB_PATH):
        build.build_phase_clocks()
    binding.LIB_PATH = build.CLOCKS_LIB_PATH           # before the first call: this process uses the diagnostic copy
    import torch
    import paper_2006_10901_amd as spdl
    import workloads as wl

    lib = binding.lib()
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    table = np.zeros(8192 * STRIDE, dtype=np.uint64)

    def report(name, info, waves_per_wg, launch):
        for _ in range(3):
            launch()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        launch()
        e1.record()
        torch.cuda.synchronize()
        rc = lib.spdl_debug_phase_clocks(table.ctypes.data_as(ctypes.c_void_p), ctypes.c_size_t(table.size))
        assert rc == 0, rc
        waves = min(8192, info["grid_x"] * max(1, info["grid_y"]) * waves_per_wg)
        t = table.reshape(8192, STRIDE)[:waves].astype(np.float64)
        t = t[t[:, 8] > 0]
        total = t[:, 8].mean()
        shares = " | ".join(f"{100 * t[:, i].mean() / total:5.1f}" for i in range(8))
        print(f"| {name} | {spdl.spdl_variant_name(0 if name.startswith('SpMM') else 1, info['variant'])} | "
              f"{e0.elapsed_time(e1) * 1e3:6.1f} | {total / 1e3:6.1f} | {shares} | {t[:, 8].max() / total:4.2f} |", flush=True)

    print("| operation | kernel | launch µs (with clocks) | thousand ticks per wave | " + " | ".join(PHASES) + " | slowest / mean |")
    print("|---|---|---|---|" + "---|" * (len(PHASES) + 1))
    for sparsity in (70, 90, 95):
        w = wl.lstm(sparsity)
        A, n = w["A"], w["n"]
        ro, ci, val = dev(A.row_offsets), dev(A.column_indices), dev(A.values)
        B, L, R = dev(w["B"]), dev(w["L"]), dev(w["R"])
        order = dev(spdl.spdl_build_row_order(A.m, A.row_offsets))
        C = torch.empty((A.m, n), device="cuda")
        out = torch.empty(A.nnz, device="cuda")
        report(f"SpMM {sparsity} %", spdl.spdl_select_spmm(A.m, A.k, n, A.nnz, 4, 0, 0), 16,
               lambda: spdl.spdl_spmm(A.m, A.k, n, A.nnz, ro, ci, val, order, B, C))
        report(f"SDDMM {sparsity} %", spdl.spdl_select_sddmm(A.m, A.k, n, A.nnz, 4, 0, 0), 16,
               lambda: spdl.spdl_sddmm(A.m, A.k, n, A.nnz, ro, ci, L, R, out))
    w = wl.attention()
    A, n = w["A"], w["n"]
    ro, ci, val = dev(A.row_offsets), dev(A.column_indices), dev(A.values)
    V = dev(w["V"])
    C = torch.empty((A.m, n), device="cuda")
    info = spdl.spdl_select_spmm(A.m, A.k, n, A.nnz, 4, 0, 0)
    report("SpMM attention head", info, info["block_threads"] // 64,
           lambda: spdl.spdl_spmm(A.m, A.k, n, A.nnz, ro, ci, val, None, V, C))


if __name__ == "__main__":
    main()
