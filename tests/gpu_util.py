"""Helpers for the GPU parity tests: move seeded inputs to the GPU, call libspdl through its
binding (C ABI underneath), bring results back, and apply the per-element tolerance rule
|gpu - oracle| <= tol * S  (S = sum of |products|, from the oracle)."""
import numpy as np
import torch

import paper_2006_10901_amd as spdl

TOL_F32 = 1e-4
TOL_F16 = 2e-3
# Results of the fp16 entry points are stored as binary16, whose values below 2^-14 are spaced
# 2^-24 apart: one round-to-nearest of the fp32 accumulator can move a tiny result by 2^-25
# whatever its scale, so the fp16 comparisons allow that much on top of tol * S.
ATOL_F16_STORE = 2.0 ** -25


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


class DevCsr:
    def __init__(self, A):
        self.m, self.k, self.nnz = A.m, A.k, A.nnz
        self.ro = dev(A.row_offsets)
        self.ci = dev(A.column_indices)
        self.val = dev(A.values)


def gpu_spmm(A, B, n, order=None, dA=None, stream=None):
    dA = dA or DevCsr(A)
    f16 = A.values.dtype == np.float16
    dB = dev(B)
    C = torch.full((A.m, n), float("nan"), dtype=dB.dtype, device="cuda")   # must be fully overwritten
    dorder = dev(order.astype(np.int32)) if order is not None else None
    fn = spdl.spdl_spmm_f16 if f16 else spdl.spdl_spmm
    fn(A.m, A.k, n, A.nnz, dA.ro, dA.ci, dA.val, dorder, dB, C, stream)
    torch.cuda.synchronize()
    return C.cpu().numpy()


def gpu_sddmm(A, L, R, n, dA=None, stream=None):
    dA = dA or DevCsr(A)
    f16 = L.dtype == np.float16
    dL, dR = dev(L), dev(R)
    out = torch.full((A.nnz,), float("nan"), dtype=dL.dtype, device="cuda")
    fn = spdl.spdl_sddmm_f16 if f16 else spdl.spdl_sddmm
    fn(A.m, A.k, n, A.nnz, dA.ro, dA.ci, dL, dR, out, stream)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def assert_close(gpu, ref, scale, tol, what=""):
    atol = ATOL_F16_STORE if gpu.dtype == np.float16 else 0.0
    gpu = gpu.astype(np.float64)
    assert gpu.shape == ref.shape, (gpu.shape, ref.shape)
    assert np.all(np.isfinite(gpu)), f"{what}: non-finite output (unwritten element?)"
    err = np.abs(gpu - ref)
    bad = err > tol * scale + atol
    if bad.any():
        idx = np.unravel_index(np.argmax(err - tol * scale), err.shape)
        raise AssertionError(
            f"{what}: {bad.sum()} of {bad.size} elements outside {tol}*S; worst at {idx}: "
            f"gpu={gpu[idx]!r} oracle={ref[idx]!r} S={scale[idx]!r}")
    with np.errstate(divide="ignore", invalid="ignore"):
        ratio = np.where(scale > 0, np.maximum(err - atol, 0.0) / scale, 0.0)
    return float(ratio.max()) if ratio.size else 0.0
