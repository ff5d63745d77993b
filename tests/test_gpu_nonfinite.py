"""Non-finite inputs: an Inf or NaN in one row of a dense operand must reach exactly the outputs
that the definition makes depend on that row (paper Sec. "Sparse Matrix Computation": SpMM sums
over the stored entries of a row only, SDDMM takes one dot product per stored entry).  Every fp32
kernel family and the direct fp16 kernels are held to that; the fp16 matrix-core SpMM multiplies
the zeros of its expanded 32-row panels by whole rows of B, and the documented consequence (NaN in
that column of C for every row, no other column touched) is asserted instead."""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def g():
    import torch
    assert torch.cuda.is_available(), "the gpu tests need a GPU"
    from tests import gpu_util
    return gpu_util


@pytest.fixture
def force():
    import paper_2006_10901_amd as spdl
    yield spdl.spdl_force_variant
    spdl.spdl_force_variant(0, -1)
    spdl.spdl_force_variant(1, -1)


def variants(op):
    import paper_2006_10901_amd as spdl
    out, v = [], 0
    while spdl.spdl_variant_name(op, v) is not None:
        out.append((v, spdl.spdl_variant_name(op, v)))
        v += 1
    return out


def place_column(A, col, rows_with):
    """A with column `col` stored in exactly the rows of rows_with (ascending rows kept ascending)."""
    rows = []
    for i in range(A.m):
        c = A.column_indices[A.row_offsets[i]:A.row_offsets[i + 1]]
        c = c[c != col]
        rows.append(np.sort(np.append(c, col)) if i in rows_with else c)
    lens = np.array([len(r) for r in rows])
    ro = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    ci = np.concatenate(rows).astype(np.int32)
    vals = np.random.default_rng(7).standard_normal(len(ci)).astype(A.values.dtype)
    vals[vals == 0] = 1
    return wl.Csr(A.m, A.k, ro, ci, vals)


def same_where_finite(gpu, ref, S, tol, atol, what):
    """Element by element: where the oracle is finite the tolerance rule holds, where it is an
    infinity the GPU has the same infinity, where it is NaN the GPU has NaN."""
    gpu = gpu.astype(np.float64)
    fin = np.isfinite(ref)
    assert np.array_equal(np.isnan(gpu), np.isnan(ref)), f"{what}: NaN pattern differs"
    assert np.array_equal(np.isinf(gpu), np.isinf(ref)), f"{what}: Inf pattern differs"
    assert np.array_equal(np.sign(gpu[np.isinf(ref)]), np.sign(ref[np.isinf(ref)])), f"{what}: sign of Inf"
    Sf = np.where(np.isfinite(S), S, 0.0)
    assert np.all(np.abs(gpu[fin] - ref[fin]) <= tol * Sf[fin] + atol), f"{what}: finite part outside tolerance"


def spmm_inputs(dtype, m=512, k=320, n=64, density=0.06):
    A = wl.uniform_mask_csr(m, k, density, 4100)
    A.values = A.values.astype(dtype)
    k0 = 137
    A = place_column(A, k0, set(range(40, 60, 3)) | {200, 202})               # 32-row panels 1 and 6 of 16
    assert (A.column_indices == k0).sum() == 9
    B = wl.dense(k, n, 4101, dtype)
    B[k0, 0] = np.inf
    B[k0, 1] = np.nan
    B[k0, 5] = -np.inf
    return A, B, k0


def test_spmm_fp32_every_family_contains_nonfinite_rows_of_B(g, oracle_lib, force):
    import paper_2006_10901_amd as spdl
    A, B, k0 = spmm_inputs(np.float32)
    n = B.shape[1]
    with np.errstate(invalid="ignore", over="ignore"):
        C, S = oracle_lib.spmm(A.m, A.k, n, A.row_offsets, A.column_indices, A.values, B)
    touched = np.array([k0 in A.column_indices[A.row_offsets[i]:A.row_offsets[i + 1]] for i in range(A.m)])
    assert np.all(np.isfinite(C[~touched])) and not np.any(np.isfinite(C[touched][:, [0, 1, 5]]))
    order = spdl.spdl_build_row_order(A.m, A.row_offsets)
    for v, name in variants(0):
        if name == "mfma":
            continue
        force(0, v)
        assert spdl.spdl_select_spmm(A.m, A.k, n, A.nnz, 4, 0, 0)["variant"] == v
        same_where_finite(g.gpu_spmm(A, B, n, order), C, S, g.TOL_F32, 0.0, f"spmm {name}")


def test_spmm_fp16_direct_kernel_contains_and_matrix_core_kernel_behaves_as_documented(g, oracle_lib, force):
    import paper_2006_10901_amd as spdl
    A, B, k0 = spmm_inputs(np.float16)
    n = B.shape[1]
    with np.errstate(invalid="ignore", over="ignore"):
        C, S = oracle_lib.spmm(A.m, A.k, n, A.row_offsets, A.column_indices, A.values, B)
    touched = np.array([k0 in A.column_indices[A.row_offsets[i]:A.row_offsets[i + 1]] for i in range(A.m)])
    by_name = dict((name, v) for v, name in variants(0))
    force(0, by_name["rowsplit"])
    same_where_finite(g.gpu_spmm(A, B, n, None), C, S, g.TOL_F16, g.ATOL_F16_STORE, "spmm f16 rowsplit")
    force(0, by_name["mfma"])
    assert spdl.spdl_variant_name(0, spdl.spdl_select_spmm(A.m, A.k, n, A.nnz, 2, 0, 0)["variant"]) == "mfma"
    got = g.gpu_spmm(A, B, n, None).astype(np.float64)
    bad_cols = [0, 1, 5]
    good_cols = [j for j in range(n) if j not in bad_cols]
    # the rows the definition affects are non-finite in the affected columns
    assert not np.any(np.isfinite(got[touched][:, bad_cols]))
    # every other column is right in every row
    same_where_finite(got[:, good_cols], C[:, good_cols], S[:, good_cols], g.TOL_F16, g.ATOL_F16_STORE, "mfma other columns")
    # the documented spill-over: every panel multiplies the zeros of its expanded block by row k0
    # of B, so the affected columns are NaN in every row of C
    assert np.all(np.isnan(got[~touched][:, bad_cols]))


def sddmm_inputs(dtype, m=512, k=320, n=128, density=0.06):
    A = wl.uniform_mask_csr(m, k, density, 4200)
    counts = np.bincount(A.column_indices, minlength=k)
    c0, c1 = [int(c) for c in np.argsort(-counts)[:2]]
    L, R = wl.dense(m, n, 4201, dtype), wl.dense(k, n, 4202, dtype)
    L[L == 0] = 1
    R[c0, 3] = np.inf
    R[c1, 70] = np.nan
    i0 = int(np.argmax(np.diff(A.row_offsets)))
    L[i0, 9] = -np.inf
    return A, L, R


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_sddmm_every_family_contains_nonfinite_rows_of_L_and_R(g, oracle_lib, force, dtype):
    import paper_2006_10901_amd as spdl
    A, L, R = sddmm_inputs(dtype)
    n = L.shape[1]
    with np.errstate(invalid="ignore", over="ignore"):
        out, S = oracle_lib.sddmm(A.m, A.k, n, A.row_offsets, A.column_indices, L, R)
    assert 0 < np.count_nonzero(~np.isfinite(out)) < A.nnz // 8
    tol, atol = (g.TOL_F32, 0.0) if dtype == np.float32 else (g.TOL_F16, g.ATOL_F16_STORE)
    for v, name in variants(1):
        if name == "mfma" and dtype == np.float32:
            continue
        if name in ("slab", "slabdma", "lane") and dtype == np.float16:
            continue                                    # fp32 only: a forced choice falls back
        force(1, v)
        same_where_finite(g.gpu_sddmm(A, L, R, n), out, S, tol, atol, f"sddmm {name} {dtype.__name__}")


def test_window_kernels_contain_nonfinite_rows_inside_and_outside_the_window(g, oracle_lib, force):
    """A banded mask, 64 columns: one non-finite row of the dense operand sits inside the band of the
    rows that reference it (it reaches them through the window in LDS), one far from the diagonal
    (gathered); rows that reference neither stay finite and right."""
    import paper_2006_10901_amd as spdl
    A = wl.banded_attention_csr(640, 128, 0.3, 4300)
    n = 64
    B, L = wl.dense(A.k, n, 4301), wl.dense(A.m, n, 4302)
    L[L == 0] = 1
    B[300, 0] = np.inf
    B[300, 7] = np.nan
    B[10, 63] = -np.inf
    touched = np.array([np.isin([300, 10], A.column_indices[A.row_offsets[i]:A.row_offsets[i + 1]]).any()
                        for i in range(A.m)])
    assert touched[300] and 100 < touched.sum() < A.m - 100
    with np.errstate(invalid="ignore", over="ignore"):
        C, S = oracle_lib.spmm(A.m, A.k, n, A.row_offsets, A.column_indices, A.values, B)
        out, So = oracle_lib.sddmm(A.m, A.k, n, A.row_offsets, A.column_indices, L, B)
    assert np.all(np.isfinite(C[~touched])) and not np.all(np.isfinite(C[touched]))
    by0, by1 = dict((nm, v) for v, nm in variants(0)), dict((nm, v) for v, nm in variants(1))
    force(0, by0["window"])
    assert spdl.spdl_select_spmm(A.m, A.k, n, A.nnz, 4, 0, 0)["variant"] == by0["window"]
    same_where_finite(g.gpu_spmm(A, B, n, None), C, S, g.TOL_F32, 0.0, "spmm window")
    force(1, by1["window"])
    assert spdl.spdl_select_sddmm(A.m, A.k, n, A.nnz, 4, 0, 0)["variant"] == by1["window"]
    same_where_finite(g.gpu_sddmm(A, L, B, n), out, So, g.TOL_F32, 0.0, "sddmm window")

