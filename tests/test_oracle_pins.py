"""Pins for the CPU oracle: every check compares it with something that is not the oracle
(a library GEMM on the densified matrix, closed forms, exact special cases, a hand-worked
fixture), chosen so that a dropped term, a wrong index, a swapped operand or a transposed
read in the oracle fails at least one of them."""
import os

import numpy as np
import pytest

import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def densify(A, dtype=np.float64):
    D = np.zeros((A.m, A.k), dtype=dtype)
    for i in range(A.m):
        s, e = A.row_offsets[i], A.row_offsets[i + 1]
        np.add.at(D[i], A.column_indices[s:e], A.values[s:e].astype(dtype))
    return D


def read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, vals = line.split(":")
            out[key] = np.array([float(x) for x in vals.split()])
    return out


def test_hand_worked_example(oracle_lib):
    g = read_golden("hand_worked_3x3.txt")
    ro = g["row_offsets"].astype(np.int32)
    ci = g["column_indices"].astype(np.int32)
    C, S = oracle_lib.spmm(3, 3, 2, ro, ci, g["values"].astype(np.float32), g["B"].reshape(3, 2).astype(np.float32))
    assert np.array_equal(C.ravel(), g["C"]) and np.array_equal(S.ravel(), g["S"])
    out, oS = oracle_lib.sddmm(3, 3, 2, ro, ci, g["L"].reshape(3, 2).astype(np.float32),
                               g["R"].reshape(3, 2).astype(np.float32))
    assert np.array_equal(out, g["out"]) and np.array_equal(oS, g["outS"])


@pytest.mark.parametrize("m,k,n,density,seed", [(17, 23, 9, 0.3, 1), (64, 40, 33, 0.5, 2), (5, 7, 1, 0.9, 3)])
def test_spmm_equals_dense_gemm_small(oracle_lib, m, k, n, density, seed):
    A = wl.uniform_mask_csr(m, k, density, seed)
    B = wl.dense(k, n, seed + 100)
    C, S = oracle_lib.spmm(m, k, n, A.row_offsets, A.column_indices, A.values, B)
    D = densify(A)
    ref = D @ B.astype(np.float64)                      # library GEMM, non-square, non-symmetric
    assert np.allclose(C, ref, rtol=1e-12, atol=1e-12)
    refS = np.abs(D) @ np.abs(B.astype(np.float64))
    assert np.allclose(S, refS, rtol=1e-12, atol=1e-12)


def test_spmm_equals_dense_gemm_config1(oracle_lib):
    w = wl.tiny()
    A = w["A"]
    C, S = oracle_lib.spmm(A.m, A.k, w["n"], A.row_offsets, A.column_indices, A.values, w["B"])
    ref = densify(A) @ w["B"].astype(np.float64)
    assert np.allclose(C, ref, rtol=1e-11, atol=1e-11)
    assert np.all(S >= np.abs(C) - 1e-9)


def test_spmm_identity_and_permutation_are_exact(oracle_lib):
    m = 37
    rng = np.random.default_rng(5)
    B = wl.dense(m, 19, 6)
    ro = np.arange(m + 1, dtype=np.int32)
    ones = np.ones(m, dtype=np.float32)
    C, S = oracle_lib.spmm(m, m, 19, ro, np.arange(m, dtype=np.int32), ones, B)
    assert np.array_equal(C, B.astype(np.float64))
    perm = rng.permutation(m).astype(np.int32)
    C, _ = oracle_lib.spmm(m, m, 19, ro, perm, ones, B)
    assert np.array_equal(C, B[perm].astype(np.float64))          # row i of C is row perm[i] of B
    scale = rng.standard_normal(m).astype(np.float32)
    C, S = oracle_lib.spmm(m, m, 19, ro, perm, scale, B)
    assert np.array_equal(C, scale.astype(np.float64)[:, None] * B[perm].astype(np.float64))
    assert np.array_equal(S, np.abs(C))


def test_spmm_all_ones_closed_form_and_empty_rows(oracle_lib):
    A = wl.adversarial_csr(60, 80, 11)
    A.values[:] = 1.0
    B = np.ones((80, 7), dtype=np.float32)
    C, S = oracle_lib.spmm(A.m, A.k, 7, A.row_offsets, A.column_indices, A.values, B)
    lens = A.row_lengths.astype(np.float64)
    assert np.array_equal(C, np.repeat(lens[:, None], 7, axis=1))
    assert np.array_equal(S, C)
    assert (lens == 0).sum() >= 3 and np.all(C[lens == 0] == 0.0)


def test_spmm_linearity_and_column_independence(oracle_lib):
    A = wl.uniform_mask_csr(40, 50, 0.3, 21)
    B = wl.dense(50, 12, 22)
    C, _ = oracle_lib.spmm(40, 50, 12, A.row_offsets, A.column_indices, A.values, B)
    C2, _ = oracle_lib.spmm(40, 50, 12, A.row_offsets, A.column_indices, A.values * np.float32(2), B)
    assert np.array_equal(C2, 2.0 * C)
    B3 = B.copy()
    B3[:, 5] = 0.0
    C3, _ = oracle_lib.spmm(40, 50, 12, A.row_offsets, A.column_indices, A.values, B3)
    keep = [j for j in range(12) if j != 5]
    assert np.array_equal(C3[:, keep], C[:, keep]) and np.all(C3[:, 5] == 0.0)


def test_spmm_unsorted_and_duplicate_columns(oracle_lib):
    # duplicates are summed, order inside a row does not matter (up to rounding in double)
    ro = np.array([0, 4, 4, 6], dtype=np.int32)
    ci = np.array([3, 0, 3, 1, 2, 2], dtype=np.int32)
    va = np.array([1, 2, 4, 8, 16, 32], dtype=np.float32)
    B = wl.dense(4, 5, 31)
    C, _ = oracle_lib.spmm(3, 4, 5, ro, ci, va, B)
    D = np.zeros((3, 4))
    D[0, 3] = 5; D[0, 0] = 2; D[0, 1] = 8; D[2, 2] = 48
    assert np.allclose(C, D @ B.astype(np.float64), rtol=1e-13, atol=1e-13)


def test_sddmm_full_mask_equals_dense_product(oracle_lib):
    m, k, n = 13, 21, 10
    L = wl.dense(m, n, 41)
    R = wl.dense(k, n, 42)
    ro = (np.arange(m + 1) * k).astype(np.int32)
    ci = np.tile(np.arange(k, dtype=np.int32), m)
    out, S = oracle_lib.sddmm(m, k, n, ro, ci, L, R)
    ref = L.astype(np.float64) @ R.astype(np.float64).T            # library GEMM with transposed RHS
    assert np.allclose(out.reshape(m, k), ref, rtol=1e-12, atol=1e-12)
    refS = np.abs(L.astype(np.float64)) @ np.abs(R.astype(np.float64)).T
    assert np.allclose(S.reshape(m, k), refS, rtol=1e-12, atol=1e-12)


def test_sddmm_sampled_positions_and_closed_forms(oracle_lib):
    A = wl.adversarial_csr(50, 64, 51)
    n = 24
    L = wl.dense(50, n, 52)
    R = wl.dense(64, n, 53)
    out, S = oracle_lib.sddmm(50, 64, n, A.row_offsets, A.column_indices, L, R)
    full = L.astype(np.float64) @ R.astype(np.float64).T
    rows = np.repeat(np.arange(50), A.row_lengths)
    assert np.allclose(out, full[rows, A.column_indices], rtol=1e-12, atol=1e-12)
    ones_out, ones_S = oracle_lib.sddmm(50, 64, n, A.row_offsets, A.column_indices,
                                        np.ones((50, n), np.float32), np.ones((64, n), np.float32))
    assert np.all(ones_out == n) and np.all(ones_S == n)


def test_sddmm_spmm_adjoint_identity(oracle_lib):
    # <SDDMM(L,R), v> == <L, SpMM(A_v, R)> for any values v on the topology
    A = wl.uniform_mask_csr(33, 45, 0.25, 61)
    n = 17
    L = wl.dense(33, n, 62)
    R = wl.dense(45, n, 63)
    out, _ = oracle_lib.sddmm(33, 45, n, A.row_offsets, A.column_indices, L, R)
    C, _ = oracle_lib.spmm(33, 45, n, A.row_offsets, A.column_indices, A.values, R)
    lhs = float(np.dot(out, A.values.astype(np.float64)))
    rhs = float(np.sum(L.astype(np.float64) * C))
    assert abs(lhs - rhs) <= 1e-10 * max(1.0, abs(lhs))


def test_fp16_decode_is_exact_for_every_finite_half(oracle_lib):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    halves = bits.view(np.float16)
    finite = np.isfinite(halves)
    vals = halves[finite]
    k = vals.shape[0]
    B = vals.reshape(k, 1)
    ro = np.arange(k + 1, dtype=np.int32)
    C, S = oracle_lib.spmm(k, k, 1, ro, np.arange(k, dtype=np.int32), np.ones(k, np.float16), B)
    assert np.array_equal(C.ravel(), vals.astype(np.float64))       # numpy's own half -> double
    assert np.array_equal(S.ravel(), np.abs(vals.astype(np.float64)))


def test_fp16_ops_match_dense_products(oracle_lib):
    A = wl.uniform_mask_csr(20, 30, 0.4, 71)
    A.values = A.values.astype(np.float16)
    B = wl.dense(30, 11, 72, np.float16)
    C, _ = oracle_lib.spmm(20, 30, 11, A.row_offsets, A.column_indices, A.values, B)
    assert np.allclose(C, densify(A) @ B.astype(np.float64), rtol=1e-12, atol=1e-12)
    L = wl.dense(20, 11, 73, np.float16)
    out, _ = oracle_lib.sddmm(20, 30, 11, A.row_offsets, A.column_indices, L, B)
    full = L.astype(np.float64) @ B.astype(np.float64).T
    rows = np.repeat(np.arange(20), A.row_lengths)
    assert np.allclose(out, full[rows, A.column_indices], rtol=1e-12, atol=1e-12)


def test_row_order_is_stable_descending_permutation(oracle_lib):
    A = wl.lognormal_rows_csr(300, 128, 0.2, 81)
    order = oracle_lib.row_order(A.m, A.row_offsets)
    lens = A.row_lengths
    assert sorted(order.tolist()) == list(range(A.m))
    assert np.all(np.diff(lens[order]) <= 0)
    same = np.diff(lens[order]) == 0
    assert np.all(np.diff(order)[same] > 0)                          # ties: ascending row index
    assert np.array_equal(order, np.argsort(-lens, kind="stable"))  # library stable sort


# ------------------------------------------------------------------ rows added after the hot path
def test_csr_softmax_against_library_and_closed_forms(oracle_lib):
    from scipy.special import softmax as lib_softmax
    A = wl.adversarial_csr(60, 90, 91)
    x = np.random.default_rng(92).standard_normal(A.nnz).astype(np.float32) * 3
    for scale in (1.0, 0.125):
        out = oracle_lib.csr_softmax(A.m, A.row_offsets, x, scale)
        for i in range(A.m):
            s, e = A.row_offsets[i], A.row_offsets[i + 1]
            if e > s:
                assert np.allclose(out[s:e], lib_softmax(scale * x[s:e].astype(np.float64)), rtol=1e-12, atol=0)
                assert abs(out[s:e].sum() - 1.0) < 1e-12
    # equal logits -> 1/len; two entries -> logistic closed form; shift invariance
    ro = np.array([0, 5, 7, 7, 8], dtype=np.int32)
    v = np.array([2, 2, 2, 2, 2, 1.5, -0.25, 9.0], dtype=np.float32)
    out = oracle_lib.csr_softmax(4, ro, v, 1.0)
    assert np.allclose(out[:5], 0.2, rtol=1e-15)
    assert np.isclose(out[5], 1.0 / (1.0 + np.exp(-0.25 - 1.5)), rtol=1e-14) and np.isclose(out[5] + out[6], 1.0)
    assert out[7] == 1.0
    shifted = oracle_lib.csr_softmax(4, ro, v + np.float32(4.0), 1.0)       # exact shift in fp32 here
    assert np.allclose(shifted, out, rtol=1e-13)
    big = oracle_lib.csr_softmax(1, np.array([0, 3], np.int32), np.array([1000, 999, -1000], np.float32), 1.0)
    assert np.all(np.isfinite(big)) and np.isclose(big[0], 1 / (1 + np.exp(-1.0)), rtol=1e-12) and big[2] == 0.0


def test_spmm_bias_relu_against_dense(oracle_lib):
    A = wl.uniform_mask_csr(30, 44, 0.3, 93)
    B = wl.dense(44, 13, 94)
    bias = np.random.default_rng(95).standard_normal(30).astype(np.float32)
    C, S = oracle_lib.spmm_bias_relu(30, 44, 13, A.row_offsets, A.column_indices, A.values, B, bias)
    ref = np.maximum(densify(A) @ B.astype(np.float64) + bias.astype(np.float64)[:, None], 0.0)
    assert np.allclose(C, ref, rtol=1e-12, atol=1e-12)
    assert (C == 0).any() and (C > 0).any()
    plain, S0 = oracle_lib.spmm(30, 44, 13, A.row_offsets, A.column_indices, A.values, B)
    assert np.allclose(S, S0 + np.abs(bias.astype(np.float64))[:, None], rtol=1e-13)
    zero_bias, _ = oracle_lib.spmm_bias_relu(30, 44, 13, A.row_offsets, A.column_indices, A.values, B, np.zeros(30, np.float32))
    assert np.array_equal(zero_bias, np.maximum(plain, 0.0))
    # the two switches: without a bias nothing is added, without the activation negatives stay
    none_relu, Sn = oracle_lib.spmm_bias_relu(30, 44, 13, A.row_offsets, A.column_indices, A.values, B, None)
    assert np.array_equal(none_relu, np.maximum(plain, 0.0)) and np.array_equal(Sn, S0)
    lin, _ = oracle_lib.spmm_bias_relu(30, 44, 13, A.row_offsets, A.column_indices, A.values, B, bias, relu=False)
    assert np.allclose(lin, densify(A) @ B.astype(np.float64) + bias.astype(np.float64)[:, None], rtol=1e-12, atol=1e-12)
    assert (lin < 0).any()


def test_transpose_topology_and_transposed_spmm(oracle_lib):
    A = wl.adversarial_csr(37, 53, 96)
    tro, tci, perm = oracle_lib.transpose_topology(A.m, A.k, A.row_offsets, A.column_indices)
    assert tro[0] == 0 and tro[-1] == A.nnz and sorted(perm.tolist()) == list(range(A.nnz))
    D = densify(A)
    T = wl.Csr(A.k, A.m, tro, tci, A.values[perm])
    assert np.array_equal(densify(T), D.T)                         # same matrix, transposed
    for c in range(A.k):
        assert np.all(np.diff(tci[tro[c]:tro[c + 1]]) > 0)         # ascending inside each row of A^T
    B = wl.dense(A.m, 9, 97)
    C, _ = oracle_lib.spmm(A.k, A.m, 9, tro, tci, T.values, B)
    assert np.allclose(C, D.T @ B.astype(np.float64), rtol=1e-12, atol=1e-12)


def test_sddmm_scaled_against_dense_hadamard(oracle_lib):
    A = wl.adversarial_csr(41, 57, 98, sorted_cols=False)
    L, R = wl.dense(41, 19, 99), wl.dense(57, 19, 100)
    out, S = oracle_lib.sddmm_scaled(A.m, A.k, 19, A.row_offsets, A.column_indices, A.values, L, R)
    P = L.astype(np.float64) @ R.astype(np.float64).T
    rows = np.repeat(np.arange(A.m), np.diff(A.row_offsets))
    ref = A.values.astype(np.float64) * P[rows, A.column_indices]          # A (Hadamard) L R^T, entry by entry
    assert np.allclose(out, ref, rtol=1e-12, atol=1e-12)
    plain, S0 = oracle_lib.sddmm(A.m, A.k, 19, A.row_offsets, A.column_indices, L, R)
    assert np.allclose(S, np.abs(A.values.astype(np.float64)) * S0, rtol=1e-13)
    ones = oracle_lib.sddmm_scaled(A.m, A.k, 19, A.row_offsets, A.column_indices, np.ones(A.nnz, np.float32), L, R)[0]
    assert np.array_equal(ones, plain)                                      # unit values: the unscaled operation
    # the scaled SDDMM summed over each row against all-ones R rows equals SpMM of A with ... a
    # rank-one check: L = u 1^T, R = w 1^T gives out[p] = a_p * n * u_i * w_c exactly representable here
    u = np.arange(1, A.m + 1, dtype=np.float32)[:, None] * np.ones((1, 4), np.float32)
    w = np.arange(1, A.k + 1, dtype=np.float32)[:, None] * np.ones((1, 4), np.float32)
    small = oracle_lib.sddmm_scaled(A.m, A.k, 4, A.row_offsets, A.column_indices, A.values, u, w)[0]
    assert np.allclose(small, A.values.astype(np.float64) * 4.0 * (rows + 1) * (A.column_indices + 1), rtol=1e-14)


def test_sddmm_nt_against_dense_product_and_transposed_form(oracle_lib):
    A = wl.adversarial_csr(33, 47, 101, sorted_cols=False)
    L, Rn = wl.dense(33, 21, 102), wl.dense(21, 47, 103)                   # Rn is n x k: not square with L
    out, S = oracle_lib.sddmm_nt(A.m, A.k, 21, A.row_offsets, A.column_indices, L, Rn)
    P = L.astype(np.float64) @ Rn.astype(np.float64)                        # plain dense product, no transpose
    rows = np.repeat(np.arange(A.m), np.diff(A.row_offsets))
    assert np.allclose(out, P[rows, A.column_indices], rtol=1e-12, atol=1e-12)
    assert np.allclose(S, (np.abs(L).astype(np.float64) @ np.abs(Rn).astype(np.float64))[rows, A.column_indices], rtol=1e-12)
    # the transposed form on the transposed operand is the same sum in the same order
    t_out, t_S = oracle_lib.sddmm(A.m, A.k, 21, A.row_offsets, A.column_indices, L, np.ascontiguousarray(Rn.T))
    assert np.array_equal(out, t_out) and np.array_equal(S, t_S)
