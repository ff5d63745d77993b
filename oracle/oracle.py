"""ctypes front end of the plain-C oracle, plus tiny pure-numpy forms of the same definitions.

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg; never by the GPU library or its binding.

spmm / sddmm return (result, scale) as float64 arrays: result is the double-precision sum of
the stored inputs' products and scale is the sum of their absolute values (the per-element
tolerance scale).  fp16 inputs are passed as numpy float16 arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "spdl_oracle.c")
_LIB = os.path.join(_HERE, "libspdl_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(t: int) -> None:
    _load().oracle_set_num_threads(ctypes.c_int(t))


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _csr_args(row_offsets, column_indices):
    ro = np.ascontiguousarray(row_offsets, dtype=np.int32)
    ci = np.ascontiguousarray(column_indices, dtype=np.int32)
    return ro, ci


def spmm(m, k, n, row_offsets, column_indices, values, B):
    """Paper Sec. 'Sparse Matrix--Matrix Multiplication Operation': C = A B."""
    lib = _load()
    ro, ci = _csr_args(row_offsets, column_indices)
    assert ro.shape == (m + 1,) and B.shape == (k, n) and values.shape == ci.shape
    C = np.empty((m, n), dtype=np.float64)
    S = np.empty((m, n), dtype=np.float64)
    if values.dtype == np.float16:
        assert B.dtype == np.float16
        v = np.ascontiguousarray(values).view(np.uint16)
        b = np.ascontiguousarray(B).view(np.uint16)
        lib.oracle_spmm_f16(m, k, n, _p(ro), _p(ci), _p(v), _p(b), _p(C), _p(S))
    else:
        v = np.ascontiguousarray(values, dtype=np.float32)
        b = np.ascontiguousarray(B, dtype=np.float32)
        lib.oracle_spmm_f32(m, k, n, _p(ro), _p(ci), _p(v), _p(b), _p(C), _p(S))
    return C, S


def sddmm(m, k, n, row_offsets, column_indices, L, R):
    """Paper Sec. 'Sampled Dense--Dense Matrix Multiplication Operation': (L R^T) at A's nonzeros."""
    lib = _load()
    ro, ci = _csr_args(row_offsets, column_indices)
    assert ro.shape == (m + 1,) and L.shape == (m, n) and R.shape == (k, n)
    nnz = ci.shape[0]
    out = np.empty(nnz, dtype=np.float64)
    S = np.empty(nnz, dtype=np.float64)
    if L.dtype == np.float16:
        assert R.dtype == np.float16
        l = np.ascontiguousarray(L).view(np.uint16)
        r = np.ascontiguousarray(R).view(np.uint16)
        lib.oracle_sddmm_f16(m, k, n, _p(ro), _p(ci), _p(l), _p(r), _p(out), _p(S))
    else:
        l = np.ascontiguousarray(L, dtype=np.float32)
        r = np.ascontiguousarray(R, dtype=np.float32)
        lib.oracle_sddmm_f32(m, k, n, _p(ro), _p(ci), _p(l), _p(r), _p(out), _p(S))
    return out, S


def sddmm_scaled(m, k, n, row_offsets, column_indices, values, L, R):
    """Paper Sec. 'Sampled Dense--Dense Matrix Multiplication Operation' (strict definition): the
    sampled products times the stored values of the sparse matrix.  fp32 inputs."""
    lib = _load()
    ro, ci = _csr_args(row_offsets, column_indices)
    nnz = ci.shape[0]
    v = np.ascontiguousarray(values, dtype=np.float32)
    l = np.ascontiguousarray(L, dtype=np.float32)
    r = np.ascontiguousarray(R, dtype=np.float32)
    assert v.shape == (nnz,) and l.shape == (m, n) and r.shape == (k, n)
    out = np.empty(nnz, dtype=np.float64)
    S = np.empty(nnz, dtype=np.float64)
    lib.oracle_sddmm_scaled_f32(m, k, n, _p(ro), _p(ci), _p(v), _p(l), _p(r), _p(out), _p(S))
    return out, S


def sddmm_nt(m, k, n, row_offsets, column_indices, L, Rn):
    """Same section, footnote: SDDMM with the right-hand operand not transposed (Rn is n x k)."""
    lib = _load()
    ro, ci = _csr_args(row_offsets, column_indices)
    nnz = ci.shape[0]
    l = np.ascontiguousarray(L, dtype=np.float32)
    r = np.ascontiguousarray(Rn, dtype=np.float32)
    assert l.shape == (m, n) and r.shape == (n, k)
    out = np.empty(nnz, dtype=np.float64)
    S = np.empty(nnz, dtype=np.float64)
    lib.oracle_sddmm_nt_f32(m, k, n, _p(ro), _p(ci), _p(l), _p(r), _p(out), _p(S))
    return out, S


def row_order(m, row_offsets):
    """Paper Sec. 'Row Binning & Row Bundling Heuristics': rows by decreasing length, stable."""
    lib = _load()
    ro = np.ascontiguousarray(row_offsets, dtype=np.int32)
    out = np.empty(m, dtype=np.int32)
    lib.oracle_row_order(m, _p(ro), _p(out))
    return out


def csr_softmax(m, row_offsets, x, scale=1.0):
    """Paper Sec. 'Application: Sparse Transformer': softmax over the stored entries of each row."""
    lib = _load()
    ro = np.ascontiguousarray(row_offsets, dtype=np.int32)
    xv = np.ascontiguousarray(x, dtype=np.float32)
    out = np.zeros(xv.shape[0], dtype=np.float64)
    lib.oracle_csr_softmax_f32(m, _p(ro), _p(xv), ctypes.c_double(scale), _p(out))
    return out


def spmm_bias_relu(m, k, n, row_offsets, column_indices, values, B, bias, relu=True):
    """Paper Sec. 'Application: Sparse MobileNetV1': C = relu(A B + bias[row]); bias None adds
    nothing, relu False leaves the sum as it is."""
    lib = _load()
    ro, ci = _csr_args(row_offsets, column_indices)
    v = np.ascontiguousarray(values, dtype=np.float32)
    b = np.ascontiguousarray(B, dtype=np.float32)
    bs = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    assert (bs is None or bs.shape == (m,)) and b.shape == (k, n)
    C = np.empty((m, n), dtype=np.float64)
    S = np.empty((m, n), dtype=np.float64)
    lib.oracle_spmm_bias_relu_f32(m, k, n, _p(ro), _p(ci), _p(v), _p(b), _p(bs) if bs is not None else None,
                                  int(bool(relu)), _p(C), _p(S))
    return C, S


def transpose_topology(m, k, row_offsets, column_indices):
    """Paper Sec. 'Discussion & Conclusion': topology of A^T and the permutation that moves the values."""
    lib = _load()
    ro, ci = _csr_args(row_offsets, column_indices)
    nnz = ci.shape[0]
    tro = np.empty(k + 1, dtype=np.int32)
    tci = np.empty(nnz, dtype=np.int32)
    perm = np.empty(nnz, dtype=np.int32)
    lib.oracle_transpose_topology(m, k, _p(ro), _p(ci), _p(tro), _p(tci), _p(perm))
    return tro, tci, perm
