"""Thin ctypes binding of libspdl's C ABI: argument marshalling only.

Every function has the name and argument order of its C entry point (include/spdl.h).  Device
arrays are torch tensors on the GPU (PyTorch supplies memory and streams, nothing else); host
arrays are numpy.  There is no fallback: if libspdl.so is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspdl.so")
_lib = None

EXPORTS = (
    "spdl_spmm", "spdl_sddmm", "spdl_spmm_f16", "spdl_sddmm_f16", "spdl_build_row_order",
    "spdl_validate_csr_host", "spdl_select_spmm", "spdl_select_sddmm", "spdl_force_variant",
    "spdl_variant_name", "spdl_status_string", "spdl_version",
    "spdl_spmm_bias_relu", "spdl_spmm_bias_relu_f16", "spdl_csr_softmax", "spdl_build_transpose_host",
    "spdl_permute_values", "spdl_sddmm_scaled", "spdl_sddmm_scaled_f16",
    "spdl_sddmm_nt", "spdl_sddmm_nt_f16", "spdl_spmm_f16_i16", "spdl_sddmm_ordered",
    "spdl_spmm_banded", "spdl_sddmm_banded", "spdl_spmm_skewed", "spdl_sddmm_skewed",
)


class SpdlError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


class LaunchInfo(ctypes.Structure):
    _fields_ = [(name, ctypes.c_int) for name in
                ("variant", "vec", "lanes_per_row", "rows_per_block", "block_threads", "grid_x", "grid_y")]

    def as_dict(self):
        return {name: getattr(self, name) for name, _ in self._fields_}


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2006_10901_amd.build` "
                "(there is no CPU fallback)")
        # PyTorch ships its own HIP runtime under the same soname as the system one.  Import
        # torch first so that libspdl binds to the runtime that owns torch's streams and
        # allocations; with the opposite order two runtimes would coexist and launches fail.
        import torch  # noqa: F401
        _lib = ctypes.CDLL(LIB_PATH)
        _lib.spdl_status_string.restype = ctypes.c_char_p
        _lib.spdl_variant_name.restype = ctypes.c_char_p
        for name in EXPORTS:
            getattr(_lib, name)            # raises AttributeError if a declared symbol is absent
    return _lib


def status_string(status: int) -> str:
    return lib().spdl_status_string(int(status)).decode()


def _check(status, where):
    if status != 0:
        raise SpdlError(status, where)


def _dev(t, dtype, name, allow_none=False):
    """Device pointer of a contiguous GPU tensor of the given torch dtype."""
    import torch
    if t is None:
        if allow_none:
            return ctypes.c_void_p(0)
        raise ValueError(f"{name} is required")
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise ValueError(f"{name} must be a GPU tensor")
    if t.dtype != dtype:
        raise ValueError(f"{name} must have dtype {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, torch.cuda.Stream):
        return ctypes.c_void_p(stream.cuda_stream)
    return ctypes.c_void_p(int(stream))


def spdl_spmm(m, k, n, nnz, row_offsets, column_indices, values, row_order, B, C, stream=None):
    import torch
    _check(lib().spdl_spmm(
        int(m), int(k), int(n), int(nnz), _dev(row_offsets, torch.int32, "row_offsets"),
        _dev(column_indices, torch.int32, "column_indices"), _dev(values, torch.float32, "values"),
        _dev(row_order, torch.int32, "row_order", allow_none=True), _dev(B, torch.float32, "B"),
        _dev(C, torch.float32, "C"), _stream(stream)), "spdl_spmm")
    return C


def spdl_sddmm(m, k, n, nnz, row_offsets, column_indices, L, R, out_values, stream=None):
    import torch
    _check(lib().spdl_sddmm(
        int(m), int(k), int(n), int(nnz), _dev(row_offsets, torch.int32, "row_offsets"),
        _dev(column_indices, torch.int32, "column_indices"), _dev(L, torch.float32, "L"),
        _dev(R, torch.float32, "R"), _dev(out_values, torch.float32, "out_values"), _stream(stream)),
        "spdl_sddmm")
    return out_values


def spdl_spmm_banded(m, k, n, nnz, row_offsets, column_indices, values, B, C, stream=None):
    import torch
    _check(lib().spdl_spmm_banded(
        int(m), int(k), int(n), int(nnz), _dev(row_offsets, torch.int32, "row_offsets"),
        _dev(column_indices, torch.int32, "column_indices"), _dev(values, torch.float32, "values"),
        _dev(B, torch.float32, "B"), _dev(C, torch.float32, "C"), _stream(stream)), "spdl_spmm_banded")
    return C


def spdl_sddmm_banded(m, k, n, nnz, row_offsets, column_indices, L, R, out_values, stream=None):
    import torch
    _check(lib().spdl_sddmm_banded(
        int(m), int(k), int(n), int(nnz), _dev(row_offsets, torch.int32, "row_offsets"),
        _dev(column_indices, torch.int32, "column_indices"), _dev(L, torch.float32, "L"),
        _dev(R, torch.float32, "R"), _dev(out_values, torch.float32, "out_values"), _stream(stream)),
        "spdl_sddmm_banded")
    return out_values


def spdl_spmm_skewed(m, k, n, nnz, row_offsets, column_indices, values, B, C, stream=None):
    import torch
    _check(lib().spdl_spmm_skewed(
        int(m), int(k), int(n), int(nnz), _dev(row_offsets, torch.int32, "row_offsets"),
        _dev(column_indices, torch.int32, "column_indices"), _dev(values, torch.float32, "values"),
        _dev(B, torch.float32, "B"), _dev(C, torch.float32, "C"), _stream(stream)), "spdl_spmm_skewed")
    return C


def spdl_sddmm_skewed(m, k, n, nnz, row_offsets, column_indices, L, R, out_values, stream=None):
    import torch
    _check(lib().spdl_sddmm_skewed(
        int(m), int(k), int(n), int(nnz), _dev(row_offsets, torch.int32, "row_offsets"),
        _dev(column_indices, torch.int32, "column_indices"), _dev(L, torch.float32, "L"),
        _dev(R, torch.float32, "R"), _dev(out_values, torch.float32, "out_values"), _stream(stream)),
        "spdl_sddmm_skewed")
    return out_values


def spdl_sddmm_ordered(m, k, n, nnz, row_offsets, column_indices, row_order, L, R, out_values, stream=None):
    import torch
    _check(lib().spdl_sddmm_ordered(
        int(m), int(k), int(n), int(nnz), _dev(row_offsets, torch.int32, "row_offsets"),
        _dev(column_indices, torch.int32, "column_indices"),
        _dev(row_order, torch.int32, "row_order", allow_none=True), _dev(L, torch.float32, "L"),
        _dev(R, torch.float32, "R"), _dev(out_values, torch.float32, "out_values"), _stream(stream)),
        "spdl_sddmm_ordered")
    return out_values


def spdl_sddmm_scaled(m, k, n, nnz, row_offsets, column_indices, values, L, R, out_values, stream=None):
    import torch
    _check(lib().spdl_sddmm_scaled(
        int(m), int(k), int(n), int(nnz), _dev(row_offsets, torch.int32, "row_offsets"),
        _dev(column_indices, torch.int32, "column_indices"), _dev(values, torch.float32, "values"),
        _dev(L, torch.float32, "L"), _dev(R, torch.float32, "R"),
        _dev(out_values, torch.float32, "out_values"), _stream(stream)), "spdl_sddmm_scaled")
    return out_values


def spdl_sddmm_scaled_f16(m, k, n, nnz, row_offsets, column_indices, values, L, R, out_values, stream=None):
    import torch
    _check(lib().spdl_sddmm_scaled_f16(
        int(m), int(k), int(n), int(nnz), _dev(row_offsets, torch.int32, "row_offsets"),
        _dev(column_indices, torch.int32, "column_indices"), _dev(values, torch.float16, "values"),
        _dev(L, torch.float16, "L"), _dev(R, torch.float16, "R"),
        _dev(out_values, torch.float16, "out_values"), _stream(stream)), "spdl_sddmm_scaled_f16")
    return out_values


def spdl_sddmm_nt(m, k, n, nnz, row_offsets, column_indices, values, L, Rn, out_values, stream=None):
    import torch
    _check(lib().spdl_sddmm_nt(
        int(m), int(k), int(n), int(nnz), _dev(row_offsets, torch.int32, "row_offsets"),
        _dev(column_indices, torch.int32, "column_indices"),
        _dev(values, torch.float32, "values", allow_none=True), _dev(L, torch.float32, "L"),
        _dev(Rn, torch.float32, "Rn"), _dev(out_values, torch.float32, "out_values"), _stream(stream)),
        "spdl_sddmm_nt")
    return out_values


def spdl_sddmm_nt_f16(m, k, n, nnz, row_offsets, column_indices, values, L, Rn, out_values, stream=None):
    import torch
    _check(lib().spdl_sddmm_nt_f16(
        int(m), int(k), int(n), int(nnz), _dev(row_offsets, torch.int32, "row_offsets"),
        _dev(column_indices, torch.int32, "column_indices"),
        _dev(values, torch.float16, "values", allow_none=True), _dev(L, torch.float16, "L"),
        _dev(Rn, torch.float16, "Rn"), _dev(out_values, torch.float16, "out_values"), _stream(stream)),
        "spdl_sddmm_nt_f16")
    return out_values


def spdl_spmm_f16_i16(m, k, n, nnz, row_offsets, column_indices, values, row_order, B, C, stream=None):
    import torch
    _check(lib().spdl_spmm_f16_i16(
        int(m), int(k), int(n), int(nnz), _dev(row_offsets, torch.int32, "row_offsets"),
        _dev(column_indices, torch.int16, "column_indices"), _dev(values, torch.float16, "values"),
        _dev(row_order, torch.int32, "row_order", allow_none=True), _dev(B, torch.float16, "B"),
        _dev(C, torch.float16, "C"), _stream(stream)), "spdl_spmm_f16_i16")
    return C


def spdl_spmm_f16(m, k, n, nnz, row_offsets, column_indices, values, row_order, B, C, stream=None):
    import torch
    _check(lib().spdl_spmm_f16(
        int(m), int(k), int(n), int(nnz), _dev(row_offsets, torch.int32, "row_offsets"),
        _dev(column_indices, torch.int32, "column_indices"), _dev(values, torch.float16, "values"),
        _dev(row_order, torch.int32, "row_order", allow_none=True), _dev(B, torch.float16, "B"),
        _dev(C, torch.float16, "C"), _stream(stream)), "spdl_spmm_f16")
    return C


def spdl_sddmm_f16(m, k, n, nnz, row_offsets, column_indices, L, R, out_values, stream=None):
    import torch
    _check(lib().spdl_sddmm_f16(
        int(m), int(k), int(n), int(nnz), _dev(row_offsets, torch.int32, "row_offsets"),
        _dev(column_indices, torch.int32, "column_indices"), _dev(L, torch.float16, "L"),
        _dev(R, torch.float16, "R"), _dev(out_values, torch.float16, "out_values"), _stream(stream)),
        "spdl_sddmm_f16")
    return out_values


def spdl_spmm_bias_relu(m, k, n, nnz, row_offsets, column_indices, values, row_order, B, bias, relu, C,
                        stream=None):
    import torch
    _check(lib().spdl_spmm_bias_relu(
        int(m), int(k), int(n), int(nnz), _dev(row_offsets, torch.int32, "row_offsets"),
        _dev(column_indices, torch.int32, "column_indices"), _dev(values, torch.float32, "values"),
        _dev(row_order, torch.int32, "row_order", allow_none=True), _dev(B, torch.float32, "B"),
        _dev(bias, torch.float32, "bias", allow_none=True), int(bool(relu)),
        _dev(C, torch.float32, "C"), _stream(stream)), "spdl_spmm_bias_relu")
    return C


def spdl_spmm_bias_relu_f16(m, k, n, nnz, row_offsets, column_indices, values, row_order, B, bias, relu, C,
                            stream=None):
    import torch
    _check(lib().spdl_spmm_bias_relu_f16(
        int(m), int(k), int(n), int(nnz), _dev(row_offsets, torch.int32, "row_offsets"),
        _dev(column_indices, torch.int32, "column_indices"), _dev(values, torch.float16, "values"),
        _dev(row_order, torch.int32, "row_order", allow_none=True), _dev(B, torch.float16, "B"),
        _dev(bias, torch.float16, "bias", allow_none=True), int(bool(relu)),
        _dev(C, torch.float16, "C"), _stream(stream)), "spdl_spmm_bias_relu_f16")
    return C


def spdl_csr_softmax(m, nnz, row_offsets, logits, scale, probabilities, stream=None):
    import torch
    _check(lib().spdl_csr_softmax(
        int(m), int(nnz), _dev(row_offsets, torch.int32, "row_offsets"),
        _dev(logits, torch.float32, "logits"), ctypes.c_float(float(scale)),
        _dev(probabilities, torch.float32, "probabilities"), _stream(stream)), "spdl_csr_softmax")
    return probabilities


def spdl_permute_values(nnz, elem_bytes, perm, values, out, stream=None):
    import torch
    dtype = {2: torch.float16, 4: torch.float32}.get(int(elem_bytes))
    if dtype is None:
        raise ValueError("elem_bytes must be 2 or 4")
    _check(lib().spdl_permute_values(
        int(nnz), int(elem_bytes), _dev(perm, torch.int32, "perm"), _dev(values, dtype, "values"),
        _dev(out, dtype, "out"), _stream(stream)), "spdl_permute_values")
    return out


def _host_i32(a, name):
    a = np.ascontiguousarray(a)
    if a.dtype != np.int32:
        raise ValueError(f"{name} must be int32")
    return a


def spdl_build_row_order(m, row_offsets_host):
    ro = _host_i32(row_offsets_host, "row_offsets_host")
    if ro.shape[0] != m + 1:
        raise ValueError("row_offsets_host must have m+1 entries")
    out = np.empty(m, dtype=np.int32)
    _check(lib().spdl_build_row_order(int(m), ro.ctypes.data_as(ctypes.c_void_p),
                                      out.ctypes.data_as(ctypes.c_void_p)), "spdl_build_row_order")
    return out


def spdl_validate_csr_host(m, k, nnz, row_offsets_host, column_indices_host):
    """Returns (status, rows_sorted)."""
    ro = _host_i32(row_offsets_host, "row_offsets_host")
    ci = _host_i32(column_indices_host, "column_indices_host")
    if ro.shape[0] != m + 1 or ci.shape[0] != nnz:
        raise ValueError("array lengths do not match m / nnz")
    flag = ctypes.c_int(0)
    st = lib().spdl_validate_csr_host(int(m), int(k), int(nnz), ro.ctypes.data_as(ctypes.c_void_p),
                                      ci.ctypes.data_as(ctypes.c_void_p), ctypes.byref(flag))
    return int(st), bool(flag.value)


def spdl_build_transpose_host(m, k, nnz, row_offsets_host, column_indices_host):
    """Returns (t_row_offsets, t_column_indices, perm) as numpy int32 arrays."""
    ro = _host_i32(row_offsets_host, "row_offsets_host")
    ci = _host_i32(column_indices_host, "column_indices_host")
    if ro.shape[0] != m + 1 or ci.shape[0] != nnz:
        raise ValueError("array lengths do not match m / nnz")
    t_ro = np.empty(k + 1, dtype=np.int32)
    t_ci = np.empty(nnz, dtype=np.int32)
    perm = np.empty(nnz, dtype=np.int32)
    _check(lib().spdl_build_transpose_host(
        int(m), int(k), int(nnz), ro.ctypes.data_as(ctypes.c_void_p), ci.ctypes.data_as(ctypes.c_void_p),
        t_ro.ctypes.data_as(ctypes.c_void_p), t_ci.ctypes.data_as(ctypes.c_void_p),
        perm.ctypes.data_as(ctypes.c_void_p)), "spdl_build_transpose_host")
    return t_ro, t_ci, perm


def _ptr_or_zero(t):
    return ctypes.c_void_p(0 if t is None else (t if isinstance(t, int) else t.data_ptr()))


def spdl_select_spmm(m, k, n, nnz, elem_bytes, B=None, C=None):
    info = LaunchInfo()
    _check(lib().spdl_select_spmm(int(m), int(k), int(n), int(nnz), int(elem_bytes),
                                  _ptr_or_zero(B), _ptr_or_zero(C), ctypes.byref(info)), "spdl_select_spmm")
    return info.as_dict()


def spdl_select_sddmm(m, k, n, nnz, elem_bytes, L=None, R=None):
    info = LaunchInfo()
    _check(lib().spdl_select_sddmm(int(m), int(k), int(n), int(nnz), int(elem_bytes),
                                   _ptr_or_zero(L), _ptr_or_zero(R), ctypes.byref(info)), "spdl_select_sddmm")
    return info.as_dict()


def spdl_force_variant(op, variant):
    _check(lib().spdl_force_variant(int(op), int(variant)), "spdl_force_variant")


def spdl_variant_name(op, variant):
    s = lib().spdl_variant_name(int(op), int(variant))
    return None if s is None else s.decode()


def spdl_status_string(status):
    return status_string(status)


def spdl_version():
    return int(lib().spdl_version())
