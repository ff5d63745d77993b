"""CPU-side checks of libspdl: the library loads, exports every declared symbol, validates
arguments before touching the GPU, and its host routines agree with the oracle."""
import ctypes
import os
import re

import numpy as np
import pytest

import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def spdl():
    import paper_2006_10901_amd as s
    s.lib()
    return s


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "spdl.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(spdl_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(spdl):
    names = declared_symbols()
    assert "spdl_spmm" in names and "spdl_sddmm" in names and len(names) >= 10
    lib = ctypes.CDLL(spdl.LIB_PATH)
    for name in names:
        assert hasattr(lib, name), name
    assert set(names) == set(spdl.EXPORTS)


def test_binding_names_match_the_abi(spdl):
    for name in declared_symbols():
        assert callable(getattr(spdl, name)), name


def test_invalid_arguments_are_rejected_without_a_gpu(spdl):
    lib = spdl.lib()
    null = ctypes.c_void_p(0)
    one = ctypes.c_void_p(256)     # never dereferenced: the checks fail first
    assert lib.spdl_spmm(-1, 4, 4, 0, one, one, one, null, one, one, null) == -1
    assert lib.spdl_spmm(4, 4, 4, 3, null, one, one, null, one, one, null) == -1
    assert lib.spdl_spmm(4, 4, 4, 3, one, null, one, null, one, one, null) == -1
    assert lib.spdl_spmm(1 << 20, 4, 1 << 12, 3, one, one, one, null, one, one, null) == -1   # m*n overflow
    assert lib.spdl_sddmm(4, 4, 4, -3, one, one, one, one, one, null) == -1
    assert lib.spdl_sddmm(4, 4, 4, 3, one, one, null, one, one, null) == -1
    assert lib.spdl_spmm_f16(4, -4, 4, 3, one, one, one, null, one, one, null) == -1
    assert lib.spdl_sddmm_f16(4, 4, 4, 3, one, one, one, one, null, null) == -1
    assert lib.spdl_spmm_banded(4, 4, 4, 3, one, null, one, one, one, null) == -1
    assert lib.spdl_sddmm_banded(4, 4, -4, 3, one, one, one, one, one, null) == -1
    assert lib.spdl_spmm_banded(0, 4, 4, 0, null, null, null, null, null, null) == 0
    assert lib.spdl_sddmm_banded(4, 4, 4, 0, one, null, one, one, null, null) == 0
    # degenerate sizes succeed without launching anything
    assert lib.spdl_spmm(0, 4, 4, 0, null, null, null, null, null, null, null) == 0
    assert lib.spdl_spmm(4, 4, 0, 0, one, null, null, null, null, null, null) == 0
    assert lib.spdl_sddmm(4, 4, 4, 0, one, null, one, one, null, null) == 0
    assert spdl.spdl_status_string(-1) == "invalid argument"
    assert spdl.spdl_status_string(0) == "ok"
    assert spdl.spdl_version() >= 100


def test_row_order_matches_oracle(spdl, oracle_lib):
    for A in (wl.lognormal_rows_csr(500, 256, 0.1, 7), wl.adversarial_csr(77, 90, 8),
              wl.uniform_mask_csr(64, 64, 0.1, 9)):
        got = spdl.spdl_build_row_order(A.m, A.row_offsets)
        assert got.dtype == np.int32
        assert np.array_equal(got, oracle_lib.row_order(A.m, A.row_offsets))
    assert spdl.spdl_build_row_order(0, np.zeros(1, np.int32)).shape == (0,)


def test_transpose_topology_matches_oracle_and_rejects_bad_input(spdl, oracle_lib):
    for A in (wl.adversarial_csr(77, 90, 21), wl.adversarial_csr(60, 45, 22, sorted_cols=False),
              wl.uniform_mask_csr(64, 200, 0.1, 23)):
        got = spdl.spdl_build_transpose_host(A.m, A.k, A.nnz, A.row_offsets, A.column_indices)
        ref = oracle_lib.transpose_topology(A.m, A.k, A.row_offsets, A.column_indices)
        for a, b in zip(got, ref):
            assert a.dtype == np.int32 and np.array_equal(a, b)
    A = wl.adversarial_csr(40, 50, 24)
    bad = A.column_indices.copy()
    bad[3] = A.k
    with pytest.raises(spdl.SpdlError) as e:
        spdl.spdl_build_transpose_host(A.m, A.k, A.nnz, A.row_offsets, bad)
    assert e.value.status == -3
    lib = spdl.lib()
    null, one = ctypes.c_void_p(0), ctypes.c_void_p(256)
    assert lib.spdl_build_transpose_host(-1, 4, 0, one, one, one, one, one) == -1
    assert lib.spdl_permute_values(5, 3, one, one, one, null) == -1
    assert lib.spdl_permute_values(0, 4, null, null, null, null) == 0
    assert lib.spdl_csr_softmax(4, 0, one, null, ctypes.c_float(1.0), null, null) == 0
    assert lib.spdl_csr_softmax(4, 3, one, null, ctypes.c_float(1.0), one, null) == -1
    assert lib.spdl_sddmm_scaled(4, 4, 4, 3, one, one, null, one, one, one, null) == -1
    assert lib.spdl_sddmm_scaled(4, 4, 4, 3, one, one, one, one, one, one, null) == -1        # values is out
    assert lib.spdl_sddmm_scaled_f16(4, 4, 4, 0, one, null, null, one, one, null, null) == 0
    assert lib.spdl_sddmm_nt(4, 4, 4, 3, one, one, null, null, one, one, null) == -1
    assert lib.spdl_sddmm_nt(4, 4, 4, 3, one, one, one, one, one, one, null) == -1            # values is out
    assert lib.spdl_sddmm_nt_f16(4, 4, 4, 0, one, null, null, one, one, null, null) == 0
    assert lib.spdl_spmm_f16_i16(4, 32768, 4, 3, one, one, one, null, one, one, null) == -1
    assert lib.spdl_spmm_f16_i16(0, 4, 4, 0, null, null, null, null, null, null, null) == 0
    assert lib.spdl_spmm_bias_relu(4, 4, 4, 3, null, one, one, null, one, one, 1, one, null) == -1
    assert lib.spdl_spmm_bias_relu_f16(-4, 4, 4, 3, one, one, one, null, one, one, 1, one, null) == -1
    e0 = spdl.spdl_build_transpose_host(0, 3, 0, np.zeros(1, np.int32), np.zeros(0, np.int32))
    assert np.array_equal(e0[0], np.zeros(4, np.int32)) and e0[1].size == 0


def test_validate_csr_host(spdl):
    A = wl.adversarial_csr(40, 50, 12)
    assert spdl.spdl_validate_csr_host(A.m, A.k, A.nnz, A.row_offsets, A.column_indices) == (0, True)
    U = wl.adversarial_csr(40, 50, 12, sorted_cols=False)
    assert spdl.spdl_validate_csr_host(U.m, U.k, U.nnz, U.row_offsets, U.column_indices) == (0, False)
    bad = A.column_indices.copy()
    bad[3] = A.k
    assert spdl.spdl_validate_csr_host(A.m, A.k, A.nnz, A.row_offsets, bad)[0] == -3
    ro = A.row_offsets.copy()
    ro[5], ro[6] = ro[6] + 1, ro[5]
    assert spdl.spdl_validate_csr_host(A.m, A.k, A.nnz, ro, A.column_indices)[0] == -3
    ro = A.row_offsets.copy()
    ro[0] = 1
    assert spdl.spdl_validate_csr_host(A.m, A.k, A.nnz, ro, A.column_indices)[0] == -3


def test_selection_uses_widest_aligned_vector(spdl):
    s = spdl.spdl_select_spmm(8192, 10240, 128, 1 << 19, 4, 0, 0)          # 99.4 % sparse, rows of 64: row splitting
    assert spdl.spdl_variant_name(0, s["variant"]) == "rowsplit"
    assert s["vec"] == 4 and s["lanes_per_row"] * s["vec"] >= 128
    s = spdl.spdl_select_spmm(8192, 10240, 128, 1 << 20, 4, 0, 0)          # 98.75 % sparse, rows of 128: gathers, four groups per row
    assert spdl.spdl_variant_name(0, s["variant"]) == "window" and s["vec"] == 4 and s["grid_y"] == 2
    s = spdl.spdl_select_spmm(8192, 10240, 128, 8 << 20, 4, 0, 0)          # 90 % sparse: LDS slabs
    assert spdl.spdl_variant_name(0, s["variant"]) == "slabdma" and s["grid_x"] == 256
    assert spdl.spdl_select_spmm(64, 64, 130, 100, 4, 0, 0)["vec"] == 2
    assert spdl.spdl_select_spmm(64, 64, 63, 100, 4, 0, 0)["vec"] == 1
    assert spdl.spdl_select_spmm(64, 64, 128, 100, 4, 4, 0)["vec"] == 1      # misaligned base
    assert spdl.spdl_select_spmm(64, 64, 128, 100, 4, 8, 16)["vec"] == 2
    assert spdl.spdl_select_spmm(64, 64, 3136, 100, 2, 0, 0)["vec"] == 8
    d = spdl.spdl_select_sddmm(8192, 10240, 128, 8 << 20, 4, 0, 0)           # 90 % sparse: two rows per lane group
    assert spdl.spdl_variant_name(1, d["variant"]) == "lane" and d["grid_x"] >= 256 and d["grid_y"] == 4
    assert d["rows_per_block"] == 128
    d = spdl.spdl_select_sddmm(8192, 10240, 128, 24 << 20, 4, 0, 0)          # 71 % sparse: one row per lane group
    assert spdl.spdl_variant_name(1, d["variant"]) == "lane" and d["rows_per_block"] == 64 and d["grid_y"] == 2
    d = spdl.spdl_select_sddmm(4096, 1024, 4096, 419430, 4, 0, 0)            # wide dot products: slab kernel
    assert spdl.spdl_variant_name(1, d["variant"]) == "slabdma"
    d = spdl.spdl_select_sddmm(8192, 10240, 130, 8 << 20, 4, 0, 0)           # n % 4 != 0: general kernel
    assert spdl.spdl_variant_name(1, d["variant"]) == "rowstrip" and d["block_threads"] == 256
    d = spdl.spdl_select_sddmm(2048, 2048, 64, 20000, 2, 0, 0)               # sparse fp16, short dot products: strip kernel
    # split by nonzeros: waves of 64 entries each, 4 waves per block
    assert spdl.spdl_variant_name(1, d["variant"]) == "group" and d["rows_per_block"] == 64
    assert d["grid_x"] == (20000 + 255) // 256
    # (with long dot products the gather kernel's latency per strip makes the dense blocks cheaper even at 2 %)
    assert spdl.spdl_variant_name(1, spdl.spdl_select_sddmm(1024, 1024, 3136, 20000, 2, 0, 0)["variant"]) == "mfma"
    # the LSTM shape in fp16: 20480 blocks of 64 x 64 for 128 columns each cost more than gathering
    assert spdl.spdl_variant_name(1, spdl.spdl_select_sddmm(8192, 10240, 128, 8 << 20, 2, 0, 0)["variant"]) == "group"
    assert spdl.spdl_variant_name(0, spdl.spdl_select_spmm(8192, 10240, 128, 8 << 20, 2, 0, 0)["variant"]) == "rowsplit"
    d = spdl.spdl_select_sddmm(1024, 1024, 3136, 100000, 2, 0, 0)            # one position in ten: dense blocks
    assert spdl.spdl_variant_name(1, d["variant"]) == "mfma" and d["grid_x"] == 8 * 8 * 4
    s = spdl.spdl_select_spmm(1024, 1024, 3136, 100000, 2, 0, 0)
    assert spdl.spdl_variant_name(0, s["variant"]) == "mfma" and s["grid_x"] == 32 * 7 and s["rows_per_block"] == 32 and s["block_threads"] == 256
    assert spdl.spdl_variant_name(0, 0) is not None and spdl.spdl_variant_name(0, 99) is None


def test_sddmm_selection_for_long_dot_products(spdl):
    """n > 128: the estimate of run times picks lane passes where rows are dense or the passes few,
    the slab kernel where they are many and rows sparse enough, the gather kernel for very sparse A
    (paper Sec. "Experiments": kernel selection by heuristics from the shape)."""
    def chosen(m, k, n, density):
        d = spdl.spdl_select_sddmm(m, k, n, int(m * k * density), 4, 0, 0)
        return spdl.spdl_variant_name(1, d["variant"])
    assert chosen(8192, 10240, 256, 0.50) == "lane"
    assert chosen(8192, 10240, 512, 0.30) == "lane"
    assert chosen(4096, 1024, 4096, 0.10) == "slabdma"          # the Transformer FFN shape
    assert chosen(4096, 1024, 4096, 0.30) == "slabdma"          # 32 passes would cost more than the overflow
    assert chosen(1024, 1024, 3136, 0.10) == "slabdma"          # the fp32 conv shape
    assert chosen(1024, 1024, 1024, 0.03) == "slabdma"          # small: never 8 passes of fixed cost
    assert chosen(8192, 10240, 256, 0.005) == "group"
    assert chosen(300, 1024, 1024, 0.10) == "slabdma"           # few rows, long dot products: gathers pay 1.1 us per 64 columns
    assert chosen(760, 231, 2048, 0.43) == "group"              # 24 workgroups of slabs on 256 compute units


def test_spmm_selection_of_the_window_kernel(spdl):
    """One or two 64-column tiles, a few hundred entries per row or more, thousands of rows, and a
    shape the slab kernel does not take: the shape of an attention head (paper Sec. "Application:
    Sparse Transformer") goes to the window kernel; anything narrower, wider, with shorter or fewer
    rows, in half precision, or dense enough for the slab kernel does not."""
    def chosen(m, k, n, nnz, eb=4):
        return spdl.spdl_variant_name(0, spdl.spdl_select_spmm(m, k, n, nnz, eb, 0, 0)["variant"])
    assert chosen(4096, 4096, 64, 1678008) == "window"            # config 4
    assert chosen(12288, 12288, 64, 12288 * 800) == "window"      # the paper's own sequence length, 6.5 % dense
    # dense enough for slabs of 64 columns: the shape alone keeps them (spdl_spmm_banded is for the caller who knows)
    assert chosen(12288, 12288, 64, int(12288 * 12288 * 0.1)) == "slabdma"
    assert chosen(8192, 8192, 64, int(8192 * 8192 * 0.1)) == "slabdma"
    assert chosen(8192, 8192, 64, int(8192 * 8192 * 0.05)) == "window"        # too sparse for slabs of 64 columns
    assert chosen(8192, 8192, 32, int(8192 * 8192 * 0.05)) == "rowsplit"     # narrow output: gathers
    assert chosen(8192, 8192, 32, int(8192 * 8192 * 0.3)) == "slabdma"
    assert chosen(8192, 8192, 8, int(8192 * 8192 * 0.3)) == "rowsplit"       # an eighth of a tile's lanes
    assert chosen(4096, 4096, 32, 1678008) == "rowsplit"
    assert chosen(4096, 4096, 128, 1678008) == "slabdma"          # 10 % dense: slabs, in workgroups of 8 waves
    assert chosen(4096, 4096, 128, int(4096 * 4096 * 0.06)) == "window"     # ... too sparse for those
    assert chosen(8192, 4096, 128, int(8192 * 4096 * 0.06)) == "slabdma"    # full-size workgroups take it
    assert chosen(8192, 10240, 128, 1677910) == "window"          # the LSTM matrix at 98 % sparsity
    assert chosen(8192, 10240, 128, 4195643) == "slabdma"         # ... at 95 %
    assert chosen(2048, 4096, 128, 2048 * 400) == "window"
    assert chosen(1024, 4096, 128, 1024 * 400) == "rowsplit"      # too few rows
    assert chosen(4096, 4096, 256, 4096 * 246) == "slabdma"
    # wider than two tiles: the window kernel only where a tile's share of B (k x 256 bytes) is too large for L2
    assert chosen(4096, 65536, 256, 4096 * 246) == "window"
    assert chosen(16384, 6000, 256, 16384 * 100) == "rowsplit"
    assert chosen(16384, 12000, 256, 16384 * 100) == "rowsplit"   # rows too short
    assert chosen(16384, 12000, 256, 16384 * 130) == "window"
    assert chosen(16384, 12000, 1024, 16384 * 130) == "window"
    assert chosen(4096, 4096, 64, int(4096 * 4096 * 0.3)) == "window"       # denser, still no slab shape: gathers
    assert chosen(2048, 2048, 64, 2048 * 300) == "rowsplit"       # few rows and not long enough
    assert chosen(2048, 2048, 64, 2048 * 400) == "window"
    assert chosen(4096, 4096, 64, 4096 * 60) == "rowsplit"        # short rows
    assert chosen(8192, 8192, 64, int(8192 * 8192 * 0.3)) == "slabdma"
    # dense matrices take the slab kernel with fewer workgroups than half the compute units
    assert chosen(6144, 2048, 64, int(6144 * 2048 * 0.35)) == "slabdma"       # 96 workgroups
    assert chosen(6144, 2048, 64, int(6144 * 2048 * 0.2)) == "window"
    assert chosen(4096, 4096, 64, int(4096 * 4096 * 0.5)) == "slabdma"        # 64 workgroups
    assert chosen(3072, 3072, 128, int(3072 * 3072 * 0.35)) == "slabdma"
    assert chosen(2048, 4096, 64, int(2048 * 4096 * 0.5)) == "window"         # 32 workgroups: too few
    # one tile per panel: the slab kernel from lower densities where the panels fill whole rounds of the machine
    assert chosen(16384, 4096, 64, int(16384 * 4096 * 0.04)) == "slabdma"     # 256 panels
    assert chosen(12288, 4096, 64, int(12288 * 4096 * 0.04)) == "window"      # 192 panels
    assert chosen(24576, 4096, 64, int(24576 * 4096 * 0.04)) == "window"      # 384 panels: from 64 * density = 3 on
    assert chosen(24576, 4096, 64, int(24576 * 4096 * 0.05)) == "slabdma"
    assert chosen(16384, 16384, 64, int(16384 * 16384 * 0.04)) == "window"    # square: could be an attention mask
    assert chosen(4096, 4096, 64, 1678008, eb=2) != "window"
    try:
        spdl.spdl_force_variant(0, 4)
        assert chosen(4096, 4096, 64, 0) == "rowsplit"            # nothing to fetch from
        assert chosen(64, 64, 130, 100) == "rowsplit"             # n % 4 != 0
        assert chosen(203, 700, 1028, 3000) == "window"
        # 32-bit byte offsets into B: k * n * 4 < 2^31, else the general kernel
        assert chosen(4096, 1 << 20, 256, 1 << 20) == "window"
        assert chosen(4096, 1 << 20, 512, 1 << 20) == "rowsplit"
    finally:
        spdl.spdl_force_variant(0, -1)


def test_sddmm_selection_of_the_window_kernel(spdl):
    def chosen(m, k, n, nnz, eb=4):
        return spdl.spdl_variant_name(1, spdl.spdl_select_sddmm(m, k, n, nnz, eb, 0, 0)["variant"])
    assert chosen(4096, 4096, 64, 1678008) == "window"            # config 4
    assert chosen(4096, 4096, 32, 1678008) == "group"
    assert chosen(4096, 4096, 128, 1678008) == "lane"
    assert chosen(2048, 8192, 64, 2048 * 400) == "group"           # too few rows
    assert chosen(4096, 4096, 64, 4096 * 100) == "group"          # short rows
    assert chosen(4096, 4096, 64, 1678008, eb=2) != "window"
    # uniform masks of that density with enough rows for full slab panels: the slab kernel
    assert chosen(8192, 2048, 64, int(8192 * 2048 * 0.1)) == "slabdma"
    assert chosen(16384, 4096, 32, int(16384 * 4096 * 0.1)) == "slabdma"
    assert chosen(8192, 8192, 64, int(8192 * 8192 * 0.05)) == "window"
    # ... from lower densities where the panels fill whole rounds of the machine (not for square matrices)
    assert chosen(16384, 4096, 64, int(16384 * 4096 * 0.065)) == "slabdma"
    assert chosen(16384, 4096, 64, int(16384 * 4096 * 0.05)) != "slabdma"
    assert chosen(12288, 4096, 64, int(12288 * 4096 * 0.065)) != "slabdma"
    assert chosen(16384, 16384, 64, int(16384 * 16384 * 0.065)) != "slabdma"
    try:
        spdl.spdl_force_variant(1, 6)
        assert chosen(203, 700, 64, 3000) == "window"
        assert chosen(203, 700, 68, 3000) == "window"
        assert chosen(203, 700, 132, 3000) == "group"             # dot products of at most 128 columns
        assert chosen(4096, 1 << 21, 128, 1 << 20) == "window"
        assert chosen(4096, 1 << 22, 128, 1 << 20) == "group"     # k * n * 4 would reach 2^31
    finally:
        spdl.spdl_force_variant(1, -1)


def test_spmm_tile_inner_slab_kernel_shape(spdl):
    """Wide outputs with two rows per lane group walk at most four tiles per workgroup (their
    accumulators stay in registers while a slab is scanned once for all of them), unless a slab holds
    more of a row than the 48 pairs of look-ahead (mean + 3 sigma)."""
    s = spdl.spdl_select_spmm(4096, 1024, 4096, 420757, 4, 0, 0)            # Transformer W1, 10 % dense
    assert spdl.spdl_variant_name(0, s["variant"]) == "slabdma"
    assert (s["rows_per_block"], s["grid_y"], s["grid_x"]) == (128, 4, 512)
    s = spdl.spdl_select_spmm(1024, 4096, 4096, 420099, 4, 0, 0)            # W2: two tiles fill the machine
    assert (s["rows_per_block"], s["grid_y"]) == (128, 2)
    s = spdl.spdl_select_spmm(4096, 1024, 4096, int(4096 * 1024 * 0.3), 4, 0, 0)   # 77 pairs per slab: the other kernel
    assert (s["rows_per_block"], s["grid_y"]) == (128, 8)


def test_forced_slab_variants_never_run_an_empty_matrix(spdl):
    """With nnz == 0 the sparse arrays and B may be null; the kernels that fetch from them
    unconditionally must not be chosen, forced or not."""
    try:
        for forced in (1, 2, 3, 4):
            spdl.spdl_force_variant(0, forced)
            for eb in (4, 2):
                s = spdl.spdl_select_spmm(4096, 4096, 128, 0, eb, 0, 0)
                assert spdl.spdl_variant_name(0, s["variant"]) == "rowsplit", (forced, eb)
            s = spdl.spdl_select_spmm(4096, 4096, 128, 1 << 20, 4, 0, 0)
            if forced in (1, 2):
                assert s["variant"] == forced
    finally:
        spdl.spdl_force_variant(0, -1)


def test_status_strings(spdl):
    lib = ctypes.CDLL(spdl.LIB_PATH)
    lib.spdl_status_string.restype = ctypes.c_char_p
    seen = {lib.spdl_status_string(c).decode() for c in (0, -1, -2, -3, -4, -5)}
    assert len(seen) == 6 and "unknown status" not in seen
    assert lib.spdl_status_string(-99).decode() == "unknown status"
    assert lib.spdl_version() >= 120


def test_bench_reads_its_traffic_figures_from_the_profile_summary():
    """roofline.traffic is not a constant of bench.py: it is the read + written MB of the kernel's
    row in profiles/lstm_sweep_hbm_traffic.md."""
    import bench
    table = bench.measured_hbm_traffic()
    assert table, "no kernel rows parsed from the profile summary"
    text = open(os.path.join(ROOT, bench.TRAFFIC_PROFILE)).read()
    for name, nbytes in table.items():
        row = [l for l in text.splitlines() if l.startswith("| " + name + " ")]
        assert len(row) == 1
        cells = [c.strip() for c in row[0].strip("|").split("|")]
        assert abs(nbytes - (float(cells[4]) + float(cells[5])) * 1e6) < 1.0
        assert nbytes > 1e6


def test_workload_statistics():
    A = wl.tiny()["A"]
    assert A.m == 512 and abs(A.nnz / 512 / 512 - 0.10) < 0.01
    F = wl.transformer_ffn(1, with_dense=False)["A"]
    lens = F.row_lengths
    assert F.m == 4096 and F.k == 1024 and abs(lens.mean() - 102.4) < 2 and lens.std() / lens.mean() < 0.15
    S = wl.conv1x1(True, with_dense=False)["A"]
    ls = S.row_lengths
    assert abs(S.nnz - 104857.6) < 0.011 * 104857.6 and ls.std() / ls.mean() > 0.8
    for A_ in (A, F, S):
        for i in range(0, A_.m, 97):
            c = A_.column_indices[A_.row_offsets[i]:A_.row_offsets[i + 1]]
            assert np.all(np.diff(c) > 0) and (len(c) == 0 or (c[0] >= 0 and c[-1] < A_.k))


def test_work_split_per_panel_avoids_a_second_round_of_workgroups():
    """A slab kernel's workgroup fills a compute unit, so more than 256 workgroups run in rounds:
    the split of a panel's work (column ranges of A in SDDMM, tiles of C in SpMM) is the one with
    the shortest chain, not the one with the most workgroups."""
    import paper_2006_10901_amd as spdl
    names = {spdl.spdl_variant_name(1, v): v for v in range(16) if spdl.spdl_variant_name(1, v)}
    try:
        for variant in ("slabdma", "lane"):
            spdl.spdl_force_variant(1, names[variant])
            # 64 panels: four column ranges each, one workgroup per compute unit (the LSTM and FFN shapes)
            info = spdl.spdl_select_sddmm(4096, 4096, 256, 4096 * 400, 4, 0, 0)
            assert (info["grid_x"], info["grid_y"]) == (256, 4)
            # 48 panels: five ranges (240 workgroups), not six (288: a second round for 32 of them)
            info = spdl.spdl_select_sddmm(3072, 3072, 256, 3072 * 300, 4, 0, 0)
            assert (info["grid_x"], info["grid_y"]) == (240, 5)
            # 96 panels: two ranges, not three
            info = spdl.spdl_select_sddmm(6144, 2048, 256, 6144 * 200, 4, 0, 0)
            assert (info["grid_x"], info["grid_y"]) == (192, 2)
    finally:
        spdl.spdl_force_variant(1, -1)
    info = spdl.spdl_select_spmm(8192, 10240, 128, 8390433, 4, 0, 0)        # the LSTM problem: unchanged
    assert spdl.spdl_variant_name(0, info["variant"]) == "slabdma" and info["grid_x"] == 256
    info = spdl.spdl_select_spmm(3072, 3072, 1024, 3072 * 300, 4, 0, 0)     # 48 panels, 16 tiles: 4 x 4 tiles, not 6 x 3
    assert spdl.spdl_variant_name(0, info["variant"]) == "slabdma" and info["grid_x"] == 192
