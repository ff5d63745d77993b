"""GPU parity: libspdl (through its C ABI) against the CPU oracle, element by element, on the
same seeded inputs.  fp32: |gpu - oracle| <= 1e-4 * S; fp16 in / fp32 accumulate: 2e-3 * S."""
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


def spmm_case(g, oracle, A, B, n, tol, order="sorted", what=""):
    C, S = oracle.spmm(A.m, A.k, n, A.row_offsets, A.column_indices, A.values, B)
    ro = oracle.row_order(A.m, A.row_offsets) if isinstance(order, str) else order
    got = g.gpu_spmm(A, B, n, ro)
    return g.assert_close(got, C, S, tol, what), got


def sddmm_case(g, oracle, A, L, R, n, tol, what=""):
    out, S = oracle.sddmm(A.m, A.k, n, A.row_offsets, A.column_indices, L, R)
    got = g.gpu_sddmm(A, L, R, n)
    return g.assert_close(got, out, S, tol, what), got


# ------------------------------------------------------------------ config 1 and exact cases
def test_config1_tiny(g, oracle_lib):
    w = wl.tiny()
    A = w["A"]
    _, c_sorted = spmm_case(g, oracle_lib, A, w["B"], w["n"], g.TOL_F32, "sorted", "cfg1 spmm")
    _, c_ident = spmm_case(g, oracle_lib, A, w["B"], w["n"], g.TOL_F32, None, "cfg1 spmm no order")
    rnd = np.random.default_rng(1).permutation(A.m).astype(np.int32)
    _, c_rand = spmm_case(g, oracle_lib, A, w["B"], w["n"], g.TOL_F32, rnd, "cfg1 spmm random order")
    # the row swizzle is a pure reordering of work: identical bits whatever the order
    assert np.array_equal(c_sorted, c_ident) and np.array_equal(c_sorted, c_rand)
    sddmm_case(g, oracle_lib, A, w["L"], w["R"], w["n"], g.TOL_F32, "cfg1 sddmm")


def test_row_order_built_by_the_library_feeds_the_kernels(g, oracle_lib):
    """The host routine's own output (not the oracle's) as row_order, on skewed rows where the
    order matters for balance: same bits as with the identity order, and equal to the oracle's
    order array."""
    import paper_2006_10901_amd as spdl
    A = wl.lognormal_rows_csr(700, 900, 0.08, 77)
    B = wl.dense(A.k, 128, 78)
    mine = spdl.spdl_build_row_order(A.m, A.row_offsets)
    assert np.array_equal(mine, oracle_lib.row_order(A.m, A.row_offsets))
    _, c_mine = spmm_case(g, oracle_lib, A, B, 128, g.TOL_F32, mine, "spmm with the library's row order")
    _, c_ident = spmm_case(g, oracle_lib, A, B, 128, g.TOL_F32, None, "spmm identity order")
    assert np.array_equal(c_mine, c_ident)


def test_sddmm_with_a_row_order_gives_the_same_bits(g, oracle_lib):
    """spdl_sddmm_ordered: the row order only moves rows between workgroups.  Skewed rows on a shape
    that takes the lane kernel and one that takes the slab kernel for wide dot products (the two
    that use the order; m is not a multiple of the panel), the library's sorted order and a random
    permutation, against the oracle and bit for bit against spdl_sddmm; and a shape whose kernel
    ignores the order."""
    import torch
    import paper_2006_10901_amd as spdl
    for (m, k, n, dens, seed) in ((2100, 900, 128, 0.12, 81), (1100, 640, 260, 0.08, 83), (300, 200, 48, 0.1, 82)):
        A = wl.lognormal_rows_csr(m, k, dens, seed)
        L, R = wl.dense(m, n, seed + 100), wl.dense(k, n, seed + 200)
        ref, plain = sddmm_case(g, oracle_lib, A, L, R, n, g.TOL_F32, "sddmm without an order")
        d = g.DevCsr(A)
        dL, dR = g.dev(L), g.dev(R)
        orders = (spdl.spdl_build_row_order(A.m, A.row_offsets),
                  np.random.default_rng(seed).permutation(m).astype(np.int32), None)
        for order in orders:
            out = torch.full((A.nnz,), float("nan"), device="cuda")
            spdl.spdl_sddmm_ordered(m, k, n, A.nnz, d.ro, d.ci, None if order is None else g.dev(order), dL, dR, out)
            torch.cuda.synchronize()
            assert np.array_equal(out.cpu().numpy(), plain)
    # a single ragged panel (m < 64 rows per workgroup slot count), lane kernel forced
    A = wl.lognormal_rows_csr(70, 260, 0.2, 84)
    L, R = wl.dense(70, 128, 184), wl.dense(260, 128, 284)
    ref, S = oracle_lib.sddmm(A.m, A.k, 128, A.row_offsets, A.column_indices, L, R)
    d = g.DevCsr(A)
    spdl.spdl_force_variant(1, 5)
    try:
        assert spdl.spdl_variant_name(1, spdl.spdl_select_sddmm(70, 260, 128, A.nnz, 4, 0, 0)["variant"]) == "lane"
        for order in (spdl.spdl_build_row_order(A.m, A.row_offsets), None):
            out = torch.full((A.nnz,), float("nan"), device="cuda")
            spdl.spdl_sddmm_ordered(70, 260, 128, A.nnz, d.ro, d.ci, None if order is None else g.dev(order),
                                    g.dev(L), g.dev(R), out)
            torch.cuda.synchronize()
            g.assert_close(out.cpu().numpy(), ref, S, g.TOL_F32, "forced lane kernel, one ragged panel")
    finally:
        spdl.spdl_force_variant(1, -1)


def test_identity_and_permutation_return_rows_of_B_exactly(g, oracle_lib):
    m, n = 300, 128
    B = wl.dense(m, n, 3)
    perm = np.random.default_rng(4).permutation(m).astype(np.int32)
    A = wl.Csr(m, m, np.arange(m + 1, dtype=np.int32), perm, np.ones(m, np.float32))
    got = g.gpu_spmm(A, B, n, None)
    assert np.array_equal(got, B[perm])
    A.values = np.random.default_rng(5).standard_normal(m).astype(np.float32)
    got = g.gpu_spmm(A, B, n, oracle_lib.row_order(m, A.row_offsets))
    assert np.array_equal(got, A.values[:, None] * B[perm])       # one correctly rounded product


def test_sddmm_full_density_mask_equals_dense_product(g, oracle_lib):
    m, k, n = 70, 96, 128
    A = wl.Csr(m, k, (np.arange(m + 1) * k).astype(np.int32), np.tile(np.arange(k, dtype=np.int32), m),
               np.zeros(m * k, np.float32))
    sddmm_case(g, oracle_lib, A, wl.dense(m, n, 6), wl.dense(k, n, 7), n, g.TOL_F32, "full mask")


# ------------------------------------------------------------------ edge cases
@pytest.mark.parametrize("n", [1, 2, 3, 4, 8, 63, 64, 65, 130, 256, 260, 1028])
def test_ragged_rows_any_n(g, oracle_lib, n):
    # rows start at every residue modulo 8, lengths 0,1,2,3,5,...; empty first and last rows
    A = wl.adversarial_csr(203, 157, 100 + n)
    spmm_case(g, oracle_lib, A, wl.dense(A.k, n, 200 + n), n, g.TOL_F32, "sorted", f"spmm n={n}")
    sddmm_case(g, oracle_lib, A, wl.dense(A.m, n, 300 + n), wl.dense(A.k, n, 400 + n), n, g.TOL_F32, f"sddmm n={n}")


@pytest.mark.parametrize("n", [3, 8, 64, 136, 264])
def test_ragged_rows_fp16(g, oracle_lib, n):
    A = wl.adversarial_csr(150, 120, 500 + n)
    A.values = A.values.astype(np.float16)
    spmm_case(g, oracle_lib, A, wl.dense(A.k, n, 600 + n, np.float16), n, g.TOL_F16, "sorted", f"spmm f16 n={n}")
    sddmm_case(g, oracle_lib, A, wl.dense(A.m, n, 700 + n, np.float16), wl.dense(A.k, n, 800 + n, np.float16),
               n, g.TOL_F16, f"sddmm f16 n={n}")


def test_unsorted_and_duplicate_columns(g, oracle_lib):
    A = wl.adversarial_csr(120, 90, 31, sorted_cols=False)
    A.column_indices[5:9] = A.column_indices[5]                      # duplicates inside a row
    n = 128
    spmm_case(g, oracle_lib, A, wl.dense(A.k, n, 32), n, g.TOL_F32, "sorted", "unsorted spmm")
    sddmm_case(g, oracle_lib, A, wl.dense(A.m, n, 33), wl.dense(A.k, n, 34), n, g.TOL_F32, "unsorted sddmm")


def test_degenerate_sizes(g, oracle_lib):
    import torch
    import paper_2006_10901_amd as spdl
    # nnz == 0: SpMM still zero-fills C
    A = wl.Csr(9, 5, np.zeros(10, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32))
    got = g.gpu_spmm(A, wl.dense(5, 12, 1), 12, None)
    assert np.array_equal(got, np.zeros((9, 12), np.float32)) and not np.signbit(got).any()
    assert g.gpu_sddmm(A, wl.dense(9, 12, 2), wl.dense(5, 12, 3), 12).shape == (0,)
    # m == 0 and n == 0 return without touching anything
    z = torch.zeros(4, dtype=torch.int32, device="cuda")
    f = torch.zeros(4, dtype=torch.float32, device="cuda")
    spdl.spdl_spmm(0, 5, 12, 0, z, z, f, None, f, f)
    spdl.spdl_spmm(4, 5, 0, 0, z, z, f, None, f, f)
    # n == 0 SDDMM: every dot product is an empty sum
    A2 = wl.adversarial_csr(20, 16, 41)
    out = torch.full((A2.nnz,), 7.0, device="cuda")
    d = g.DevCsr(A2)
    spdl.spdl_sddmm(A2.m, A2.k, 0, A2.nnz, d.ro, d.ci, f, f, out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), np.zeros(A2.nnz, np.float32))


def test_offset_views_and_poisoned_neighbours(g, oracle_lib):
    """Arrays handed over as views at odd offsets inside larger buffers whose surroundings hold
    NaN / out-of-range indices: an over-read that is used, or a write outside C, shows up."""
    import torch
    import paper_2006_10901_amd as spdl
    A = wl.adversarial_csr(97, 80, 51)
    n = 20
    B = wl.dense(A.k, n, 52)
    C, S = oracle_lib.spmm(A.m, A.k, n, A.row_offsets, A.column_indices, A.values, B)
    out, oS = oracle_lib.sddmm(A.m, A.k, n, A.row_offsets, A.column_indices, wl.dense(A.m, n, 53), B)
    for pad in (1, 3, 5):
        def embed(a, poison, dtype):
            buf = torch.full((a.size + 2 * 64,), poison, dtype=dtype, device="cuda")
            view = buf[pad + 32: pad + 32 + a.size]
            view.copy_(torch.from_numpy(np.ascontiguousarray(a).ravel()))
            return buf, view
        _, ro = embed(A.row_offsets, 1 << 30, torch.int32)
        _, ci = embed(A.column_indices, 1 << 30, torch.int32)
        _, va = embed(A.values, float("nan"), torch.float32)
        _, dB = embed(B, float("nan"), torch.float32)
        _, dL = embed(wl.dense(A.m, n, 53), float("nan"), torch.float32)
        cbuf, dC = embed(np.zeros((A.m, n), np.float32), 123.0, torch.float32)
        obuf, dO = embed(np.zeros(A.nnz, np.float32), 123.0, torch.float32)
        spdl.spdl_spmm(A.m, A.k, n, A.nnz, ro, ci, va, None, dB, dC)
        spdl.spdl_sddmm(A.m, A.k, n, A.nnz, ro, ci, dL, dB, dO)
        torch.cuda.synchronize()
        g.assert_close(dC.cpu().numpy().reshape(A.m, n), C, S, g.TOL_F32, f"view pad={pad} spmm")
        g.assert_close(dO.cpu().numpy(), out, oS, g.TOL_F32, f"view pad={pad} sddmm")
        for buf, size in ((cbuf, A.m * n), (obuf, A.nnz)):
            host = buf.cpu().numpy()
            assert np.all(host[:pad + 32] == 123.0) and np.all(host[pad + 32 + size:] == 123.0)


def test_sddmm_may_overwrite_the_values_array_and_other_streams_work(g, oracle_lib):
    import torch
    import paper_2006_10901_amd as spdl
    A = wl.uniform_mask_csr(256, 300, 0.2, 61)
    n = 64
    L, R = wl.dense(A.m, n, 62), wl.dense(A.k, n, 63)
    out, S = oracle_lib.sddmm(A.m, A.k, n, A.row_offsets, A.column_indices, L, R)
    d = g.DevCsr(A)
    st = torch.cuda.Stream()
    dL, dR = g.dev(L), g.dev(R)
    torch.cuda.synchronize()
    with torch.cuda.stream(st):
        spdl.spdl_sddmm(A.m, A.k, n, A.nnz, d.ro, d.ci, dL, dR, d.val, st)
    st.synchronize()
    g.assert_close(d.val.cpu().numpy(), out, S, g.TOL_F32, "in-place sddmm on a side stream")


# ------------------------------------------------------------------ full-size configurations
@pytest.mark.parametrize("sparsity", wl.LSTM_SPARSITIES)
def test_config2_lstm(g, oracle_lib, sparsity):
    w = wl.lstm(sparsity)
    A = w["A"]
    assert A.m == 8192 and A.k == 10240
    r, _ = spmm_case(g, oracle_lib, A, w["B"], 128, g.TOL_F32, "sorted", f"lstm {sparsity}% spmm")
    r2, _ = sddmm_case(g, oracle_lib, A, w["L"], w["R"], 128, g.TOL_F32, f"lstm {sparsity}% sddmm")
    print(f"lstm {sparsity}%: nnz={A.nnz} max err/S spmm={r:.2e} sddmm={r2:.2e}")


@pytest.mark.parametrize("which", [1, 2])
def test_config3_transformer_ffn(g, oracle_lib, which):
    w = wl.transformer_ffn(which)
    A = w["A"]
    r, _ = spmm_case(g, oracle_lib, A, w["B"], 4096, g.TOL_F32, "sorted", f"ffn W{which} spmm")
    r2, _ = sddmm_case(g, oracle_lib, A, w["L"], w["R"], 4096, g.TOL_F32, f"ffn W{which} sddmm")
    print(f"ffn W{which}: nnz={A.nnz} max err/S spmm={r:.2e} sddmm={r2:.2e}")


def test_config4_sparse_attention(g, oracle_lib):
    import torch
    import paper_2006_10901_amd as spdl
    topo = wl.attention(0)["A"]
    lens = topo.row_lengths
    assert abs(topo.nnz / 4096 / 4096 - 0.10) < 0.003 and lens.max() / max(lens.min(), 1) < 4
    order = oracle_lib.row_order(topo.m, topo.row_offsets)
    d = g.DevCsr(topo)
    for head in range(8):
        w = wl.attention(head, topo)
        Q, K, V = w["Q"], w["K"], w["V"]
        out, S = oracle_lib.sddmm(4096, 4096, 64, topo.row_offsets, topo.column_indices, Q, K)
        got = g.gpu_sddmm(topo, Q, K, 64, dA=d)
        g.assert_close(got, out, S, g.TOL_F32, f"attention head {head} sddmm")
        # SpMM stage on the oracle's scores (rounded to fp32 once)
        scores = wl.Csr(4096, 4096, topo.row_offsets, topo.column_indices, out.astype(np.float32))
        C, CS = oracle_lib.spmm(4096, 4096, 64, topo.row_offsets, topo.column_indices, scores.values, V)
        gotC = g.gpu_spmm(scores, V, 64, order)
        g.assert_close(gotC, C, CS, g.TOL_F32, f"attention head {head} spmm")
        if head == 0:
            # the chained GPU pipeline (GPU scores feed the GPU SpMM): its input error adds
            # 1e-4 * S_sddmm[p] * |V| per term on top of the SpMM's own budget
            dv = g.dev(V)
            sc = torch.empty(topo.nnz, device="cuda")
            Cc = torch.empty((4096, 64), device="cuda")
            spdl.spdl_sddmm(4096, 4096, 64, topo.nnz, d.ro, d.ci, g.dev(Q), g.dev(K), sc)
            spdl.spdl_spmm(4096, 4096, 64, topo.nnz, d.ro, d.ci, sc, g.dev(order), dv, Cc)
            torch.cuda.synchronize()
            extra, _ = oracle_lib.spmm(4096, 4096, 64, topo.row_offsets, topo.column_indices,
                                       S.astype(np.float32), np.abs(V))
            g.assert_close(Cc.cpu().numpy(), C, (CS + extra) * 1.001, g.TOL_F32, "attention chained")


@pytest.mark.parametrize("skewed", [False, True])
def test_config5_conv1x1_fp16(g, oracle_lib, skewed):
    w = wl.conv1x1(skewed)
    A = w["A"]
    r, _ = spmm_case(g, oracle_lib, A, w["B"], 3136, g.TOL_F16, "sorted", f"conv skewed={skewed} spmm f16")
    r2, _ = sddmm_case(g, oracle_lib, A, w["L"], w["R"], 3136, g.TOL_F16, f"conv skewed={skewed} sddmm f16")
    print(f"conv skewed={skewed}: nnz={A.nnz} max err/S spmm={r:.2e} sddmm={r2:.2e}")


# ------------------------------------------------------------------ every kernel family, forced
@pytest.fixture
def force():
    import paper_2006_10901_amd as spdl
    yield spdl.spdl_force_variant
    spdl.spdl_force_variant(0, -1)
    spdl.spdl_force_variant(1, -1)


def spmm_variants():
    import paper_2006_10901_amd as spdl
    out, v = [], 0
    while spdl.spdl_variant_name(0, v) is not None:
        out.append(v)
        v += 1
    return out


@pytest.mark.parametrize("n", [4, 64, 68, 128, 200, 1028])
def test_forced_spmm_variants_ragged(g, oracle_lib, force, n):
    import paper_2006_10901_amd as spdl
    A = wl.adversarial_csr(203, 700, 900 + n)             # k spans several LDS slabs
    B = wl.dense(A.k, n, 901 + n)
    C, S = oracle_lib.spmm(A.m, A.k, n, A.row_offsets, A.column_indices, A.values, B)
    order = oracle_lib.row_order(A.m, A.row_offsets)
    results = []
    for v in spmm_variants():
        if spdl.spdl_variant_name(0, v) == "mfma":
            continue                                      # fp16 only, see the mixed-precision tests
        force(0, v)
        sel = spdl.spdl_select_spmm(A.m, A.k, n, A.nnz, 4, 0, 0)
        assert sel["variant"] == v
        got = g.gpu_spmm(A, B, n, order)
        g.assert_close(got, C, S, g.TOL_F32, f"variant {spdl.spdl_variant_name(0, v)} n={n}")
        # (when several lane groups share a row, the row-splitting kernel adds partial sums, and
        # the window kernel always does)
        if spdl.spdl_variant_name(0, v) != "window" and (
                sel["block_threads"] != 256 or sel["rows_per_block"] * sel["lanes_per_row"] == 256):
            results.append(got)
    # every family adds a row's products in stored order with fused multiply-adds: same bits
    assert len(results) >= 2
    for r in results[1:]:
        assert np.array_equal(r, results[0])


def test_forced_spmm_variants_unsorted_rows_and_uniform_mask(g, oracle_lib, force):
    import paper_2006_10901_amd as spdl
    U = wl.adversarial_csr(150, 600, 77, sorted_cols=False)
    U.column_indices[5:9] = U.column_indices[5]
    D = wl.uniform_mask_csr(333, 1000, 0.2, 78)
    for A in (U, D):
        n = 128
        B = wl.dense(A.k, n, 79)
        C, S = oracle_lib.spmm(A.m, A.k, n, A.row_offsets, A.column_indices, A.values, B)
        for v in spmm_variants():
            force(0, v)
            for order in (None, oracle_lib.row_order(A.m, A.row_offsets)):
                got = g.gpu_spmm(A, B, n, order)
                g.assert_close(got, C, S, g.TOL_F32, f"variant {spdl.spdl_variant_name(0, v)}")


def sddmm_variants():
    import paper_2006_10901_amd as spdl
    out, v = [], 0
    while spdl.spdl_variant_name(1, v) is not None:
        out.append(v)
        v += 1
    return out


@pytest.mark.parametrize("n", [4, 64, 68, 128, 200, 1028])
def test_forced_sddmm_variants_ragged(g, oracle_lib, force, n):
    import paper_2006_10901_amd as spdl
    for A in (wl.adversarial_csr(203, 700, 950 + n), wl.adversarial_csr(90, 300, 951 + n, sorted_cols=False)):
        L, R = wl.dense(A.m, n, 952 + n), wl.dense(A.k, n, 953 + n)
        out, S = oracle_lib.sddmm(A.m, A.k, n, A.row_offsets, A.column_indices, L, R)
        for v in sddmm_variants():
            if spdl.spdl_variant_name(1, v) == "mfma":
                continue                                  # fp16 only, see the mixed-precision tests
            force(1, v)
            chosen = spdl.spdl_variant_name(1, spdl.spdl_select_sddmm(A.m, A.k, n, A.nnz, 4, 0, 0)["variant"])
            # (the lane kernel takes dot products of more than 128 columns in passes of 128; the window
            # kernel is for dot products of at most 128 columns)
            name = spdl.spdl_variant_name(1, v)
            assert chosen == ("group" if name == "window" and n > 128 else name)
            got = g.gpu_sddmm(A, L, R, n)
            g.assert_close(got, out, S, g.TOL_F32, f"sddmm variant {spdl.spdl_variant_name(1, v)} n={n}")


@pytest.mark.parametrize("shape", [(700, 4100, 128), (333, 1500, 100), (200, 9000, 68), (130, 640, 264)])
def test_sddmm_column_parts_on_rows_with_clustered_columns(g, oracle_lib, force, shape):
    """The slab kernels split A's columns over workgroups and find where each part of a row starts by
    a search whose first probes are placed by interpolation, as if the row's columns were spread
    evenly.  Rows whose columns are clustered at one end, at both ends, around a random centre or
    run with gaps are where that guess is wrong by as much as it can be: every variant against the
    oracle."""
    import paper_2006_10901_amd as spdl
    m, k, n = shape
    A = wl.clustered_rows_csr(m, k, 7000 + m)
    L, R = wl.dense(m, n, 7001 + m), wl.dense(k, n, 7002 + m)
    ref, S = oracle_lib.sddmm(A.m, A.k, n, A.row_offsets, A.column_indices, L, R)
    for v in sddmm_variants():
        if spdl.spdl_variant_name(1, v) == "mfma":
            continue
        force(1, v)
        g.assert_close(g.gpu_sddmm(A, L, R, n), ref, S, g.TOL_F32,
                       f"clustered columns, sddmm variant {spdl.spdl_variant_name(1, v)}, shape {shape}")


@pytest.mark.parametrize("n", [132, 256, 388])
def test_sddmm_long_dot_products_of_dense_rows(g, oracle_lib, n):
    """Rows too dense for the slab kernel's 32 partial sums per row and slab, dot products longer
    than 128 columns: the lane kernel runs once per 128 columns and adds up in the output array.
    A uniform mask, ragged last chunk, rows that are not ascending (recomputed as a whole, whatever
    the earlier passes left), and the scaled form."""
    import torch
    import paper_2006_10901_amd as spdl
    cases = [wl.uniform_mask_csr(1500, 1000, 0.3, 970 + n), wl.adversarial_csr(600, 300, 971 + n, sorted_cols=False)]
    for idx, A in enumerate(cases):
        L, R = wl.dense(A.m, n, 972 + n), wl.dense(A.k, n, 973 + n)
        ref, S = oracle_lib.sddmm(A.m, A.k, n, A.row_offsets, A.column_indices, L, R)
        try:
            spdl.spdl_force_variant(1, 5)            # (what is chosen by default depends on the estimate of run times)
            chosen = spdl.spdl_variant_name(1, spdl.spdl_select_sddmm(A.m, A.k, n, A.nnz, 4, 0, 0)["variant"])
            assert chosen == "lane"
            g.assert_close(g.gpu_sddmm(A, L, R, n), ref, S, g.TOL_F32, f"lane sddmm in passes, n={n}")
            d = g.DevCsr(A)
            out = torch.full((A.nnz,), float("nan"), device="cuda")
            spdl.spdl_sddmm_scaled(A.m, A.k, n, A.nnz, d.ro, d.ci, d.val, g.dev(L), g.dev(R), out)
            torch.cuda.synchronize()
            v = A.values.astype(np.float64)
            g.assert_close(out.cpu().numpy(), v * ref, np.abs(v) * S, g.TOL_F32, f"scaled, in passes, n={n}")
        finally:
            spdl.spdl_force_variant(1, -1)


def test_forced_sddmm_variants_fp16_and_long_rows(g, oracle_lib, force):
    import paper_2006_10901_amd as spdl
    A = wl.uniform_mask_csr(300, 2000, 0.3, 960)          # ~600 nonzeros per row: several waves per row
    n = 136
    for dt, tol in ((np.float32, g.TOL_F32), (np.float16, g.TOL_F16)):
        L, R = wl.dense(A.m, n, 961, dt), wl.dense(A.k, n, 962, dt)
        out, S = oracle_lib.sddmm(A.m, A.k, n, A.row_offsets, A.column_indices, L, R)
        for v in sddmm_variants():
            force(1, v)
            got = g.gpu_sddmm(A, L, R, n)
            g.assert_close(got, out, S, tol, f"sddmm variant {spdl.spdl_variant_name(1, v)} {dt.__name__}")


@pytest.mark.parametrize("n", [36, 64, 100, 128])
def test_window_kernels_on_banded_masks(g, oracle_lib, force, n):
    """The window kernels (one window of 256 rows of the dense operand in LDS per 8 or 16 sparse rows,
    gathers for the rest) on masks with a band: a row count that is not a multiple of 16, fewer
    columns than a window holds, a band that is not on the diagonal of a rectangular matrix, a
    uniform mask, for which no window is placed, and a causal mask (band to the left of the diagonal).  SDDMM gives the bits of the nonzero-split kernel."""
    import paper_2006_10901_amd as spdl
    v0 = {spdl.spdl_variant_name(0, v): v for v in spmm_variants()}
    v1 = {spdl.spdl_variant_name(1, v): v for v in sddmm_variants()}
    shifted = wl.banded_attention_csr(600, 128, 0.3, 2105 + n)
    shifted = wl.Csr(600, 1500, shifted.row_offsets, (shifted.column_indices + 700).astype(np.int32), shifted.values)
    cases = [wl.banded_attention_csr(1000, 128, 0.2, 2100 + n), wl.banded_attention_csr(200, 64, 0.5, 2101 + n),
             shifted, wl.uniform_mask_csr(500, 3000, 0.1, 2102 + n), wl.causal_attention_csr(900, 256, 0.05, 2106 + n)]
    for idx, A in enumerate(cases):
        B, L = wl.dense(A.k, n, 2103 + n), wl.dense(A.m, n, 2104 + n)
        C, S = oracle_lib.spmm(A.m, A.k, n, A.row_offsets, A.column_indices, A.values, B)
        force(0, v0["window"])
        assert spdl.spdl_select_spmm(A.m, A.k, n, A.nnz, 4, 0, 0)["variant"] == v0["window"]
        g.assert_close(g.gpu_spmm(A, B, n, None), C, S, g.TOL_F32, f"window spmm case {idx} n={n}")
        out, So = oracle_lib.sddmm(A.m, A.k, n, A.row_offsets, A.column_indices, L, B)
        force(1, v1["window"])
        assert spdl.spdl_select_sddmm(A.m, A.k, n, A.nnz, 4, 0, 0)["variant"] == v1["window"]
        got = g.gpu_sddmm(A, L, B, n)
        g.assert_close(got, out, So, g.TOL_F32, f"window sddmm case {idx} n={n}")
        force(1, v1["group"])
        assert np.array_equal(got, g.gpu_sddmm(A, L, B, n))
        force(0, -1)
        force(1, -1)
        # the entry points for banded masks choose the same kernels by themselves: same bits
        import torch
        d = g.DevCsr(A)
        Cb = torch.full((A.m, n), float("nan"), device="cuda")
        ob = torch.full((A.nnz,), float("nan"), device="cuda")
        spdl.spdl_spmm_banded(A.m, A.k, n, A.nnz, d.ro, d.ci, d.val, g.dev(B), Cb)
        spdl.spdl_sddmm_banded(A.m, A.k, n, A.nnz, d.ro, d.ci, g.dev(L), g.dev(B), ob)
        torch.cuda.synchronize()
        g.assert_close(Cb.cpu().numpy(), C, S, g.TOL_F32, f"spmm_banded case {idx} n={n}")
        assert np.array_equal(ob.cpu().numpy(), got)


def test_banded_entry_points_fall_back_when_the_window_kernels_do_not_apply(g, oracle_lib):
    """n % 4 != 0 (SpMM), dot products of more than 128 columns (SDDMM), a matrix without entries:
    the entry points for banded masks then run what spdl_spmm / spdl_sddmm run."""
    import torch
    import paper_2006_10901_amd as spdl
    A = wl.banded_attention_csr(300, 64, 0.4, 2200)
    d = g.DevCsr(A)
    for n in (130, 200):
        B, L = wl.dense(A.k, n, 2201 + n), wl.dense(A.m, n, 2202 + n)
        C, S = oracle_lib.spmm(A.m, A.k, n, A.row_offsets, A.column_indices, A.values, B)
        out, So = oracle_lib.sddmm(A.m, A.k, n, A.row_offsets, A.column_indices, L, B)
        Cb = torch.full((A.m, n), float("nan"), device="cuda")
        ob = torch.full((A.nnz,), float("nan"), device="cuda")
        spdl.spdl_spmm_banded(A.m, A.k, n, A.nnz, d.ro, d.ci, d.val, g.dev(B), Cb)
        spdl.spdl_sddmm_banded(A.m, A.k, n, A.nnz, d.ro, d.ci, g.dev(L), g.dev(B), ob)
        torch.cuda.synchronize()
        g.assert_close(Cb.cpu().numpy(), C, S, g.TOL_F32, f"spmm_banded n={n}")
        g.assert_close(ob.cpu().numpy(), out, So, g.TOL_F32, f"sddmm_banded n={n}")
    E = wl.Csr(40, 50, np.zeros(41, dtype=np.int32), np.zeros(0, dtype=np.int32), np.zeros(0, dtype=np.float32))
    Ce = torch.full((40, 64), float("nan"), device="cuda")
    none_i, none_f = torch.empty(0, dtype=torch.int32, device="cuda"), torch.empty(0, device="cuda")
    spdl.spdl_spmm_banded(E.m, E.k, 64, 0, g.dev(E.row_offsets), none_i, none_f, torch.zeros((E.k, 64), device="cuda"), Ce)
    torch.cuda.synchronize()
    assert not Ce.cpu().numpy().any()


def _with_dense_rows(A, rows, seed):
    """A copy of A in which the given rows hold every column."""
    rng = np.random.default_rng(seed)
    lens = np.diff(A.row_offsets).astype(np.int64)
    lens[sorted(rows)] = A.k
    ro = np.zeros(A.m + 1, dtype=np.int64)
    np.cumsum(lens, out=ro[1:])
    ci = np.empty(ro[-1], dtype=np.int32)
    for i in range(A.m):
        ci[ro[i]:ro[i + 1]] = (np.arange(A.k) if i in rows
                               else A.column_indices[A.row_offsets[i]:A.row_offsets[i + 1]])
    return wl.Csr(A.m, A.k, ro.astype(np.int32), ci, rng.standard_normal(int(ro[-1])).astype(np.float32))


@pytest.mark.parametrize("n", [64, 100])
def test_sddmm_window_kernel_shares_the_tail_of_long_rows(g, oracle_lib, force, n):
    """The SDDMM window kernel gives a wave the first 512 entries of its row; what a longer row
    holds beyond them is dealt to all waves of the workgroup.  A banded mask in which some rows hold
    every column (first, last, two neighbours in one workgroup, one in a ragged last workgroup) and
    one holds exactly 512 and one 513 entries, against the oracle and bit for bit against the
    nonzero-split kernel."""
    import paper_2006_10901_amd as spdl
    base = wl.banded_attention_csr(1003, 64, 0.12, 4100 + n)
    A = _with_dense_rows(base, {0, 17, 18, 500, 1002}, 4101 + n)
    lens = np.diff(A.row_offsets).astype(np.int64)
    for r, want in ((40, 512), (41, 513)):
        lens[r] = want
    ro = np.zeros(A.m + 1, dtype=np.int64)
    np.cumsum(lens, out=ro[1:])
    ci = np.empty(ro[-1], dtype=np.int32)
    for i in range(A.m):
        old = A.column_indices[A.row_offsets[i]:A.row_offsets[i + 1]]
        ci[ro[i]:ro[i + 1]] = old if lens[i] == len(old) else np.arange(lens[i])
    A = wl.Csr(A.m, A.k, ro.astype(np.int32), ci, np.ones(int(ro[-1]), np.float32))
    L, R = wl.dense(A.m, n, 4102 + n), wl.dense(A.k, n, 4103 + n)
    ref, S = oracle_lib.sddmm(A.m, A.k, n, A.row_offsets, A.column_indices, L, R)
    names = {spdl.spdl_variant_name(1, v): v for v in sddmm_variants()}
    force(1, names["window"])
    assert spdl.spdl_variant_name(1, spdl.spdl_select_sddmm(A.m, A.k, n, A.nnz, 4, 0, 0)["variant"]) == "window"
    got = g.gpu_sddmm(A, L, R, n)
    g.assert_close(got, ref, S, g.TOL_F32, f"window sddmm, long rows, n={n}")
    force(1, names["group"])
    assert np.array_equal(got, g.gpu_sddmm(A, L, R, n))


@pytest.mark.parametrize("n", [64, 100])
def test_spmm_window_kernel_shares_the_tail_of_long_rows(g, oracle_lib, force, n):
    """The SpMM window kernel gives a wave the first 512 pairs of its row; what a longer row holds
    beyond them is dealt to all waves of the workgroup, whose partial sums the owner adds.  The
    same mask as for the SDDMM kernel (rows that hold every column: first, last, two neighbours in
    one workgroup, one in a ragged last workgroup; one row of exactly 512 and one of 513 entries)
    with random values, one and two column tiles, with and without the fused bias + ReLU."""
    import torch
    import paper_2006_10901_amd as spdl
    base = wl.banded_attention_csr(1003, 64, 0.12, 4200 + n)
    A = _with_dense_rows(base, {0, 17, 18, 500, 1002}, 4201 + n)
    lens = np.diff(A.row_offsets).astype(np.int64)
    for r, want in ((40, 512), (41, 513)):
        lens[r] = want
    ro = np.zeros(A.m + 1, dtype=np.int64)
    np.cumsum(lens, out=ro[1:])
    ci = np.empty(ro[-1], dtype=np.int32)
    for i in range(A.m):
        old = A.column_indices[A.row_offsets[i]:A.row_offsets[i + 1]]
        ci[ro[i]:ro[i + 1]] = old if lens[i] == len(old) else np.arange(lens[i])
    vals = np.random.default_rng(4202 + n).standard_normal(int(ro[-1])).astype(np.float32)
    A = wl.Csr(A.m, A.k, ro.astype(np.int32), ci, vals)
    B = wl.dense(A.k, n, 4203 + n)
    names = {spdl.spdl_variant_name(0, v): v for v in spmm_variants()}
    force(0, names["window"])
    assert spdl.spdl_variant_name(0, spdl.spdl_select_spmm(A.m, A.k, n, A.nnz, 4, 0, 0)["variant"]) == "window"
    C, S = oracle_lib.spmm(A.m, A.k, n, A.row_offsets, A.column_indices, A.values, B)
    g.assert_close(g.gpu_spmm(A, B, n, None), C, S, g.TOL_F32, f"window spmm, long rows, n={n}")
    bias = np.random.default_rng(4204 + n).standard_normal(A.m).astype(np.float32)
    C, S = oracle_lib.spmm_bias_relu(A.m, A.k, n, A.row_offsets, A.column_indices, A.values, B, bias, True)
    d = g.DevCsr(A)
    out = torch.full((A.m, n), float("nan"), dtype=torch.float32, device="cuda")
    spdl.spdl_spmm_bias_relu(A.m, A.k, n, A.nnz, d.ro, d.ci, d.val, None, g.dev(B), g.dev(bias), True, out)
    torch.cuda.synchronize()
    g.assert_close(out.cpu().numpy(), C, S, g.TOL_F32, f"window spmm + bias + relu, long rows, n={n}")


def test_spmm_wide_outputs_tile_inner_slab_kernel(g, oracle_lib, force):
    """Outputs wide enough for two rows per lane group and several tiles per workgroup: the slab
    kernel that scans a slab once for all its tiles.  A ragged last tile, a density at the edge of
    its look-ahead, rows that hold every column (more pairs in a slab than one scan takes: extra
    rounds in every tile's stage), rows that are not ascending, with and without a row order, and the
    fused bias + ReLU."""
    import torch
    import paper_2006_10901_amd as spdl
    cases = [(wl.uniform_mask_csr(2048, 700, 0.10, 2300), 2000),
             (wl.uniform_mask_csr(2048, 1300, 0.12, 2301), 2052),
             (_with_dense_rows(wl.uniform_mask_csr(2048, 900, 0.08, 2302), {0, 77, 1029, 2047}, 2303), 2304),
             (wl.adversarial_csr(2100, 600, 2304, sorted_cols=False), 2500)]
    slabdma = [v for v in spmm_variants() if spdl.spdl_variant_name(0, v) == "slabdma"][0]
    force(0, slabdma)            # (the very sparse last case would otherwise take the gather kernel)
    for idx, (A, n) in enumerate(cases):
        B = wl.dense(A.k, n, 2310 + idx)
        sel = spdl.spdl_select_spmm(A.m, A.k, n, A.nnz, 4, 0, 0)
        assert sel["variant"] == slabdma and sel["rows_per_block"] == 128
        assert 2 <= sel["grid_y"] <= 4
        C, S = oracle_lib.spmm(A.m, A.k, n, A.row_offsets, A.column_indices, A.values, B)
        for order in (None, spdl.spdl_build_row_order(A.m, A.row_offsets)):
            g.assert_close(g.gpu_spmm(A, B, n, order), C, S, g.TOL_F32, f"tile-inner slab case {idx}")
    A, n = cases[0]
    B = wl.dense(A.k, n, 2310)
    bias = np.random.default_rng(2320).standard_normal(A.m).astype(np.float32)
    C, S = oracle_lib.spmm_bias_relu(A.m, A.k, n, A.row_offsets, A.column_indices, A.values, B, bias, True)
    d = g.DevCsr(A)
    out = torch.full((A.m, n), float("nan"), device="cuda")
    spdl.spdl_spmm_bias_relu(A.m, A.k, n, A.nnz, d.ro, d.ci, d.val, None, g.dev(B), g.dev(bias), 1, out)
    torch.cuda.synchronize()
    g.assert_close(out.cpu().numpy(), C, S, g.TOL_F32, "tile-inner slab, bias + ReLU")


def test_entry_points_for_rows_of_unequal_length(g, oracle_lib):
    """spdl_spmm_skewed / spdl_sddmm_skewed: the same results as spdl_spmm / spdl_sddmm through the
    kernels that do not care how long a row is.  Log-normal row lengths (a few rows of thousands of
    entries), short and long dot products, a shape the preferred kernels cannot take (n % 4 != 0:
    runs as through the plain entry points), an empty matrix."""
    import torch
    import paper_2006_10901_amd as spdl
    cases = [(wl.lognormal_rows_csr(3000, 4000, 0.05, 5100, sigma_ln=1.5), 64),
             (wl.lognormal_rows_csr(2500, 3000, 0.08, 5101, sigma_ln=1.2), 128),
             (wl.lognormal_rows_csr(1500, 2100, 0.06, 5102, sigma_ln=1.3), 200),
             (wl.lognormal_rows_csr(1300, 1700, 0.10, 5103, sigma_ln=1.0), 520),
             (wl.lognormal_rows_csr(700, 900, 0.10, 5104, sigma_ln=1.0), 30),
             (wl.uniform_mask_csr(40, 50, 0.0, 5105), 64)]
    for A, n in cases:
        what = f"m={A.m} k={A.k} n={n} nnz={A.nnz}"
        d = g.DevCsr(A)
        B = wl.dense(A.k, n, 5110 + n)
        C, S = oracle_lib.spmm(A.m, A.k, n, A.row_offsets, A.column_indices, A.values, B)
        out = torch.full((A.m, n), float("nan"), dtype=torch.float32, device="cuda")
        spdl.spdl_spmm_skewed(A.m, A.k, n, A.nnz, d.ro, d.ci, d.val, g.dev(B), out)
        torch.cuda.synchronize()
        g.assert_close(out.cpu().numpy(), C, S, g.TOL_F32, "spmm_skewed " + what)
        L, R = wl.dense(A.m, n, 5111 + n), wl.dense(A.k, n, 5112 + n)
        ref, S = oracle_lib.sddmm(A.m, A.k, n, A.row_offsets, A.column_indices, L, R)
        out = torch.full((A.nnz,), float("nan"), dtype=torch.float32, device="cuda")
        spdl.spdl_sddmm_skewed(A.m, A.k, n, A.nnz, d.ro, d.ci, g.dev(L), g.dev(R), out)
        torch.cuda.synchronize()
        g.assert_close(out.cpu().numpy(), ref, S, g.TOL_F32, "sddmm_skewed " + what)


# ------------------------------------------------------------------ matrix-core kernels (fp16)
def _f16(A):
    A.values = A.values.astype(np.float16)
    return A


@pytest.mark.parametrize("n", [8, 24, 136, 264, 520])
def test_mfma_kernels_edge_cases(g, oracle_lib, force, n):
    import paper_2006_10901_amd as spdl
    dup = wl.adversarial_csr(150, 600, 1101, sorted_cols=False)
    dup.column_indices[5:9] = dup.column_indices[5]                 # duplicates inside a row
    cases = [wl.adversarial_csr(203, 700, 1100 + n),                # m % 32 != 0, k % 16 != 0, empty rows
             dup,
             wl.adversarial_csr(70, 2500, 1102 + n),                 # k spans three panel chunks
             wl.uniform_mask_csr(64, 96, 0.5, 1103 + n)]
    for A in cases:
        A = _f16(A)
        B = wl.dense(A.k, n, 1104 + n, np.float16)
        L, R = wl.dense(A.m, n, 1105 + n, np.float16), wl.dense(A.k, n, 1106 + n, np.float16)
        force(0, 3)
        force(1, 4)
        assert spdl.spdl_variant_name(0, spdl.spdl_select_spmm(A.m, A.k, n, A.nnz, 2, 0, 0)["variant"]) == "mfma"
        assert spdl.spdl_variant_name(1, spdl.spdl_select_sddmm(A.m, A.k, n, A.nnz, 2, 0, 0)["variant"]) == "mfma"
        spmm_case(g, oracle_lib, A, B, n, g.TOL_F16, "sorted", f"mfma spmm n={n} m={A.m} k={A.k}")
        sddmm_case(g, oracle_lib, A, L, R, n, g.TOL_F16, f"mfma sddmm n={n} m={A.m} k={A.k}")
        # the direct-gather kernels on the same inputs (what n % 8 != 0 or a sparser matrix would run)
        force(0, 0)
        force(1, 1)
        spmm_case(g, oracle_lib, A, B, n, g.TOL_F16, "sorted", f"rowsplit spmm f16 n={n}")
        sddmm_case(g, oracle_lib, A, L, R, n, g.TOL_F16, f"group sddmm f16 n={n}")


def test_mfma_spmm_row_lengths_and_short_contractions(g, oracle_lib, force):
    # Row lengths around the sizes the panel expansion works in (64 entries per load, 128 fetched
    # ahead, 256 per further round), and contractions shorter than the depth of the pipeline of B
    # loads (16 rows per step, six steps in registers), with and without a ragged last step.
    import paper_2006_10901_amd as spdl
    lengths = [0, 1, 63, 64, 65, 127, 128, 129, 191, 192, 193, 383, 384, 385, 640, 1500, 0, 2, 700, 130] * 2
    cases = [wl.row_lengths_csr(len(lengths), 1500, lengths, 1200)]
    for k in (16, 17, 31, 32, 40, 95, 96, 97, 112):
        cases.append(wl.uniform_mask_csr(50, k, 0.6, 1201 + k))
    for A in cases:
        A = _f16(A)
        for n in (8, 264):
            B = wl.dense(A.k, n, 1250 + n, np.float16)
            force(0, 3)
            assert spdl.spdl_variant_name(0, spdl.spdl_select_spmm(A.m, A.k, n, A.nnz, 2, 0, 0)["variant"]) == "mfma"
            spmm_case(g, oracle_lib, A, B, n, g.TOL_F16, "sorted", f"mfma spmm n={n} m={A.m} k={A.k}")
    # below 16 columns of A the kernel is not taken, forced or not
    A = _f16(wl.uniform_mask_csr(50, 12, 0.6, 1290))
    force(0, 3)
    assert spdl.spdl_variant_name(0, spdl.spdl_select_spmm(A.m, A.k, 64, A.nnz, 2, 0, 0)["variant"]) == "rowsplit"
    spmm_case(g, oracle_lib, A, wl.dense(A.k, 64, 1291, np.float16), 64, g.TOL_F16, "sorted", "k=12 fp16")


def test_mfma_spmm_rows_across_many_column_chunks(g, oracle_lib, force):
    """The panel of the matrix-core SpMM is expanded once per chunk of 1024 columns of A, each row
    continuing where the chunk before left it.  Five chunks; rows that hold every column, rows whose
    entries all lie in one late chunk or skip the middle chunks, rows with 64 / 128 / 256 entries
    per chunk exactly (the sizes of the expansion's rounds), a row with one entry in the last
    column, empty rows, and rows that are not ascending (computed apart), all in one panel and
    again spread over several."""
    import paper_2006_10901_amd as spdl
    k = 5000
    rng = np.random.default_rng(1300)
    def cols(kind):
        if kind == "full":
            return np.arange(k)
        if kind == "late":
            return np.arange(4100, 4100 + 700)
        if kind == "ends":
            return np.concatenate([np.arange(0, 300), np.arange(4096, 4096 + 300)])
        if kind == "last":
            return np.array([k - 1])
        if kind == "empty":
            return np.array([], dtype=np.int64)
        if kind.startswith("per"):
            per = int(kind[3:])
            return np.concatenate([c * 1024 + np.sort(rng.choice(900, per, replace=False)) for c in range(5)])
        if kind == "random":
            return np.sort(rng.choice(k, int(rng.integers(1, 3000)), replace=False))
        if kind == "shuffled":
            return rng.permutation(np.sort(rng.choice(k, 1500, replace=False)))
        raise ValueError(kind)
    kinds = ["full", "late", "ends", "last", "empty", "per64", "per128", "per256", "per65", "random", "shuffled", "full",
             "random", "late", "per129", "random"]
    for rows in (kinds, kinds * 5 + ["full", "empty", "shuffled"]):
        per_row = [cols(kd) for kd in rows]
        ro = np.zeros(len(rows) + 1, dtype=np.int32)
        ro[1:] = np.cumsum([len(c) for c in per_row])
        ci = np.concatenate(per_row).astype(np.int32)
        vals = rng.standard_normal(len(ci)).astype(np.float16)
        A = wl.Csr(len(rows), k, ro, ci, vals)
        for n in (8, 264):
            B = wl.dense(k, n, 1301 + n, np.float16)
            force(0, 3)
            assert spdl.spdl_variant_name(0, spdl.spdl_select_spmm(A.m, A.k, n, A.nnz, 2, 0, 0)["variant"]) == "mfma"
            spmm_case(g, oracle_lib, A, B, n, g.TOL_F16, "sorted", f"mfma spmm, five chunks, n={n} m={A.m}")


def test_mfma_kernels_are_the_default_for_moderately_sparse_fp16(g):
    import paper_2006_10901_amd as spdl
    assert spdl.spdl_variant_name(0, spdl.spdl_select_spmm(1024, 1024, 3136, 104000, 2, 0, 0)["variant"]) == "mfma"
    assert spdl.spdl_variant_name(1, spdl.spdl_select_sddmm(1024, 1024, 3136, 104000, 2, 0, 0)["variant"]) == "mfma"
    # one stored position in a hundred: gathering rows of B is cheaper than dense panels (SpMM); for SDDMM the
    # dense blocks stay cheaper at this length of the dot products, but not for short ones
    assert spdl.spdl_variant_name(0, spdl.spdl_select_spmm(1024, 1024, 3136, 10400, 2, 0, 0)["variant"]) == "rowsplit"
    assert spdl.spdl_variant_name(1, spdl.spdl_select_sddmm(1024, 1024, 3136, 10400, 2, 0, 0)["variant"]) == "mfma"
    assert spdl.spdl_variant_name(1, spdl.spdl_select_sddmm(2048, 2048, 64, 41000, 2, 0, 0)["variant"]) == "group"
    # fp32 never takes them, n % 8 != 0 neither
    assert spdl.spdl_variant_name(0, spdl.spdl_select_spmm(1024, 1024, 3136, 104000, 4, 0, 0)["variant"]) != "mfma"
    assert spdl.spdl_variant_name(0, spdl.spdl_select_spmm(1024, 1024, 3132, 104000, 2, 0, 0)["variant"]) == "rowsplit"


def test_rowsplit_with_several_lane_groups_per_row(g, oracle_lib, force):
    # few long rows: the row-splitting kernel spreads each row over 2, 4 or 8 lane groups
    import paper_2006_10901_amd as spdl
    force(0, 0)
    seen = set()
    for m, k, dens, n, dt in ((300, 4000, 0.3, 64, np.float32), (64, 3000, 0.5, 32, np.float32),
                              (500, 2000, 0.2, 128, np.float32), (300, 4000, 0.3, 64, np.float16),
                              (40, 5000, 0.4, 200, np.float32)):
        A = wl.uniform_mask_csr(m, k, dens, 3000 + m)
        A.row_offsets = A.row_offsets.copy()
        if dt == np.float16:
            A.values = A.values.astype(np.float16)
        B = wl.dense(k, n, 3001 + m, dt)
        sel = spdl.spdl_select_spmm(m, k, n, A.nnz, 2 if dt == np.float16 else 4, 0, 0)
        seen.add(256 // (sel["rows_per_block"] * sel["lanes_per_row"]))
        spmm_case(g, oracle_lib, A, B, n, g.TOL_F16 if dt == np.float16 else g.TOL_F32, "sorted",
                  f"rowsplit segments m={m} n={n} {dt.__name__}")
    assert max(seen) >= 4 and len(seen) >= 2, seen
