"""GPU parity of the operations around SpMM/SDDMM: softmax over CSR rows, SpMM with the fused
bias + ReLU epilogue, and SpMM with the transposed sparse matrix, each against the CPU oracle.

Tolerances.  Softmax (fp32): relative 1e-4 plus absolute 1e-37.  The kernel rounds scale*x once,
subtracts the row maximum, calls an exponential good to a few ulp whose argument error
2^-24*|scale*x| becomes a relative error of the same size, sums at most len positive terms
(relative error <= len * 2^-24 however they are grouped) and divides: about
(2*|scale*x|max + log2(len) + 8) * 2^-24 in all, below 1e-4 up to |scale*x| ~ 800; the absolute
term covers results that underflow fp32.  Bias + ReLU: the SpMM rule, 1e-4 * (S + |bias|) for
fp32 and 2e-3 * (S + |bias|) + 2^-25 for fp16 storage (ReLU never increases an error)."""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu

SOFTMAX_RTOL = 1e-4
SOFTMAX_ATOL = 1e-37


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


def gpu_softmax(g, m, ro, x, scale, in_place=False):
    import torch
    import paper_2006_10901_amd as spdl
    dx = g.dev(x)
    out = dx if in_place else torch.full_like(dx, float("nan"))
    spdl.spdl_csr_softmax(m, x.shape[0], g.dev(ro), dx, scale, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def check_softmax(got, ref, what):
    assert np.all(np.isfinite(got)), f"{what}: non-finite or unwritten output"
    err = np.abs(got.astype(np.float64) - ref)
    bad = err > SOFTMAX_RTOL * ref + SOFTMAX_ATOL
    assert not bad.any(), f"{what}: {bad.sum()} outside tolerance, worst {err.max():.3e}"


# ------------------------------------------------------------------ softmax
def test_softmax_row_lengths_around_every_boundary(g, oracle_lib):
    # empty rows, single entries, the wave width, the register-resident limit (1024) and beyond
    lengths = np.array([0, 1, 2, 63, 64, 65, 0, 127, 128, 129, 1023, 1024, 1025, 0, 3000, 5000, 7, 0],
                       dtype=np.int64)
    m = lengths.size
    ro = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    x = (4.0 * np.random.default_rng(501).standard_normal(int(ro[-1]))).astype(np.float32)
    for scale in (1.0, 0.125, -2.5):
        ref = oracle_lib.csr_softmax(m, ro, x, scale)
        got = gpu_softmax(g, m, ro, x, scale)
        check_softmax(got, ref, f"softmax scale={scale}")
        sums = np.add.reduceat(got.astype(np.float64), ro[:-1][lengths > 0])
        assert np.allclose(sums, 1.0, atol=1e-5)
    # one-entry rows are exactly 1
    assert gpu_softmax(g, m, ro, x, 1.0)[ro[1]] == 1.0


def test_softmax_large_magnitudes_and_in_place(g, oracle_lib):
    rng = np.random.default_rng(502)
    lengths = rng.integers(1, 400, size=300)
    ro = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    x = rng.uniform(-300.0, 300.0, size=int(ro[-1])).astype(np.float32)   # exp() alone would overflow
    x[ro[5]:ro[6]] = 88.5                                                # equal logits: uniform row
    ref = oracle_lib.csr_softmax(300, ro, x, 1.0)
    got = gpu_softmax(g, 300, ro, x, 1.0)
    check_softmax(got, ref, "softmax large")
    assert np.all(got[ro[5]:ro[6]] == np.float32(1.0) / np.float32(lengths[5]))
    again = gpu_softmax(g, 300, ro, x, 1.0, in_place=True)
    assert np.array_equal(again, got)


def test_softmax_attention_scores_full_size(g, oracle_lib):
    # the Sparse Transformer path: scores from SDDMM, scaled by 1/sqrt(d_k), softmax, then SpMM
    import torch
    import paper_2006_10901_amd as spdl
    w = wl.attention(0)
    A, Q, K, V = w["A"], w["Q"], w["K"], w["V"]
    scores, _ = oracle_lib.sddmm(4096, 4096, 64, A.row_offsets, A.column_indices, Q, K)
    scores = scores.astype(np.float32)
    ref = oracle_lib.csr_softmax(4096, A.row_offsets, scores, 0.125)
    got = gpu_softmax(g, 4096, A.row_offsets, scores, 0.125)
    check_softmax(got, ref, "attention softmax")
    # chained on the GPU: SDDMM -> softmax (in place) -> SpMM, against the oracle's chain.  The
    # scores carry 1e-4*S_sddmm of error, which the softmax turns into a relative error of
    # 2 * 0.125 * that (numerator and normaliser), small next to the SpMM budget used here.
    d = g.DevCsr(A)
    sc = torch.empty(A.nnz, device="cuda")
    C = torch.empty((4096, 64), device="cuda")
    spdl.spdl_sddmm(4096, 4096, 64, A.nnz, d.ro, d.ci, g.dev(Q), g.dev(K), sc)
    spdl.spdl_csr_softmax(4096, A.nnz, d.ro, sc, 0.125, sc)
    spdl.spdl_spmm(4096, 4096, 64, A.nnz, d.ro, d.ci, sc, None, g.dev(V), C)
    torch.cuda.synchronize()
    Cref, S = oracle_lib.spmm(4096, 4096, 64, A.row_offsets, A.column_indices, ref.astype(np.float32), V)
    g.assert_close(C.cpu().numpy(), Cref, S, 1e-3, "attention chain with softmax")


def test_softmax_degenerate_sizes(g):
    import torch
    import paper_2006_10901_amd as spdl
    ro = torch.zeros(5, dtype=torch.int32, device="cuda")
    x = torch.empty(0, device="cuda")
    spdl.spdl_csr_softmax(4, 0, ro, x, 1.0, x)
    spdl.spdl_csr_softmax(0, 0, ro, x, 1.0, x)
    with pytest.raises(spdl.SpdlError):
        spdl.spdl_csr_softmax(-1, 0, ro, x, 1.0, x)
    torch.cuda.synchronize()


# ------------------------------------------------------------------ bias + ReLU epilogue
def gpu_spmm_epilogue(g, A, B, n, bias, relu, order):
    import torch
    import paper_2006_10901_amd as spdl
    f16 = A.values.dtype == np.float16
    d = g.DevCsr(A)
    dB = g.dev(B)
    C = torch.full((A.m, n), float("nan"), dtype=dB.dtype, device="cuda")
    fn = spdl.spdl_spmm_bias_relu_f16 if f16 else spdl.spdl_spmm_bias_relu
    fn(A.m, A.k, n, A.nnz, d.ro, d.ci, d.val, g.dev(order) if order is not None else None, dB,
       g.dev(bias) if bias is not None else None, relu, C)
    torch.cuda.synchronize()
    return C.cpu().numpy()


def spmm_variants():
    import paper_2006_10901_amd as spdl
    out, v = [], 0
    while spdl.spdl_variant_name(0, v) is not None:
        out.append(v)
        v += 1
    return out


@pytest.mark.parametrize("n", [4, 68, 200])
def test_bias_relu_every_variant(g, oracle_lib, force, n):
    import paper_2006_10901_amd as spdl
    A = wl.adversarial_csr(203, 700, 1900 + n)
    B = wl.dense(A.k, n, 1901 + n)
    bias = np.random.default_rng(1902 + n).standard_normal(A.m).astype(np.float32)
    order = oracle_lib.row_order(A.m, A.row_offsets)
    for b, relu in ((bias, True), (bias, False), (None, True), (None, False)):
        C, S = oracle_lib.spmm_bias_relu(A.m, A.k, n, A.row_offsets, A.column_indices, A.values, B, b, relu)
        results = []
        for v in spmm_variants():
            force(0, v)
            got = gpu_spmm_epilogue(g, A, B, n, b, relu, order)
            g.assert_close(got, C, S, g.TOL_F32, f"{spdl.spdl_variant_name(0, v)} bias={b is not None} relu={relu}")
            if relu:
                assert (got >= 0).all() and (got == 0).any()
            if spdl.spdl_variant_name(0, v) != "window":         # (adds four partial sums per row)
                results.append(got)
        for r in results[1:]:
            assert np.array_equal(r, results[0])
        force(0, -1)
    # without bias and activation the entry point is plain SpMM, bit for bit
    assert np.array_equal(gpu_spmm_epilogue(g, A, B, n, None, False, order), g.gpu_spmm(A, B, n, order))


@pytest.mark.parametrize("skewed", [False, True])
def test_bias_relu_conv1x1_fp16_full_size(g, oracle_lib, skewed):
    # the MobileNet use: 1x1 convolution weights as the sparse matrix, bias per output channel
    w = wl.conv1x1(skewed)
    A, B, n = w["A"], w["B"], w["n"]
    bias = (0.5 * np.random.default_rng(wl.seed_for(5, 7)).standard_normal(A.m)).astype(np.float16)
    # binary16 -> binary32 is exact, so the fp32 oracle on the widened inputs is the fp16 oracle
    C, S = oracle_lib.spmm_bias_relu(A.m, A.k, n, A.row_offsets, A.column_indices, A.values.astype(np.float32),
                                     B.astype(np.float32), bias.astype(np.float32), True)
    got = gpu_spmm_epilogue(g, A, B, n, bias, True, oracle_lib.row_order(A.m, A.row_offsets))
    g.assert_close(got, C, S, g.TOL_F16, f"conv bias relu f16 skewed={skewed}")


def test_bias_relu_lstm_shape_fp32_default_kernel(g, oracle_lib):
    import paper_2006_10901_amd as spdl
    w = wl.lstm(90)
    A, B, n = w["A"], w["B"], w["n"]
    assert spdl.spdl_variant_name(0, spdl.spdl_select_spmm(A.m, A.k, n, A.nnz, 4, 0, 0)["variant"]) == "slabdma"
    bias = np.random.default_rng(wl.seed_for(2, 77)).standard_normal(A.m).astype(np.float32)
    C, S = oracle_lib.spmm_bias_relu(A.m, A.k, n, A.row_offsets, A.column_indices, A.values, B, bias, True)
    got = gpu_spmm_epilogue(g, A, B, n, bias, True, oracle_lib.row_order(A.m, A.row_offsets))
    g.assert_close(got, C, S, g.TOL_F32, "lstm-90 bias relu")


# ------------------------------------------------------------------ transposed SpMM
@pytest.mark.parametrize("case", ["adversarial", "ffn"])
def test_transposed_spmm(g, oracle_lib, case):
    import torch
    import paper_2006_10901_amd as spdl
    if case == "adversarial":
        A = wl.adversarial_csr(333, 517, 2100, sorted_cols=False)
        n = 72
    else:
        A = wl.transformer_ffn(1, with_dense=False)["A"]
        n = 256
    B = wl.dense(A.m, n, 2101)
    tro, tci, perm = spdl.spdl_build_transpose_host(A.m, A.k, A.nnz, A.row_offsets, A.column_indices)
    otro, otci, operm = oracle_lib.transpose_topology(A.m, A.k, A.row_offsets, A.column_indices)
    assert np.array_equal(tro, otro) and np.array_equal(tci, otci) and np.array_equal(perm, operm)
    dval = g.dev(A.values)
    tval = torch.full_like(dval, float("nan"))
    spdl.spdl_permute_values(A.nnz, 4, g.dev(perm), dval, tval)
    torch.cuda.synchronize()
    assert np.array_equal(tval.cpu().numpy(), A.values[operm])
    h = g.dev(A.values.astype(np.float16))
    th = torch.empty_like(h)
    spdl.spdl_permute_values(A.nnz, 2, g.dev(perm), h, th)
    torch.cuda.synchronize()
    assert np.array_equal(th.cpu().numpy(), A.values.astype(np.float16)[operm])
    # A^T B through the ordinary SpMM on the cached transposed topology
    C, S = oracle_lib.spmm(A.k, A.m, n, otro, otci, A.values[operm], B)
    T = wl.Csr(A.k, A.m, tro, tci, tval.cpu().numpy())
    got = g.gpu_spmm(T, B, n, oracle_lib.row_order(A.k, otro))
    g.assert_close(got, C, S, g.TOL_F32, f"transposed spmm {case}")


# ------------------------------------------------------------------ general SDDMM (scaled by A's values)
def gpu_sddmm_scaled(g, A, L, R, n):
    import torch
    import paper_2006_10901_amd as spdl
    f16 = L.dtype == np.float16
    d = g.DevCsr(A)
    dL, dR = g.dev(L), g.dev(R)
    out = torch.full((A.nnz,), float("nan"), dtype=dL.dtype, device="cuda")
    fn = spdl.spdl_sddmm_scaled_f16 if f16 else spdl.spdl_sddmm_scaled
    fn(A.m, A.k, n, A.nnz, d.ro, d.ci, d.val, dL, dR, out)
    torch.cuda.synchronize()
    assert np.array_equal(d.val.cpu().numpy(), A.values)          # the values are an input only
    return out.cpu().numpy()


def sddmm_variants():
    import paper_2006_10901_amd as spdl
    out, v = [], 0
    while spdl.spdl_variant_name(1, v) is not None:
        out.append(v)
        v += 1
    return out


@pytest.mark.parametrize("n", [4, 68, 128, 200])
def test_sddmm_scaled_every_variant(g, oracle_lib, force, n):
    import paper_2006_10901_amd as spdl
    for sorted_cols in (True, False):
        A = wl.adversarial_csr(203, 700, 2300 + n, sorted_cols=sorted_cols)
        L, R = wl.dense(A.m, n, 2301 + n), wl.dense(A.k, n, 2302 + n)
        ref, S = oracle_lib.sddmm_scaled(A.m, A.k, n, A.row_offsets, A.column_indices, A.values, L, R)
        for v in sddmm_variants():
            force(1, v)
            got = gpu_sddmm_scaled(g, A, L, R, n)
            g.assert_close(got, ref, S, g.TOL_F32, f"scaled sddmm {spdl.spdl_variant_name(1, v)} n={n} sorted={sorted_cols}")
        force(1, -1)


def test_sddmm_scaled_full_size_and_fp16(g, oracle_lib):
    import torch
    import paper_2006_10901_amd as spdl
    w = wl.lstm(90)
    A, L, R, n = w["A"], w["L"], w["R"], w["n"]
    assert spdl.spdl_variant_name(1, spdl.spdl_select_sddmm(A.m, A.k, n, A.nnz, 4, 0, 0)["variant"]) == "lane"
    ref, S = oracle_lib.sddmm_scaled(A.m, A.k, n, A.row_offsets, A.column_indices, A.values, L, R)
    g.assert_close(gpu_sddmm_scaled(g, A, L, R, n), ref, S, g.TOL_F32, "lstm-90 scaled sddmm")
    c = wl.conv1x1(True)
    A, L, R, n = c["A"], c["L"], c["R"], c["n"]
    # binary16 -> binary32 is exact, so the fp32 oracle on the widened inputs is the fp16 oracle
    ref, S = oracle_lib.sddmm_scaled(A.m, A.k, n, A.row_offsets, A.column_indices, A.values.astype(np.float32),
                                     L.astype(np.float32), R.astype(np.float32))
    g.assert_close(gpu_sddmm_scaled(g, A, L, R, n), ref, S, g.TOL_F16, "conv skewed scaled sddmm f16")
    # the values array may not double as the output
    d = g.DevCsr(w["A"])
    with pytest.raises(spdl.SpdlError):
        spdl.spdl_sddmm_scaled(d.m, d.k, 128, d.nnz, d.ro, d.ci, d.val, g.dev(w["L"]), g.dev(w["R"]), d.val)
    torch.cuda.synchronize()


def test_epilogue_and_scaling_on_the_matrix_core_kernels(g, oracle_lib, force):
    import paper_2006_10901_amd as spdl
    A = wl.adversarial_csr(203, 700, 2400)
    A.values = A.values.astype(np.float16)
    n = 136
    B = wl.dense(A.k, n, 2401, np.float16)
    bias = np.random.default_rng(2402).standard_normal(A.m).astype(np.float16)
    force(0, 3)
    force(1, 4)
    for b, relu in ((bias, True), (bias, False), (None, True)):
        C, S = oracle_lib.spmm_bias_relu(A.m, A.k, n, A.row_offsets, A.column_indices, A.values.astype(np.float32),
                                         B.astype(np.float32), None if b is None else b.astype(np.float32), relu)
        got = gpu_spmm_epilogue(g, A, B, n, b, relu, None)
        g.assert_close(got, C, S, g.TOL_F16, f"mfma spmm bias={b is not None} relu={relu}")
    L, R = wl.dense(A.m, n, 2403, np.float16), wl.dense(A.k, n, 2404, np.float16)
    ref, S = oracle_lib.sddmm_scaled(A.m, A.k, n, A.row_offsets, A.column_indices, A.values.astype(np.float32),
                                     L.astype(np.float32), R.astype(np.float32))
    g.assert_close(gpu_sddmm_scaled(g, A, L, R, n), ref, S, g.TOL_F16, "mfma scaled sddmm")


# ------------------------------------------------------------------ non-transposed right-hand operand
@pytest.mark.parametrize("n", [1, 7, 64, 130])
def test_sddmm_nt(g, oracle_lib, n):
    import torch
    import paper_2006_10901_amd as spdl
    for sorted_cols in (True, False):
        A = wl.adversarial_csr(203, 157, 2500 + n, sorted_cols=sorted_cols)
        L, Rn = wl.dense(A.m, n, 2501 + n), wl.dense(n, A.k, 2502 + n)
        ref, S = oracle_lib.sddmm_nt(A.m, A.k, n, A.row_offsets, A.column_indices, L, Rn)
        d = g.DevCsr(A)
        out = torch.full((A.nnz,), float("nan"), device="cuda")
        spdl.spdl_sddmm_nt(A.m, A.k, n, A.nnz, d.ro, d.ci, None, g.dev(L), g.dev(Rn), out)
        torch.cuda.synchronize()
        g.assert_close(out.cpu().numpy(), ref, S, g.TOL_F32, f"sddmm nt n={n}")
        # with the element-wise scaling: values[p] times the same sum
        out.fill_(float("nan"))
        spdl.spdl_sddmm_nt(A.m, A.k, n, A.nnz, d.ro, d.ci, d.val, g.dev(L), g.dev(Rn), out)
        torch.cuda.synchronize()
        v = A.values.astype(np.float64)
        g.assert_close(out.cpu().numpy(), v * ref, np.abs(v) * S, g.TOL_F32, f"scaled sddmm nt n={n}")
        # fp16 operands (exactly representable in fp32, so the fp32 oracle on the widened inputs applies)
        Lh, Rh = L.astype(np.float16), Rn.astype(np.float16)
        refh, Sh = oracle_lib.sddmm_nt(A.m, A.k, n, A.row_offsets, A.column_indices, Lh.astype(np.float32),
                                       Rh.astype(np.float32))
        outh = torch.full((A.nnz,), float("nan"), dtype=torch.float16, device="cuda")
        spdl.spdl_sddmm_nt_f16(A.m, A.k, n, A.nnz, d.ro, d.ci, None, g.dev(Lh), g.dev(Rh), outh)
        torch.cuda.synchronize()
        g.assert_close(outh.cpu().numpy(), refh, Sh, g.TOL_F16, f"sddmm nt f16 n={n}")


@pytest.mark.parametrize("n", [4, 64, 100, 128])
def test_sddmm_nt_slab_path(g, oracle_lib, n):
    """k % 4 == 0, n % 4 == 0, n <= 128, 16-byte aligned operands: the slabs of Rn are fetched as
    they lie and transposed inside LDS.  Ragged last slab (160 = 128 + 32 columns), rows that are
    not ascending (redone entry by entry), the scaled form."""
    import torch
    import paper_2006_10901_amd as spdl
    cases = [wl.adversarial_csr(203, 160, 2600 + n, sorted_cols=True),
             wl.adversarial_csr(203, 160, 2600 + n, sorted_cols=False),
             wl.uniform_mask_csr(700, 1000, 0.3, 2650 + n),        # 8 slabs, three look-ahead chunks
             wl.uniform_mask_csr(64, 132, 0.9, 2660 + n)]          # nearly dense rows: several rounds per slab
    for A in cases:
        L, Rn = wl.dense(A.m, n, 2601 + n), wl.dense(n, A.k, 2602 + n)
        ref, S = oracle_lib.sddmm_nt(A.m, A.k, n, A.row_offsets, A.column_indices, L, Rn)
        d = g.DevCsr(A)
        out = torch.full((A.nnz,), float("nan"), device="cuda")
        spdl.spdl_sddmm_nt(A.m, A.k, n, A.nnz, d.ro, d.ci, None, g.dev(L), g.dev(Rn), out)
        torch.cuda.synchronize()
        g.assert_close(out.cpu().numpy(), ref, S, g.TOL_F32, f"sddmm nt {A.m}x{A.k} n={n}")
        out.fill_(float("nan"))
        spdl.spdl_sddmm_nt(A.m, A.k, n, A.nnz, d.ro, d.ci, d.val, g.dev(L), g.dev(Rn), out)
        torch.cuda.synchronize()
        v = A.values.astype(np.float64)
        g.assert_close(out.cpu().numpy(), v * ref, np.abs(v) * S, g.TOL_F32, f"scaled sddmm nt {A.m}x{A.k} n={n}")


def test_sddmm_nt_lstm_full_size(g, oracle_lib):
    """The weight-gradient shape of the LSTM problem at 90 % sparsity with R given as its transpose
    (128 x 10240): every output against the oracle, and bit for bit against the transposed entry point,
    which forms each dot product in the same order."""
    import torch
    import paper_2006_10901_amd as spdl
    w = wl.lstm(90)
    A, L, R = w["A"], w["L"], w["R"]
    Rn = np.ascontiguousarray(R.T)
    ref, S = oracle_lib.sddmm_nt(A.m, A.k, 128, A.row_offsets, A.column_indices, L, Rn)
    d = g.DevCsr(A)
    out = torch.full((A.nnz,), float("nan"), device="cuda")
    spdl.spdl_sddmm_nt(A.m, A.k, 128, A.nnz, d.ro, d.ci, None, g.dev(L), g.dev(Rn), out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    g.assert_close(got, ref, S, g.TOL_F32, "lstm 90 % sddmm nt")
    assert np.array_equal(got, g.gpu_sddmm(A, L, R, 128, dA=d))


def test_sddmm_nt_attention_size_equals_transposed_form(g, oracle_lib):
    # the attention scores of one head, computed from K^T (64 x 4096) instead of K
    import torch
    import paper_2006_10901_amd as spdl
    w = wl.attention(0)
    A, Q, K = w["A"], w["Q"], w["K"]
    ref, S = oracle_lib.sddmm_nt(4096, 4096, 64, A.row_offsets, A.column_indices, Q, np.ascontiguousarray(K.T))
    d = g.DevCsr(A)
    out = torch.full((A.nnz,), float("nan"), device="cuda")
    spdl.spdl_sddmm_nt(4096, 4096, 64, A.nnz, d.ro, d.ci, None, g.dev(Q), g.dev(np.ascontiguousarray(K.T)), out)
    torch.cuda.synchronize()
    g.assert_close(out.cpu().numpy(), ref, S, g.TOL_F32, "attention scores from K^T")


# ------------------------------------------------------------------ 16-bit column indices
@pytest.mark.parametrize("n", [8, 50, 136])
def test_spmm_f16_with_int16_indices(g, oracle_lib, force, n):
    import torch
    import paper_2006_10901_amd as spdl
    dup = wl.adversarial_csr(150, 600, 2601, sorted_cols=False)
    dup.column_indices[5:9] = dup.column_indices[5]
    for A in (wl.adversarial_csr(203, 700, 2600 + n), dup, wl.adversarial_csr(70, 2500, 2602 + n)):
        A.values = A.values.astype(np.float16)
        B = wl.dense(A.k, n, 2603 + n, np.float16)
        C, S = oracle_lib.spmm(A.m, A.k, n, A.row_offsets, A.column_indices, A.values, B)
        d = g.DevCsr(A)
        ci16 = g.dev(A.column_indices.astype(np.int16))
        order = g.dev(oracle_lib.row_order(A.m, A.row_offsets))
        for variant in (-1, 0, 3):                      # the heuristic's choice, row splitting, matrix cores
            force(0, variant)
            got = torch.full((A.m, n), float("nan"), dtype=torch.float16, device="cuda")
            spdl.spdl_spmm_f16_i16(A.m, A.k, n, A.nnz, d.ro, ci16, d.val, order, g.dev(B), got)
            torch.cuda.synchronize()
            g.assert_close(got.cpu().numpy(), C, S, g.TOL_F16, f"int16 indices n={n} variant={variant}")
        force(0, -1)
    with pytest.raises(spdl.SpdlError):                 # k does not fit 16 signed bits
        spdl.spdl_spmm_f16_i16(4, 40000, 8, 0, d.ro, ci16, d.val, None, g.dev(B), got)
