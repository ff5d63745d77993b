"""Seeded synthetic inputs shaped like the paper's workloads.

Only random draws and index bookkeeping live here: no SpMM / SDDMM arithmetic.
Both the CPU oracle's tests and the GPU path's tests / benchmark take their
inputs from this module, so the two sides always see identical arrays.

Workload shapes follow the paper's experiments (Sec. "Sparse Recurrent Neural
Networks", Fig. 1 caption, Sec. "Application: Sparse Transformer",
Sec. "Application: Sparse MobileNetV1", and the load-imbalance figure); the
paper's own matrices are not available, so every topology is drawn from a
distribution with the same sparsity and row-length statistics.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np

BASE_SEED = 20200610


def seed_for(config_id: int, variant: int = 0) -> int:
    return BASE_SEED + 100 * config_id + variant


@dataclass
class Csr:
    m: int
    k: int
    row_offsets: np.ndarray      # int32 [m+1]
    column_indices: np.ndarray   # int32 [nnz], ascending inside each row
    values: np.ndarray           # float32 [nnz]

    @property
    def nnz(self) -> int:
        return int(self.row_offsets[-1])

    @property
    def row_lengths(self) -> np.ndarray:
        return np.diff(self.row_offsets)


def _from_mask_rows(m, k, rows_cols, rng, sigma):
    lens = np.fromiter((len(c) for c in rows_cols), dtype=np.int64, count=m)
    ro = np.zeros(m + 1, dtype=np.int64)
    np.cumsum(lens, out=ro[1:])
    assert ro[-1] < 2**31
    ci = (np.concatenate(rows_cols) if m else np.zeros(0)).astype(np.int32)
    vals = (rng.standard_normal(int(ro[-1]), dtype=np.float32) * np.float32(sigma))
    return Csr(m, k, ro.astype(np.int32), ci, vals.astype(np.float32))


def uniform_mask_csr(m, k, density, seed, sigma=1.0, chunk_rows=512) -> Csr:
    """Each of the m*k entries is kept independently with probability `density`."""
    rng = np.random.default_rng(seed)
    lens = np.zeros(m, dtype=np.int64)
    cols = []
    for r0 in range(0, m, chunk_rows):
        r1 = min(m, r0 + chunk_rows)
        keep = rng.random((r1 - r0, k), dtype=np.float32) < np.float32(density)
        rr, cc = np.nonzero(keep)            # row-major order: ascending columns per row
        lens[r0:r1] = np.bincount(rr, minlength=r1 - r0)
        cols.append(cc.astype(np.int32))
    ro = np.zeros(m + 1, dtype=np.int64)
    np.cumsum(lens, out=ro[1:])
    assert ro[-1] < 2**31
    ci = np.concatenate(cols) if cols else np.zeros(0, np.int32)
    vals = rng.standard_normal(int(ro[-1]), dtype=np.float32) * np.float32(sigma)
    return Csr(m, k, ro.astype(np.int32), ci.astype(np.int32), vals.astype(np.float32))


def row_lengths_csr(m, k, lengths, seed, sigma=1.0) -> Csr:
    """Row i gets lengths[i] distinct columns drawn uniformly, sorted ascending."""
    rng = np.random.default_rng(seed)
    rows = []
    for i in range(m):
        cnt = int(lengths[i])
        if cnt == 0:
            rows.append(np.zeros(0, np.int32))
        elif cnt == k:
            rows.append(np.arange(k, dtype=np.int32))
        else:
            rows.append(np.sort(rng.choice(k, size=cnt, replace=False)).astype(np.int32))
    return _from_mask_rows(m, k, rows, rng, sigma)


def binomial_rows_csr(m, k, density, seed, sigma=1.0) -> Csr:
    rng = np.random.default_rng(seed)
    lengths = rng.binomial(k, density, size=m)
    return row_lengths_csr(m, k, lengths, seed + 1, sigma)


def lognormal_rows_csr(m, k, density, seed, sigma_ln=1.0, sigma=1.0) -> Csr:
    """Skewed rows: lengths ~ LogNormal(mu, sigma_ln) with mean density*k, clipped to [0,k],
    then rescaled so the total count is within 1 % of density*m*k."""
    rng = np.random.default_rng(seed)
    mean = density * k
    mu = math.log(mean) - 0.5 * sigma_ln * sigma_ln
    raw = rng.lognormal(mu, sigma_ln, size=m)
    target = density * m * k
    lengths = np.clip(np.rint(raw), 0, k)
    for _ in range(20):
        tot = lengths.sum()
        if abs(tot - target) <= 0.01 * target:
            break
        raw = raw * (target / max(tot, 1.0))
        lengths = np.clip(np.rint(raw), 0, k)
    return row_lengths_csr(m, k, lengths.astype(np.int64), seed + 1, sigma)


def banded_attention_csr(seq, band, density, seed, sigma=1.0) -> Csr:
    """Dense band |i-j| <= band/2 plus off-band entries kept with probability
    proportional to 1/|i-j|, scaled so the overall density is `density`."""
    rng = np.random.default_rng(seed)
    half = band // 2
    i = np.arange(seq)[:, None]
    j = np.arange(seq)[None, :]
    dist = np.abs(i - j)
    in_band = dist <= half
    w = np.where(in_band, 0.0, 1.0 / np.maximum(dist, 1))
    extras = density * seq * seq - in_band.sum()
    assert extras > 0
    p = np.minimum(1.0, w * (extras / w.sum()))
    keep = in_band | (rng.random((seq, seq)) < p)
    rr, cc = np.nonzero(keep)
    lens = np.bincount(rr, minlength=seq)
    ro = np.zeros(seq + 1, dtype=np.int64)
    np.cumsum(lens, out=ro[1:])
    vals = rng.standard_normal(int(ro[-1]), dtype=np.float32) * np.float32(sigma)
    return Csr(seq, seq, ro.astype(np.int32), cc.astype(np.int32), vals)


def causal_attention_csr(seq, band, off_density, seed, sigma=1.0) -> Csr:
    """Causal mask: the band i - band < j <= i, plus entries to the left of it kept with probability
    proportional to 1/(i - j), scaled so that `off_density` of those positions are kept (the mask of
    paper Sec. "Application: Sparse Transformer": band 256, 5 % off the band, sequence 12,288)."""
    rng = np.random.default_rng(seed)
    i = np.arange(seq)[:, None]
    j = np.arange(seq)[None, :]
    d = i - j
    left = d >= band
    w = np.where(left, 1.0 / np.maximum(d, 1), 0.0)
    p = np.minimum(1.0, w * (off_density * left.sum() / max(w.sum(), 1e-30)))
    keep = ((d >= 0) & (d < band)) | (rng.random((seq, seq)) < p)
    rr, cc = np.nonzero(keep)
    ro = np.zeros(seq + 1, dtype=np.int64)
    np.cumsum(np.bincount(rr, minlength=seq), out=ro[1:])
    vals = rng.standard_normal(int(ro[-1]), dtype=np.float32) * np.float32(sigma)
    return Csr(seq, seq, ro.astype(np.int32), cc.astype(np.int32), vals)


def clustered_rows_csr(m, k, seed, sigma=1.0) -> Csr:
    """Rows whose columns are anything but evenly spread over [0, k): each row draws a pattern at
    random: all columns in a narrow range at the left end, at the right end or around a random
    centre; two clusters at both ends; every second row of a dense run; or spread evenly.  Columns
    ascending inside a row.  (A test input for searches that guess positions by interpolation.)"""
    rng = np.random.default_rng(seed)
    rows = []
    for _ in range(m):
        kind = int(rng.integers(0, 6))
        width = int(rng.integers(1, max(2, k // 8)))
        if kind == 0:
            pool = np.arange(0, min(k, width))
        elif kind == 1:
            pool = np.arange(max(0, k - width), k)
        elif kind == 2:
            c = int(rng.integers(0, k))
            pool = np.arange(max(0, c - width // 2), min(k, c + width // 2 + 1))
        elif kind == 3:
            pool = np.concatenate([np.arange(0, min(k // 2, width)), np.arange(max(k // 2, k - width), k)])
        elif kind == 4:
            c = int(rng.integers(0, max(1, k - 2 * width)))
            pool = np.arange(c, min(k, c + 2 * width), 2)
        else:
            pool = np.arange(k)
        take = int(rng.integers(0, len(pool) + 1))
        if rng.random() < 0.3:
            take = len(pool)
        rows.append(np.sort(rng.choice(pool, size=take, replace=False)).astype(np.int32))
    return _from_mask_rows(m, k, rows, rng, sigma)


def dense(rows, cols, seed, dtype=np.float32) -> np.ndarray:
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((rows, cols), dtype=np.float32)
    return x.astype(dtype)          # fp16: one round-to-nearest-even of the fp32 draw


def adversarial_csr(m, k, seed, max_len=None, sorted_cols=True, sigma=1.0) -> Csr:
    """Small matrix whose rows start at every residue modulo 8: lengths cycle through
    0,1,2,3,5,7,8,9,... with empty rows first, last and in the middle."""
    rng = np.random.default_rng(seed)
    max_len = min(k, max_len or k)
    pattern = [0, 1, 2, 3, 5, 0, 7, 8, 9, 4, 13, 16, 17, 31, 33, 6, 64, 65, 0, 11]
    lengths = np.array([min(max_len, pattern[i % len(pattern)] + (i // len(pattern)) % 3) for i in range(m)])
    lengths[0] = 0
    lengths[-1] = 0
    rows = []
    for i in range(m):
        c = rng.choice(k, size=int(lengths[i]), replace=False).astype(np.int32)
        rows.append(np.sort(c) if sorted_cols else c)
    return _from_mask_rows(m, k, rows, rng, sigma)


# ---------------------------------------------------------------------------
# The five benchmark configurations
# ---------------------------------------------------------------------------
LSTM_SPARSITIES = (70, 80, 90, 95, 98)


def tiny(seed=None):
    s = seed_for(1) if seed is None else seed
    A = uniform_mask_csr(512, 512, 0.10, s)
    return dict(A=A, n=128, B=dense(512, 128, s + 1), L=dense(512, 128, s + 2), R=dense(512, 128, s + 3))


def lstm(sparsity_pct: int, with_dense=True):
    """Weight-sparse LSTM: A is (4*hidden) x (input+hidden) = 8192 x 10240, batch 128."""
    s = seed_for(2, sparsity_pct)
    A = uniform_mask_csr(8192, 10240, 1.0 - sparsity_pct / 100.0, s, sigma=0.02)
    out = dict(A=A, n=128)
    if with_dense:
        out.update(B=dense(10240, 128, s + 1), L=dense(8192, 128, s + 2), R=dense(10240, 128, s + 3))
    return out


def transformer_ffn(which: int, with_dense=True):
    """which=1: W1 4096x1024; which=2: W2 1024x4096; 4096 tokens, 90 % sparse."""
    s = seed_for(3, which)
    m, k = (4096, 1024) if which == 1 else (1024, 4096)
    A = binomial_rows_csr(m, k, 0.10, s, sigma=0.02)
    out = dict(A=A, n=4096)
    if with_dense:
        out.update(B=dense(k, 4096, s + 2), L=dense(m, 4096, s + 3), R=dense(k, 4096, s + 4))
    return out


def attention(head: int = 0, topology=None):
    s = seed_for(4)
    A = topology if topology is not None else banded_attention_csr(4096, 256, 0.10, s)
    hs = s + 10 * (head + 1)
    return dict(A=A, n=64, Q=dense(4096, 64, hs), K=dense(4096, 64, hs + 1), V=dense(4096, 64, hs + 2))


def conv1x1(skewed: bool, with_dense=True):
    s = seed_for(5, 1 if skewed else 0)
    if skewed:
        A = lognormal_rows_csr(1024, 1024, 0.10, s)
    else:
        A = uniform_mask_csr(1024, 1024, 0.10, s)
    A.values = A.values.astype(np.float16)
    out = dict(A=A, n=3136)
    if with_dense:
        out.update(B=dense(1024, 3136, s + 2, np.float16), L=dense(1024, 3136, s + 3, np.float16),
                   R=dense(1024, 3136, s + 4, np.float16))
    return out


def imbalance_sweep(cov: float, seed=None):
    """8192 x 2048 at 75 % sparsity with a chosen row-length coefficient of variation
    (the load-imbalance figure's problem); lengths are gamma distributed, total fixed."""
    s = seed_for(6, int(round(cov * 100))) if seed is None else seed
    rng = np.random.default_rng(s)
    m, k, mean = 8192, 2048, 512.0
    if cov <= 0:
        lengths = np.full(m, int(mean))
    else:
        shape = 1.0 / (cov * cov)
        lengths = np.clip(np.rint(rng.gamma(shape, mean / shape, size=m)), 0, k)
        lengths = np.clip(np.rint(lengths * (mean * m / lengths.sum())), 0, k)
    A = row_lengths_csr(m, k, lengths.astype(np.int64), s + 1)
    return dict(A=A, n=128, B=dense(k, 128, s + 2))
