// SDDMM, window family: the counterpart of the window SpMM kernel for sparse matrices whose
// entries cluster around a band (the attention masks of paper Sec. "Application: Sparse
// Transformer") and dot products of at most 128 columns (one attention head).  A workgroup owns
// NW consecutive sparse rows, one per wave, and copies ONE window of 256 consecutive rows of R
// into LDS, placed where its rows have most of their entries.  A row is cut into strips of 16
// consecutive entries, dealt to the wave's four 16-lane groups; a strip whose 16 columns all lie
// inside the window reads its rows of R from LDS, any other strip gathers them from global
// memory exactly as the nonzero-split kernel does.  The arithmetic of a strip is that kernel's
// (four columns of the dot product per lane, one partial sum per entry, a transposing reduction
// that leaves entry t's result in lane t), so both give the same bits.
// Any CSR input gives the right result; the window's position is only a matter of speed.
// NC = chunks of 64 columns of the dot product (1 or 2); the window holds 256 rows x 64 NC columns
// of R, chunk after chunk.  Needs n <= 64 NC, n % 4 == 0, 16-byte aligned L and R, k * n < 2^29.
#pragma once
#include "common.hpp"
#include "sddmm_group.hpp"
#include "spmm_window.hpp"

namespace spdl {

constexpr int kWinOwn = 512;     // entries of its own row that a wave walks alone, at least (a multiple of 64)

template <int NW, int NC>
__global__ __launch_bounds__(64 * NW, 4) void sddmm_window_kernel(
    int m, int k, int n, int nnz, const int* __restrict__ row_offsets,
    const int* __restrict__ column_indices, const float* __restrict__ L, const float* __restrict__ R,
    float* __restrict__ out, const float* __restrict__ scale) {
  constexpr int W = 256;
  constexpr int kChunkBytes = W * 64 * 4;           // one 64-column chunk of the window
  constexpr int kCopies = W / (4 * NW);
  static_assert(W % (4 * NW) == 0, "every wave copies the same number of 4-row pieces");
  extern __shared__ __attribute__((aligned(16))) char lds_raw[];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = uniform(tid >> 6);
  const int sub = lane >> 4;
  const int l16 = lane & 15;
  // this lane's four columns of chunk c: 64 c + 4 l16 .. + 3 (past n: the chunk's first four, times zero)
  bool col_ok[NC];
  int lane_b[NC];
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    col_ok[c] = 64 * c + l16 * 4 < n;
    lane_b[c] = col_ok[c] ? l16 * 16 : 0;
  }

  const int r0 = blockIdx.x * NW;
  const int r1 = min(m, r0 + NW) - 1;
  // the offsets of all rows of the workgroup (for the rows that are shared at the end), requested
  // with everything else of the set-up and moved to scalar registers once they have arrived
  int ro_raw[NW + 1];
#pragma unroll
  for (int i = 0; i <= NW; ++i) ro_raw[i] = row_offsets[min(r0 + i, m)];
  const int c0 = win_place<W>(row_offsets, column_indices, r0, r1, k);

  // The window copy, chunk after chunk: copy i of wave w fills window rows (i*NW + w)*4 .. +3 (256
  // bytes each in LDS), lane L row L/16 of those and columns 4*(L%16) .. +3 of the chunk; rows past
  // k are clamped to row k-1 and columns past n to the chunk's first (nothing valid reads those).
  if (c0 < k) {
    const unsigned dst = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)lds_raw +
                         (unsigned)wave * (4 * 64 * 4);
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const char* base = reinterpret_cast<const char*>(R + 64 * c);
#pragma unroll
      for (int i = 0; i < kCopies; ++i) {
        const int lrow = (i * NW + wave) * 4 + sub;
        const unsigned voff = (unsigned)min(c0 + lrow, k - 1) * (unsigned)n * 4u + (unsigned)lane_b[c];
        const unsigned m0v = dst + (unsigned)(c * kChunkBytes + i * (NW * 4 * 64 * 4));
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                     :: "s"(m0v), "v"(voff), "s"(base) : "memory", "m0");
      }
    }
  }

  const int row = r0 + wave;
  const bool row_ok = row < m;
  const int p_begin = row_ok ? row_offsets[row] : 0;
  const int p_end = row_ok ? row_offsets[row + 1] : 0;

  // this lane's four columns per chunk of sparse row r of L (zero past n)
  float l[NC][4];
  auto load_l = [&](const float* Lrow) {
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      Pack<float, 4>::load(Lrow + 64 * c + (col_ok[c] ? l16 * 4 : 0), l[c]);
#pragma unroll
      for (int v = 0; v < 4; ++v) l[c][v] = col_ok[c] ? l[c][v] : 0.f;
    }
  };

  // Strips at begin + 16 sub, + stride, ... below end, of the sparse row whose entries end at
  // row_end and whose row of L is in l (Lrow for the gathered strips).
  auto walk = [&](int begin, int end, int stride, int row_end, const float* Lrow) {
    // the column of this lane's entry of the strip at `at`; past the row end the last entry's again
    auto fetch = [&](int at) { return column_indices[max(min(at + l16, row_end - 1), 0)]; };
    int at = begin + 16 * sub;
    int cc = fetch(at);
    for (; __any(at < end); at += stride) {
      const int cn = fetch(at + stride);
      const unsigned rel = (unsigned)(cc - c0);
      const unsigned long long m_in = __builtin_amdgcn_ballot_w64(rel < (unsigned)W);
      const bool group_in = ((unsigned)(m_in >> (16 * sub)) & 0xffffu) == 0xffffu;
      if (at < end) {
        if (group_in) {
          const int off = (int)(rel * 256u);
          float partial[16];
#pragma unroll
          for (int t = 0; t < 16; ++t) partial[t] = 0.f;
#pragma unroll
          for (int c = 0; c < NC; ++c) {
            f32x4 r[16];
            const char* chunk = lds_raw + c * kChunkBytes + lane_b[c];
#define SPDL_W1(T0) \
            r[T0] = *reinterpret_cast<const f32x4*>(chunk + __builtin_amdgcn_update_dpp(0, off, 0x150 + (T0), 0xf, 0xf, false));
            SPDL_W1(0) SPDL_W1(1) SPDL_W1(2) SPDL_W1(3) SPDL_W1(4) SPDL_W1(5) SPDL_W1(6) SPDL_W1(7)
            SPDL_W1(8) SPDL_W1(9) SPDL_W1(10) SPDL_W1(11) SPDL_W1(12) SPDL_W1(13) SPDL_W1(14) SPDL_W1(15)
#undef SPDL_W1
#pragma unroll
            for (int t = 0; t < 16; ++t) {
              partial[t] = __builtin_fmaf(l[c][0], r[t].x, partial[t]);
              partial[t] = __builtin_fmaf(l[c][1], r[t].y, partial[t]);
              partial[t] = __builtin_fmaf(l[c][2], r[t].z, partial[t]);
              partial[t] = __builtin_fmaf(l[c][3], r[t].w, partial[t]);
            }
          }
          const float total = reduce16x16(partial, l16);
          if (at + l16 < row_end) sddmm_store<float>(out, scale, at + l16, total);
        } else {
          sddmm_strip_direct_at<float>(n, at, row_end, l16, cc * n, Lrow, R, out, scale);
        }
      }
      cc = cn;
    }
  };

  const float* Lown = L + (size_t)(row_ok ? row : 0) * n;
  load_l(Lown);
  __builtin_amdgcn_s_waitcnt(0);      // the window copy
  __syncthreads();
  int ro_all[NW + 1];
#pragma unroll
  for (int i = 0; i <= NW; ++i) ro_all[i] = uniform(ro_raw[i]);

  // Every wave walks the first kWinOwn entries of its own row.  What a longer row holds beyond them
  // is dealt to all waves of the workgroup, 64 entries at a time (every entry's result is its own,
  // so nothing has to be added up): a row of thousands of entries among rows of hundreds would
  // otherwise keep one wave busy long after the others are done (a matrix with log-normal row
  // lengths, 4096 x 4096 at 6 %, n = 64: 60 us against 17 for the nonzero-split kernel).
  // The share a wave walks alone grows with the mean row length of the matrix (9/8 of it, rounded
  // up to whole rounds), so rows that are long but alike are not shared at all.
  const int mean = nnz / m;
  const int own = max(kWinOwn, (mean + (mean >> 3) + 63) & ~63);
  walk(p_begin, min(p_end, p_begin + own), 64, p_end, Lown);
#pragma unroll
  for (int i = 0; i < NW; ++i) {
    const int rb = ro_all[i], re = ro_all[i + 1];        // (rows past m: empty)
    if (re - rb <= own) continue;
    const float* Lrow = L + (size_t)(r0 + i) * n;
    load_l(Lrow);
    // (the first 64 entries of row i's tail go to wave i, the next to wave i + 1, ...: short tails
    // of several rows then do not all land on the first waves)
    walk(rb + own + 64 * ((wave + NW - i) & (NW - 1)), re, 64 * NW, re, Lrow);
  }
}

}  // namespace spdl
