// SpMM, window family: for sparse matrices whose entries cluster around a band (the attention
// masks of paper Sec. "Application: Sparse Transformer": a dense band along the diagonal plus
// scattered entries elsewhere).  A workgroup owns NW consecutive sparse rows, one per wave, and one
// 64-column tile of C.  It copies ONE window of W consecutive rows of B into LDS, placed where the
// workgroup's rows have most of their entries, and every entry whose column falls inside the
// window takes its row of B from LDS (reuse across the workgroup's rows: neighbouring rows of a
// band share almost all their columns); every other entry gathers its row of B from global
// memory as the row-splitting kernel does.  There is no walk over all of B as in the slab
// kernels, so the rows' scattered entries cost one gather each and nothing else.
//
// A 16-lane group covers the 64 columns of the tile, four per lane (paper Sec. "Subwarp
// Tiling"); the four groups of a wave share the wave's row: the row is read 64 (value, column)
// pairs at a time, group s taking pairs 16 s .. 16 s + 15 and lane t of the group pair t, the next
// 64 requested before the current ones are used, and the four partial sums are added at the end.
// (One row per group would leave a sequence of 4096 rows with one wave per SIMD, and each wave
// with four times as many dependent memory latencies in a row.)  Pairs inside the
// window are multiplied exactly as in the slab kernels (LDS offset pre-scaled once per pair,
// DPP row broadcast of the value inside the multiply-add, the all-zero LDS row for lanes
// without a pair).  Pairs outside it: the byte offset of the row of B is broadcast lane by
// lane, the groups that have such a pair at that position load 16 bytes per lane under the
// execution mask, and all sixteen loads of a chunk are in flight before the first is used.
// The registers those loads fill are cleared first whenever some lane of the wave has no pair to
// gather at some position, so the multiply by that lane's zero value meets a zero and never a
// non-finite number left over from an earlier row of B.
//
// Any CSR input gives the right result: nothing depends on the order of a row's entries, and
// the window's position is only a matter of speed.  A wave walks the first 512 pairs of its row
// alone (or 9/8 of the mean row length, if that is more); what a longer row holds beyond them is dealt to all waves of the workgroup (64 pairs per
// wave and round, gathers only), whose partial sums meet in LDS and are added by the row's owner,
// so a few very long rows among short ones do not leave one wave working while the others have
// finished.  Workgroups without such a row do not synchronise again once the window is in place.
// Needs n % 4 == 0, 16-byte aligned B and C, k * n * 4 < 2^31.
#pragma once
#include "common.hpp"
#include "spmm_slab.hpp"

namespace spdl {

constexpr int kWinTile = 64;                 // output columns per tile (= kSlabTile: the same inner steps)

template <int NW>
struct WinShape {
  static constexpr int kRows = NW;                           // sparse rows per workgroup
  static constexpr int kW = 256;                             // rows of B in the window
  static constexpr int kPartialOff = (kW + 1) * kWinTile * 4; // after the window and the all-zero row:
  static constexpr int kLdsBytes = kPartialOff + NW * kWinTile * 4;   // one row of partial sums per wave
};

constexpr int kWinOwnPairs = 512;            // entries of its own row that a wave walks alone (a multiple of 64)

// The tail of a long row, shared by the waves of a workgroup: pairs begin + 16 sub .. per group,
// + stride, ... below end, every one gathered from global memory (no window), four loads in
// flight per group.  Returns this lane's four columns of the partial sum.  Lean on
// purpose: the main kernel has no registers to spare, and this runs only for rows of more than
// kWinOwnPairs entries.  A lane without a pair at a position skips the load and the multiply-add,
// so nothing outside a row's own entries reaches its sum.
__device__ __forceinline__ f32x4 win_tail_gather(const int* __restrict__ column_indices,
                                                          const float* __restrict__ values, const char* gbase,
                                                          int begin, int end, int stride, int n, int sub, int l16) {
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int at = begin + 16 * sub; __any(at < end); at += stride) {
    const bool valid = at + l16 < end;
    const int idx = valid ? at + l16 : begin;
    const float a = valid ? values[idx] : 0.f;
    const int goff = valid ? (int)((unsigned)column_indices[idx] * (unsigned)n * 4u) : (int)0x80000000;
#define SPDL_TAIL1(T)                                                                                          \
  const int o##T = __builtin_amdgcn_update_dpp(0, goff, 0x150 + (T), 0xf, 0xf, false);                          \
  const float av##T = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, a), 0x150 + (T), 0xf, 0xf, false)); \
  f32x4 b##T = {0.f, 0.f, 0.f, 0.f};                                                                            \
  if (o##T >= 0) b##T = *reinterpret_cast<const f32x4*>(gbase + (unsigned)o##T);
#define SPDL_TAILF(T)                                                                                          \
  if (o##T >= 0) {                                                                                              \
    acc.x = __builtin_fmaf(av##T, b##T.x, acc.x);                                                               \
    acc.y = __builtin_fmaf(av##T, b##T.y, acc.y);                                                               \
    acc.z = __builtin_fmaf(av##T, b##T.z, acc.z);                                                               \
    acc.w = __builtin_fmaf(av##T, b##T.w, acc.w);                                                               \
  }
#define SPDL_TAIL4(A, B, C, D)                                                                                 \
  {                                                                                                             \
    SPDL_TAIL1(A) SPDL_TAIL1(B) SPDL_TAIL1(C) SPDL_TAIL1(D)                                                     \
    SPDL_TAILF(A) SPDL_TAILF(B) SPDL_TAILF(C) SPDL_TAILF(D)                                                     \
  }
    SPDL_TAIL4(0, 1, 2, 3) SPDL_TAIL4(4, 5, 6, 7) SPDL_TAIL4(8, 9, 10, 11) SPDL_TAIL4(12, 13, 14, 15)
#undef SPDL_TAIL1
#undef SPDL_TAILF
#undef SPDL_TAIL4
  }
  return acc;
}

// Column of the entry at quantile j/4 of the row [b, e), e > b (a wave-uniform load).
__device__ __forceinline__ int win_quantile(const int* __restrict__ ci, int b, int e, int j) {
  return ci[uniform(b + (int)(((long long)(e - b - 1) * j) >> 2))];
}

// Where the window goes: between a low quantile of the workgroup's first row r0 and a high
// quantile of its last row r1, for the pair of quantiles (0, 1/2), (1/4, 3/4), (1/2, 1) that
// spans the fewest columns; the window is centred on that span.  A band with scattered entries
// on one or both sides puts two adjacent quarters of a row's entries inside the band.  Returns
// the window's first column, or k (no window: nothing is inside it) when half of the rows'
// entries do not fit into W columns.  Wave-uniform.
template <int W>
__device__ __forceinline__ int win_place(const int* __restrict__ row_offsets, const int* __restrict__ column_indices,
                                         int r0, int r1, int k) {
  int c0 = 0;
  const int b0 = row_offsets[r0], e0 = row_offsets[r0 + 1];
  const int b1 = row_offsets[r1], e1 = row_offsets[r1 + 1];
  // an empty first or last row lends the other one's entries
  const int lb = e0 > b0 ? b0 : b1, le = e0 > b0 ? e0 : e1;
  const int hb = e1 > b1 ? b1 : b0, he = e1 > b1 ? e1 : e0;
  if (le > lb && he > hb) {
    int best = 0x7fffffff, centre = 0;
#pragma unroll
    for (int a = 0; a < 3; ++a) {
      const int lo = win_quantile(column_indices, lb, le, a);
      const int hi = win_quantile(column_indices, hb, he, a + 2);
      const int span = hi >= lo ? hi - lo : 0x7ffffffe;
      if (span < best) { best = span; centre = lo + (span >> 1); }
    }
    c0 = max(0, min(centre - W / 2, k - W));
    if (best > W) c0 = k;
  }
  return uniform(c0);
}

template <int NW>
__global__ __launch_bounds__(64 * NW, 4) void spmm_window_kernel(
    int m, int k, int n, int nnz, const int* __restrict__ row_offsets,
    const int* __restrict__ column_indices, const float* __restrict__ values, const float* __restrict__ B,
    float* __restrict__ C, const float* __restrict__ bias, int relu) {
  using Sh = WinShape<NW>;
  constexpr int W = Sh::kW;
  constexpr int kZeroOff = W * kWinTile * 4;
  constexpr int kCopies = W / (4 * NW);                 // 1 KB direct-to-LDS loads per wave
  static_assert(W % (4 * NW) == 0, "every wave copies the same number of 4-row pieces");
  extern __shared__ __attribute__((aligned(16))) char lds_raw[];

  PhaseClocks clocks;
  clocks.start();
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = uniform(tid >> 6);
  const int sub = lane >> 4;
  const int l16 = lane & 15;
  const int lane_b = l16 * 16;
  const int panel = blockIdx.x;
  const int tile = blockIdx.y;
  const int col = tile * kWinTile + l16 * 4;
  const bool col_ok = col < n;
  const int last_nz = nnz - 1;

  if (tid < kWinTile) *reinterpret_cast<float*>(lds_raw + kZeroOff + tid * 4) = 0.f;

  const int r0 = panel * Sh::kRows;
  const int r1 = min(m, r0 + Sh::kRows) - 1;
  // the offsets of all rows of the workgroup (for the rows that are shared at the end), requested
  // with everything else of the set-up and moved to scalar registers once they have arrived
  int ro_raw[NW + 1];
#pragma unroll
  for (int i = 0; i <= NW; ++i) ro_raw[i] = row_offsets[min(r0 + i, m)];
  const int c0 = win_place<W>(row_offsets, column_indices, r0, r1, k);

  // The window copy: copy i of wave w fills window rows (i*NW + w)*4 .. +3, lane L row L/16 of
  // those and columns 4*(L%16) .. +3 of the tile; rows past k are clamped to row k-1 and
  // columns past n to the tile's first column (nothing valid reads those).
  if (c0 < k) {
    const unsigned col_off = col_ok ? (unsigned)(l16 * 16) : 0u;
    const char* base = reinterpret_cast<const char*>(B + tile * kWinTile);
    const unsigned dst = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)lds_raw +
                         (unsigned)wave * (4 * kWinTile * 4);
#pragma unroll
    for (int i = 0; i < kCopies; ++i) {
      const int lrow = (i * NW + wave) * 4 + sub;
      const unsigned voff = (unsigned)min(c0 + lrow, k - 1) * (unsigned)n * 4u + col_off;
      const unsigned m0v = dst + (unsigned)i * (NW * 4 * kWinTile * 4);
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                   :: "s"(m0v), "v"(voff), "s"(base) : "memory", "m0");
    }
  }

  const int row = r0 + wave;
  const bool row_ok = row < m;
  const int p_begin = (row_ok ? row_offsets[row] : 0) + 16 * sub;
  const int p_row_end = row_ok ? row_offsets[row + 1] : 0;

  auto fetch = [&](int at, int& c, float& a) {
    const unsigned o = (unsigned)min(at + l16, last_nz) << 2;
    c = *reinterpret_cast<const int*>(reinterpret_cast<const char*>(column_indices) + o);
    a = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(values) + o);
  };
  int cc, cn;
  float aa, an;
  fetch(p_begin, cc, aa);

  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  // rows of B gathered from global memory, one per pair of a chunk (four arrays of four: the
  // multiply-add macro takes an array of four)
  f32x4 g0[4], g1[4], g2[4], g3[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) g0[t] = g1[t] = g2[t] = g3[t] = f32x4{0.f, 0.f, 0.f, 0.f};
  const char* gbase = reinterpret_cast<const char*>(B + (col_ok ? col : 0));

  clocks.lap(kPhaseSetup);
  __builtin_amdgcn_s_waitcnt(0);      // the window copy and the first chunk
  clocks.lap(kPhaseWait);
  __syncthreads();
  clocks.lap(kPhaseBarrier);
  int ro_all[NW + 1];
#pragma unroll
  for (int i = 0; i <= NW; ++i) ro_all[i] = uniform(ro_raw[i]);
  // A wave walks at most `own` pairs of its row alone (the rest of a longer row: below): 9/8 of the
  // mean row length of the matrix, in whole rounds, so rows that are long but alike are not shared
  // at all.
  const int mean = nnz / m;
  const int own = max(kWinOwnPairs, (mean + (mean >> 3) + 63) & ~63);
  const int p_end = min(p_row_end, p_begin - 16 * sub + own);

  for (int at = p_begin; __any(at < p_end); at += 64) {
    fetch(at + 64, cn, an);
    const bool valid = at + l16 < p_end;
    const unsigned rel = (unsigned)(cc - c0);
    const bool inwin = valid && rel < (unsigned)W;
    const bool outw = valid && !inwin;
    const unsigned long long m_in = __builtin_amdgcn_ballot_w64(inwin);
    const unsigned long long m_out = __builtin_amdgcn_ballot_w64(outw);
    clocks.lap(kPhaseScan);
    if (m_in != 0) {
      // positions 0 .. cmax-1 of the chunk hold every pair inside the window, in any group
      const unsigned lo = (unsigned)m_in, hi = (unsigned)(m_in >> 32);
      const unsigned any16 = (lo | (lo >> 16) | hi | (hi >> 16)) & 0xffffu;
      const int cmax = 32 - __builtin_clz(any16);
      const float av = inwin ? aa : 0.f;
      const int off = inwin ? (int)(rel * (kWinTile * 4)) : kZeroOff;
      slab_steps(acc, av, off, lds_raw, lane_b, cmax);
    }
    clocks.lap(kPhaseSteps);
    if (m_out != 0) {
      const float av = outw ? aa : 0.f;
      // byte offset of the pair's row of B; the sign bit marks "no gather for this pair"
      const int goff = outw ? (int)((unsigned)cc * (unsigned)n * 4u) : (int)0x80000000;
      const unsigned lo = (unsigned)m_out, hi = (unsigned)(m_out >> 32);
      const unsigned any16 = (lo | (lo >> 16) | hi | (hi >> 16)) & 0xffffu;
      if (m_out != ~0ull) {
#pragma unroll
        for (int t = 0; t < 4; ++t) g0[t] = g1[t] = g2[t] = g3[t] = f32x4{0.f, 0.f, 0.f, 0.f};
      }
#define SPDL_WIN_GATHER(G, T)                                                                    \
  {                                                                                              \
    const int o = __builtin_amdgcn_update_dpp(0, goff, 0x150 + (T), 0xf, 0xf, false);            \
    if (o >= 0) G[(T) & 3] = *reinterpret_cast<const f32x4*>(gbase + (unsigned)o);               \
  }
      // all the loads of the chunk first (blocks of four positions that no group needs are
      // skipped), then the multiply-adds
      if (any16 & 0x000fu) { SPDL_WIN_GATHER(g0, 0) SPDL_WIN_GATHER(g0, 1) SPDL_WIN_GATHER(g0, 2) SPDL_WIN_GATHER(g0, 3) }
      if (any16 & 0x00f0u) { SPDL_WIN_GATHER(g1, 4) SPDL_WIN_GATHER(g1, 5) SPDL_WIN_GATHER(g1, 6) SPDL_WIN_GATHER(g1, 7) }
      if (any16 & 0x0f00u) { SPDL_WIN_GATHER(g2, 8) SPDL_WIN_GATHER(g2, 9) SPDL_WIN_GATHER(g2, 10) SPDL_WIN_GATHER(g2, 11) }
      if (any16 & 0xf000u) { SPDL_WIN_GATHER(g3, 12) SPDL_WIN_GATHER(g3, 13) SPDL_WIN_GATHER(g3, 14) SPDL_WIN_GATHER(g3, 15) }
#undef SPDL_WIN_GATHER
      if (any16 & 0x000fu) slab_fma16_q0(acc, av, g0);
      if (any16 & 0x00f0u) slab_fma16_q1(acc, av, g1);
      if (any16 & 0x0f00u) slab_fma16_q2(acc, av, g2);
      if (any16 & 0xf000u) slab_fma16_q3(acc, av, g3);
    }
    clocks.lap(kPhaseGather);
    cc = cn;
    aa = an;
  }

  // What a row holds beyond kWinOwnPairs pairs is dealt to all waves of the workgroup, 64 pairs at
  // a time; their partial sums go through LDS to the wave that owns the row.  A row of thousands of
  // entries among rows of hundreds would otherwise keep one wave busy long after the others are
  // done.  (The loop is the same for every wave of the workgroup, so its barriers are met by all.)
  float* partials = reinterpret_cast<float*>(lds_raw + Sh::kPartialOff);
#pragma unroll
  for (int i = 0; i < NW; ++i) {
    const int rb = ro_all[i], re = ro_all[i + 1];       // (rows past m: empty)
    if (re - rb <= own) continue;
    f32x4 part = win_tail_gather(column_indices, values, gbase, rb + own + 64 * wave, re, 64 * NW, n, sub, l16);
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      part[v] += __shfl_xor(part[v], 16, kWave);
      part[v] += __shfl_xor(part[v], 32, kWave);
    }
    if (sub == 0) *reinterpret_cast<f32x4*>(partials + wave * kWinTile + l16 * 4) = part;
    __syncthreads();
    if (wave == i && sub == 0) {
#pragma unroll
      for (int w2 = 0; w2 < NW; ++w2) {
        const f32x4 pv = *reinterpret_cast<const f32x4*>(partials + w2 * kWinTile + l16 * 4);
        acc[0] += pv.x; acc[1] += pv.y; acc[2] += pv.z; acc[3] += pv.w;
      }
    }
    __syncthreads();
  }

#pragma unroll
  for (int v = 0; v < 4; ++v) {
    acc[v] += __shfl_xor(acc[v], 16, kWave);
    acc[v] += __shfl_xor(acc[v], 32, kWave);
  }
  if (row_ok && col_ok && sub == 0) {
    spmm_epilogue<float, 4>(acc, bias, row, relu);
    Pack<float, 4>::store(C + (size_t)row * n + col, acc);
  }
  clocks.lap(kPhaseRest);
  clocks.store((blockIdx.y * gridDim.x + blockIdx.x) * NW + wave);
}

}  // namespace spdl
