// SpMM in mixed precision on the matrix cores (paper Sec. "Mixed Precision": fp16 operands,
// fp32 accumulation).  A panel of 32 sparse rows is expanded into a dense fp16 block in LDS
// (zeros where A stores nothing) and multiplied with MFMA: on this chip the dense fp16 matrix
// rate is some thirty times the fp32 vector rate, so for the moderately sparse matrices of deep
// learning the multiplications by zero cost less than gathering one row of B per stored entry.
// Sparsity still saves the memory and the traffic of A.
//
// A workgroup owns one panel (32 or 64 rows) and WAVES tiles of 256 output columns.  The panel
// is expanded once per chunk of up to kMfmaChunk columns of A and shared by the waves.  For a
// step of 16 columns of A, lane (c, h) of a wave loads rows k0+8h .. k0+8h+7 of B, columns
// n0+8c .. n0+8c+7 (eight 16-byte loads; the 32 lanes of a half read 512 contiguous bytes of each
// row), transposes the 8x8 block inside its registers with byte permutes, and so obtains, for
// each j < 8, the second MFMA operand of the 32 output columns n0+8c+j: B needs no staging and
// no transposed copy although the contraction runs over its slow dimension.  The eight
// results of a lane for one row are eight adjacent columns: one 16-byte store.
//
// Rows whose indices are not strictly ascending (duplicates included) cannot be expanded by
// plain stores; they are found while the panel is filled and computed by direct gathers.
// Needs n % 8 == 0 and 16-byte aligned B and C.  The row order is not used: dense work is the
// same for every row.
#pragma once
#include "common.hpp"
#include "sddmm_mfma.hpp"

namespace spdl {

constexpr int kMfmaChunk = 1024;         // columns of A expanded at a time
constexpr int kMfmaSets = 6;             // steps of B rows held in registers per wave
constexpr int kMfmaPad = 8;              // halves of padding per panel row: row stride = 16 mod 128 bytes

// LDS: the panel of 32*rb rows (reused at the end to add up the k-parts' accumulators, rb * 32 KB
// per tile), the flags of rows that cannot be expanded, the panel's row offsets.
__host__ __device__ __forceinline__ int spmm_mfma_lds_bytes(int k, int waves, int rb) {
  const int kc = ((k + 15) & ~15) < kMfmaChunk ? ((k + 15) & ~15) : kMfmaChunk;
  const int panel = 32 * rb * (kc + kMfmaPad) * 2, sums = waves * rb * 128 * 64 * 4;
  return (panel > sums ? panel : sums) + (64 * rb + 1) * 4;
}

// WAVES tiles of 256 columns per workgroup, and KP waves per tile that split the steps of the
// contraction between them (more loads in flight per CU; their accumulators are added up
// through LDS at the end).  RB blocks of 32 rows per panel: with two, every fragment of B feeds
// two MFMAs and B is read from L2 half as often.
template <int WAVES, int KP, typename I = int, int RB = 1>
__global__ __launch_bounds__(64 * WAVES * KP) void spmm_mfma_kernel(
    int m, int k, int n, int tiles_n, const int* __restrict__ row_offsets,
    const I* __restrict__ column_indices, const _Float16* __restrict__ values,
    const _Float16* __restrict__ B, _Float16* __restrict__ C, const _Float16* __restrict__ bias, int relu) {
  extern __shared__ __attribute__((aligned(16))) char lds_raw[];
  constexpr int THREADS = 64 * WAVES * KP;
  const int kc_max = min((k + 15) & ~15, kMfmaChunk);
  const int stride = kc_max + kMfmaPad;                 // halves per panel row
  _Float16* panel = reinterpret_cast<_Float16*>(lds_raw);
  constexpr int PR = 32 * RB;                           // rows of the panel
  int* bad = reinterpret_cast<int*>(lds_raw + spmm_mfma_lds_bytes(k, WAVES, RB) - (2 * PR + 1) * 4);   // rows that cannot be expanded
  int* rowptr = bad + PR;                                           // the panel's PR + 1 row offsets

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = uniform(tid >> 6);
  const int tile_w = wave % WAVES;                      // which of the workgroup's tiles
  const int kpart = wave / WAVES;                       // which share of the steps
  const int c = lane & 31;
  const int h = lane >> 5;
  const int groups = (tiles_n + WAVES - 1) / WAVES;
  const int panel_id = blockIdx.x / groups;
  const int tile = (blockIdx.x - panel_id * groups) * WAVES + tile_w;
  const bool active = tile < tiles_n;                   // idle waves still take part in the barriers
  const int i0 = panel_id * PR;
  const int n0 = tile * 256;
  const int col = n0 + 8 * c;                           // this lane's eight output columns
  const bool col_ok = active && col < n;
  const _Float16* bp = B + (col_ok ? col : 0);

  if (tid < PR) bad[tid] = 0;
  if (tid < PR + 1) rowptr[tid] = row_offsets[min(i0 + tid, m)];

  f32x16 acc[RB][8];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int t = 0; t < 16; ++t) acc[rb][j][t] = 0.f;

  for (int kc0 = 0; kc0 < k; kc0 += kMfmaChunk) {
    const int kc = min(k - kc0, kMfmaChunk);
    const int all_steps = (kc + 15) >> 4;
    const int per_part = (all_steps + KP - 1) / KP;
    const int s_begin = min(all_steps, kpart * per_part);
    const int steps = min(all_steps, s_begin + per_part) - s_begin;      // this wave's steps: s_begin ..
    // second operand source: rows kc0 + 16*(s_begin + s) + 8h + r of B, r < 8: a scalar base that
    // moves with the step plus this lane's fixed byte offset (8h rows down, `col` columns in).
    // Steps that would reach past the last row of B take the slow form with clamped rows (the
    // panel holds zeros there).
    // (rows of B are kept as four 32-bit words each: the byte permutes work on those)
    constexpr int NS = RB == 1 ? kMfmaSets : 4;        // register sets: loads run NS-1 steps ahead
    u32x4 w[NS][8];
    const unsigned lane_off = (unsigned)((8 * h * n + (col_ok ? col : 0)) * 2);
    auto load_rows = [&](int s, u32x4 (&ws)[8]) {
      const int k0 = kc0 + 16 * (s_begin + s);
      if (k0 + 16 <= k) {
        const char* base = reinterpret_cast<const char*>(B + (size_t)k0 * n);
#pragma unroll
        for (int r = 0; r < 8; ++r)
          ws[r] = *reinterpret_cast<const u32x4*>(base + (size_t)r * n * 2 + lane_off);
      } else {
#pragma unroll
        for (int r = 0; r < 8; ++r)
          ws[r] = *reinterpret_cast<const u32x4*>(bp + (size_t)min(k0 + 8 * h + r, k - 1) * n);
      }
    };
    if (active) {
      // the first loads go out before the panel is built: they do not depend on it
#pragma unroll
      for (int u = 0; u < NS - 1; ++u)
        if (u < steps) load_rows(u, w[u]);
    }
    __syncthreads();                                     // the previous chunk's reads are done
    for (int o = tid * 16; o < PR * stride * 2; o += THREADS * 16)
      *reinterpret_cast<f32x4*>(lds_raw + o) = f32x4{0.f, 0.f, 0.f, 0.f};
    __syncthreads();
    // Expansion.  The panel's entries are one contiguous piece of the CSR arrays; the threads
    // take them round-robin, eight at a time (coalesced loads, all issued before the first
    // store), and each thread follows the row boundaries with a cursor into the 33 offsets.
    {
      constexpr int EB = 8;
      const int pbeg = rowptr[0], pend = rowptr[PR];
      int rr = 0;
      for (int base = pbeg + tid; base < pend; base += EB * THREADS) {
        int cidx[EB], prev[EB];
        _Float16 a[EB];
#pragma unroll
        for (int u = 0; u < EB; ++u) {
          const int p = min(base + u * THREADS, pend - 1);
          cidx[u] = (int)column_indices[p];
          prev[u] = (int)column_indices[max(p - 1, pbeg)];
          a[u] = values[p];
        }
#pragma unroll
        for (int u = 0; u < EB; ++u) {
          const int p = base + u * THREADS;
          if (p < pend) {
            while (rowptr[rr + 1] <= p) ++rr;              // rows in between are empty
            if (kc0 == 0 && p > rowptr[rr] && prev[u] >= cidx[u]) bad[rr] = 1;
            const unsigned rel = (unsigned)(cidx[u] - kc0);
            if (rel < (unsigned)kc) panel[rr * stride + rel] = a[u];
          }
        }
      }
    }
    __syncthreads();
    if (active) {
      // first operands: rows c, 32 + c, .. of the panel, columns 16*s + 8h .. +7 of the chunk
      const _Float16* ap = panel + c * stride + 8 * h + 16 * s_begin;
      auto step = [&](int s, const u32x4 (&ws)[8]) {
        f16x8 a[RB];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) a[rb] = *reinterpret_cast<const f16x8*>(ap + 32 * rb * stride + 16 * s);
        // 8x8 transpose of halves inside the lane: operand j, word q = (ws[2q][j], ws[2q+1][j])
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          u32x4 packed;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const unsigned sel = (j & 1) ? 0x07060302u : 0x05040100u;
            packed[q] = __builtin_amdgcn_perm(ws[2 * q + 1][j / 2], ws[2 * q][j / 2], sel);
          }
#pragma unroll
          for (int rb = 0; rb < RB; ++rb)
            acc[rb][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[rb], __builtin_bit_cast(f16x8, packed), acc[rb][j],
                                                                0, 0, 0);
        }
      };
      int s0 = 0;
      for (; s0 + NS <= steps; s0 += NS) {
#pragma unroll
        for (int u = 0; u < NS; ++u) {
          if (s0 + u + NS - 1 < steps) load_rows(s0 + u + NS - 1, w[(u + NS - 1) % NS]);
          step(s0 + u, w[u]);
        }
      }
#pragma unroll
      for (int u = 0; u < NS - 1; ++u)
        if (s0 + u < steps) step(s0 + u, w[u]);       // their loads are already under way
    }
  }
  // The k-parts' accumulators are added up through LDS (the panel is no longer needed), one
  // part at a time: element (rb, j, t) of lane l of tile w at float index
  // (((w*RB + rb)*8 + j)*16 + t)*64 + l.
  if constexpr (KP > 1) {
    float* sums = reinterpret_cast<float*>(lds_raw) + tile_w * (RB * 128 * 64) + lane;
    for (int q = 1; q < KP; ++q) {
      __syncthreads();
      if (kpart == q) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
          for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int t = 0; t < 16; ++t) sums[((rb * 8 + j) * 16 + t) * 64] = acc[rb][j][t];
      }
      __syncthreads();
      if (kpart == 0) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
          for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int t = 0; t < 16; ++t) acc[rb][j][t] += sums[((rb * 8 + j) * 16 + t) * 64];
      }
    }
  } else {
    __syncthreads();
  }
  if (!active || kpart != 0) return;

  // Register t of lane (c, h) in accumulator (rb, j) is row 32*rb + 8*(t/4) + 4h + t%4, column
  // n0 + 8c + j.
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int t = 0; t < 16; ++t) {
      const int rr = 32 * rb + 8 * (t / 4) + 4 * h + (t % 4);
      const int row = i0 + rr;
      if (row < m && col_ok && !bad[rr]) {
        float v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = acc[rb][j][t];
        spmm_epilogue<_Float16, 8>(v, bias, row, relu);
        Pack<_Float16, 8>::store(C + (size_t)row * n + col, v);
      }
    }
  // rows that could not be expanded: direct gathers, four columns per lane
  for (int rr = 0; rr < PR; ++rr) {
    if (!bad[rr]) continue;
    const int row = i0 + rr;
    const int col4 = n0 + 4 * lane;
    const bool ok = col4 < n;
    float v[4] = {0.f, 0.f, 0.f, 0.f};
    for (int p = row_offsets[row]; p < row_offsets[row + 1]; ++p) {
      const float a = (float)values[p];
      float b[4];
      Pack<_Float16, 4>::load(B + (size_t)(int)column_indices[p] * n + (ok ? col4 : 0), b);
#pragma unroll
      for (int j = 0; j < 4; ++j) v[j] = __builtin_fmaf(a, b[j], v[j]);
    }
    spmm_epilogue<_Float16, 4>(v, bias, row, relu);
    if (ok) Pack<_Float16, 4>::store(C + (size_t)row * n + col4, v);
  }
}

}  // namespace spdl
