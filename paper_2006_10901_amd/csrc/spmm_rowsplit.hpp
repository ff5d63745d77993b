// SpMM, row-splitting family: a group of G lanes owns one sparse row and a 1-D tile of
// G*VEC output columns (paper Sec. "Hierarchical 1-Dimensional Tiling" and "Subwarp Tiling").
// Dense rows of B are gathered straight from global memory, one vector load per lane per
// nonzero.  This is the general kernel: any n, any alignment, any column order inside a row.
#pragma once
#include "common.hpp"

namespace spdl {

// I is the type of the column indices (int32, or int16 in the mixed-precision form of paper Sec.
// "Mixed Precision", which halves the index traffic).
// SEG lane groups of one wave share a row: group s takes the batches s, s+SEG, ... of the row's
// nonzeros and the partial sums are added across the groups at the end.  Used when there are too
// few rows to fill the machine with one group per row (each lane then walks a shorter list).
template <typename T, int VEC, int G, typename I = int, int SEG = 1>
__global__ __launch_bounds__(256) void spmm_rowsplit_kernel(
    int m, int n, const int* __restrict__ row_offsets,
    const I* __restrict__ column_indices, const T* __restrict__ values, const int* __restrict__ row_order,
    const T* __restrict__ B, T* __restrict__ C, const T* __restrict__ bias, int relu) {
  static_assert(G * SEG <= kWave, "the groups that share a row sit in one wave");
  constexpr int U = (G == kWave && VEC * sizeof(T) <= 16) ? 16 : 8;   // nonzeros in flight per lane
  const int sub = threadIdx.x / G;
  const int lane = threadIdx.x % G;
  // Row binning and bundling (paper Sec. "Row Swizzle Load Balancing"): the rows of one wave
  // are adjacent in the row order (a bundle of similar lengths, so the lanes of a wave finish
  // together), while the four waves of a block take bundles a quarter of the order apart, so
  // every block, and with it every CU, gets the same mix of long and short rows.
  constexpr int RPW = kWave / (G * SEG);               // rows per wave
  const int wave_in_block = threadIdx.x / kWave;
  const int seg = sub % SEG;
  const int slot = (wave_in_block * (int)gridDim.x + (int)blockIdx.x) * RPW + (sub / SEG) % RPW;
  if (slot >= m) return;
  int row = row_order ? row_order[slot] : slot;          // row swizzle: one extra load
  if (G * SEG == kWave) row = uniform(row);              // whole wave on one row: scalar loads
  const int col = (blockIdx.y * G + lane) * VEC;
  const bool active = col < n;
  const int start = row_offsets[row];
  const int end = row_offsets[row + 1];
  const T* Bcol = B + (active ? col : 0);

  float acc[VEC];
#pragma unroll
  for (int v = 0; v < VEC; ++v) acc[v] = 0.f;

  int p = start + seg * U;
  // Full batches of U nonzeros.  The values and column indices of the next batch are requested
  // before the gathers of the current one are waited for, so a batch costs one memory latency
  // (the rows of B), not two in a row (indices, then rows).
  float a[U];
  int c[U];
  if (p + U <= end) {
#pragma unroll
    for (int u = 0; u < U; ++u) { a[u] = (float)values[p + u]; c[u] = (int)column_indices[p + u]; }
  }
  for (; p + U <= end; p += SEG * U) {
    float b[U][VEC];
#pragma unroll
    for (int u = 0; u < U; ++u) Pack<T, VEC>::load(Bcol + (size_t)c[u] * n, b[u]);
    float an[U];
    int cn[U];
    const int pn = p + SEG * U;
    if (pn + U <= end) {
#pragma unroll
      for (int u = 0; u < U; ++u) { an[u] = (float)values[pn + u]; cn[u] = (int)column_indices[pn + u]; }
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int v = 0; v < VEC; ++v) acc[v] = __builtin_fmaf(a[u], b[u][v], acc[v]);
#pragma unroll
    for (int u = 0; u < U; ++u) { a[u] = an[u]; c[u] = cn[u]; }
  }
  // after the full batches, p is the start of this group's next batch: past the row end for every
  // group but the one that owns the short last batch
  for (; p < end; ++p) {
    const float a = (float)values[p];
    float b[VEC];
    Pack<T, VEC>::load(Bcol + (size_t)(int)column_indices[p] * n, b);
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = __builtin_fmaf(a, b[v], acc[v]);
  }
  if (SEG > 1) {
#pragma unroll
    for (int d = G; d < G * SEG; d *= 2)
#pragma unroll
      for (int v = 0; v < VEC; ++v) acc[v] += __shfl_xor(acc[v], d, kWave);
    if (seg != 0) return;
  }
  spmm_epilogue<T, VEC>(acc, bias, row, relu);
  if (active) Pack<T, VEC>::store(C + (size_t)row * n + col, acc);
}

}  // namespace spdl
