// SDDMM with the right-hand operand not transposed (paper Sec. "Sampled Dense--Dense Matrix
// Multiplication Operation", footnote: the general form; with Rn of shape n x k the reads are
// coalesced without any work): out[p] = sum_j L[i,j] * Rn[j, c_p], optionally times values[p].
// One lane per stored entry (consecutive entries of a row have ascending columns, so for a
// fixed j the lanes of a wave read one row of Rn left to right); each lane finds its row with
// a binary search in the row offsets.  The plain fallback (two loads per multiply-add, any n,
// any alignment, fp32 and fp16): fp32 dot products of up to 128 columns with k % 4 == 0 go through
// the lane kernel's NT mode instead, which transposes slabs of Rn inside LDS.
#pragma once
#include "common.hpp"

namespace spdl {

template <typename T>
__global__ __launch_bounds__(256) void sddmm_nt_kernel(
    int m, int k, int n, int nnz, const int* __restrict__ row_offsets,
    const int* __restrict__ column_indices, const T* __restrict__ L, const T* __restrict__ Rn,
    T* __restrict__ out, const T* __restrict__ scale) {
  const int p = blockIdx.x * 256 + threadIdx.x;
  if (p >= nnz) return;
  int lo = 0, hi = m;                          // invariant: row_offsets[lo] <= p < row_offsets[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (row_offsets[mid] <= p) lo = mid; else hi = mid;
  }
  const T* l = L + (size_t)lo * n;
  const T* r = Rn + column_indices[p];
  float acc = 0.f;
  int j = 0;
  for (; j + 8 <= n; j += 8) {
    float a[8], b[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      a[u] = (float)l[j + u];
      b[u] = (float)r[(size_t)(j + u) * k];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) acc = __builtin_fmaf(a[u], b[u], acc);
  }
  for (; j < n; ++j) acc = __builtin_fmaf((float)l[j], (float)r[(size_t)j * k], acc);
  sddmm_store<T>(out, scale, p, acc);
}

}  // namespace spdl
