// SDDMM, row-strip family: one wave owns strips of 32 consecutive nonzeros of one sparse row
// (paper Sec. "Sampled Dense--Dense Matrix Multiplication", 1-D tiling over nonzero strips).
// The 64 lanes split the dot-product dimension so that rows of L and R are read contiguously;
// each lane keeps a partial sum for every nonzero of the strip and a transposing butterfly
// over the lanes finishes the sums (same section, reduction with shuffles).
// `split` waves share a row, taking strips round-robin, so the grid is m*split waves and no
// wave is launched for strips that cannot exist.
#pragma once
#include "common.hpp"

namespace spdl {

constexpr int kStrip = 32;

// Lane l ends with the sum over all 64 lanes of element e(l) = bit-reversal of (l & 31).
__device__ __forceinline__ float strip_reduce32(float (&v)[kStrip], int lane) {
#pragma unroll
  for (int b = 0; b < 5; ++b) {
    const int h = (kStrip >> b) / 2;
    const int mask = 1 << b;
    const bool up = (lane & mask) != 0;
#pragma unroll
    for (int i = 0; i < h; ++i) {
      const float send = up ? v[i] : v[i + h];
      const float keep = up ? v[i + h] : v[i];
      v[i] = keep + __shfl_xor(send, mask, kWave);
    }
  }
  return v[0] + __shfl_xor(v[0], 32, kWave);
}

template <typename T, int VEC>
__global__ __launch_bounds__(256) void sddmm_rowstrip_kernel(
    int m, int n, int split, const int* __restrict__ row_offsets,
    const int* __restrict__ column_indices, const T* __restrict__ L, const T* __restrict__ R,
    T* __restrict__ out, const T* __restrict__ scale) {
  const int lane = threadIdx.x % kWave;
  const int wave = uniform(blockIdx.x * 4 + threadIdx.x / kWave);
  const int row = wave / split;
  const int part = wave - row * split;
  if (row >= m) return;
  const int start = row_offsets[row];
  const int end = row_offsets[row + 1];
  const T* Lrow = L + (size_t)row * n;
  const int e = (int)(__builtin_bitreverse32((unsigned)lane) >> 27);   // element this lane ends with

  for (int s = start + part * kStrip; s < end; s += split * kStrip) {
    const int last = end - 1;
    float partial[kStrip];
#pragma unroll
    for (int t = 0; t < kStrip; ++t) partial[t] = 0.f;

    for (int j0 = 0; j0 < n; j0 += kWave * VEC) {
      const int j = j0 + lane * VEC;
      const bool active = j < n;
      const int jj = active ? j : 0;
      float l[VEC];
      Pack<T, VEC>::load(Lrow + jj, l);
      if (!active) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) l[v] = 0.f;
      }
#pragma unroll
      for (int t0 = 0; t0 < kStrip; t0 += 8) {
        float r[8][VEC];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          // positions past the row's end re-read its last entry; their sums are never stored
          const int q = s + t0 + u;
          const int c = column_indices[q < last ? q : last];
          Pack<T, VEC>::load(R + (size_t)c * n + jj, r[u]);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
          for (int v = 0; v < VEC; ++v)
            partial[t0 + u] = __builtin_fmaf(l[v], r[u][v], partial[t0 + u]);
      }
    }
    const float total = strip_reduce32(partial, lane);
    if (lane < kStrip && s + e < end) sddmm_store<T>(out, scale, s + e, total);
  }
}

}  // namespace spdl
