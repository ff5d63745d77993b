// Softmax over the stored entries of every CSR row (paper Sec. "Application: Sparse
// Transformer": the softmax of the sparse attention scores), on logits multiplied by `scale`
// (1/sqrt(d_k) in attention).  One wave per row.  Rows of up to 1024 entries are read once and
// kept in registers; longer rows are read three times (maximum, sum, normalise).  8 bytes of
// HBM traffic per entry: the kernel is bandwidth-bound.  out may alias x.
#pragma once
#include "common.hpp"

namespace spdl {

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v = fmaxf(v, __shfl_xor(v, d, kWave));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, kWave);
  return v;
}

__global__ __launch_bounds__(256) void csr_softmax_kernel(int m, const int* __restrict__ row_offsets,
                                                          const float* x, float scale, float* out) {
  constexpr int kKeep = 16;                       // entries per lane kept in registers
  const int lane = threadIdx.x & 63;
  const int row = uniform(blockIdx.x * 4 + (threadIdx.x >> 6));
  if (row >= m) return;
  const int s = row_offsets[row];
  const int e = row_offsets[row + 1];
  const int len = e - s;
  if (len <= 0) return;
  const float ninf = -__builtin_inff();
  if (len <= kKeep * kWave) {
    const int nit = (len + kWave - 1) / kWave;
    float v[kKeep];
    float mx = ninf;
#pragma unroll
    for (int i = 0; i < kKeep; ++i) {
      v[i] = ninf;
      if (i < nit) {
        const int idx = s + i * kWave + lane;
        if (idx < e) v[i] = scale * x[idx];
        mx = fmaxf(mx, v[i]);
      }
    }
    mx = wave_max(mx);
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < kKeep; ++i)
      if (i < nit) {
        v[i] = expf(v[i] - mx);                  // exp(-inf) = 0 for the lanes past the row end
        sum += v[i];
      }
    const float inv = 1.f / wave_sum(sum);
#pragma unroll
    for (int i = 0; i < kKeep; ++i)
      if (i < nit) {
        const int idx = s + i * kWave + lane;
        if (idx < e) out[idx] = v[i] * inv;
      }
  } else {
    float mx = ninf;
    for (int idx = s + lane; idx < e; idx += kWave) mx = fmaxf(mx, scale * x[idx]);
    mx = wave_max(mx);
    float sum = 0.f;
    for (int idx = s + lane; idx < e; idx += kWave) sum += expf(scale * x[idx] - mx);
    const float inv = 1.f / wave_sum(sum);
    for (int idx = s + lane; idx < e; idx += kWave) out[idx] = expf(scale * x[idx] - mx) * inv;
  }
}

// out[t] = values[perm[t]]: moves the values of A into the order of A^T's entries (paper Sec.
// "Discussion & Conclusion": the transpose of the values as a cached permutation).
template <typename T>
__global__ __launch_bounds__(256) void permute_values_kernel(int nnz, const int* __restrict__ perm,
                                                             const T* __restrict__ values, T* __restrict__ out) {
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t < nnz) out[t] = values[perm[t]];
}

}  // namespace spdl
