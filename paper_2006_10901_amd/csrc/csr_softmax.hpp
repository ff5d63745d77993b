// Softmax over the stored entries of every CSR row (paper Sec. "Application: Sparse
// Transformer": the softmax of the sparse attention scores), on logits multiplied by `scale`
// (1/sqrt(d_k) in attention).  One wave per row.  Rows of up to 1024 entries are read once and
// kept in registers; longer rows are read three times (maximum, sum, normalise).  8 bytes of
// HBM traffic per entry: the kernel is bandwidth-bound.  out may alias x.
#pragma once
#include "common.hpp"

namespace spdl {

// Wave-wide reductions whose result is in every lane: four row rotations (DPP) leave each
// 16-lane row's result in all of its lanes, the four rows are then combined through scalar
// registers.
#define SPDL_ROR_F32(V, N) \
  __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, V), 0x120 + (N), 0xf, 0xf, false))
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, SPDL_ROR_F32(v, 8));
  v = fmaxf(v, SPDL_ROR_F32(v, 4));
  v = fmaxf(v, SPDL_ROR_F32(v, 2));
  v = fmaxf(v, SPDL_ROR_F32(v, 1));
  const float a = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 0));
  const float b = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 16));
  const float c = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 32));
  const float d = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 48));
  return fmaxf(fmaxf(a, b), fmaxf(c, d));
}
__device__ __forceinline__ float wave_sum(float v) {
  v += SPDL_ROR_F32(v, 8);
  v += SPDL_ROR_F32(v, 4);
  v += SPDL_ROR_F32(v, 2);
  v += SPDL_ROR_F32(v, 1);
  const float a = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 0));
  const float b = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 16));
  const float c = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 32));
  const float d = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 48));
  return (a + b) + (c + d);
}
#undef SPDL_ROR_F32

// A row of up to 64*NIT entries, read once and kept in registers (NIT per lane).  All loads are
// issued before anything is done with them: positions past the row end re-read its last entry
// and count as -infinity.
template <int NIT>
__device__ __forceinline__ void softmax_row_in_registers(int s, int e, int lane, const float* x, float scale,
                                                         float* out) {
  const float ninf = -__builtin_inff();
  float v[NIT];
#pragma unroll
  for (int i = 0; i < NIT; ++i) v[i] = x[min(s + i * kWave + lane, e - 1)];
  float mx = ninf;
#pragma unroll
  for (int i = 0; i < NIT; ++i) {
    v[i] = (s + i * kWave + lane < e) ? scale * v[i] : ninf;
    mx = fmaxf(mx, v[i]);
  }
  mx = wave_max(mx);
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < NIT; ++i) {
    v[i] = expf(v[i] - mx);                    // exp(-inf) = 0 for the positions past the row end
    sum += v[i];
  }
  const float inv = 1.f / wave_sum(sum);
#pragma unroll
  for (int i = 0; i < NIT; ++i) {
    const int idx = s + i * kWave + lane;
    if (idx < e) out[idx] = v[i] * inv;
  }
}

__global__ __launch_bounds__(256) void csr_softmax_kernel(int m, const int* __restrict__ row_offsets,
                                                          const float* x, float scale, float* out) {
  const int lane = threadIdx.x & 63;
  const int row = uniform(blockIdx.x * 4 + (threadIdx.x >> 6));
  if (row >= m) return;
  const int s = row_offsets[row];
  const int e = row_offsets[row + 1];
  const int len = e - s;
  if (len <= 0) return;
  if (len <= 1 * kWave) softmax_row_in_registers<1>(s, e, lane, x, scale, out);
  else if (len <= 2 * kWave) softmax_row_in_registers<2>(s, e, lane, x, scale, out);
  else if (len <= 4 * kWave) softmax_row_in_registers<4>(s, e, lane, x, scale, out);
  else if (len <= 8 * kWave) softmax_row_in_registers<8>(s, e, lane, x, scale, out);
  else if (len <= 16 * kWave) softmax_row_in_registers<16>(s, e, lane, x, scale, out);
  else {
    const float ninf = -__builtin_inff();
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
