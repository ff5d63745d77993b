// SDDMM, group family: a 16-lane group owns 16 consecutive nonzeros of one sparse row (a
// strip, paper Sec. "Sampled Dense--Dense Matrix Multiplication": 1-D tiling over strips of
// consecutive nonzeros).  The lanes split the dot-product dimension four columns at a time,
// so rows of L and R are read contiguously; every lane keeps one partial sum per nonzero of
// the strip, and a transposing reduction over the 16 lanes leaves nonzero t's dot product in
// lane t, which stores it (same section: partial results for all outputs of the tile, then a
// reduction with shuffles).  Column indices are loaded once per strip, pre-scaled to row
// offsets of R, and handed out by DPP row broadcasts.
// Needs n % 4 == 0, 16-byte aligned L and R (8-byte for fp16) and k*n < 2^31.
#pragma once
#include "common.hpp"

namespace spdl {

// x[t] holds this lane's partial sum for nonzero t (16 lanes, 16 nonzeros).  Returns the
// complete sum of nonzero (lane & 15).  row_ror:n hands lane l the value of lane l-n (mod 16).
// Row rotations with bank masks do the first
// two halvings in two instructions per surviving value; the last two use quad permutes.
__device__ __forceinline__ float reduce16x16(float (&x)[16], int l16) {
#define SPDL_ROR(DST, SRC, ROT, BANKS)                                                         \
  asm volatile("s_nop 1\n\tv_add_f32_dpp %0, %1, %1 row_ror:" #ROT " row_mask:0xf bank_mask:" #BANKS \
               : "+v"(DST) : "v"(SRC));
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    SPDL_ROR(x[t], x[t], 8, 0x3)          // lanes 0-7:  x[t]   += x[t]   from lane+8
    SPDL_ROR(x[t], x[t + 8], 8, 0xc)      // lanes 8-15: x[t+8] += x[t+8] from lane-8, kept in x[t]
  }
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    SPDL_ROR(x[t], x[t], 12, 0x5)         // lanes with bit 2 clear: += lane+4 (rotate right by 12)
    SPDL_ROR(x[t], x[t + 4], 4, 0xa)      // lanes with bit 2 set:   x[t+4] += lane-4, kept in x[t]
  }
#undef SPDL_ROR
  const bool b1 = (l16 & 2) != 0;
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const float keep = b1 ? x[t + 2] : x[t];
    const float send = b1 ? x[t] : x[t + 2];
    x[t] = keep + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(
                      0, __builtin_bit_cast(int, send), 0x4e /* quad_perm [2,3,0,1] */, 0xf, 0xf, false));
  }
  const bool b0 = (l16 & 1) != 0;
  const float keep = b0 ? x[1] : x[0];
  const float send = b0 ? x[0] : x[1];
  return keep + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(
                    0, __builtin_bit_cast(int, send), 0xb1 /* quad_perm [1,0,3,2] */, 0xf, 0xf, false));
}

// Dot products of one strip of up to 16 consecutive nonzeros [q, q+16) ∩ [q, end) of `row`,
// rows of L and R gathered straight from global memory.  Called by all 16 lanes of a group.
template <typename T>
__device__ __forceinline__ void sddmm_strip_direct(int n, int q, int end, int l16, const T* __restrict__ Lrow,
                                                   const int* __restrict__ column_indices,
                                                   const T* __restrict__ R, T* __restrict__ out) {
  const int cidx = q + l16;
  const int roff = column_indices[min(cidx, end - 1)] * n;     // past the end: last entry again
  float partial[16];
#pragma unroll
  for (int t = 0; t < 16; ++t) partial[t] = 0.f;
  for (int col0 = 0; col0 < n; col0 += 64) {
    const int col = col0 + 4 * l16;
    const bool ok = col < n;
    const int colc = ok ? col : 0;
    float l[4];
    Pack<T, 4>::load(Lrow + colc, l);
    if (!ok) l[0] = l[1] = l[2] = l[3] = 0.f;
    const int lane_off = colc;
#define SPDL_R4(T0)                                                                             \
  {                                                                                             \
    float r[4][4];                                                                              \
    Pack<T, 4>::load(R + (__builtin_amdgcn_update_dpp(0, roff, 0x150 + (T0), 0xf, 0xf, false) + lane_off), r[0]);     \
    Pack<T, 4>::load(R + (__builtin_amdgcn_update_dpp(0, roff, 0x150 + (T0) + 1, 0xf, 0xf, false) + lane_off), r[1]); \
    Pack<T, 4>::load(R + (__builtin_amdgcn_update_dpp(0, roff, 0x150 + (T0) + 2, 0xf, 0xf, false) + lane_off), r[2]); \
    Pack<T, 4>::load(R + (__builtin_amdgcn_update_dpp(0, roff, 0x150 + (T0) + 3, 0xf, 0xf, false) + lane_off), r[3]); \
    _Pragma("unroll") for (int u = 0; u < 4; ++u)                                               \
      _Pragma("unroll") for (int v = 0; v < 4; ++v)                                             \
        partial[(T0) + u] = __builtin_fmaf(l[v], r[u][v], partial[(T0) + u]);                   \
  }
    SPDL_R4(0) SPDL_R4(4) SPDL_R4(8) SPDL_R4(12)
#undef SPDL_R4
  }
  const float total = reduce16x16(partial, l16);
  if (cidx < end) out[cidx] = (T)total;
}

template <typename T>
__global__ __launch_bounds__(256) void sddmm_group_kernel(
    int m, int n, int split, const int* __restrict__ row_offsets,
    const int* __restrict__ column_indices, const T* __restrict__ L, const T* __restrict__ R,
    T* __restrict__ out) {
  const int lane = threadIdx.x & 63;
  const int sub = lane >> 4;
  const int l16 = lane & 15;
  const int wave = uniform(blockIdx.x * 4 + (threadIdx.x >> 6));
  const int row = wave / split;
  const int part = wave - row * split;
  if (row >= m) return;
  const int start = row_offsets[row];
  const int end = row_offsets[row + 1];
  const T* Lrow = L + (size_t)row * n;
  // the four groups of a wave take strips part*4+sub, then every split*4-th one
  for (int q0 = start + part * 64; q0 < end; q0 += split * 64)
    sddmm_strip_direct<T>(n, q0 + sub * 16, end, l16, Lrow, column_indices, R, out);
}

}  // namespace spdl
