// SDDMM in mixed precision on the matrix cores (paper Sec. "Mixed Precision": fp16 operands,
// fp32 accumulation).  On this chip the dense fp16 matrix rate is some thirty times the fp32
// vector rate, so for the moderately sparse matrices of deep learning it is cheaper to compute
// a whole 32x32 block of L R^T with MFMA and keep only the entries A stores there than to
// gather one row of R per stored entry.  The contraction runs over n, which is the contiguous
// dimension of both row-major operands, so every lane loads its operand fragments straight
// from global memory, 16 bytes at a time; nothing is staged.
//
// A workgroup owns one 64x64 block of A's index space.  Which stored entries fall into the
// block: for each of its 64 rows a binary search gives the first entry with column >= c0 and
// the first with column >= c0 + 64.  Whatever the column order inside a row, the ranges of
// consecutive blocks cover the row (the first block starts at the row start, the last ends at
// the row end), and every entry of a range is produced by the wave that owns the range: from
// the block if its column lies inside it, else (rows that are not ascending) by a plain dot
// product.  Dense work is the same for every block, so row lengths do not unbalance anything.
//
// Needs n % 8 == 0 and 16-byte aligned L and R.
#pragma once
#include "common.hpp"

namespace spdl {

typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ f16x8 load_h8(const _Float16* p) { return *reinterpret_cast<const f16x8*>(p); }

// Dot product of two rows of length n by one lane (entries whose column lies outside the block
// that owns their range; only rows that are not ascending have them).
__device__ __attribute__((noinline)) float sddmm_lane_dot(const _Float16* __restrict__ l,
                                                          const _Float16* __restrict__ r, int n) {
  float acc = 0.f;
  for (int j = 0; j < n; j += 8) {
    const f16x8 a = load_h8(l + j), b = load_h8(r + j);
#pragma unroll
    for (int t = 0; t < 8; ++t) acc = __builtin_fmaf((float)a[t], (float)b[t], acc);
  }
  return acc;
}

constexpr int kSddmmMfmaLdsBytes = 4 * 64 * 65 * 4 + 2 * 64 * 4;

// One workgroup (four waves) owns one 64x64 block of A's index space.  Each wave computes the
// whole block, as 2x2 MFMA tiles, over a quarter of the contraction (four operand loads feed four
// MFMAs: half the traffic per multiply of a 32x32 block, and four times the loads in flight
// of one wave per block); the four partial blocks are laid side by side in LDS and added, in a
// fixed order, only at the positions A stores.
__global__ __launch_bounds__(256) void sddmm_mfma_kernel(
    int m, int k, int n, int tiles_k, const int* __restrict__ row_offsets,
    const int* __restrict__ column_indices, const _Float16* __restrict__ L, const _Float16* __restrict__ R,
    _Float16* __restrict__ out, const _Float16* __restrict__ scale) {
  extern __shared__ __attribute__((aligned(16))) char lds_raw[];
  float (*part)[64][65] = reinterpret_cast<float (*)[64][65]>(lds_raw);          // [wave][row][column]
  int (*bound)[64] = reinterpret_cast<int (*)[64]>(lds_raw + 4 * 64 * 65 * 4);   // [0]: range start, [1]: end
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = uniform(tid >> 6);
  const int r = lane & 31;
  const int half = lane >> 5;
  const int tile_i = blockIdx.x / tiles_k;
  const int tile_c = blockIdx.x - tile_i * tiles_k;
  const int i0 = tile_i * 64;
  const int c0 = tile_c * 64;

  // Range of row i0 + t%64 that this block owns: threads 0..63 search for c0, 64..127 for c0 + 64.
  if (tid < 128) {
    const int row = i0 + (tid & 63);
    const int which = tid >> 6;
    int rs = 0, re = 0;
    if (row < m) {
      rs = row_offsets[row];
      re = row_offsets[row + 1];
    }
    int lo = rs, hi = re;
    const int key = c0 + 64 * which;
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (column_indices[mid] < key) lo = mid + 1; else hi = mid;
    }
    if (which == 0 && tile_c == 0) lo = rs;
    if (which == 1 && tile_c == tiles_k - 1) lo = re;
    bound[which][tid & 63] = lo;
  }

  // Partial block of L R^T over this wave's share of the 16-column steps.  Lane (r, half) holds
  // columns 8*half .. 8*half+7 of a step, of rows i0+r and i0+32+r of L (first operands) and
  // rows c0+r and c0+32+r of R (second operands); rows past the end of either matrix are clamped,
  // their results are never looked at.
  const int steps_all = (n + 15) >> 4;
  const int per_wave = (steps_all + 3) >> 2;
  const int s_begin = min(steps_all, wave * per_wave);
  const int s_end = min(steps_all, s_begin + per_wave);
  const int full_end = min(s_end, n >> 4);             // steps before this are complete for both halves
  const _Float16* lp[2];
  const _Float16* rp[2];
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    lp[b] = L + (size_t)min(i0 + 32 * b + r, m - 1) * n + 8 * half;
    rp[b] = R + (size_t)min(c0 + 32 * b + r, k - 1) * n + 8 * half;
  }
  f32x16 acc[2][2];
#pragma unroll
  for (int bi = 0; bi < 2; ++bi)
#pragma unroll
    for (int bc = 0; bc < 2; ++bc)
#pragma unroll
      for (int t = 0; t < 16; ++t) acc[bi][bc][t] = 0.f;

  constexpr int U = 4;                                  // steps per register set
  f16x8 a0[U][2], b0v[U][2], a1[U][2], b1v[U][2];
  auto load_set = [&](int s, f16x8 (&a)[U][2], f16x8 (&b)[U][2]) {
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        a[u][q] = load_h8(lp[q] + (s + u) * 16);
        b[u][q] = load_h8(rp[q] + (s + u) * 16);
      }
  };
  auto mma_set = [&](const f16x8 (&a)[U][2], const f16x8 (&b)[U][2]) {
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int bi = 0; bi < 2; ++bi)
#pragma unroll
        for (int bc = 0; bc < 2; ++bc)
          acc[bi][bc] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[u][bi], b[u][bc], acc[bi][bc], 0, 0, 0);
  };
  // two register sets: the loads of one are in flight while the other is multiplied
  int s = s_begin;
  if (s + U <= full_end) load_set(s, a0, b0v);
  for (; s + 2 * U <= full_end; s += 2 * U) {
    load_set(s + U, a1, b1v);
    mma_set(a0, b0v);
    if (s + 3 * U <= full_end) load_set(s + 2 * U, a0, b0v);
    mma_set(a1, b1v);
  }
  if (s + U <= full_end) {
    mma_set(a0, b0v);
    s += U;
  }
  // the remaining steps one at a time, the very last one possibly half empty (n % 16 == 8)
  for (; s < s_end; ++s) {
    const bool in = 16 * s + 8 * half < n;
    // (the pointers already point 8*half columns into the row: step back for the lanes past the end)
    const int o = in ? 16 * s : -8 * half;
    f16x8 a[2], b[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      a[q] = load_h8(lp[q] + o);
      b[q] = load_h8(rp[q] + o);
      if (!in) {
#pragma unroll
        for (int t = 0; t < 8; ++t) a[q][t] = b[q][t] = (_Float16)0.f;
      }
    }
#pragma unroll
    for (int bi = 0; bi < 2; ++bi)
#pragma unroll
      for (int bc = 0; bc < 2; ++bc)
        acc[bi][bc] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[bi], b[bc], acc[bi][bc], 0, 0, 0);
  }

  // Register t of lane (c, half) in tile (bi, bc) is element (32*bi + 8*(t/4) + 4*half + t%4, 32*bc + c).
#pragma unroll
  for (int bi = 0; bi < 2; ++bi)
#pragma unroll
    for (int bc = 0; bc < 2; ++bc)
#pragma unroll
      for (int t = 0; t < 16; ++t)
        part[wave][32 * bi + 8 * (t / 4) + 4 * half + (t % 4)][32 * bc + r] = acc[bi][bc][t];
  __syncthreads();

  // Four threads per row take alternate entries of its range.
  const int rr = tid >> 2;
  const int row = i0 + rr;
  const int b0 = bound[0][rr];
  const int b1 = max(b0, bound[1][rr]);
  for (int p = b0 + (tid & 3); p < b1; p += 4) {
    const int c = column_indices[p];
    const unsigned cc = (unsigned)(c - c0);
    float v;
    if (cc < 64u) v = ((part[0][rr][cc] + part[1][rr][cc]) + part[2][rr][cc]) + part[3][rr][cc];
    else v = sddmm_lane_dot(L + (size_t)row * n, R + (size_t)c * n, n);
    sddmm_store<_Float16>(out, scale, p, v);
  }
}

}  // namespace spdl
