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
// The element offset in R of the row that lane l16 of a group gathers for the strip [q, q+16) of a
// sparse row ending at `end`: its own nonzero's column, past the end the last entry's again.
__device__ __forceinline__ int sddmm_strip_offset(int n, int q, int end, int l16,
                                                  const int* __restrict__ column_indices) {
  return column_indices[min(q + l16, end - 1)] * n;
}

template <typename T>
__device__ __forceinline__ void sddmm_strip_direct_at(int n, int q, int end, int l16, int roff,
                                                      const T* __restrict__ Lrow, const T* __restrict__ R,
                                                      T* __restrict__ out, const T* __restrict__ scale = nullptr) {
  const int cidx = q + l16;
  float partial[16];
#pragma unroll
  for (int t = 0; t < 16; ++t) partial[t] = 0.f;
  for (int col0 = 0; col0 < n; col0 += 64) {
    const int col = col0 + 4 * l16;
    const bool ok = col < n;
    const int colc = ok ? col : 0;
    const int lane_off = colc;
    // All sixteen gathers are issued before the first multiply-add (the scheduling barrier keeps
    // the compiler from interleaving them with the arithmetic, which it otherwise does whenever
    // the surrounding control flow changes, leaving two loads in flight instead of sixteen).
    float r[16][4];
#define SPDL_R1(T0) \
    Pack<T, 4>::load(R + (__builtin_amdgcn_update_dpp(0, roff, 0x150 + (T0), 0xf, 0xf, false) + lane_off), r[T0]);
    SPDL_R1(0) SPDL_R1(1) SPDL_R1(2) SPDL_R1(3) SPDL_R1(4) SPDL_R1(5) SPDL_R1(6) SPDL_R1(7)
    SPDL_R1(8) SPDL_R1(9) SPDL_R1(10) SPDL_R1(11) SPDL_R1(12) SPDL_R1(13) SPDL_R1(14) SPDL_R1(15)
#undef SPDL_R1
    float l[4];
    Pack<T, 4>::load(Lrow + colc, l);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int v = 0; v < 4; ++v) l[v] = ok ? l[v] : 0.f;
#pragma unroll
    for (int t = 0; t < 16; ++t)
#pragma unroll
      for (int v = 0; v < 4; ++v) partial[t] = __builtin_fmaf(l[v], r[t][v], partial[t]);
  }
  const float total = reduce16x16(partial, l16);
  if (cidx < end) sddmm_store<T>(out, scale, cidx, total);
}

template <typename T>
__device__ __forceinline__ void sddmm_strip_direct(int n, int q, int end, int l16, const T* __restrict__ Lrow,
                                                   const int* __restrict__ column_indices,
                                                   const T* __restrict__ R, T* __restrict__ out,
                                                   const T* __restrict__ scale = nullptr) {
  sddmm_strip_direct_at<T>(n, q, end, l16, sddmm_strip_offset(n, q, end, l16, column_indices), Lrow, R, out, scale);
}

// Work is split by nonzeros, not by rows: every wave owns `per_wave` consecutive entries of
// the CSR arrays (a multiple of 64), finds the row of its first entry with a binary search in
// the row offsets, and walks on from there.  The walk is wave-uniform (scalar loads and
// arithmetic): it cuts the range into strips of up to 16 entries that end at row ends and
// deals them to the four 16-lane groups, four at a time, so consecutive strips of one row
// share its L row in cache and short rows still keep all four groups busy.  Outputs are
// independent, so rows shared by several waves need no reduction, and the load per wave is
// the same whatever the row lengths are (the balance the paper gets for SpMM from the row
// swizzle, Sec. "Row Swizzle Load Balancing", without needing a row order in the interface).
template <typename T>
__global__ __launch_bounds__(256) void sddmm_group_kernel(
    int m, int n, int nnz, int per_wave, const int* __restrict__ row_offsets,
    const int* __restrict__ column_indices, const T* __restrict__ L, const T* __restrict__ R,
    T* __restrict__ out, const T* __restrict__ scale) {
  const int l16 = threadIdx.x & 15;
  const int sub = (threadIdx.x & 63) >> 4;
  const int wave = uniform(blockIdx.x * 4 + (threadIdx.x >> 6));
  const long long first = (long long)wave * per_wave;
  if (first >= nnz) return;
  int p = (int)first;
  const int range_end = (int)min((long long)nnz, first + per_wave);
  // Last row whose offset is <= p: the row of entry p (rows in between are empty).  A 64-way
  // search, one probe per lane: three rounds of dependent loads for up to 2^18 rows.
  const int lane = threadIdx.x & 63;
  int lo = 0, hi = m;                          // invariant: row_offsets[lo] <= p < row_offsets[hi]
  while (hi - lo > 1) {
    const int step = (hi - lo + 63) >> 6;
    const int probe = lo + (lane + 1) * step;
    const bool le = probe < hi && row_offsets[min(probe, hi)] <= p;     // true for a prefix of the lanes
    const int cnt = __builtin_popcountll(__builtin_amdgcn_ballot_w64(le));
    lo += cnt * step;
    hi = min(hi, lo + step);
  }
  int row = lo;
  int row_end = row_offsets[row + 1];
  // The walk runs one round ahead of the arithmetic: the column indices of the next round's strips
  // are requested before the current round's gathers are waited for, so a round costs one memory
  // latency (the rows of R), not two in a row (indices, then rows).
  int cur_row = 0, cur_q = 0, cur_end = 0, cur_off = 0;
  bool have = false;
  while (true) {
    int my_row = 0, my_q = 0, my_end = 0;
    const bool next = p < range_end;
    if (next) {
      while (row_end <= p) {                     // p reached the end of this row: next non-empty row
        ++row;
        row_end = row_offsets[row + 1];
      }
      const int seg_end = min(row_end, range_end);
      if (p + 64 <= seg_end) {                   // four full strips of the same row
        my_row = row;
        my_q = p + 16 * sub;
        my_end = seg_end;
        p += 64;
      } else {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          if (p < range_end) {
            while (row_end <= p) {
              ++row;
              row_end = row_offsets[row + 1];
            }
            const int e = min(row_end, range_end);
            if (sub == g) { my_row = row; my_q = p; my_end = e; }
            p = min(p + 16, e);
          }
        }
      }
    }
    int my_off = 0;
    if (my_q < my_end) my_off = sddmm_strip_offset(n, my_q, my_end, l16, column_indices);
    if (have && cur_q < cur_end)
      sddmm_strip_direct_at<T>(n, cur_q, cur_end, l16, cur_off, L + (size_t)cur_row * n, R, out, scale);
    if (!next) break;
    cur_row = my_row; cur_q = my_q; cur_end = my_end; cur_off = my_off;
    have = true;
  }
}

}  // namespace spdl
