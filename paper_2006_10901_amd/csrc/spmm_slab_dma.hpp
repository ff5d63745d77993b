// SpMM, slab family with asynchronous global->LDS copies: same decomposition as the
// producer/consumer slab kernel (64 sparse rows x 64-column tiles per workgroup, B streamed
// through LDS in slabs of S rows, 16-lane groups with DPP-broadcast multiply-adds), but all
// 16 waves compute, one sparse row per 16-lane group, and each wave moves its share of the
// next slab with direct-to-LDS loads (no staging registers, no LDS store instructions).
// Vector-memory loads retire in order, so the first wait for sparse elements inside a stage
// also waits for that wave's four slab loads; they were issued at the start of the stage and
// have had a round of arithmetic to complete.
#pragma once
#include "common.hpp"
#include "spmm_slab.hpp"

namespace spdl {

template <int S>
__global__ __launch_bounds__(kSlabThreads) void spmm_slab_dma_kernel(
    int m, int k, int n, int nnz, int tiles_n, int tiles_per_wg, int panels,
    const int* __restrict__ row_offsets, const int* __restrict__ column_indices,
    const float* __restrict__ values, const int* __restrict__ row_order, const float* __restrict__ B,
    float* __restrict__ C) {
  using T = float;
  extern __shared__ __attribute__((aligned(16))) char lds_raw[];
  constexpr int kBufBytes = (S + 1) * kSlabTile * 4;      // S data rows + one all-zero row
  constexpr int kZeroOff = S * kSlabTile * 4;
  constexpr int kCopies = S / 64;                         // 1 KB direct-to-LDS loads per wave per slab

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int sub = lane >> 4;
  const int l16 = lane & 15;
  const int lane_b = l16 * 16;

  const int groups_n = (tiles_n + tiles_per_wg - 1) / tiles_per_wg;
  const int per_block = 8 * groups_n;
  const int blk = blockIdx.x / per_block;
  const int rem = blockIdx.x - blk * per_block;
  const int panel = blk * 8 + (rem & 7);
  if (panel >= panels) return;
  const int tile_begin = (rem >> 3) * tiles_per_wg;
  const int tile_end = min(tiles_n, tile_begin + tiles_per_wg);
  const int nslabs = (k + S - 1) / S;
  const int stages = (tile_end - tile_begin) * nslabs;

  if (tid < 2 * kSlabTile)
    *reinterpret_cast<float*>(lds_raw + (tid >> 6) * kBufBytes + kZeroOff + (tid & 63) * 4) = 0.f;

  // Slab copy: copy i of wave w fills slab rows (i*16 + w)*4 .. +3; lane L brings row L/16 of
  // those, columns 4*(L%16) .. +3, and the hardware places lane L's 16 bytes at base + 16*L.
  // Rows past k and columns past n are clamped into B: nothing valid ever reads them.
  auto copy_stage = [&](int q) {
    const int tile = tile_begin + q / nslabs;
    const int slab = q - (q / nslabs) * nslabs;
    const int colg = tile * kSlabTile + l16 * 4;
    const float* src = B + (colg < n ? colg : 0);
    char* dst = lds_raw + (q & 1) * kBufBytes;
#pragma unroll
    for (int i = 0; i < kCopies; ++i) {
      const int lrow = (i * 16 + wave) * 4;
      const int r = min(slab * S + lrow + sub, k - 1);
      __builtin_amdgcn_global_load_lds(src + (size_t)r * n,
                                       (__attribute__((address_space(3))) void*)(dst + lrow * (kSlabTile * 4)),
                                       16, 0, 0);
    }
  };

  SlabRow row;
  {
    const int slot = panel * kSlabRows + wave * 4 + sub;
    row.row = -1;
    row.p_begin = row.row_end = 0;
    if (slot < m) {
      const int r = row_order ? row_order[slot] : slot;
      row.row = r;
      row.p_begin = row_offsets[r];
      row.row_end = row_offsets[r + 1];
    }
  }
  float acc[4];

  copy_stage(0);
  __builtin_amdgcn_s_waitcnt(0);     // vmcnt(0): this wave's copies have landed in LDS
  __syncthreads();
  int q = 0;
  for (int tile = tile_begin; tile < tile_end; ++tile) {
    const int col = tile * kSlabTile + l16 * 4;
    const bool col_ok = col < n;
    row.p = row.p_begin;
    acc[0] = acc[1] = acc[2] = acc[3] = 0.f;
    slab_fetch<T>(row, l16, nnz - 1, column_indices, values);
    for (int s = 0; s < nslabs; ++s, ++q) {
      if (q + 1 < stages) copy_stage(q + 1);
      const char* buf = lds_raw + (q & 1) * kBufBytes;
      slab_consume<T, S>(row, acc, buf, s * S, sub, l16, lane_b, nnz - 1, column_indices, values);
      __builtin_amdgcn_s_waitcnt(0);
      __syncthreads();
    }
    if (row.p != row.row_end) {
      acc[0] = acc[1] = acc[2] = acc[3] = 0.f;
      const T* Bcol = B + (col_ok ? col : 0);
      for (int t = row.p_begin; t < row.row_end; ++t) {
        const float a = (float)values[t];
        float b[4];
        Pack<T, 4>::load(Bcol + (size_t)column_indices[t] * n, b);
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[v] = __builtin_fmaf(a, b[v], acc[v]);
      }
    }
    if (row.row >= 0 && col_ok) Pack<T, 4>::store(C + (size_t)row.row * n + col, acc);
  }
}

}  // namespace spdl
