// SpMM, slab family: a workgroup of 16 waves owns 64 sparse rows and a 64-column tile of C.
// B is streamed through LDS in slabs of S consecutive rows (double buffered), so every B
// element is fetched from global memory once per workgroup and then re-read from LDS by each
// sparse row that has a nonzero in that column: reuse of B across rows, which the paper names
// as the way past its shared-memory bandwidth limit (Sec. "Discussion & Conclusion").
//
// Inside a wave each 16-lane group owns one sparse row (paper Sec. "Subwarp Tiling": four
// rows per wave, bundled by length through the row order).  A group fetches 16 consecutive
// (value, column) pairs of its row with one load each, and the pairs are handed to the
// group's lanes one at a time by DPP row broadcasts inside the multiply-add itself.  The
// column index is pre-scaled to an LDS byte offset once per pair (Sec. "Index Pre-Scaling").
//
// Requires ascending column indices inside a row for the slab walk; a row that is not in
// ascending order is noticed (its cursor does not reach the row end) and redone by direct
// gathers, so results are always right.  Needs n % 4 == 0 and 16-byte aligned B and C.
#pragma once
#include "common.hpp"

namespace spdl {

constexpr int kSlabTile = 64;        // output columns per workgroup
constexpr int kSlabRows = 64;        // sparse rows per workgroup
constexpr int kSlabThreads = 1024;

// Four consecutive pairs of every 16-lane group: four LDS addresses and 128-bit LDS reads,
// then sixteen multiply-adds whose first operand is lane T of the group (DPP row_newbcast).
// PRE is "s_nop 1" on the first use after `av` was written by a VALU instruction: a DPP read
// needs two wait states after a VALU write and the compiler cannot see inside the asm.
#define SPDL_DPP_FMA4(T, BV, PRE)                                                              \
  asm volatile(PRE                                                                             \
               "v_fmac_f32_dpp %0, %4, %5 row_newbcast:" #T " row_mask:0xf bank_mask:0xf\n\t"  \
               "v_fmac_f32_dpp %1, %4, %6 row_newbcast:" #T " row_mask:0xf bank_mask:0xf\n\t"  \
               "v_fmac_f32_dpp %2, %4, %7 row_newbcast:" #T " row_mask:0xf bank_mask:0xf\n\t"  \
               "v_fmac_f32_dpp %3, %4, %8 row_newbcast:" #T " row_mask:0xf bank_mask:0xf"       \
               : "+v"(acc0), "+v"(acc1), "+v"(acc2), "+v"(acc3)                                \
               : "v"(av), "v"(BV.x), "v"(BV.y), "v"(BV.z), "v"(BV.w));

#define SPDL_DPP_ADDR(T) (__builtin_amdgcn_update_dpp(0, off, 0x150 + (T), 0xf, 0xf, false) + lane_b)

#define SPDL_DPP_GROUP(T0, T1, T2, T3, PRE)                                                    \
  {                                                                                            \
    const f32x4 b0 = *reinterpret_cast<const f32x4*>(buf + SPDL_DPP_ADDR(T0));                 \
    const f32x4 b1 = *reinterpret_cast<const f32x4*>(buf + SPDL_DPP_ADDR(T1));                 \
    const f32x4 b2 = *reinterpret_cast<const f32x4*>(buf + SPDL_DPP_ADDR(T2));                 \
    const f32x4 b3 = *reinterpret_cast<const f32x4*>(buf + SPDL_DPP_ADDR(T3));                 \
    SPDL_DPP_FMA4(T0, b0, PRE)                                                                 \
    SPDL_DPP_FMA4(T1, b1, "")                                                                  \
    SPDL_DPP_FMA4(T2, b2, "")                                                                  \
    SPDL_DPP_FMA4(T3, b3, "")                                                                  \
  }

template <typename T, int S>
__global__ __launch_bounds__(kSlabThreads) void spmm_slab_kernel(
    int m, int k, int n, int tiles_n, int panels, const int* __restrict__ row_offsets,
    const int* __restrict__ column_indices, const T* __restrict__ values,
    const int* __restrict__ row_order, const T* __restrict__ B, T* __restrict__ C) {
  extern __shared__ __attribute__((aligned(16))) char lds_raw[];
  constexpr int kBufBytes = (S + 1) * kSlabTile * 4;      // S data rows + one all-zero row
  constexpr int kZeroOff = S * kSlabTile * 4;
  constexpr int kPasses = S * 16 / kSlabThreads;          // float4 loads per thread per slab

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int sub = lane >> 4;
  const int l16 = lane & 15;
  const int lane_b = l16 * 16;

  // Workgroup id -> (panel, tile): the tiles of one row panel get ids that are equal modulo 8,
  // so they run on the same XCD and the panel's part of A is fetched into one L2 only.
  const int per_group = 8 * tiles_n;
  const int grp = blockIdx.x / per_group;
  const int rem = blockIdx.x - grp * per_group;
  const int tile = rem >> 3;
  const int panel = grp * 8 + (rem & 7);
  if (panel >= panels) return;

  const int slot = panel * kSlabRows + wave * 4 + sub;
  int row = -1, p = 0, row_end = 0;
  if (slot < m) {
    row = row_order ? row_order[slot] : slot;
    p = row_offsets[row];
    row_end = row_offsets[row + 1];
  }
  const int p_begin = p;
  const int col = tile * kSlabTile + l16 * 4;
  const bool col_ok = col < n;

  // staging of B: thread -> (row within pass, 4 columns)
  const int srow = tid >> 4;
  const bool scol_ok = (tile * kSlabTile + (tid & 15) * 4) < n;
  const T* Bst = B + (size_t)(tile * kSlabTile + (scol_ok ? (tid & 15) * 4 : 0));
  float stage[kPasses][4];
  auto gload = [&](int slab) {
#pragma unroll
    for (int j = 0; j < kPasses; ++j) {
      const int r = slab * S + j * 64 + srow;
      if (r < k && scol_ok) {
        Pack<T, 4>::load(Bst + (size_t)r * n, stage[j]);
      } else {
        stage[j][0] = stage[j][1] = stage[j][2] = stage[j][3] = 0.f;
      }
    }
  };
  auto lstore = [&](int bufi) {
#pragma unroll
    for (int j = 0; j < kPasses; ++j) {
      f32x4 v = {stage[j][0], stage[j][1], stage[j][2], stage[j][3]};
      *reinterpret_cast<f32x4*>(lds_raw + bufi * kBufBytes + ((j * 64 + srow) * kSlabTile + (tid & 15) * 4) * 4) = v;
    }
  };
  if (tid < 2 * kSlabTile)
    *reinterpret_cast<float*>(lds_raw + (tid >> 6) * kBufBytes + kZeroOff + (tid & 63) * 4) = 0.f;

  float acc0 = 0.f, acc1 = 0.f, acc2 = 0.f, acc3 = 0.f;
  const int nslabs = (k + S - 1) / S;
  gload(0);
  lstore(0);
  __syncthreads();

  for (int s = 0; s < nslabs; ++s) {
    if (s + 1 < nslabs) gload(s + 1);
    const int slab_start = s * S;
    const char* buf = lds_raw + (s & 1) * kBufBytes;
    while (true) {
      const int idx = p + l16;
      const bool inrow = idx < row_end;
      int c = 0x7fffffff;
      float a = 0.f;
      if (inrow) {
        c = column_indices[idx];
        a = (float)values[idx];
      }
      const unsigned rel = (unsigned)(c - slab_start);
      const bool valid = rel < (unsigned)S;
      const unsigned long long mask = __ballot(valid);
      const unsigned piece = (unsigned)(mask >> (sub * 16)) & 0xffffu;
      const int cnt = __builtin_ctz(~piece | 0x10000u);          // leading pairs inside the slab
      const int cmax = max(max(__builtin_amdgcn_readlane(cnt, 0), __builtin_amdgcn_readlane(cnt, 16)),
                           max(__builtin_amdgcn_readlane(cnt, 32), __builtin_amdgcn_readlane(cnt, 48)));
      if (cmax == 0) break;
      const bool use = l16 < cnt;
      const float av = use ? a : 0.f;
      const int off = use ? (int)(rel * (kSlabTile * 4)) : kZeroOff;   // LDS byte offset of the B row
      SPDL_DPP_GROUP(0, 1, 2, 3, "s_nop 1\n\t")
      if (cmax > 4) {
        SPDL_DPP_GROUP(4, 5, 6, 7, "")
        if (cmax > 8) {
          SPDL_DPP_GROUP(8, 9, 10, 11, "")
          if (cmax > 12) SPDL_DPP_GROUP(12, 13, 14, 15, "")
        }
      }
      p += cnt;
      if (cmax < 16) break;
    }
    if (s + 1 < nslabs) lstore((s + 1) & 1);
    __syncthreads();
  }

  // A row whose column indices are not ascending leaves its cursor short of the row end:
  // redo that row from scratch with direct gathers.
  if (p != row_end) {
    acc0 = acc1 = acc2 = acc3 = 0.f;
    const T* Bcol = B + (col_ok ? col : 0);
    for (int q = p_begin; q < row_end; ++q) {
      const float a = (float)values[q];
      float b[4];
      Pack<T, 4>::load(Bcol + (size_t)column_indices[q] * n, b);
      acc0 = __builtin_fmaf(a, b[0], acc0);
      acc1 = __builtin_fmaf(a, b[1], acc1);
      acc2 = __builtin_fmaf(a, b[2], acc2);
      acc3 = __builtin_fmaf(a, b[3], acc3);
    }
  }
  if (row >= 0 && col_ok) {
    const float out[4] = {acc0, acc1, acc2, acc3};
    Pack<T, 4>::store(C + (size_t)row * n + col, out);
  }
}

#undef SPDL_DPP_GROUP
#undef SPDL_DPP_ADDR
#undef SPDL_DPP_FMA4

}  // namespace spdl
