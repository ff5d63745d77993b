// SpMM, slab family: a workgroup owns 64 sparse rows (one panel) and walks over one or more
// 64-column tiles of C.  B is streamed through LDS in slabs of S consecutive rows, so every
// B element is fetched from global memory once per workgroup and then re-read from LDS by
// each sparse row that has a nonzero in that column: reuse of B across rows, which the paper
// names as the way past its shared-memory bandwidth limit (Sec. "Discussion & Conclusion").
//
// The 16 waves are specialised.  Waves 8..15 are producers: they only move B slabs from
// global memory into the LDS buffer that is not being read (two buffers).  Waves 0..7 are
// consumers.  Vector-memory loads retire in order, so a wave that had both a slab prefetch
// and its sparse-row loads in flight would stall on the slab every time it needed the next
// sparse elements; with the split, consumers wait only for their own short loads.
//
// Inside a consumer wave each 16-lane group owns two sparse rows (paper Sec. "Subwarp
// Tiling"; rows bundled by length through the row order).  A group fetches 16 consecutive
// (value, column) pairs of its row with one load each, one round ahead, and the pairs are
// handed to the group's lanes one at a time by DPP row broadcasts inside the multiply-add.
// The column index is pre-scaled to an LDS byte offset once per pair (Sec. "Index
// Pre-Scaling").  Every row's products are added in stored order with fused multiply-adds.
//
// The slab walk needs ascending column indices inside a row; a row that is not ascending is
// noticed (its cursor does not reach the row end) and redone by direct gathers, so results
// are always right.  Needs n % 4 == 0 and 16-byte aligned B and C.
#pragma once
#include "common.hpp"

namespace spdl {

constexpr int kSlabTile = 64;          // output columns per tile
constexpr int kSlabRows = 64;          // sparse rows per workgroup
constexpr int kSlabThreads = 1024;
constexpr int kSlabConsumers = 512;    // threads of the consumer waves

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
               : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3])                        \
               : "v"(av), "v"(BV.x), "v"(BV.y), "v"(BV.z), "v"(BV.w));

#define SPDL_DPP_ADDR(T) (__builtin_amdgcn_update_dpp(0, off, 0x150 + (T), 0xf, 0xf, false) + lane_b)

// Loads of one group of four pairs into BQ[0..3], and its sixteen multiply-adds.
#define SPDL_DPP_LOAD4(BQ, T0, T1, T2, T3)                                                     \
  BQ[0] = *reinterpret_cast<const f32x4*>(buf + SPDL_DPP_ADDR(T0));                            \
  BQ[1] = *reinterpret_cast<const f32x4*>(buf + SPDL_DPP_ADDR(T1));                            \
  BQ[2] = *reinterpret_cast<const f32x4*>(buf + SPDL_DPP_ADDR(T2));                            \
  BQ[3] = *reinterpret_cast<const f32x4*>(buf + SPDL_DPP_ADDR(T3));

// One asm statement per group, so that the wait in front of it can leave exactly the four
// younger reads of the next group outstanding.
#define SPDL_DPP_FMA16(BQ, T0, T1, T2, T3, PRE)                                                              \
  asm volatile(PRE                                                                                            \
               "v_fmac_f32_dpp %0, %4, %5 row_newbcast:" #T0 " row_mask:0xf bank_mask:0xf\n\t"                \
               "v_fmac_f32_dpp %1, %4, %6 row_newbcast:" #T0 " row_mask:0xf bank_mask:0xf\n\t"                \
               "v_fmac_f32_dpp %2, %4, %7 row_newbcast:" #T0 " row_mask:0xf bank_mask:0xf\n\t"                \
               "v_fmac_f32_dpp %3, %4, %8 row_newbcast:" #T0 " row_mask:0xf bank_mask:0xf\n\t"                \
               "v_fmac_f32_dpp %0, %4, %9 row_newbcast:" #T1 " row_mask:0xf bank_mask:0xf\n\t"                \
               "v_fmac_f32_dpp %1, %4, %10 row_newbcast:" #T1 " row_mask:0xf bank_mask:0xf\n\t"               \
               "v_fmac_f32_dpp %2, %4, %11 row_newbcast:" #T1 " row_mask:0xf bank_mask:0xf\n\t"               \
               "v_fmac_f32_dpp %3, %4, %12 row_newbcast:" #T1 " row_mask:0xf bank_mask:0xf\n\t"               \
               "v_fmac_f32_dpp %0, %4, %13 row_newbcast:" #T2 " row_mask:0xf bank_mask:0xf\n\t"               \
               "v_fmac_f32_dpp %1, %4, %14 row_newbcast:" #T2 " row_mask:0xf bank_mask:0xf\n\t"               \
               "v_fmac_f32_dpp %2, %4, %15 row_newbcast:" #T2 " row_mask:0xf bank_mask:0xf\n\t"               \
               "v_fmac_f32_dpp %3, %4, %16 row_newbcast:" #T2 " row_mask:0xf bank_mask:0xf\n\t"               \
               "v_fmac_f32_dpp %0, %4, %17 row_newbcast:" #T3 " row_mask:0xf bank_mask:0xf\n\t"               \
               "v_fmac_f32_dpp %1, %4, %18 row_newbcast:" #T3 " row_mask:0xf bank_mask:0xf\n\t"               \
               "v_fmac_f32_dpp %2, %4, %19 row_newbcast:" #T3 " row_mask:0xf bank_mask:0xf\n\t"               \
               "v_fmac_f32_dpp %3, %4, %20 row_newbcast:" #T3 " row_mask:0xf bank_mask:0xf"                    \
               : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3])                                       \
               : "v"(av), "v"(BQ[0].x), "v"(BQ[0].y), "v"(BQ[0].z), "v"(BQ[0].w), "v"(BQ[1].x), "v"(BQ[1].y), \
                 "v"(BQ[1].z), "v"(BQ[1].w), "v"(BQ[2].x), "v"(BQ[2].y), "v"(BQ[2].z), "v"(BQ[2].w),          \
                 "v"(BQ[3].x), "v"(BQ[3].y), "v"(BQ[3].z), "v"(BQ[3].w));

// The up to 16 steps of one round: pair t of every group (value av, LDS offset off, both held
// by lane t of the group) times its B row, for t < cmax rounded up to a multiple of four.
// The reads one group of four ahead are issued whether or not that group is needed (every
// offset is a valid LDS address), so that the wait before each block of multiply-adds can
// leave exactly the younger four reads outstanding.
__device__ __forceinline__ void slab_steps(float (&acc)[4], float av, int off, const char* buf, int lane_b,
                                           int cmax) {
  f32x4 bx[4], by[4];
  SPDL_DPP_LOAD4(bx, 0, 1, 2, 3)
  SPDL_DPP_LOAD4(by, 4, 5, 6, 7)
  SPDL_DPP_FMA16(bx, 0, 1, 2, 3, "s_nop 1\n\t")
  if (cmax > 4) {
    SPDL_DPP_LOAD4(bx, 8, 9, 10, 11)
    SPDL_DPP_FMA16(by, 4, 5, 6, 7, "")
    if (cmax > 8) {
      SPDL_DPP_LOAD4(by, 12, 13, 14, 15)
      SPDL_DPP_FMA16(bx, 8, 9, 10, 11, "")
      if (cmax > 12) { SPDL_DPP_FMA16(by, 12, 13, 14, 15, "") }
    }
  }
}

// State of one sparse row inside a 16-lane group.
struct SlabRow {
  int row, p_begin, p, row_end;
  int c_next;
  float a_next;
};

// The loads are unconditional (index clamped into the arrays, result discarded past the row
// end): a load under a branch would make the compiler wait for it at once, and the point of
// fetching a round ahead is to leave it in flight.  Byte offsets are 32-bit so that the loads
// use a scalar base plus a vector offset (nnz < 2^29 is checked on the host).
template <typename T>
__device__ __forceinline__ void slab_fetch(SlabRow& r, int l16, int last_nz, const int* __restrict__ ci,
                                           const T* __restrict__ val) {
  const int idx = r.p + l16;
  const unsigned safe = (unsigned)min(idx, last_nz);
  const int c = *reinterpret_cast<const int*>(reinterpret_cast<const char*>(ci) + (safe << 2));
  const float a = (float)*reinterpret_cast<const T*>(reinterpret_cast<const char*>(val) + safe * (unsigned)sizeof(T));
  const bool in = idx < r.row_end;
  r.c_next = in ? c : 0x7fffffff;
  r.a_next = in ? a : 0.f;
}

// All of one row's pairs that fall into the slab [slab_start, slab_start + S).
template <typename T, int S>
__device__ __forceinline__ void slab_consume(SlabRow& r, float (&acc)[4], const char* buf,
                                             int slab_start, int sub, int l16, int lane_b, int last_nz,
                                             const int* __restrict__ ci, const T* __restrict__ val) {
  constexpr int kZeroOff = S * kSlabTile * 4;
  const int sub8 = sub * 8;
  while (true) {
    const unsigned rel = (unsigned)(r.c_next - slab_start);
    const bool valid = rel < (unsigned)S;
    // Everything derived from the wave mask is wave-uniform and stays in scalar registers:
    // per-group counts of leading pairs inside the slab, their maximum, and the four counts
    // packed into one word from which each lane extracts its group's.
    const unsigned long long mask = __ballot(valid);
    if (mask == 0) break;
    const unsigned lo = (unsigned)mask, hi = (unsigned)(mask >> 32);
    const int c0 = leading16(lo & 0xffffu), c1 = leading16(lo >> 16);
    const int c2 = leading16(hi & 0xffffu), c3 = leading16(hi >> 16);
    const int cmax = max(max(c0, c1), max(c2, c3));
    if (cmax == 0) break;
    const unsigned packed = (unsigned)c0 | ((unsigned)c1 << 8) | ((unsigned)c2 << 16) | ((unsigned)c3 << 24);
    const int cnt = (int)((packed >> sub8) & 0xffu);
    // A pair inside the slab is used even if it is not among the leading ones (rows that are
    // not ascending): the cursor then stops short of the row end and the row is redone.
    const float av = valid ? r.a_next : 0.f;
    const int off = valid ? (int)(rel * (kSlabTile * 4)) : kZeroOff;   // LDS byte offset of the B row
    r.p += cnt;
    slab_fetch<T>(r, l16, last_nz, ci, val);                        // next round's pairs
    // LDS reads of the next group of four pairs are issued before the multiply-adds of the
    // current one, so their latency overlaps arithmetic inside the wave.
    // The reads one group ahead are issued whether or not that group is needed (every offset
    // is a valid LDS address), so that the wait before each block of multiply-adds can leave
    // exactly the younger four reads outstanding.
    f32x4 bx[4], by[4];
    SPDL_DPP_LOAD4(bx, 0, 1, 2, 3)
    SPDL_DPP_LOAD4(by, 4, 5, 6, 7)
    SPDL_DPP_FMA16(bx, 0, 1, 2, 3, "s_nop 1\n\t")
    if (cmax > 4) {
      SPDL_DPP_LOAD4(bx, 8, 9, 10, 11)
      SPDL_DPP_FMA16(by, 4, 5, 6, 7, "")
      if (cmax > 8) {
        SPDL_DPP_LOAD4(by, 12, 13, 14, 15)
        SPDL_DPP_FMA16(bx, 8, 9, 10, 11, "")
        if (cmax > 12) { SPDL_DPP_FMA16(by, 12, 13, 14, 15, "") }
      }
    }
    if (cmax < 16) break;
  }
}

template <typename T, int S>
__global__ __launch_bounds__(kSlabThreads) void spmm_slab_kernel(
    int m, int k, int n, int nnz, int tiles_n, int tiles_per_wg, int panels,
    const int* __restrict__ row_offsets, const int* __restrict__ column_indices,
    const T* __restrict__ values, const int* __restrict__ row_order, const T* __restrict__ B,
    T* __restrict__ C, const T* __restrict__ bias, int relu) {
  extern __shared__ __attribute__((aligned(16))) char lds_raw[];
  constexpr int kBufBytes = (S + 1) * kSlabTile * 4;      // S data rows + one all-zero row
  constexpr int kZeroOff = S * kSlabTile * 4;
  constexpr int kPasses = S * 16 / (kSlabThreads - kSlabConsumers);   // float4 loads per producer thread

  const int tid = threadIdx.x;

  // Workgroup id -> (panel, tile group): the tile groups of one row panel get ids that are
  // equal modulo 8, so they run on the same XCD and the panel's part of A stays in one L2.
  const int groups_n = (tiles_n + tiles_per_wg - 1) / tiles_per_wg;
  int panel, tile_group;
  if (!slab_wg_map(blockIdx.x, panels, groups_n, panel, tile_group)) return;
  const int tile_begin = tile_group * tiles_per_wg;
  const int tile_end = min(tiles_n, tile_begin + tiles_per_wg);
  const int nslabs = (k + S - 1) / S;
  const int stages = (tile_end - tile_begin) * nslabs;

  if (tid < 2 * kSlabTile)
    *reinterpret_cast<float*>(lds_raw + (tid >> 6) * kBufBytes + kZeroOff + (tid & 63) * 4) = 0.f;

  if (tid >= kSlabConsumers) {
    // ---------------------------------------------------------------- producer waves
    const int pt = tid - kSlabConsumers;
    const int srow = pt >> 4;                 // 0..31
    const int scol = (pt & 15) * 4;
    // Two register sets: the loads of stage q+2 are issued before stage q+1 is written to
    // LDS, so two slabs are in flight per workgroup.  Every load is unconditional (row and
    // column clamped into B, stage index clamped to the last one): the wait before a store
    // can then leave exactly the younger set outstanding.  Slab rows past k and tile columns
    // past n hold clamped copies that no valid column index or stored output ever touches.
    float stage[2][kPasses][4];
    const int last_stage = stages - 1;
    auto gload = [&](int q, float (&st)[kPasses][4]) {
      q = min(q, last_stage);
      const int tile = tile_begin + q / nslabs;
      const int slab = q - (q / nslabs) * nslabs;
      const int colg = tile * kSlabTile + scol;
      const T* src = B + (colg < n ? colg : 0);
#pragma unroll
      for (int j = 0; j < kPasses; ++j) {
        const int r = min(slab * S + j * 32 + srow, k - 1);
        Pack<T, 4>::load(src + (size_t)r * n, st[j]);
      }
    };
    auto lstore = [&](int q, const float (&st)[kPasses][4]) {
      char* dst = lds_raw + (q & 1) * kBufBytes;
#pragma unroll
      for (int j = 0; j < kPasses; ++j) {
        f32x4 v = {st[j][0], st[j][1], st[j][2], st[j][3]};
        *reinterpret_cast<f32x4*>(dst + ((j * 32 + srow) * kSlabTile + scol) * 4) = v;
      }
    };
    gload(0, stage[0]);
    gload(1, stage[1]);
    lstore(0, stage[0]);
    __syncthreads();
    // at the top of iteration q: stage q is in LDS, stage q+1 is in flight to set 1
    for (int q = 0; q < stages; q += 2) {
      gload(q + 2, stage[0]);
      if (q + 1 < stages) lstore(q + 1, stage[1]);
      __syncthreads();
      gload(q + 3, stage[1]);
      if (q + 1 < stages) {
        if (q + 2 < stages) lstore(q + 2, stage[0]);
        __syncthreads();
      }
    }
    return;
  }

  // ------------------------------------------------------------------ consumer waves
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int sub = lane >> 4;
  const int l16 = lane & 15;
  const int lane_b = l16 * 16;

  SlabRow rows[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    // a wave's 8 rows are adjacent in the row order; a workgroup takes every panels-th bundle
    const int slot = ((wave * panels + panel) * 4 + sub) * 2 + j;
    rows[j].row = -1;
    rows[j].p_begin = rows[j].row_end = 0;
    if (slot < m) {
      const int row = row_order ? row_order[slot] : slot;
      rows[j].row = row;
      rows[j].p_begin = row_offsets[row];
      rows[j].row_end = row_offsets[row + 1];
    }
  }
  float acc[2][4];

  __syncthreads();
  int q = 0;
  for (int tile = tile_begin; tile < tile_end; ++tile) {
    const int col = tile * kSlabTile + l16 * 4;
    const bool col_ok = col < n;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      rows[j].p = rows[j].p_begin;
      acc[j][0] = acc[j][1] = acc[j][2] = acc[j][3] = 0.f;
      slab_fetch<T>(rows[j], l16, nnz - 1, column_indices, values);
    }
    for (int s = 0; s < nslabs; ++s, ++q) {
      const char* buf = lds_raw + (q & 1) * kBufBytes;
#pragma unroll
      for (int j = 0; j < 2; ++j)
        slab_consume<T, S>(rows[j], acc[j], buf, s * S, sub, l16, lane_b, nnz - 1, column_indices, values);
      __syncthreads();
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      // A row whose column indices are not ascending leaves its cursor short of the row end:
      // redo that row from scratch with direct gathers.
      if (rows[j].p != rows[j].row_end) {
        acc[j][0] = acc[j][1] = acc[j][2] = acc[j][3] = 0.f;
        const T* Bcol = B + (col_ok ? col : 0);
        for (int t = rows[j].p_begin; t < rows[j].row_end; ++t) {
          const float a = (float)values[t];
          float b[4];
          Pack<T, 4>::load(Bcol + (size_t)column_indices[t] * n, b);
#pragma unroll
          for (int v = 0; v < 4; ++v) acc[j][v] = __builtin_fmaf(a, b[v], acc[j][v]);
        }
      }
      if (rows[j].row >= 0 && col_ok) {
        spmm_epilogue<T, 4>(acc[j], bias, rows[j].row, relu);
        Pack<T, 4>::store(C + (size_t)rows[j].row * n + col, acc[j]);
      }
    }
  }
}

// The sixteen multiply-adds of pairs 4Q .. 4Q+3 of every group as functions, for kernels that
// bring the rows of B in some other way (bq[j] = the four columns of this lane in the row of B of
// pair 4Q+j; av = the group's values, lane t holding pair t).
#define SPDL_DEF_FMA16(NAME, T0, T1, T2, T3)                                                      \
  __device__ __forceinline__ void NAME(float (&acc)[4], float av, const f32x4 (&bq)[4]) {          \
    SPDL_DPP_FMA16(bq, T0, T1, T2, T3, "s_nop 1\n\t")                                             \
  }
SPDL_DEF_FMA16(slab_fma16_q0, 0, 1, 2, 3)
SPDL_DEF_FMA16(slab_fma16_q1, 4, 5, 6, 7)
SPDL_DEF_FMA16(slab_fma16_q2, 8, 9, 10, 11)
SPDL_DEF_FMA16(slab_fma16_q3, 12, 13, 14, 15)
#undef SPDL_DEF_FMA16
#undef SPDL_DPP_FMA16
#undef SPDL_DPP_LOAD4
#undef SPDL_DPP_ADDR
#undef SPDL_DPP_FMA4

}  // namespace spdl
