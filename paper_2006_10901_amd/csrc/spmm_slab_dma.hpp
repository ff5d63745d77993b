// SpMM, slab family with asynchronous global->LDS copies: same decomposition as the
// producer/consumer slab kernel (64 sparse rows x 64-column tiles per workgroup, B streamed
// through LDS in slabs of S rows, 16-lane groups with DPP-broadcast multiply-adds), but all
// 16 waves compute, one sparse row per 16-lane group, and each wave moves its share of the
// next slab with direct-to-LDS loads (no staging registers, no LDS store instructions).
//
// A wait for sparse elements that were requested after the slab copies also waits for the
// copies, so waits inside a stage are avoided: the kernel works in double rounds of 32
// (value, column) pairs per row, the next 32 pairs are requested as soon as the cursor is
// known, before the arithmetic of the current double round, and they are first needed in the
// next stage.  The only wait is the one at the end of a stage, for everything (copies and pair
// loads alike have had the stage's arithmetic to complete); no assumption is made about the
// order in which copies and ordinary loads retire.  A row with more than 32 pairs in a slab
// takes further double rounds, each behind a full wait.
#pragma once
#include "common.hpp"
#include "spmm_slab.hpp"

namespace spdl {

// RPG = sparse rows per 16-lane group (1 or 2): the workgroup owns 64*RPG rows.  Two rows per
// group halve the traffic of B and the number of stages per unit of work when the output has
// enough tiles to fill the machine anyway.
template <int S, int RPG>
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

  SlabRow rows[RPG];
#pragma unroll
  for (int j = 0; j < RPG; ++j) {
    // Row binning (paper Sec. "Row Swizzle Load Balancing"): a wave's 4*RPG rows are adjacent
    // in the row order (a bundle of similar lengths), and a workgroup takes every panels-th
    // bundle, so each workgroup gets the same mix of long and short bundles.
    const int slot = ((wave * panels + panel) * 4 + sub) * RPG + j;
    rows[j].row = -1;
    rows[j].p_begin = rows[j].row_end = 0;
    if (slot < m) {
      const int r = row_order ? row_order[slot] : slot;
      rows[j].row = r;
      rows[j].p_begin = row_offsets[r];
      rows[j].row_end = row_offsets[r + 1];
    }
  }
  const int last_nz = nnz - 1;
  const int sub8 = sub * 8;
  float acc[RPG][4];

  // Pairs [at, at+16) and [at+16, at+32) of each row, lane t of the group holding pair t.  The
  // loaded words are kept raw (no arithmetic on them here): the compiler waits for a load at
  // its first use, and the first use is in the next stage, after the full wait that ends
  // every stage.  32-bit byte offsets from scalar bases (nnz < 2^29 is checked on the host).
  int cA[RPG], cB[RPG], at[RPG];
  float aA[RPG], aB[RPG];
  auto fetch32 = [&](int j, int from) {
    at[j] = from;
    const int idx = from + l16;
    const unsigned oa = (unsigned)min(idx, last_nz) << 2, ob = (unsigned)min(idx + 16, last_nz) << 2;
    const char* cbase = reinterpret_cast<const char*>(column_indices);
    const char* vbase = reinterpret_cast<const char*>(values);
    cA[j] = *reinterpret_cast<const int*>(cbase + oa);
    aA[j] = *reinterpret_cast<const float*>(vbase + oa);
    cB[j] = *reinterpret_cast<const int*>(cbase + ob);
    aB[j] = *reinterpret_cast<const float*>(vbase + ob);
  };
  // every vector-memory operation of this wave (pair loads, slab copies) has completed
  auto wait_everything = [&]() { __builtin_amdgcn_s_waitcnt(0); };

  // One double round of row j in the slab starting at slab_start.  Returns true when all 32
  // fetched pairs of some group were used, i.e. the slab may hold more pairs of that row.
  // `restart`: this is the last slab of a tile and another tile follows, so once the row is done
  // here the next pairs needed are those at the row start again.
  auto double_round = [&](int j, const char* buf, int slab_start, bool restart) -> bool {
    const int idx = at[j] + l16;
    const unsigned relA = (unsigned)(cA[j] - slab_start), relB = (unsigned)(cB[j] - slab_start);
    const bool inA = idx < rows[j].row_end && relA < (unsigned)S;
    const unsigned long long mA = __ballot(inA);
    const unsigned lo = (unsigned)mA, hi = (unsigned)(mA >> 32);
    const int a0 = leading16(lo & 0xffffu), a1 = leading16(lo >> 16);
    const int a2 = leading16(hi & 0xffffu), a3 = leading16(hi >> 16);
    const int cmaxA = max(max(a0, a1), max(a2, a3));
    const unsigned packedA = (unsigned)a0 | ((unsigned)a1 << 8) | ((unsigned)a2 << 16) | ((unsigned)a3 << 24);
    const int cntA = (int)((packedA >> sub8) & 0xffu);
    // the second 16 continue the first 16 only where those were all consumed
    const bool inB = cntA == 16 && idx + 16 < rows[j].row_end && relB < (unsigned)S;
    const unsigned long long mB = __ballot(inB);
    const unsigned lo2 = (unsigned)mB, hi2 = (unsigned)(mB >> 32);
    const int b0 = leading16(lo2 & 0xffffu), b1 = leading16(lo2 >> 16);
    const int b2 = leading16(hi2 & 0xffffu), b3 = leading16(hi2 >> 16);
    const int cmaxB = max(max(b0, b1), max(b2, b3));
    const unsigned packedB = (unsigned)b0 | ((unsigned)b1 << 8) | ((unsigned)b2 << 16) | ((unsigned)b3 << 24);
    const int cntB = (int)((packedB >> sub8) & 0xffu);
    const float avA = inA ? aA[j] : 0.f, avB = inB ? aB[j] : 0.f;
    const int offA = inA ? (int)(relA * (kSlabTile * 4)) : kZeroOff;
    const int offB = inB ? (int)(relB * (kSlabTile * 4)) : kZeroOff;
    rows[j].p += cntA + cntB;
    // next 32 pairs, first needed in the next stage (or in the next double round of this one)
    fetch32(j, (restart && cmaxB < 16) ? rows[j].p_begin : rows[j].p);
    if (cmaxA > 0) slab_steps(acc[j], avA, offA, buf, lane_b, cmaxA);
    if (cmaxB > 0) slab_steps(acc[j], avB, offB, buf, lane_b, cmaxB);
    return cmaxB == 16;
  };

  copy_stage(0);
#pragma unroll
  for (int j = 0; j < RPG; ++j) fetch32(j, rows[j].p_begin);
  wait_everything();
  __builtin_amdgcn_s_barrier();
  int q = 0;
  for (int tile = tile_begin; tile < tile_end; ++tile) {
    const int col = tile * kSlabTile + l16 * 4;
    const bool col_ok = col < n;
#pragma unroll
    for (int j = 0; j < RPG; ++j) {
      rows[j].p = rows[j].p_begin;          // the pairs at the row start are already in registers
      acc[j][0] = acc[j][1] = acc[j][2] = acc[j][3] = 0.f;
    }
    for (int s = 0; s < nslabs; ++s, ++q) {
      // A use of the youngest pair register before the copies are issued: the compiler places
      // its wait for the pair loads here, where they completed long ago (full wait at the end
      // of the previous stage), instead of after the copies, where it would wait for those too.
      asm volatile("v_mov_b32 %0, %0" : "+v"(aB[RPG - 1]));
      if (q + 1 < stages) copy_stage(q + 1);
      const char* buf = lds_raw + (q & 1) * kBufBytes;
#pragma unroll
      for (int j = 0; j < RPG; ++j) {
        const bool restart = s == nslabs - 1 && tile + 1 < tile_end;
        // The first double round stands outside the loop: inside it the compiler would have to
        // wait for the previous iteration's loads, and with them for the copies just issued.
        if (double_round(j, buf, s * S, restart))
          while (double_round(j, buf, s * S, restart)) {}        // more than 32 pairs in this slab
      }
      wait_everything();
      __builtin_amdgcn_s_barrier();
    }
#pragma unroll
    for (int j = 0; j < RPG; ++j) {
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
      if (rows[j].row >= 0 && col_ok) Pack<T, 4>::store(C + (size_t)rows[j].row * n + col, acc[j]);
    }
  }
}

}  // namespace spdl
