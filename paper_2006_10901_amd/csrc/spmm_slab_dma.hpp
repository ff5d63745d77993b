// SpMM, slab family with asynchronous global->LDS copies: same decomposition as the
// producer/consumer slab kernel (64 sparse rows x 64-column tiles per workgroup, B streamed
// through LDS in slabs of S rows, 16-lane groups with DPP-broadcast multiply-adds), but all
// 16 waves compute, one sparse row per 16-lane group, and each wave moves its share of the
// next slab with direct-to-LDS loads (no staging registers, no LDS store instructions).
//
// A wait for sparse elements that were requested after the slab copies also waits for the
// copies, so waits inside a stage are avoided: the kernel works in long rounds of 16*NCH
// (value, column) pairs per row, the next pairs are requested as soon as the cursor is
// known, before the arithmetic of the current round, and they are first needed in the
// next stage.  The only wait is the one at the end of a stage, for everything (copies and pair
// loads alike have had the stage's arithmetic to complete); no assumption is made about the
// order in which copies and ordinary loads retire.  A row with more than 16*NCH pairs in a
// slab takes further rounds, each behind a full wait.
#pragma once
#include "common.hpp"
#include "spmm_slab.hpp"

namespace spdl {

// RPG = sparse rows per 16-lane group (1 or 2): the workgroup owns 64*RPG rows.  Two rows per
// group halve the traffic of B and the number of stages per unit of work when the output has
// enough tiles to fill the machine anyway.
// NCH = chunks of 16 pairs fetched ahead per row (chosen by the host from the density so that
// a row's pairs inside one slab usually fit).
// NW = waves per workgroup: 16 (one workgroup per CU), or 8 with slabs half as large, so that two
// workgroups share a CU: panels of 32*RPG rows, for outputs with fewer than 256 tiles of 64 x 64,
// which would otherwise leave compute units without a workgroup.
template <int S, int RPG, int NCH, int NW = 16>
__global__ __launch_bounds__(64 * NW) void spmm_slab_dma_kernel(
    int m, int k, int n, int nnz, int tiles_n, int tiles_per_wg, int panels,
    const int* __restrict__ row_offsets, const int* __restrict__ column_indices,
    const float* __restrict__ values, const int* __restrict__ row_order, const float* __restrict__ B,
    float* __restrict__ C, const float* __restrict__ bias, int relu) {
  using T = float;
  extern __shared__ __attribute__((aligned(16))) char lds_raw[];
  constexpr int kBufBytes = (S + 1) * kSlabTile * 4;      // S data rows + one all-zero row
  constexpr int kZeroOff = S * kSlabTile * 4;
  constexpr int kCopies = S / (4 * NW);                   // 1 KB direct-to-LDS loads per wave per slab

  PhaseClocks clocks;
  clocks.start();
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = uniform(tid >> 6);
  const int sub = lane >> 4;
  const int l16 = lane & 15;
  const int lane_b = l16 * 16;

  const int groups_n = (tiles_n + tiles_per_wg - 1) / tiles_per_wg;
  int panel, tile_group;
  if (!slab_wg_map(blockIdx.x, panels, groups_n, panel, tile_group)) return;
  const int tile_begin = tile_group * tiles_per_wg;
  const int tile_end = min(tiles_n, tile_begin + tiles_per_wg);
  const int nslabs = (k + S - 1) / S;
  const int stages = (tile_end - tile_begin) * nslabs;

  if (tid < 2 * kSlabTile)
    *reinterpret_cast<float*>(lds_raw + (tid >> 6) * kBufBytes + kZeroOff + (tid & 63) * 4) = 0.f;

  // Slab copy: copy i of wave w fills slab rows (i*NW + w)*4 .. +3; lane L brings row L/16 of
  // those, columns 4*(L%16) .. +3, and the hardware places lane L's 16 bytes at M0 + 16*L.
  // The address is a scalar base (start of the slab in B, moved from stage to stage with scalar
  // arithmetic) plus a per-lane byte offset that is the same in every stage except a ragged
  // last slab, whose rows past k are clamped to row k-1, and a ragged last tile, whose columns
  // past n are clamped to the tile's first column: nothing valid ever reads those.
  // (S * n * 4 < 2^31 is checked on the host.)
  unsigned row_off[kCopies], row_off_last[kCopies];
  const int last_rows = k - (nslabs - 1) * S;               // rows of the last slab, 1..S
#pragma unroll
  for (int i = 0; i < kCopies; ++i) {
    const int lrow = (i * NW + wave) * 4 + sub;
    row_off[i] = (unsigned)lrow * (unsigned)n * 4u;
    row_off_last[i] = (unsigned)min(lrow, last_rows - 1) * (unsigned)n * 4u;
  }
  // The copies are issued from inline assembly: the compiler treats its own direct-to-LDS loads
  // as touching both memory paths and then turns every later wait, for LDS reads and for pair
  // loads alike, into a wait for everything.  Their completion is covered by the explicit full
  // wait and barrier that end every stage.  M0 (the LDS destination) is not used by anything
  // the compiler generates in this kernel.
  auto copy_stage = [&](int q) {
    const int t = q / nslabs;
    const int slab = q - t * nslabs;
    const int tile = tile_begin + t;
    const bool ragged_tile = tile * kSlabTile + l16 * 4 >= n;
    const unsigned col_off = ragged_tile ? 0u : (unsigned)(l16 * 16);
    const char* base = reinterpret_cast<const char*>(B + (size_t)slab * S * n + tile * kSlabTile);
    const unsigned dst = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)(lds_raw + (q & 1) * kBufBytes) +
                         (unsigned)wave * (4 * kSlabTile * 4);
    const bool last = slab == nslabs - 1;
#pragma unroll
    for (int i = 0; i < kCopies; ++i) {
      const unsigned voff = (last ? row_off_last[i] : row_off[i]) + col_off;
      const unsigned m0v = dst + (unsigned)i * (NW * 4 * kSlabTile * 4);
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                   :: "s"(m0v), "v"(voff), "s"(base) : "memory", "m0");
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

  // The next 16*NCH pairs of each row from position `at`, chunk i holding pairs
  // [at + 16 i, at + 16 i + 16), lane t of the group holding pair t.  The loaded words are kept
  // raw (no arithmetic on them here): the compiler waits for a load at its first use, and the
  // first use is in the next stage, after the full wait that ends every stage.  32-bit byte
  // offsets from scalar bases (nnz < 2^29 is checked on the host).
  int cc[RPG][NCH], at[RPG];
  float aa[RPG][NCH];
  auto fetch_pairs = [&](int j, int from) {
    at[j] = from;
    const char* cbase = reinterpret_cast<const char*>(column_indices);
    const char* vbase = reinterpret_cast<const char*>(values);
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const unsigned o = (unsigned)min(from + l16 + 16 * i, last_nz) << 2;
      cc[j][i] = *reinterpret_cast<const int*>(cbase + o);
      aa[j][i] = *reinterpret_cast<const float*>(vbase + o);
    }
  };
  // every vector-memory operation of this wave (pair loads, slab copies) has completed
  auto wait_everything = [&]() { __builtin_amdgcn_s_waitcnt(0); };

  // One long round of row j in the slab starting at slab_start: the leading pairs of the
  // fetched 16*NCH that fall into the slab.  Returns true when all of them were used by some
  // group, i.e. the slab may hold more pairs of that row.
  // `restart`: this is the last slab of a tile and another tile follows, so once the row is done
  // here the next pairs needed are those at the row start again.
  auto long_round = [&](int j, const char* buf, int slab_start, bool restart) -> bool {
    const int idx = at[j] + l16;
    float av[NCH];
    int off[NCH], cmax[NCH];
    // Everything derived from wave masks is wave-uniform and stays in scalar registers: the
    // mask of usable pairs, the four groups' counts of leading usable pairs (one byte each in
    // `counts`), their maximum, and the groups that may go on to the next chunk.
    unsigned long long gate = ~0ull;      // groups whose previous chunk was consumed completely
    unsigned counts = 0;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const unsigned rel = (unsigned)(cc[j][i] - slab_start);
      const unsigned long long mk = __builtin_amdgcn_ballot_w64(idx + 16 * i < rows[j].row_end) &
                                    __builtin_amdgcn_ballot_w64(rel < (unsigned)S) & gate;
      const unsigned lo = (unsigned)mk, hi = (unsigned)(mk >> 32);
      const int c0 = leading16(lo & 0xffffu), c1 = leading16(lo >> 16);
      const int c2 = leading16(hi & 0xffffu), c3 = leading16(hi >> 16);
      cmax[i] = scalar_max(scalar_max(c0, c1), scalar_max(c2, c3));
      counts += (unsigned)c0 | ((unsigned)c1 << 8) | ((unsigned)c2 << 16) | ((unsigned)c3 << 24);
      if (i + 1 < NCH)
        gate = (c0 == 16 ? 0xffffull : 0ull) | (c1 == 16 ? 0xffffull << 16 : 0ull) |
               (c2 == 16 ? 0xffffull << 32 : 0ull) | (c3 == 16 ? 0xffffull << 48 : 0ull);
      // a pair inside the slab is used even if it is not among the leading ones (rows that
      // are not ascending): the cursor then stops short of the row end and the row is redone
      const bool in = __builtin_amdgcn_inverse_ballot_w64(mk);
      av[i] = in ? aa[j][i] : 0.f;
      off[i] = in ? (int)(rel * (kSlabTile * 4)) : kZeroOff;
    }
    rows[j].p += (int)((counts >> sub8) & 0xffu);
    const bool more = cmax[NCH - 1] == 16;
    // the next pairs, first needed in the next stage (or in the next long round of this one)
    fetch_pairs(j, (restart && !more) ? rows[j].p_begin : rows[j].p);
    clocks.lap(kPhaseScan);
#pragma unroll
    for (int i = 0; i < NCH; ++i)
      if (cmax[i] > 0) slab_steps(acc[j], av[i], off[i], buf, lane_b, cmax[i]);
    clocks.lap(kPhaseSteps);
    return more;
  };

  copy_stage(0);
#pragma unroll
  for (int j = 0; j < RPG; ++j) fetch_pairs(j, rows[j].p_begin);
  wait_everything();
  __builtin_amdgcn_s_barrier();
  clocks.lap(kPhaseSetup);
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
      asm volatile("v_mov_b32 %0, %0" : "+v"(aa[RPG - 1][NCH - 1]));
      clocks.lap(kPhaseRest);
      if (q + 1 < stages) copy_stage(q + 1);
      clocks.lap(kPhaseIssue);
      const char* buf = lds_raw + (q & 1) * kBufBytes;
#pragma unroll
      for (int j = 0; j < RPG; ++j) {
        const bool restart = s == nslabs - 1 && tile + 1 < tile_end;
        // The first long round stands outside the loop: inside it the compiler would have to
        // wait for the previous iteration's loads, and with them for the copies just issued.
        if (long_round(j, buf, s * S, restart))
          while (long_round(j, buf, s * S, restart)) {}          // more than 16*NCH pairs in this slab
      }
      wait_everything();
      clocks.lap(kPhaseWait);
      __builtin_amdgcn_s_barrier();
      clocks.lap(kPhaseBarrier);
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
      if (rows[j].row >= 0 && col_ok) {
        spmm_epilogue<T, 4>(acc[j], bias, rows[j].row, relu);
        Pack<T, 4>::store(C + (size_t)rows[j].row * n + col, acc[j]);
      }
    }
  }
  clocks.lap(kPhaseRest);
  clocks.store(blockIdx.x * NW + wave);
}

}  // namespace spdl
