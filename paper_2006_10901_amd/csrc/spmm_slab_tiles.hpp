// SpMM, slab family for wide outputs: the copy-based slab kernel with the loop nest turned
// round.  That kernel walks its output tiles one after the other and, inside a tile, the slabs
// of B; everything it works out about a sparse row and a slab (which of the fetched pairs lie in
// the slab, their LDS offsets, the new cursor) is worked out again for every tile, although it
// depends on the row and the slab only.  Here a workgroup keeps the accumulators of up to TPW
// tiles in registers and walks slab by slab: the pairs of a slab are scanned once, and the TPW
// stages that follow (one per tile: copy of the tile's part of the slab, multiply-adds) reuse the
// masked values and offsets from registers.  The look-ahead for the next slab is requested at the
// scan and has TPW stages to arrive.
//
// A row with more than 16*NCH pairs inside one slab needs further rounds in that slab, 16 pairs at
// a time, each behind a full wait; they are not kept, every tile's stage fetches and scans them
// again.  The host picks this kernel only where that is rare (NCH chunks cover the mean count of a
// slab plus three standard deviations).
#pragma once
#include "common.hpp"
#include "spmm_slab.hpp"

namespace spdl {

template <int S, int RPG, int NCH, int TPW>
__global__ __launch_bounds__(1024) void spmm_slab_tiles_kernel(
    int m, int k, int n, int nnz, int tiles_n, int tiles_per_wg, int panels,
    const int* __restrict__ row_offsets, const int* __restrict__ column_indices,
    const float* __restrict__ values, const int* __restrict__ row_order, const float* __restrict__ B,
    float* __restrict__ C, const float* __restrict__ bias, int relu) {
  constexpr int NW = 16;
  extern __shared__ __attribute__((aligned(16))) char lds_raw[];
  constexpr int kBufBytes = (S + 1) * kSlabTile * 4;
  constexpr int kZeroOff = S * kSlabTile * 4;
  constexpr int kCopies = S / (4 * NW);

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
  const int ntiles = min(tiles_n, tile_begin + tiles_per_wg) - tile_begin;      // 1 .. TPW
  const int nslabs = (k + S - 1) / S;
  const int stages = ntiles * nslabs;                       // stage q = (slab q / ntiles, tile q % ntiles)

  if (tid < 2 * kSlabTile)
    *reinterpret_cast<float*>(lds_raw + (tid >> 6) * kBufBytes + kZeroOff + (tid & 63) * 4) = 0.f;

  unsigned row_off[kCopies], row_off_last[kCopies];
  const int last_rows = k - (nslabs - 1) * S;
#pragma unroll
  for (int i = 0; i < kCopies; ++i) {
    const int lrow = (i * NW + wave) * 4 + sub;
    row_off[i] = (unsigned)lrow * (unsigned)n * 4u;
    row_off_last[i] = (unsigned)min(lrow, last_rows - 1) * (unsigned)n * 4u;
  }
  // Slab copies as in the copy-based kernel (issued from assembly, completion covered by the full
  // wait that ends every stage); the stages are copied in order, so source and destination are
  // running scalar state.
  const size_t slab_bytes = (size_t)S * (size_t)n * 4;
  const char* slab_base = reinterpret_cast<const char*>(B + (size_t)tile_begin * kSlabTile);
  int cp_slab = 0, cp_t = 0;
  unsigned cp_dst = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)lds_raw +
                    (unsigned)wave * (4 * kSlabTile * 4);
  unsigned cp_flip = (unsigned)kBufBytes;
  auto copy_stage = [&]() {
    const bool ragged_tile = (tile_begin + cp_t) * kSlabTile + l16 * 4 >= n;
    const unsigned col_off = ragged_tile ? 0u : (unsigned)(l16 * 16);
    const char* base = slab_base + (size_t)cp_t * (kSlabTile * 4);
    const bool last = cp_slab == nslabs - 1;
#pragma unroll
    for (int i = 0; i < kCopies; ++i) {
      const unsigned voff = (last ? row_off_last[i] : row_off[i]) + col_off;
      const unsigned m0v = cp_dst + (unsigned)i * (NW * 4 * kSlabTile * 4);
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                   :: "s"(m0v), "v"(voff), "s"(base) : "memory", "m0");
    }
    cp_dst += cp_flip;
    cp_flip = 0u - cp_flip;
    if (++cp_t == ntiles) {
      cp_t = 0;
      ++cp_slab;
      slab_base += slab_bytes;
    }
  };

  SlabRow rows[RPG];
#pragma unroll
  for (int j = 0; j < RPG; ++j) {
    const int slot = ((wave * panels + panel) * 4 + sub) * RPG + j;
    rows[j].row = -1;
    rows[j].p_begin = rows[j].row_end = 0;
    if (slot < m) {
      const int r = row_order ? row_order[slot] : slot;
      rows[j].row = r;
      rows[j].p_begin = row_offsets[r];
      rows[j].row_end = row_offsets[r + 1];
    }
    rows[j].p = rows[j].p_begin;
  }
  const int last_nz = nnz - 1;
  const int sub8 = sub * 8;
  float acc[TPW][RPG][4];
#pragma unroll
  for (int t = 0; t < TPW; ++t)
#pragma unroll
    for (int j = 0; j < RPG; ++j) acc[t][j][0] = acc[t][j][1] = acc[t][j][2] = acc[t][j][3] = 0.f;

  int cc[RPG][NCH];
  float aa[RPG][NCH];
  auto fetch_pairs = [&](int j, int from) {
    const char* cbase = reinterpret_cast<const char*>(column_indices);
    const char* vbase = reinterpret_cast<const char*>(values);
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const unsigned o = (unsigned)min(from + l16 + 16 * i, last_nz) << 2;
      cc[j][i] = *reinterpret_cast<const int*>(cbase + o);
      aa[j][i] = *reinterpret_cast<const float*>(vbase + o);
    }
  };
  auto wait_everything = [&]() { __builtin_amdgcn_s_waitcnt(0); };

  copy_stage();
#pragma unroll
  for (int j = 0; j < RPG; ++j) fetch_pairs(j, rows[j].p_begin);
  wait_everything();
  __builtin_amdgcn_s_barrier();

  int q = 0;
  for (int s = 0; s < nslabs; ++s) {
    // The scan of the slab: for every row the leading pairs of the look-ahead that lie in it.
    float av[RPG][NCH];
    int off[RPG][NCH], cmax[RPG][NCH];
    bool over[RPG];                       // wave-uniform
    const int slab_start = s * S;
#pragma unroll
    for (int j = 0; j < RPG; ++j) {
      const int idx = rows[j].p + l16;
      unsigned long long gate = ~0ull;
      unsigned counts = 0, lastc = 0;
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        const unsigned rel = (unsigned)(cc[j][i] - slab_start);
        const unsigned long long mk = __builtin_amdgcn_ballot_w64(idx + 16 * i < rows[j].row_end) &
                                      __builtin_amdgcn_ballot_w64(rel < (unsigned)S) & gate;
        const unsigned lo = (unsigned)mk, hi = (unsigned)(mk >> 32);
        const int c0 = leading16(lo & 0xffffu), c1 = leading16(lo >> 16);
        const int c2 = leading16(hi & 0xffffu), c3 = leading16(hi >> 16);
        cmax[j][i] = scalar_max(scalar_max(c0, c1), scalar_max(c2, c3));
        lastc = (unsigned)c0 | ((unsigned)c1 << 8) | ((unsigned)c2 << 16) | ((unsigned)c3 << 24);
        counts += lastc;
        if (i + 1 < NCH)
          gate = (c0 == 16 ? 0xffffull : 0ull) | (c1 == 16 ? 0xffffull << 16 : 0ull) |
                 (c2 == 16 ? 0xffffull << 32 : 0ull) | (c3 == 16 ? 0xffffull << 48 : 0ull);
        const bool in = __builtin_amdgcn_inverse_ballot_w64(mk);
        av[j][i] = in ? aa[j][i] : 0.f;
        off[j][i] = in ? (int)(rel * (kSlabTile * 4)) : kZeroOff;
      }
      rows[j].p += (int)((counts >> sub8) & 0xffu);
      // every fetched pair of some row lay in the slab: it may hold more of that row
      over[j] = cmax[j][NCH - 1] == 16;
      fetch_pairs(j, rows[j].p);
    }
    // One stage per tile: the tile's part of the slab is in LDS, the next part is on its way.
#pragma unroll
    for (int t = 0; t < TPW; ++t) {
      if (t < ntiles) {
        if (q + 1 < stages) copy_stage();
        const char* buf = lds_raw + (q & 1) * kBufBytes;
#pragma unroll
        for (int j = 0; j < RPG; ++j)
#pragma unroll
          for (int i = 0; i < NCH; ++i)
            if (cmax[j][i] > 0) slab_steps(acc[t][j], av[j][i], off[j][i], buf, lane_b, cmax[j][i]);
        // The rare rest of a row that has more pairs in this slab than the look-ahead holds.
#pragma unroll
        for (int j = 0; j < RPG; ++j) {
          if (over[j]) {
            int pe = rows[j].p;                 // where the scan stopped (the same in every tile's stage)
            while (true) {
              const unsigned o = (unsigned)min(pe + l16, last_nz) << 2;
              const int c = *reinterpret_cast<const int*>(reinterpret_cast<const char*>(column_indices) + o);
              const float a = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(values) + o);
              const unsigned rel = (unsigned)(c - slab_start);
              const unsigned long long mk = __builtin_amdgcn_ballot_w64(pe + l16 < rows[j].row_end) &
                                            __builtin_amdgcn_ballot_w64(rel < (unsigned)S);
              const unsigned lo = (unsigned)mk, hi = (unsigned)(mk >> 32);
              const int c0 = leading16(lo & 0xffffu), c1 = leading16(lo >> 16);
              const int c2 = leading16(hi & 0xffffu), c3 = leading16(hi >> 16);
              const int cm = scalar_max(scalar_max(c0, c1), scalar_max(c2, c3));
              if (cm == 0) break;
              const unsigned packed = (unsigned)c0 | ((unsigned)c1 << 8) | ((unsigned)c2 << 16) | ((unsigned)c3 << 24);
              const int cnt = (int)((packed >> sub8) & 0xffu);
              // (only the leading pairs here: one behind the first pair outside the slab belongs to
              // a row that is not ascending, which is redone at the end anyway)
              const bool in = l16 < cnt;
              const float xv = in ? a : 0.f;
              const int xo = in ? (int)(rel * (kSlabTile * 4)) : kZeroOff;
              pe += cnt;
              slab_steps(acc[t][j], xv, xo, buf, lane_b, cm);
              if (cm < 16) break;
            }
            if (t == ntiles - 1) {              // the slab is done with: the cursor and the look-ahead move on
              rows[j].p = pe;
              fetch_pairs(j, pe);
            }
          }
        }
        wait_everything();
        __builtin_amdgcn_s_barrier();
        ++q;
      }
    }
  }

#pragma unroll
  for (int t = 0; t < TPW; ++t) {
    if (t < ntiles) {
      const int col = (tile_begin + t) * kSlabTile + l16 * 4;
      const bool col_ok = col < n;
#pragma unroll
      for (int j = 0; j < RPG; ++j) {
        if (rows[j].p != rows[j].row_end) {
          acc[t][j][0] = acc[t][j][1] = acc[t][j][2] = acc[t][j][3] = 0.f;
          const float* Bcol = B + (col_ok ? col : 0);
          for (int e = rows[j].p_begin; e < rows[j].row_end; ++e) {
            const float a = values[e];
            float b[4];
            Pack<float, 4>::load(Bcol + (size_t)column_indices[e] * n, b);
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[t][j][v] = __builtin_fmaf(a, b[v], acc[t][j][v]);
          }
        }
        if (rows[j].row >= 0 && col_ok) {
          spmm_epilogue<float, 4>(acc[t][j], bias, rows[j].row, relu);
          Pack<float, 4>::store(C + (size_t)rows[j].row * n + col, acc[t][j]);
        }
      }
    }
  }
}

}  // namespace spdl
