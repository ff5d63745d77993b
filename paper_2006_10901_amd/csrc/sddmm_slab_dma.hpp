// SDDMM, slab family with asynchronous global->LDS copies: same decomposition as the
// producer/consumer slab kernel (64 sparse rows and a run of slabs of R per workgroup, strips of
// 16 nonzeros per 16-lane group, transposing reduction), but all 16 waves compute, one sparse
// row per 16-lane group, and each wave moves its share of the next stage with direct-to-LDS
// loads (no staging registers, no LDS store instructions).
#pragma once
#include "common.hpp"
#include "sddmm_slab.hpp"

namespace spdl {

template <int U, int S, bool DEFERRED>
__global__ __launch_bounds__(kSdThreads) void sddmm_slab_dma_kernel(
    int m, int k, int n, int nnz, int ksplit, int slabs_per_part, int panels,
    const int* __restrict__ row_offsets, const int* __restrict__ column_indices,
    const float* __restrict__ L, const float* __restrict__ R, float* __restrict__ out,
    const float* __restrict__ scale, const int* __restrict__ row_order) {
  using T = float;
  extern __shared__ __attribute__((aligned(16))) char lds_raw[];
  constexpr int CW = 64 * U;                    // columns per stage
  constexpr int ROWB = CW * 4;                  // bytes per R row in LDS
  constexpr int kBufBytes = (S + 1) * ROWB;     // S rows of R + one all-zero row
  constexpr int kZeroOff = S * ROWB;
  constexpr int kRowsPerCopy = 1024 / ROWB;     // slab rows moved by one 1 KB wave copy
  constexpr int kCopies = S / kRowsPerCopy / 16;  // copies per wave per stage
  constexpr int kLanesPerRow = 64 / kRowsPerCopy;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = uniform(tid >> 6);
  const int sub = lane >> 4;
  const int l16 = lane & 15;
  const int lane_b = l16 * 16;
  const int last_nz = nnz - 1;

  int panel, kpart;
  if (!slab_wg_map(blockIdx.x, panels, ksplit, panel, kpart)) return;
  const int k0 = kpart * slabs_per_part * S;
  const int k1 = min(k, k0 + slabs_per_part * S);
  const int nslabs = (k1 - k0 + S - 1) / S;
  const int ncc = DEFERRED ? (n + CW - 1) / CW : 1;
  const int stages = nslabs * ncc;
  const int last_stage = stages - 1;

  if (tid < 2 * CW)
    *reinterpret_cast<float*>(lds_raw + (tid / CW) * kBufBytes + kZeroOff + (tid % CW) * 4) = 0.f;

  // Copy i of wave w fills slab rows (i*16 + w)*kRowsPerCopy .. ; lane L brings 16 bytes of row
  // L / kLanesPerRow, and the hardware places lane L's bytes at M0 + 16*L.  The address is a
  // scalar base (start of the slab and column chunk in R, moved from stage to stage with scalar
  // arithmetic) plus a per-lane byte offset that is the same in every stage except a ragged
  // last slab, whose rows past k are clamped to row k-1, and a ragged last column chunk, whose
  // columns past n are clamped to the chunk's first column: nothing valid ever reads those.
  // (S * n * 4 < 2^31 is checked on the host.)
  unsigned row_off[kCopies], row_off_last[kCopies];
  const int last_rows = k - (k0 + (nslabs - 1) * S);        // rows of the last slab, 1..S
#pragma unroll
  for (int i = 0; i < kCopies; ++i) {
    const int lrow = (i * 16 + wave) * kRowsPerCopy + lane / kLanesPerRow;
    row_off[i] = (unsigned)lrow * (unsigned)n * 4u;
    row_off_last[i] = (unsigned)min(lrow, last_rows - 1) * (unsigned)n * 4u;
  }
  // The copies are issued from inline assembly: the compiler treats its own direct-to-LDS loads
  // as touching both memory paths and then turns every later wait, for LDS reads and for index
  // loads alike, into a wait for everything.  Their completion is covered by the explicit full
  // wait and barrier that end every stage.  M0 (the LDS destination) is not used by anything
  // the compiler generates in this kernel.
  auto copy_stage = [&](int q) {
    q = min(q, last_stage);
    const int slab = q / ncc;
    const int cc = q - slab * ncc;
    const int lcol = (lane % kLanesPerRow) * 4;
    const unsigned col_off = cc * CW + lcol < n ? (unsigned)(lcol * 4) : 0u;
    const char* base = reinterpret_cast<const char*>(R + (size_t)(k0 + slab * S) * n + cc * CW);
    const unsigned dst = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)(lds_raw + (q & 1) * kBufBytes) +
                         (unsigned)wave * 1024u;
    const bool last = slab == nslabs - 1;
#pragma unroll
    for (int i = 0; i < kCopies; ++i) {
      const unsigned voff = (last ? row_off_last[i] : row_off[i]) + col_off;
      const unsigned m0v = dst + (unsigned)i * (16u * 1024u);
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                   :: "s"(m0v), "v"(voff), "s"(base) : "memory", "m0");
    }
  };

  SdRow r;
  {
    // With a row order (rows by decreasing length): the four rows of a wave are adjacent in the
    // order and a workgroup takes every panels-th such bundle, as in SpMM.
    const int slot = row_order ? (wave * panels + panel) * 4 + sub : panel * kSdRows + wave * 4 + sub;
    const int row = slot < m && row_order ? row_order[slot] : slot;
    r.row = row < m ? row : -1;
    const int rb = row < m ? row_offsets[row] : 0;
    r.row_end = row < m ? row_offsets[row + 1] : 0;
    // both ends of the range side by side, the first round of probes placed by interpolation: two
    // memory latencies before the first slab instead of six
    int lo[2] = {rb, k1 >= k ? r.row_end : rb}, hi[2] = {k0 <= 0 ? rb : r.row_end, r.row_end};
    const int key[2] = {k0, k1};
    sd_lower_bound16_batch<2>(column_indices, lo, hi, key, sub, l16, last_nz, k);
    r.p_start = lo[0];
    r.p_end = max(lo[1], r.p_start);
    r.p = r.p_start;
    sd_fetch<DEFERRED>(r, l16, last_nz, column_indices);
  }
  const T* Lrow = L + (size_t)max(r.row, 0) * n;

  float l[U][4];
  auto load_l = [&](int cc, float (&dst)[U][4]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int col = cc * CW + u * 64 + 4 * l16;
      const bool ok = col < n && r.row >= 0;
      Pack<T, 4>::load(Lrow + (ok ? col : 0), dst[u]);
      if (!ok) dst[u][0] = dst[u][1] = dst[u][2] = dst[u][3] = 0.f;
    }
  };
  float l_next[U][4];
  if (DEFERRED) load_l(0, l_next);
  else load_l(0, l);

  copy_stage(0);
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  int q = 0;
  for (int s = 0; s < nslabs; ++s) {
    const int slab_start = k0 + s * S;
    if constexpr (!DEFERRED) {
      copy_stage(q + 1);
      const char* buf = lds_raw + (q & 1) * kBufBytes;
      while (true) {
        unsigned rel;
        int cnt;
        const int cmax = sd_scan<S>(r.c_next, slab_start, sub, rel, cnt);
        if (cmax == 0) break;
        const int off = l16 < cnt ? (int)(rel * ROWB) : kZeroOff;
        const int p_old = r.p;
        r.p += cnt;
        sd_fetch<false>(r, l16, last_nz, column_indices);
        float partial[16];
        sd_steps<U, true>(partial, l, buf, off, lane_b, cmax);
        const float total = reduce16x16(partial, l16);
        if (l16 < cnt) sddmm_store<T>(out, scale, p_old + l16, total);
        if (cmax < 16) break;
      }
      __builtin_amdgcn_s_waitcnt(0);
      __syncthreads();
      ++q;
    } else {
      float partial[2][16];
      int off[2], cnt[2], cmax[2];
      unsigned rel;
      cmax[0] = sd_scan<S>(r.c_next, slab_start, sub, rel, cnt[0]);
      off[0] = l16 < cnt[0] ? (int)(rel * ROWB) : kZeroOff;
      int c1;
      cmax[1] = sd_scan<S>(r.c_next2, slab_start, sub, rel, c1);
      c1 = cnt[0] == 16 ? c1 : 0;              // the second strip only continues a full first one
      cnt[1] = c1;
      cmax[1] = cmax[0] == 16 ? cmax[1] : 0;
      off[1] = l16 < c1 ? (int)(rel * ROWB) : kZeroOff;
      const int p_old = r.p;
      r.p += cnt[0] + c1;
      sd_fetch<true>(r, l16, last_nz, column_indices);
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int t = 0; t < 16; ++t) partial[h][t] = 0.f;
      for (int cc = 0; cc < ncc; ++cc, ++q) {
        copy_stage(q + 1);
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
          for (int v = 0; v < 4; ++v) l[u][v] = l_next[u][v];
        load_l(cc + 1 < ncc ? cc + 1 : 0, l_next);
        const char* buf = lds_raw + (q & 1) * kBufBytes;
#pragma unroll
        for (int h = 0; h < 2; ++h)
          if (cmax[h] > 0) sd_steps<U>(partial[h], l, buf, off[h], lane_b, cmax[h]);
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
      }
#pragma unroll
      for (int h = 0; h < 2; ++h)
        if (cmax[h] > 0) {
          const float total = reduce16x16(partial[h], l16);
          if (l16 < cnt[h]) sddmm_store<T>(out, scale, p_old + 16 * h + l16, total);
        }
      // more than 32 nonzeros of this row in this slab: the rest by direct gathers
      int more = cmax[1];
      while (more == 16) {
        int c2;
        more = sd_scan<S>(r.c_next, slab_start, sub, rel, c2);
        if (more == 0) break;
        if (c2 > 0) sd_strip_direct_call<T>(n, r.p, r.p + c2, l16, Lrow, column_indices, R, out, scale);
        r.p += c2;
        sd_fetch<true>(r, l16, last_nz, column_indices);
      }
    }
  }

  // A range whose cursor did not stop exactly at its end was not ascending: redo it directly.
  if (r.p != r.p_end && r.row >= 0)
    for (int t = r.p_start; t < r.p_end; t += 16)
      sd_strip_direct_call<T>(n, t, r.p_end, l16, Lrow, column_indices, R, out, scale);
}

}  // namespace spdl
