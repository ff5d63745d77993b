// SDDMM, slab family: a workgroup owns 64 sparse rows (one panel) and a range of columns of A
// (a run of consecutive slabs of S rows of R).  Every output belongs to exactly one slab, so
// splitting the columns of A over workgroups needs no reduction.  R is streamed through LDS
// slab by slab, and for wide dot products also in chunks of 64*U columns, by producer waves
// (waves 8..15); consumer waves (0..7) compute.  Reuse of R rows across the 64 sparse rows
// of the panel replaces the per-nonzero gathers from L1/L2 of the strip kernels.
//
// In a consumer wave each 16-lane group owns two sparse rows.  A group takes strips of up to
// 16 consecutive nonzeros from its row's cursor (paper Sec. "Sampled Dense--Dense Matrix
// Multiplication": 1-D tiling over strips of consecutive nonzeros); the lanes split the
// dot-product dimension, each lane keeps one partial sum per nonzero of the strip, and a
// transposing reduction over the 16 lanes leaves nonzero t's result in lane t, which stores
// it.  Column indices are pre-scaled to LDS byte offsets and broadcast by DPP.
//
// With one column chunk (n <= 64*U) a strip is finished inside its slab, and a row takes as
// many strips per slab as it needs.  With several chunks, up to two strips (32 nonzeros) per
// row and slab keep their partial sums in registers while the chunks of the slab stream by;
// the host picks the slab height so that more than 32 is rare, and any further nonzeros of
// the row in that slab are done by direct gathers.
//
// Row ranges per column range come from a 16-way search that assumes ascending column
// indices.  Whatever the search returns, the ranges of consecutive column ranges tile the row,
// and a range whose cursor does not end exactly at its end (indices not ascending) is redone
// by direct gathers, so results are right for any CSR input.
// Needs n % 4 == 0, 16-byte aligned L and R.
#pragma once
#include "common.hpp"
#include "sddmm_group.hpp"

namespace spdl {

constexpr int kSdRows = 64;
constexpr int kSdThreads = 1024;
constexpr int kSdConsumers = 512;

// First position in [lo, hi) whose column index is >= key (ascending input assumed); all 16
// lanes of a group cooperate, every group of the wave runs its own search in lockstep.
__device__ __forceinline__ int sd_lower_bound16(const int* __restrict__ ci, int lo, int hi, int key,
                                                int sub, int l16, int last_nz) {
  while (__any(hi > lo)) {
    const int len = hi - lo;
    const int step = (len + 15) >> 4;
    const int probe = lo + (l16 + 1) * step - 1;
    const bool in = len > 0 && probe < hi;
    const int v = ci[min(max(probe, 0), last_nz)];
    const bool less = in && v < key;
    const unsigned long long mask = __ballot(less);
    const unsigned piece = (unsigned)(mask >> (sub * 16)) & 0xffffu;
    const int cnt = __builtin_ctz(~piece | 0x10000u);
    const int nlo = lo + cnt * step;
    const int nhi = min(hi, nlo + step - 1);
    lo = len > 0 ? nlo : lo;
    hi = len > 0 ? max(nhi, nlo) : hi;
  }
  return lo;
}

// NB such searches at once (lo[b], hi[b], key[b]; the result is left in lo[b]): the probes of all
// of them are loaded before any is looked at, so a round costs one memory latency however many
// searches there are.  A search with lo == hi is already finished.
//
// kcols > 0 (the number of columns of A) adds a first round that looks where the bound would be if
// the row's columns were spread evenly: sixteen probes around lo + len * key / kcols, spaced so that
// they span about eight standard deviations of that position for a random row.  Where the bound
// lies between two of them, a second round finishes the search for rows of up to a few thousand
// entries (three rounds without); where it does not, the round still halves nothing worse than the
// side it excludes, and the plain rounds go on from there.  Every round is a memory latency that
// the whole workgroup waits for before its first slab.
template <int NB>
__device__ __forceinline__ void sd_lower_bound16_batch(const int* __restrict__ ci, int (&lo)[NB], int (&hi)[NB],
                                                       const int (&key)[NB], int sub, int l16, int last_nz,
                                                       int kcols = 0) {
  bool any_open = false;
#pragma unroll
  for (int b = 0; b < NB; ++b) any_open = any_open || hi[b] > lo[b];
  if (kcols > 0 && __any(any_open)) {
    int v[NB], g0[NB], sp[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const int len = hi[b] - lo[b];
      const float f = (float)key[b] / (float)kcols;
      const float var = (float)len * f * (1.f - f);
      sp[b] = (int)(0.5f * __builtin_sqrtf(var > 0.f ? var : 0.f)) + 1;
      g0[b] = lo[b] + (int)((float)len * f) - ((15 * sp[b]) >> 1);
      const int probe = min(max(g0[b] + l16 * sp[b], lo[b]), max(hi[b] - 1, lo[b]));
      v[b] = ci[min(max(probe, 0), last_nz)];
    }
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const int len = hi[b] - lo[b];
      const bool less = len > 0 && v[b] < key[b];
      const unsigned long long mask = __ballot(less);
      const unsigned piece = (unsigned)(mask >> (sub * 16)) & 0xffffu;
      const int cnt = __builtin_ctz(~piece | 0x10000u);
      const int top = max(hi[b] - 1, lo[b]);
      const int below = min(max(g0[b] + (cnt - 1) * sp[b], lo[b]), top);      // last probe found less
      const int at = min(max(g0[b] + cnt * sp[b], lo[b]), top);               // first probe found not less
      const int nlo = cnt > 0 ? below + 1 : lo[b];
      const int nhi = cnt < 16 ? at : hi[b];
      lo[b] = len > 0 ? nlo : lo[b];
      hi[b] = len > 0 ? max(nhi, nlo) : hi[b];
    }
  }
  while (true) {
    bool open = false;
#pragma unroll
    for (int b = 0; b < NB; ++b) open = open || hi[b] > lo[b];
    if (!__any(open)) break;
    int v[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const int step = (hi[b] - lo[b] + 15) >> 4;
      const int probe = lo[b] + (l16 + 1) * step - 1;
      v[b] = ci[min(max(probe, 0), last_nz)];
    }
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const int len = hi[b] - lo[b];
      const int step = (len + 15) >> 4;
      const int probe = lo[b] + (l16 + 1) * step - 1;
      const bool less = len > 0 && probe < hi[b] && v[b] < key[b];
      const unsigned long long mask = __ballot(less);
      const unsigned piece = (unsigned)(mask >> (sub * 16)) & 0xffffu;
      const int cnt = __builtin_ctz(~piece | 0x10000u);
      const int nlo = lo[b] + cnt * step;
      const int nhi = min(hi[b], nlo + step - 1);
      lo[b] = len > 0 ? nlo : lo[b];
      hi[b] = len > 0 ? max(nhi, nlo) : hi[b];
    }
  }
}

// Out-of-line copy of the direct strip for the rare paths of the slab kernel, so that its
// registers do not count against the main loop.
template <typename T>
__device__ __attribute__((noinline)) void sd_strip_direct_call(int n, int q, int end, int l16, const T* Lrow,
                                                               const int* column_indices, const T* R, T* out,
                                                               const T* scale) {
  sddmm_strip_direct<T>(n, q, end, l16, Lrow, column_indices, R, out, scale);
}

struct SdRow {
  int row, p_start, p_end, row_end, p;
  int c_next;     // columns of the 16 nonzeros at the cursor (lane t: cursor + t)
  int c_next2;    // ... and of the 16 after them (two-strip mode only)
};

// Unconditional loads at clamped positions, so that they can stay in flight; 32-bit byte
// offsets from a scalar base (nnz < 2^29 is checked on the host).
template <bool TWO>
__device__ __forceinline__ void sd_fetch(SdRow& r, int l16, int last_nz, const int* __restrict__ ci) {
  const int idx = r.p + l16;
  const char* base = reinterpret_cast<const char*>(ci);
  const int c = *reinterpret_cast<const int*>(base + ((unsigned)min(idx, last_nz) << 2));
  r.c_next = idx < r.row_end ? c : 0x7fffffff;
  if (TWO) {
    const int c2 = *reinterpret_cast<const int*>(base + ((unsigned)min(idx + 16, last_nz) << 2));
    r.c_next2 = idx + 16 < r.row_end ? c2 : 0x7fffffff;
  }
}

// Leading nonzeros of the fetched strip that fall into [slab_start, slab_start + S): count for
// this group (cnt), maximum over the wave's groups (return value), slab-relative column.
// Everything derived from the wave mask is wave-uniform and stays in scalar registers.
template <int S>
__device__ __forceinline__ int sd_scan(int c, int slab_start, int sub, unsigned& rel, int& cnt) {
  rel = (unsigned)(c - slab_start);
  const unsigned long long mask = __builtin_amdgcn_ballot_w64(rel < (unsigned)S);
  const unsigned lo = (unsigned)mask, hi = (unsigned)(mask >> 32);
  const int c0 = __builtin_ctz(~(lo & 0xffffu) | 0x10000u), c1 = __builtin_ctz(~(lo >> 16) | 0x10000u);
  const int c2 = __builtin_ctz(~(hi & 0xffffu) | 0x10000u), c3 = __builtin_ctz(~(hi >> 16) | 0x10000u);
  const unsigned packed = (unsigned)c0 | ((unsigned)c1 << 8) | ((unsigned)c2 << 16) | ((unsigned)c3 << 24);
  cnt = (int)((packed >> (sub * 8)) & 0xffu);
  return max(max(c0, c1), max(c2, c3));
}

#define SPDL_SD_ADDR(T) (__builtin_amdgcn_update_dpp(0, off, 0x150 + (T), 0xf, 0xf, false) + lane_b)

// partial[T] (+)= dot(l, row of R at the LDS offset broadcast from lane T); with FRESH the sum
// starts from the first product instead of from a zero that would have to be written first
#define SPDL_SD_STEP(T)                                                                        \
  {                                                                                            \
    const int addr = SPDL_SD_ADDR(T);                                                          \
    _Pragma("unroll") for (int u = 0; u < U; ++u) {                                            \
      const f32x4 b = *reinterpret_cast<const f32x4*>(buf + addr + u * 256);                   \
      partial[T] = (FRESH && u == 0) ? l[u][0] * b.x : __builtin_fmaf(l[u][0], b.x, partial[T]); \
      partial[T] = __builtin_fmaf(l[u][1], b.y, partial[T]);                                   \
      partial[T] = __builtin_fmaf(l[u][2], b.z, partial[T]);                                   \
      partial[T] = __builtin_fmaf(l[u][3], b.w, partial[T]);                                   \
    }                                                                                          \
  }

// The up to 16 steps of one strip, in groups of four.  FRESH: `partial` holds nothing yet; the
// sums of the steps that are not run are set to zero (the reduction adds all sixteen).
template <int U, bool FRESH = false>
__device__ __forceinline__ void sd_steps(float (&partial)[16], const float (&l)[U][4], const char* buf,
                                         int off, int lane_b, int cmax) {
  // The empty asm statements pin each group's sums where they are computed: without them the
  // compiler sinks the multiply-adds below the following branches and keeps every LDS read
  // alive until then, which spills.
#define SPDL_SD_PIN(T0) \
  asm volatile("" : "+v"(partial[T0]), "+v"(partial[T0 + 1]), "+v"(partial[T0 + 2]), "+v"(partial[T0 + 3]));
#define SPDL_SD_ZERO(T0) \
  if (FRESH) { _Pragma("unroll") for (int z = (T0); z < 16; ++z) partial[z] = 0.f; }
  SPDL_SD_STEP(0) SPDL_SD_STEP(1) SPDL_SD_STEP(2) SPDL_SD_STEP(3)
  SPDL_SD_PIN(0)
  if (cmax > 4) {
    SPDL_SD_STEP(4) SPDL_SD_STEP(5) SPDL_SD_STEP(6) SPDL_SD_STEP(7)
    SPDL_SD_PIN(4)
    if (cmax > 8) {
      SPDL_SD_STEP(8) SPDL_SD_STEP(9) SPDL_SD_STEP(10) SPDL_SD_STEP(11)
      SPDL_SD_PIN(8)
      if (cmax > 12) {
        SPDL_SD_STEP(12) SPDL_SD_STEP(13) SPDL_SD_STEP(14) SPDL_SD_STEP(15)
        SPDL_SD_PIN(12)
      } else {
        SPDL_SD_ZERO(12)
      }
    } else {
      SPDL_SD_ZERO(8)
    }
  } else {
    SPDL_SD_ZERO(4)
  }
#undef SPDL_SD_ZERO
#undef SPDL_SD_PIN
}

template <typename T, int U, int S, bool DEFERRED>
__global__ __launch_bounds__(kSdThreads) void sddmm_slab_kernel(
    int m, int k, int n, int nnz, int ksplit, int slabs_per_part, int panels,
    const int* __restrict__ row_offsets, const int* __restrict__ column_indices,
    const T* __restrict__ L, const T* __restrict__ R, T* __restrict__ out, const T* __restrict__ scale) {
  extern __shared__ __attribute__((aligned(16))) char lds_raw[];
  constexpr int CW = 64 * U;                    // columns per stage
  constexpr int ROWB = CW * 4;                  // bytes per R row in LDS
  constexpr int kBufBytes = (S + 1) * ROWB;     // S rows of R + one all-zero row
  constexpr int kZeroOff = S * ROWB;
  constexpr int kRowsPerPass = (kSdThreads - kSdConsumers) / (16 * U);
  constexpr int kPasses = S / kRowsPerPass;     // float4 loads per producer thread per stage

  const int tid = threadIdx.x;
  // workgroup id -> (panel, column range); the ranges of one panel share an XCD
  int panel, kpart;
  if (!slab_wg_map(blockIdx.x, panels, ksplit, panel, kpart)) return;
  const int k0 = kpart * slabs_per_part * S;
  const int k1 = min(k, k0 + slabs_per_part * S);
  const int nslabs = (k1 - k0 + S - 1) / S;
  const int ncc = DEFERRED ? (n + CW - 1) / CW : 1;
  const int stages = nslabs * ncc;

  if (tid < 2 * CW)
    *reinterpret_cast<float*>(lds_raw + (tid / CW) * kBufBytes + kZeroOff + (tid % CW) * 4) = 0.f;

  if (tid >= kSdConsumers) {
    // ---------------------------------------------------------------- producer waves
    const int pt = tid - kSdConsumers;
    const int srow = pt / (16 * U);
    const int scol = (pt % (16 * U)) * 4;
    float stage[2][kPasses][4];
    const int last_stage = stages - 1;
    auto gload = [&](int q, float (&st)[kPasses][4]) {
      q = min(q, last_stage);
      const int slab = q / ncc;
      const int cc = q - slab * ncc;
      const int colg = cc * CW + scol;
      const T* src = R + (colg < n ? colg : 0);
#pragma unroll
      for (int j = 0; j < kPasses; ++j) {
        const int r = min(k0 + slab * S + j * kRowsPerPass + srow, k - 1);
        Pack<T, 4>::load(src + (size_t)r * n, st[j]);
      }
    };
    auto lstore = [&](int q, const float (&st)[kPasses][4]) {
      char* dst = lds_raw + (q & 1) * kBufBytes;
#pragma unroll
      for (int j = 0; j < kPasses; ++j) {
        f32x4 v = {st[j][0], st[j][1], st[j][2], st[j][3]};
        *reinterpret_cast<f32x4*>(dst + (j * kRowsPerPass + srow) * ROWB + scol * 4) = v;
      }
    };
    gload(0, stage[0]);
    gload(1, stage[1]);
    lstore(0, stage[0]);
    __syncthreads();
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
  const int last_nz = nnz - 1;

  SdRow rows[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int row = panel * kSdRows + (wave * 4 + sub) * 2 + j;
    SdRow& r = rows[j];
    r.row = row < m ? row : -1;
    const int rb = row < m ? row_offsets[row] : 0;
    r.row_end = row < m ? row_offsets[row + 1] : 0;
    // [p_start, p_end): this row's nonzeros with column in [k0, k1) if the row is ascending
    r.p_start = k0 <= 0 ? rb : sd_lower_bound16(column_indices, rb, r.row_end, k0, sub, l16, last_nz);
    r.p_end = k1 >= k ? r.row_end : sd_lower_bound16(column_indices, rb, r.row_end, k1, sub, l16, last_nz);
    r.p_end = max(r.p_end, r.p_start);
    r.p = r.p_start;
    sd_fetch<DEFERRED>(r, l16, last_nz, column_indices);
  }

  float l[2][U][4];
  auto load_l = [&](int cc, float (&dst)[2][U][4]) {
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int u = 0; u < U; ++u) {
        // unconditional load at a clamped position, zeroed afterwards where out of range
        const int col = cc * CW + u * 64 + 4 * l16;
        const bool ok = col < n && rows[j].row >= 0;
        Pack<T, 4>::load(L + (size_t)(ok ? rows[j].row : 0) * n + (ok ? col : 0), dst[j][u]);
        if (!ok) dst[j][u][0] = dst[j][u][1] = dst[j][u][2] = dst[j][u][3] = 0.f;
      }
  };
  float l_next[2][U][4];          // L slices of the next column chunk, fetched a stage ahead
  if (DEFERRED) load_l(0, l_next);
  else load_l(0, l);

  __syncthreads();
  int q = 0;
  for (int s = 0; s < nslabs; ++s) {
    const int slab_start = k0 + s * S;
    if constexpr (!DEFERRED) {
      const char* buf = lds_raw + (q & 1) * kBufBytes;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        SdRow& r = rows[j];
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
          sd_steps<U, true>(partial, l[j], buf, off, lane_b, cmax);
          const float total = reduce16x16(partial, l16);
          if (l16 < cnt) sddmm_store<T>(out, scale, p_old + l16, total);
          if (cmax < 16) break;
        }
      }
      __syncthreads();
      ++q;
    } else {
      float partial[2][2][16];                 // [row][strip][nonzero]
      int off[2][2], cnt[2][2], cmax[2][2], p_old[2];
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        unsigned rel;
        cmax[j][0] = sd_scan<S>(rows[j].c_next, slab_start, sub, rel, cnt[j][0]);
        off[j][0] = l16 < cnt[j][0] ? (int)(rel * ROWB) : kZeroOff;
        int c1;
        cmax[j][1] = sd_scan<S>(rows[j].c_next2, slab_start, sub, rel, c1);
        c1 = cnt[j][0] == 16 ? c1 : 0;          // the second strip only continues a full first one
        cnt[j][1] = c1;
        cmax[j][1] = cmax[j][0] == 16 ? cmax[j][1] : 0;
        off[j][1] = l16 < c1 ? (int)(rel * ROWB) : kZeroOff;
        p_old[j] = rows[j].p;
        rows[j].p += cnt[j][0] + c1;
        sd_fetch<true>(rows[j], l16, last_nz, column_indices);
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int t = 0; t < 16; ++t) partial[j][h][t] = 0.f;
      }
      for (int cc = 0; cc < ncc; ++cc, ++q) {
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int u = 0; u < U; ++u)
#pragma unroll
            for (int v = 0; v < 4; ++v) l[j][u][v] = l_next[j][u][v];
        load_l(cc + 1 < ncc ? cc + 1 : 0, l_next);
        const char* buf = lds_raw + (q & 1) * kBufBytes;
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int h = 0; h < 2; ++h)
            if (cmax[j][h] > 0) sd_steps<U>(partial[j][h], l[j], buf, off[j][h], lane_b, cmax[j][h]);
        __syncthreads();
      }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        SdRow& r = rows[j];
#pragma unroll
        for (int h = 0; h < 2; ++h)
          if (cmax[j][h] > 0) {
            const float total = reduce16x16(partial[j][h], l16);
            if (l16 < cnt[j][h]) sddmm_store<T>(out, scale, p_old[j] + 16 * h + l16, total);
          }
        // more than 32 nonzeros of this row in this slab: the rest by direct gathers
        int more = cmax[j][1];
        while (more == 16) {
          unsigned rel;
          int c2;
          more = sd_scan<S>(r.c_next, slab_start, sub, rel, c2);
          if (more == 0) break;
          if (c2 > 0)
            sd_strip_direct_call<T>(n, r.p, r.p + c2, l16, L + (size_t)max(r.row, 0) * n, column_indices, R, out, scale);
          r.p += c2;
          sd_fetch<true>(r, l16, last_nz, column_indices);
        }
      }
    }
  }

  // A range whose cursor did not stop exactly at its end was not ascending: redo it directly.
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const SdRow& r = rows[j];
    if (r.p != r.p_end && r.row >= 0)
      for (int t = r.p_start; t < r.p_end; t += 16)
        sd_strip_direct_call<T>(n, t, r.p_end, l16, L + (size_t)r.row * n, column_indices, R, out, scale);
  }
}

#undef SPDL_SD_STEP
#undef SPDL_SD_ADDR

}  // namespace spdl
