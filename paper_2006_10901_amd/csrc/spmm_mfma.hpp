// SpMM in mixed precision on the matrix cores (paper Sec. "Mixed Precision": fp16 operands,
// fp32 accumulation).  A panel of 32 sparse rows is expanded into a dense fp16 block in LDS
// (zeros where A stores nothing) and multiplied with MFMA: on this chip the dense fp16 matrix
// rate is some thirty times the fp32 vector rate, so for the moderately sparse matrices of deep
// learning the multiplications by zero cost less than gathering one row of B per stored entry.
// Sparsity still saves the memory and the traffic of A.
//
// A workgroup owns one panel (32 or 64 rows) and WAVES tiles of 256 output columns.  The panel
// is expanded once per chunk of up to kMfmaChunk columns of A and shared by the waves.  For a
// step of 16 columns of A, lane (c, h) of a wave loads rows k0+8h .. k0+8h+7 of B, columns
// n0+8c .. n0+8c+7 (eight 16-byte loads; the 32 lanes of a half read 512 contiguous bytes of each
// row), transposes the 8x8 block inside its registers with byte permutes, and so obtains, for
// each j < 8, the second MFMA operand of the 32 output columns n0+8c+j: B needs no staging and
// no transposed copy although the contraction runs over its slow dimension.  The eight
// results of a lane for one row are eight adjacent columns: one 16-byte store.
//
// Rows whose indices are not strictly ascending (duplicates included) cannot be expanded by
// plain stores; they are found while the panel is filled and computed by direct gathers.
// Needs n % 8 == 0, k >= 16 and 16-byte aligned B and C.  The row order is not used: dense work
// is the same for every row.
//
// What bounds it: every MFMA of a 32-row panel needs a fresh 1 KB fragment of B, and a CU's
// vector memory path delivers about 64 bytes per clock (some 100-120 GB/s measured for
// L2-resident data with copy-only kernels) against the 32 clocks of an MFMA: the main loop runs
// at the rate at which B arrives (1 MB per workgroup), not at the matrix cores' rate.  Timed
// inside the kernel on the 1x1 convolution (k = 1024, n = 3136; 20 us in all): 2.4 us until the
// first loads are out, 4 us to clear and fill the panel (mostly waiting for loads), 10.6 us main
// loop, 1.1 us to add the two k-parts, 1.9 us to convert and store.
#pragma once
#include "common.hpp"
#include "sddmm_mfma.hpp"

namespace spdl {

constexpr int kMfmaChunk = 1024;         // columns of A expanded at a time
constexpr int kMfmaSets = 6;             // steps of B rows held in registers per wave
constexpr int kMfmaPad = 8;              // halves of padding per panel row: row stride = 16 mod 128 bytes

// LDS: the panel of 32*rb rows (reused at the end to add up the k-parts' accumulators, rb * 32 KB
// per tile), the flags of rows that cannot be expanded.
__host__ __device__ __forceinline__ int spmm_mfma_lds_bytes(int k, int waves, int rb) {
  const int kc = ((k + 15) & ~15) < kMfmaChunk ? ((k + 15) & ~15) : kMfmaChunk;
  const int panel = 32 * rb * (kc + kMfmaPad) * 2, sums = waves * rb * 128 * 64 * 4;
  return (panel > sums ? panel : sums) + 32 * rb * 4;
}

// WAVES tiles of 256 columns per workgroup, and KP waves per tile that split the steps of the
// contraction between them (more loads in flight per CU; their accumulators are added up
// through LDS at the end).  RB blocks of 32 rows per panel: with two, every fragment of B feeds
// two MFMAs and B is read from L2 half as often.
template <int WAVES, int KP, typename I = int, int RB = 1>
__global__ __launch_bounds__(64 * WAVES * KP) void spmm_mfma_kernel(
    int m, int k, int n, int tiles_n, const int* __restrict__ row_offsets,
    const I* __restrict__ column_indices, const _Float16* __restrict__ values,
    const _Float16* __restrict__ B, _Float16* __restrict__ C, const _Float16* __restrict__ bias, int relu) {
  extern __shared__ __attribute__((aligned(16))) char lds_raw[];
  constexpr int THREADS = 64 * WAVES * KP;
  const int kc_max = min((k + 15) & ~15, kMfmaChunk);
  const int stride = kc_max + kMfmaPad;                 // halves per panel row
  _Float16* panel = reinterpret_cast<_Float16*>(lds_raw);
  constexpr int PR = 32 * RB;                           // rows of the panel
  int* bad = reinterpret_cast<int*>(lds_raw + spmm_mfma_lds_bytes(k, WAVES, RB) - PR * 4);   // rows that cannot be expanded

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = uniform(tid >> 6);
  const int tile_w = wave % WAVES;                      // which of the workgroup's tiles
  const int kpart = wave / WAVES;                       // which share of the steps
  const int c = lane & 31;
  const int h = lane >> 5;
  const int groups = (tiles_n + WAVES - 1) / WAVES;
  const int panel_id = blockIdx.x / groups;
  const int tile = (blockIdx.x - panel_id * groups) * WAVES + tile_w;
  const bool active = tile < tiles_n;                   // idle waves still take part in the barriers
  const int i0 = panel_id * PR;
  const int n0 = tile * 256;
  const int col = n0 + 8 * c;                           // this lane's eight output columns
  const bool col_ok = active && col < n;
  const _Float16* bp = B + (col_ok ? col : 0);

  if (tid < PR) bad[tid] = 0;

  f32x16 acc[RB][8];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int t = 0; t < 16; ++t) acc[rb][j][t] = 0.f;

  // Where each of this wave's rows continues in the next chunk of columns (rows in ascending order:
  // the entries of a chunk follow those of the chunk before).  The first chunk walks whole rows,
  // which is also what finds the rows that are not ascending; later chunks start at the cursor and
  // stop at the first 64 entries that reach past the chunk.
  int cursor[(32 * RB) / (THREADS / 64)];
  for (int kc0 = 0; kc0 < k; kc0 += kMfmaChunk) {
    const int kc = min(k - kc0, kMfmaChunk);
    const int all_steps = (kc + 15) >> 4;
    const int per_part = (all_steps + KP - 1) / KP;
    const int s_begin = min(all_steps, kpart * per_part);
    const int steps = min(all_steps, s_begin + per_part) - s_begin;      // this wave's steps: s_begin ..
    // Second operand source: rows kc0 + 16*(s_begin + s) + 8h + r of B, r < 8: a scalar base that
    // moves with the step and the row plus this lane's fixed 32-bit byte offset (8h rows down,
    // `col` columns in), so a load needs no vector arithmetic at all.  The loads are issued from
    // inline assembly and waited for with explicit counts (they complete in the order issued, and
    // inside the main loop they are the only vector-memory operations): the compiler's own
    // placement of waits made every step wait for all loads in flight, which left one step's
    // loads to cover the whole latency.  A wait names the registers it releases as operands, so
    // that no use of them can be moved above it.  The one step that would reach past the last
    // row of B (k % 16 != 0) is kept out of this pipeline and done at the end with clamped rows
    // (the panel holds zeros there).
    // (rows of B are kept as four 32-bit words each: the byte permutes work on those)
    constexpr int NS = RB == 1 ? kMfmaSets : 4;        // register sets: loads run NS-1 steps ahead
    u32x4 w[NS][8];
    const unsigned lane_off = (unsigned)((8 * h * n + (col_ok ? col : 0)) * 2);
    const bool ragged_last = kc0 + 16 * (s_begin + steps) > k && steps > 0;   // this wave's last step is the ragged one
    const int full_steps = steps - (ragged_last ? 1 : 0);
    // A step past this wave's last full one loads nothing useful: it re-reads the start of rows 0
    // and 8 of B (cache hits; k >= 16 is required), so that the number of loads behind any set is
    // the same at every step and one wait count serves them all.  The vector offset is the same
    // register for every load of the kernel.
    auto load_rows = [&](int s, u32x4 (&ws)[8]) {
      const bool real = s < full_steps;
      const char* base = reinterpret_cast<const char*>(B + (real ? (size_t)(kc0 + 16 * (s_begin + s)) * n : (size_t)0));
      const size_t row_bytes = real ? (size_t)n * 2 : (size_t)0;
      const unsigned voff = lane_off;
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        const char* row_base = base + (size_t)r * row_bytes;
        asm volatile("global_load_dwordx4 %0, %1, %2" : "=&v"(ws[r]) : "v"(voff), "s"(row_base) : "memory");
      }
    };
    // the set is complete once only the NS - 1 later sets (8 loads each) are outstanding
    auto await_rows = [&](u32x4 (&ws)[8]) {
      static_assert(NS == 6 || NS == 4, "wait counts below");
      if constexpr (NS == 6)
        asm volatile("s_waitcnt vmcnt(40)"
                     : "+v"(ws[0]), "+v"(ws[1]), "+v"(ws[2]), "+v"(ws[3]), "+v"(ws[4]), "+v"(ws[5]), "+v"(ws[6]),
                       "+v"(ws[7])::"memory");
      else
        asm volatile("s_waitcnt vmcnt(24)"
                     : "+v"(ws[0]), "+v"(ws[1]), "+v"(ws[2]), "+v"(ws[3]), "+v"(ws[4]), "+v"(ws[5]), "+v"(ws[6]),
                       "+v"(ws[7])::"memory");
    };
    // keeps a set's registers allocated up to this point (a load into them may still be in flight)
    auto hold_rows = [&](u32x4 (&ws)[8]) {
      asm volatile("" : "+v"(ws[0]), "+v"(ws[1]), "+v"(ws[2]), "+v"(ws[3]), "+v"(ws[4]), "+v"(ws[5]), "+v"(ws[6]),
                   "+v"(ws[7])::"memory");
    };
    if (active) {
      // the first loads go out before the panel is built: they do not depend on it
#pragma unroll
      for (int u = 0; u < NS - 1; ++u) load_rows(u, w[u]);
    }
    // Expansion.  A wave takes every fourth row of the panel (or so: one in THREADS/64) and its
    // lanes take the row's entries 64 at a time: coalesced loads, no search for the row of an
    // entry, and the loads of each row's first 128 entries are all issued before the panel is
    // even cleared.  Longer rows finish in a loop.  An entry whose column is not above its
    // predecessor's marks the row as not expandable (the predecessor is the lane below, or lane
    // 63 of the previous 64).
    constexpr int NW = THREADS / 64, RW = PR / NW;       // waves, rows per wave
    constexpr int PRE = RB == 1 ? 2 : 1;                // sixty-fours of a row fetched ahead
    int row_begin[RW], row_end[RW];
    int cfirst[RW][PRE];
    _Float16 afirst[RW][PRE];
#pragma unroll
    for (int i = 0; i < RW; ++i) {
      const int rr = wave + NW * i;
      row_begin[i] = uniform(row_offsets[min(i0 + rr, m)]);
      row_end[i] = uniform(row_offsets[min(i0 + rr + 1, m)]);
      if (kc0 > 0) row_begin[i] = cursor[i];
    }
    const int kend = kc0 + kc;
#pragma unroll
    for (int i = 0; i < RW; ++i)
#pragma unroll
      for (int e = 0; e < PRE; ++e) {
        const int p = row_begin[i] + 64 * e + lane;
        cfirst[i][e] = 0;
        afirst[i][e] = (_Float16)0.f;
        if (p < row_end[i]) {
          cfirst[i][e] = (int)column_indices[p];
          afirst[i][e] = values[p];
        }
      }
    __syncthreads();                                     // the previous chunk's reads are done
    for (int o = tid * 16; o < PR * stride * 2; o += THREADS * 16)
      *reinterpret_cast<f32x4*>(lds_raw + o) = f32x4{0.f, 0.f, 0.f, 0.f};
    __syncthreads();
#pragma unroll
    for (int i = 0; i < RW; ++i) {
      const int rr = wave + NW * i;
      _Float16* prow = panel + rr * stride;
      int below = 0;                                     // column of the previous 64's lane 63
      bool unordered = false;
      int before_end = 0;                                // entries seen whose column lies before the chunk's end
      bool past = false;                                 // some entry seen lies past the chunk
      auto place = [&](int p, int cidx, _Float16 a, bool head) {
        const int prev = __shfl_up(cidx, 1);
        const bool valid = p < row_end[i];
        if (valid) {
          if (!head && (lane == 0 ? below : prev) >= cidx) unordered = true;
          const unsigned rel = (unsigned)(cidx - kc0);
          if (rel < (unsigned)kc) prow[rel] = a;
        }
        if (k > kMfmaChunk) {                            // (one chunk: no cursor to keep)
          const unsigned long long inside = __builtin_amdgcn_ballot_w64(valid && cidx < kend);
          before_end += __builtin_popcountll(inside);
          past = past || __builtin_amdgcn_ballot_w64(valid && cidx >= kend) != 0;
        }
        below = __builtin_amdgcn_readlane(cidx, 63);
      };
#pragma unroll
      for (int e = 0; e < PRE; ++e)
        if (row_begin[i] + 64 * e < row_end[i])
          place(row_begin[i] + 64 * e + lane, cfirst[i][e], afirst[i][e], e == 0 && lane == 0);
      for (int base = row_begin[i] + 64 * PRE; base < row_end[i]; base += 256) {   // long rows: 256 entries per round
        if (kc0 > 0 && past) break;                      // (ascending rows: nothing further belongs to this chunk)
        int cmore[4];
        _Float16 amore[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int q = min(base + 64 * e + lane, row_end[i] - 1);
          cmore[e] = (int)column_indices[q];
          amore[e] = values[q];
        }
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (base + 64 * e < row_end[i]) place(base + 64 * e + lane, cmore[e], amore[e], false);
      }
      if (kc0 == 0 && __builtin_amdgcn_ballot_w64(unordered) != 0 && lane == 0) bad[rr] = 1;
      cursor[i] = row_begin[i] + before_end;
    }
    // Some of the expansion's loads are used on one path only; the compiler would otherwise wait
    // for them inside the main loop, where its wait also drains the loads of B.  (vmcnt 0; the
    // other two counters are left alone.)
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    if (active) {
      // first operands: rows c, 32 + c, .. of the panel, columns 16*s + 8h .. +7 of the chunk
      const _Float16* ap = panel + c * stride + 8 * h + 16 * s_begin;
      // (the fragment of a step is read from LDS one step ahead: with one wave per SIMD nothing
      // else would cover the LDS latency)
      f16x8 a_next[RB];
      auto read_panel = [&](int s) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) a_next[rb] = *reinterpret_cast<const f16x8*>(ap + 32 * rb * stride + 16 * s);
      };
      auto step = [&](int s, const u32x4 (&ws)[8]) {
        f16x8 a[RB];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) a[rb] = a_next[rb];
        if (s + 1 < steps) read_panel(s + 1);
        // 8x8 transpose of halves inside the lane: operand j, word q = (ws[2q][j], ws[2q+1][j])
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          u32x4 packed;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const unsigned sel = (j & 1) ? 0x07060302u : 0x05040100u;
            packed[q] = __builtin_amdgcn_perm(ws[2 * q + 1][j / 2], ws[2 * q][j / 2], sel);
          }
#pragma unroll
          for (int rb = 0; rb < RB; ++rb)
            acc[rb][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[rb], __builtin_bit_cast(f16x8, packed), acc[rb][j],
                                                                0, 0, 0);
        }
      };
      if (steps > 0) read_panel(0);
      for (int s0 = 0; s0 < full_steps; s0 += NS) {
#pragma unroll
        for (int u = 0; u < NS; ++u) {
          const int s = s0 + u;
          load_rows(s + NS - 1, w[(u + NS - 1) % NS]);
          await_rows(w[u]);
          if (s < full_steps) step(s, w[u]);
        }
      }
      // the loads still in flight fetch nothing that is used; they must land before their
      // registers serve anything else
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
      for (int u = 0; u < NS; ++u) hold_rows(w[u]);
      if (ragged_last) {
        const int k0 = kc0 + 16 * (s_begin + full_steps);
        u32x4 tail[8];
#pragma unroll
        for (int r = 0; r < 8; ++r)
          tail[r] = *reinterpret_cast<const u32x4*>(bp + (size_t)min(k0 + 8 * h + r, k - 1) * n);
        step(full_steps, tail);
      }
    }
  }
  // The k-parts' accumulators are added up through LDS (the panel is no longer needed), one
  // part at a time: elements (rb, j, 4g .. 4g+3) of lane l of tile w are the four floats at index
  // ((((w*RB + rb)*8 + j)*4 + g)*64 + l)*4, so both sides move 16 bytes per access.  The last
  // part is not added into the accumulators (which live in the accumulation registers: reading,
  // adding and writing them back costs three instructions per element) but on the way out, when
  // they are read for the stores anyway.
  f32x4* sums = reinterpret_cast<f32x4*>(lds_raw) + tile_w * (RB * 32 * 64) + lane;
  auto put_sums = [&]() {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g)
          sums[((rb * 8 + j) * 4 + g) * 64] =
              f32x4{acc[rb][j][4 * g], acc[rb][j][4 * g + 1], acc[rb][j][4 * g + 2], acc[rb][j][4 * g + 3]};
  };
  for (int q = 1; q + 1 < KP; ++q) {
    __syncthreads();
    if (kpart == q) put_sums();
    __syncthreads();
    if (kpart == 0) {
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const f32x4 v = sums[((rb * 8 + j) * 4 + g) * 64];
#pragma unroll
            for (int t = 0; t < 4; ++t) acc[rb][j][4 * g + t] += v[t];
          }
    }
  }
  __syncthreads();
  if constexpr (KP > 1) {
    if (kpart == KP - 1) put_sums();
    __syncthreads();
  }
  if (!active || kpart != 0) return;

  // which rows could not be expanded, as a mask in scalar registers
  const unsigned long long bad_mask = __builtin_amdgcn_ballot_w64(lane < PR && bad[lane & (PR - 1)] != 0);

  // Register t of lane (c, h) in accumulator (rb, j) is row 32*rb + 8*(t/4) + 4h + t%4, column
  // n0 + 8c + j.
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      f32x4 last[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) last[j] = KP > 1 ? sums[((rb * 8 + j) * 4 + g) * 64] : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) {
        const int rr = 32 * rb + 8 * g + 4 * h + tt;
        const int row = i0 + rr;
        if (row < m && col_ok && !((bad_mask >> rr) & 1)) {
          float v[8];
#pragma unroll
          for (int j = 0; j < 8; ++j) v[j] = acc[rb][j][4 * g + tt] + last[j][tt];
          spmm_epilogue<_Float16, 8>(v, bias, row, relu);
          Pack<_Float16, 8>::store(C + (size_t)row * n + col, v);
        }
      }
    }
  // rows that could not be expanded: direct gathers, four columns per lane
  for (unsigned long long left = bad_mask; left != 0; left &= left - 1) {
    const int rr = __builtin_ctzll(left);
    const int row = i0 + rr;
    const int col4 = n0 + 4 * lane;
    const bool ok = col4 < n;
    float v[4] = {0.f, 0.f, 0.f, 0.f};
    for (int p = row_offsets[row]; p < row_offsets[row + 1]; ++p) {
      const float a = (float)values[p];
      float b[4];
      Pack<_Float16, 4>::load(B + (size_t)(int)column_indices[p] * n + (ok ? col4 : 0), b);
#pragma unroll
      for (int j = 0; j < 4; ++j) v[j] = __builtin_fmaf(a, b[j], v[j]);
    }
    spmm_epilogue<_Float16, 4>(v, bias, row, relu);
    if (ok) Pack<_Float16, 4>::store(C + (size_t)row * n + col4, v);
  }
}

}  // namespace spdl
