// SDDMM in mixed precision on the matrix cores (paper Sec. "Mixed Precision": fp16 operands,
// fp32 accumulation).  On this chip the dense fp16 matrix rate is some thirty times the fp32
// vector rate, so for the moderately sparse matrices of deep learning it is cheaper to compute
// a whole 32x32 block of L R^T with MFMA and keep only the entries A stores there than to
// gather one row of R per stored entry.  The contraction runs over n, which is the contiguous
// dimension of both row-major operands.
//
// A workgroup owns one 64x64 block of A's index space.  Which stored entries fall into the
// block: for each of its 64 rows a binary search gives the first entry with column >= c0 and
// the first with column >= c0 + 64.  Whatever the column order inside a row, the ranges of
// consecutive blocks cover the row (the first block starts at the row start, the last ends at
// the row end), and every entry of a range is produced by the wave that owns the range: from
// the block if its column lies inside it, else (rows that are not ascending) by a plain dot
// product.  Dense work is the same for every block, so row lengths do not unbalance anything.
//
// Needs n % 8 == 0 and 16-byte aligned L and R.
#pragma once
#include "common.hpp"

namespace spdl {

typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ f16x8 load_h8(const _Float16* p) { return *reinterpret_cast<const f16x8*>(p); }

// Dot product of two rows of length n by one lane (entries whose column lies outside the block
// that owns their range; only rows that are not ascending have them).
__device__ __attribute__((noinline)) float sddmm_lane_dot(const _Float16* __restrict__ l,
                                                          const _Float16* __restrict__ r, int n) {
  float acc = 0.f;
  for (int j = 0; j < n; j += 8) {
    const f16x8 a = load_h8(l + j), b = load_h8(r + j);
#pragma unroll
    for (int t = 0; t < 8; ++t) acc = __builtin_fmaf((float)a[t], (float)b[t], acc);
  }
  return acc;
}

constexpr int kSmK = 128;                              // columns of L and R per stage (16 pieces of 16 bytes)
constexpr int kSmRing = 4;                             // stages resident in LDS (three being fetched)
constexpr int kSmOperandBytes = 64 * kSmK * 2;         // 64 rows of one operand
constexpr int kSmStageBytes = 2 * kSmOperandBytes;     // L rows, then R rows
constexpr int kSddmmMfmaLdsBytes = kSmRing * kSmStageBytes + 2 * 64 * 4;   // the ring (reused for the block) + ranges

// One workgroup (four waves) owns one 64x64 block of A's index space.  The contraction runs
// over n, 128 columns per stage.  The 64 rows of L and of R of the block are brought in by
// direct-to-LDS loads: sixteen lanes read the 256 contiguous bytes of one row, and each lane
// fetches the piece that belongs at its place in a swizzled layout (piece p of row r at slot
// p xor (r mod 16)), so that the sixteen lanes of an operand read, which want the same piece of
// sixteen rows, hit sixteen different bank groups.  Three stages are in flight while one is
// multiplied (there is little arithmetic per byte here: the loads must be kept going); one
// barrier per stage.  The copies are issued from inline assembly and waited for with explicit
// counts: apart from two early index loads they are the only vector-memory operations inside
// the loop, and they complete in the order issued.  At the end the partial blocks go to LDS and
// the threads pick out the positions A stores.
//
// What bounds it: a CU pulls L2-resident data at some 120 GB/s at best and about 90 GB/s through
// a ring with a barrier per stage (both measured with copy-only kernels), i.e. 0.35 us for a
// 32 KB stage, against 0.1 us of MFMA; LDS reads compete with the copies' LDS writes, which is
// why every byte is read only once (see the accumulators below).  Measured: 0.45 - 0.6 us per
// stage.  Larger blocks would need fewer bytes per product but leave most CUs without a block at
// the sizes of the 1x1 convolution (256 blocks of 64x64).
// (Measured and dropped: a fifth wave running ahead to pull the lines into L2, staging through
// registers instead of direct-to-LDS loads, and reading a stage's fragments one iteration ahead
// of their MFMAs; none was faster.)
__global__ __launch_bounds__(256) void sddmm_mfma_kernel(
    int m, int k, int n, int tiles_k, const int* __restrict__ row_offsets,
    const int* __restrict__ column_indices, const _Float16* __restrict__ L, const _Float16* __restrict__ R,
    _Float16* __restrict__ out, const _Float16* __restrict__ scale) {
  extern __shared__ __attribute__((aligned(16))) char lds_raw[];
  float (*part)[64][65] = reinterpret_cast<float (*)[64][65]>(lds_raw);           // [wave][row][column], after the loop
  int (*bound)[64] = reinterpret_cast<int (*)[64]>(lds_raw + kSmRing * kSmStageBytes);   // [0]: range start, [1]: end
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = uniform(tid >> 6);
  const int r = lane & 31;
  const int half = lane >> 5;
  // Block id -> (tile_i, tile_c).  Consecutive workgroup ids go round-robin to the 8 XCDs, each
  // with its own L2; XCD x gets the sub-grid (x/4 of 2 row halves) x (x%4 of 4 column quarters), so
  // that its workgroups, which advance through n together, share the rows of L and R they stream.
  const int tiles_m = (m + 63) >> 6;
  const int TI = (tiles_m + 1) >> 1, TC = (tiles_k + 3) >> 2;
  const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
  const int tile_i = (xcd >> 2) * TI + local / TC;
  const int tile_c = (xcd & 3) * TC + local % TC;
  if (tile_i >= tiles_m || tile_c >= tiles_k || local / TC >= TI) return;   // whole workgroup, before any barrier
  const int i0 = tile_i * 64;
  const int c0 = tile_c * 64;

  // Copies.  A stage is 32 copies of 1 KB (4 rows each); wave w issues copies 8w .. 8w+7: waves 0
  // and 1 bring L, waves 2 and 3 bring R.  Copy j of a wave fills rows 4*(8*(w%2) + j) .. +3 of
  // its operand; lane t brings row t/16 of those, the piece (t%16) xor (row%16), to slot t%16.
  // Rows past the end of either matrix are clamped (their results are never looked at); pieces
  // past column n are clamped to the stage's first piece and their products are zeroed below.
  const int stages = (n + kSmK - 1) / kSmK;
  const _Float16* operand = wave < 2 ? L : R;
  const int row_limit = (wave < 2 ? m : k) - 1, row_base = wave < 2 ? i0 : c0;
  unsigned voff[8];
  int vpiece[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int row = 4 * (8 * (wave & 1) + j) + (lane >> 4);
    vpiece[j] = (lane & 15) ^ (row & 15);
    voff[j] = (unsigned)min(row_base + row, row_limit) * (unsigned)n * 2u;
  }
  const unsigned lds_base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)lds_raw;
  auto issue_stage = [&](int s) {
    const char* base = reinterpret_cast<const char*>(operand + (size_t)s * kSmK);
    const unsigned dst = lds_base + (unsigned)((s % kSmRing) * kSmStageBytes + (wave >> 1) * kSmOperandBytes +
                                               (wave & 1) * (kSmOperandBytes / 2));
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const bool in = s * kSmK + vpiece[j] * 8 < n;
      const unsigned off = voff[j] + (in ? (unsigned)vpiece[j] * 16u : 0u);     // past n: the stage's first piece
      const unsigned m0v = dst + (unsigned)j * 1024u;
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                   :: "s"(m0v), "v"(off), "s"(base) : "memory", "m0");
    }
  };

  // Every wave accumulates the whole 64x64 block over its quarter of each stage (columns
  // 32*wave .. +31 of the stage's 128): every byte of a stage is then read from LDS once, by one
  // wave, where a split of the block into four 32x32 tiles reads it twice (LDS reads and the copies'
  // LDS writes share one port, and the tile split keeps it busier than the matrix cores).  The four
  // partial blocks are added when the entries are sampled.
  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int t = 0; t < 16; ++t) acc[i][j][t] = 0.f;
  // operand fragments: lane (r, half) reads piece 4*wave + 2*step + half of rows r and 32 + r of L
  // and of R, from their swizzled slots (rows r and 32 + r share r % 16)
  const int a_row_off = r * (kSmK * 2), b_row_off = kSmOperandBytes + r * (kSmK * 2);

#pragma unroll
  for (int s = 0; s < kSmRing - 1; ++s)
    if (s < stages) issue_stage(s);

  // Range of row i0 + t%64 that this block owns: threads 0..63 search for c0, 64..127 for c0 + 64
  // (a chain of dependent loads: it runs while the first stages arrive).
  if (tid < 128) {
    const int row = i0 + (tid & 63);
    const int which = tid >> 6;
    int rs = 0, re = 0;
    if (row < m) {
      rs = row_offsets[row];
      re = row_offsets[row + 1];
    }
    int lo = rs, hi = re;
    const int key = c0 + 64 * which;
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (column_indices[mid] < key) lo = mid + 1; else hi = mid;
    }
    if (which == 0 && tile_c == 0) lo = rs;
    if (which == 1 && tile_c == tiles_k - 1) lo = re;
    bound[which][tid & 63] = lo;
  }

  int pre_b0 = 0, pre_b1 = 0, pre_c0 = 0, pre_c1 = 0;
  for (int s = 0; s < stages; ++s) {
    // stage s has arrived when at most the copies of the (up to two) later stages are outstanding
    if (s + 2 < stages) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
    else if (s + 1 < stages) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();                                   // everyone's copies of stage s are in; stage s-1 is consumed
    if (s == 0) {
      // the ranges are visible now: fetch this thread's first two column indices, to be used after the loop
      pre_b0 = bound[0][tid >> 2];
      pre_b1 = max(pre_b0, bound[1][tid >> 2]);
      const int p = pre_b0 + (tid & 3);
      if (p < pre_b1) pre_c0 = column_indices[p];
      if (p + 4 < pre_b1) pre_c1 = column_indices[p + 4];
    }
    if (s + kSmRing - 1 < stages) issue_stage(s + kSmRing - 1);
    const char* buf = lds_raw + (s % kSmRing) * kSmStageBytes;
    const bool ragged = (s + 1) * kSmK > n;
#pragma unroll
    for (int step = 0; step < 2; ++step) {
      const int p = 4 * wave + 2 * step + half;
      const int slot = (p ^ (r & 15)) << 4;
      f16x8 a0 = *reinterpret_cast<const f16x8*>(buf + a_row_off + slot);
      f16x8 a1 = *reinterpret_cast<const f16x8*>(buf + a_row_off + 32 * (kSmK * 2) + slot);
      const f16x8 b0 = *reinterpret_cast<const f16x8*>(buf + b_row_off + slot);
      const f16x8 b1 = *reinterpret_cast<const f16x8*>(buf + b_row_off + 32 * (kSmK * 2) + slot);
      if (ragged && s * kSmK + p * 8 >= n) {
#pragma unroll
        for (int t = 0; t < 8; ++t) a0[t] = a1[t] = (_Float16)0.f;
      }
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, b0, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, b1, acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1, b0, acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1, b1, acc[1][1], 0, 0, 0);
    }
  }
  __syncthreads();                                     // the ring is free: it now holds the four partial blocks

  // Register t of lane (r, half) in acc[i][j] is element (32*i + 8*(t/4) + 4*half + t%4, 32*j + r).
  float (*mine)[65] = part[wave];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int t = 0; t < 16; ++t) mine[32 * i + 8 * (t / 4) + 4 * half + (t % 4)][32 * j + r] = acc[i][j][t];
  __syncthreads();

  // Four threads per row take alternate entries of its range.
  const int rr = tid >> 2;
  const int row = i0 + rr;
  const int b0 = pre_b0, b1 = pre_b1;
  for (int p = b0 + (tid & 3), it = 0; p < b1; p += 4, ++it) {
    const int c = it == 0 ? pre_c0 : it == 1 ? pre_c1 : column_indices[p];
    const unsigned cc = (unsigned)(c - c0);
    float val;
    if (cc < 64u) val = (part[0][rr][cc] + part[1][rr][cc]) + (part[2][rr][cc] + part[3][rr][cc]);
    else val = sddmm_lane_dot(L + (size_t)row * n, R + (size_t)c * n, n);
    sddmm_store<_Float16>(out, scale, p, val);
  }
}

}  // namespace spdl
