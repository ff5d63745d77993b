// SDDMM, lane family (fp32, dot products of up to 128 columns): the slab decomposition (a
// workgroup owns a panel of sparse rows and a run of slabs of R, streamed through LDS by
// direct-to-LDS copies; paper Sec. "Sampled Dense--Dense Matrix Multiplication Operation" for
// the strips of consecutive nonzeros), but every nonzero's dot product is formed by four lanes
// from start to end, each on its own quarter of the columns.  No partial sums are transposed
// across the group, no address is formed per LDS read, and both operands of every multiply-add
// are in the lane's own registers: a plain v_fmac_f32 issues in about three clocks per wave on
// this chip, the forms that take an operand from another lane (DPP) or from a scalar register in
// four and a half.
//
// A 16-lane group works on a strip of 4 consecutive nonzeros of one sparse row.  Lane 4t+h
// (t = 0..3, h = 0..3) owns nonzero t and quarter h of the dot product (columns 32h .. 32h+31).
// In step s = 0..3 it multiplies the eight columns 32h + 8((t-s) mod 4) .. of its quarter: its
// R row supplies them with two 16-byte LDS reads at a fixed offset from the row's address, and
// the matching values of L sit in registers, loaded once per kernel in exactly the order the
// lane will use them (32 registers per sparse row).  The four quarters are added with two quad
// permutes.  Per nonzero and lane: 32 multiply-adds, 4 address additions, 8 LDS reads.
//
// Bank conflicts: the 16 lanes of a group read 16 different rows of R at once, so the layout
// alone cannot keep them apart; the rotation by t does.  A slab holds the two 64-column halves
// of its rows in two regions of 256-byte rows, the second region shifted by 16 bytes.  In step s
// lane 4t+h reads bytes 128(h mod 2) + 32((t-s) mod 4) .. +31 of a row in region h/2: over the
// group these are the sixteen different 16-byte bank groups of the 64 banks, whatever the rows.
//
// Lanes whose nonzero does not exist (ragged strip, row done in this slab) read the first row
// of the slab and their result is dropped: nothing outside a nonzero's own rows of L and R can
// reach its output.
//
// Stage pipeline: the copy of the next slab and the loads of the next column indices are issued
// at the start of a stage, the results of a stage are stored at the start of the next one, and
// every stage ends with a wait for everything plus a barrier: whatever is waited for has had the
// whole stage to complete.
//
// Rows must be ascending for the slab walk; a row that is not is noticed when its nonzeros
// inside a slab are not a prefix of the look-ahead, its cursor is frozen, and the row is redone
// by direct gathers after the last slab.
// Needs n % 4 == 0, n <= 128 per launch, 16-byte aligned L and R.
//
// Row order (optional): see the row setup below.
//
// Longer dot products: the host runs the kernel once per chunk of 128 columns (L and R advanced by
// the chunk's first column c0, row stride ld = the full length, n = the chunk's width).  ACCUM
// passes (c0 > 0) add their sums to what out holds from the passes before: the old value of an
// entry is fetched together with the look-ahead of the column indices, one stage before the
// entry is stored.  Every pass walks A again, so this pays for rows that are too dense for the slab
// kernel that keeps partial sums in registers across the chunks (sddmm_slab_dma, at most 32 entries
// per row and slab).
//
// NT: the right-hand operand is given not transposed (n x k, row-major: the general SDDMM of
// the same section's footnote).  A slab is then 128 consecutive columns of every row of Rn.  It
// is fetched as it lies (rows of 512 contiguous bytes, direct-to-LDS, while the previous slab
// is being worked on) into a staging area and transposed from there into the layout above by
// LDS reads and writes, between two barriers; one slab buffer instead of two.  Needs k % 4 == 0
// and a 16-byte aligned Rn as well.
#pragma once
#include "common.hpp"
#include "sddmm_slab.hpp"

namespace spdl {

constexpr int kLaneS = 128;                          // rows of R per slab
constexpr int kLaneRegion = kLaneS * 256 + 16;       // one 64-column half of a slab
constexpr int kLaneBuf = 2 * kLaneRegion;
constexpr int kLaneLdsBytes = 2 * kLaneBuf;
// NT staging: rows 2i and 2i+1 of the slab of Rn interleaved in 16-byte pieces (piece q of row
// 2i+r at 32 q + 16 r), 32 bytes of padding per pair: the 16-byte piece q of row c then starts in
// bank group (c + 2 q) mod 16, so sixteen lanes reading one piece each of sixteen consecutive
// rows do not collide.
constexpr int kLanePairBytes = 1024 + 32;
constexpr int kLaneNtLdsBytes = kLaneBuf + 64 * kLanePairBytes;

// The two 16-byte LDS reads of one step: 32 bytes of the R row at byte offset `off`, from the
// lane's position `at` (start of LDS + the step's offset inside a row, formed once) on: one
// address addition per step.
__device__ __forceinline__ void lane_read(const char* at, int off, f32x4& b0, f32x4& b1) {
  const char* a = at + off;
  b0 = *reinterpret_cast<const f32x4*>(a);
  b1 = *reinterpret_cast<const f32x4*>(a + 16);
}

// Sum of v over the 16 lanes of a group, in every lane (four DPP row rotations).
__device__ __forceinline__ int group_sum16(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x128 /* row_ror:8 */, 0xf, 0xf, false);
  v += __builtin_amdgcn_update_dpp(0, v, 0x124 /* row_ror:4 */, 0xf, 0xf, false);
  v += __builtin_amdgcn_update_dpp(0, v, 0x122 /* row_ror:2 */, 0xf, 0xf, false);
  v += __builtin_amdgcn_update_dpp(0, v, 0x121 /* row_ror:1 */, 0xf, 0xf, false);
  return v;
}

// Value of lane Q of each quad, in all four lanes of the quad.
template <int Q>
__device__ __forceinline__ int quad_bcast(int v) {
  return __builtin_amdgcn_mov_dpp(v, Q * 0x55 /* quad_perm [Q,Q,Q,Q] */, 0xf, 0xf, false);
}

// Sum of a over the four lanes of a quad, in every lane.
__device__ __forceinline__ float quad_sum(float a) {
  a += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, a), 0xb1 /* [1,0,3,2] */,
                                                             0xf, 0xf, false));
  a += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, a), 0x4e /* [2,3,0,1] */,
                                                             0xf, 0xf, false));
  return a;
}

// RPG  = sparse rows per 16-lane group: the workgroup owns 64*RPG consecutive rows.
// NCHD = the look-ahead per row, in chunks of 16 column indices: a row may have up to 16*NCHD
//        nonzeros in one slab before it needs a second round in that slab (a full wait).
template <int RPG, int NCHD, bool SCALED, bool NT = false, bool ACCUM = false>
__global__ __launch_bounds__(kSdThreads) void sddmm_lane_kernel(
    int m, int k, int n, int nnz, int ksplit, int slabs_per_part, int panels,
    const int* __restrict__ row_offsets, const int* __restrict__ column_indices,
    const float* __restrict__ L, const float* __restrict__ R, float* __restrict__ out,
    const float* __restrict__ scale, const int* __restrict__ row_order, int ld, int c0) {
  static_assert(!(NT && ACCUM), "the not-transposed form takes dot products of up to 128 columns");
  constexpr int S = kLaneS;
  constexpr int WIN = 16 * NCHD;                // nonzeros per round
  constexpr int kCopies = S * 2 / 4 / 16;       // 1 KB direct-to-LDS loads per wave per slab
  extern __shared__ __attribute__((aligned(16))) char lds_raw[];
  PhaseClocks clocks;
  clocks.start();

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = uniform(tid >> 6);
  const int sub = lane >> 4;
  const int l16 = lane & 15;
  const int t4 = l16 >> 2;
  const int h4 = l16 & 3;
  // Position inside a chunk of 16 nonzeros of the one whose column index this lane loads (and
  // whose result it stores): strip q of the chunk is nonzeros 4q .. 4q+3, nonzero 4q+t is
  // worked on by the quad t and kept by its lane q.
  const int perm = 4 * h4 + t4;
  const int last_nz = nnz - 1;

  int panel, kpart;
  if (!slab_wg_map(blockIdx.x, panels, ksplit, panel, kpart)) return;
  const int k0 = kpart * slabs_per_part * S;
  const int k1 = min(k, k0 + slabs_per_part * S);
  const int nslabs = (k1 - k0 + S - 1) / S;

  // Slab copy: copy i of wave w moves four rows of one region (1 KB); lane L brings 16 bytes of
  // row L/16, and the hardware places lane L's bytes at M0 + 16 L.  The address is a scalar
  // base (start of the slab in R) plus a per-lane byte offset that is the same in every stage
  // except the last slab, whose rows past k are clamped to row k-1; columns past n are clamped
  // to the row's first columns (the matching values of L are zero).  S * n * 4 < 2^31 is
  // checked on the host.
  unsigned src_off[kCopies], src_off_last[kCopies];
  int dst_off[kCopies];
  const int last_rows = k - (k0 + (nslabs - 1) * S);          // rows of R from the last slab's start
#pragma unroll
  for (int i = 0; i < kCopies; ++i) {
    const int idx = i * 16 + wave;
    const int reg = idx & 1, rblock = idx >> 1;
    const int lrow = rblock * 4 + sub;
    const int col = reg * 64 + l16 * 4;
    const unsigned colb = col < n ? (unsigned)col * 4u : 0u;
    src_off[i] = (unsigned)lrow * (unsigned)ld * 4u + colb;
    src_off_last[i] = (unsigned)min(lrow, last_rows - 1) * (unsigned)ld * 4u + colb;
    dst_off[i] = reg * kLaneRegion + rblock * 1024;
  }
  const unsigned lds_base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)lds_raw;
  // Issued from inline assembly: the compiler counts its own direct-to-LDS loads on both memory
  // counters and then turns every later wait into a wait for everything; their completion is
  // covered by the explicit full wait that ends every stage.
  auto copy_stage = [&](int q) {
    const char* base = reinterpret_cast<const char*>(R + (size_t)(k0 + q * S) * ld);
    const unsigned dst = lds_base + (unsigned)((q & 1) * kLaneBuf);
    const bool last = q == nslabs - 1;
#pragma unroll
    for (int i = 0; i < kCopies; ++i) {
      const unsigned voff = last ? src_off_last[i] : src_off[i];
      const unsigned m0v = dst + (unsigned)dst_off[i];
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                   :: "s"(m0v), "v"(voff), "s"(base) : "memory", "m0");
    }
  };

  // NT: copy i of wave w fetches rows c = 2 (16 i + w) and c + 1 of Rn (even lanes the first, odd
  // lanes the second), columns slab start + 4 (lane / 2) .. + 3: lane L's 16 bytes land at
  // M0 + 16 L, which is the interleaved staging layout.  Rows past n are clamped to row 0 (the
  // matching values of L are zero), column quads past k to the slab's first quad (no valid
  // nonzero refers to them).
  auto fetch_slab_nt = [&](int q) {
    const int slab_start = k0 + q * S;
    const int quad = slab_start + 4 * (lane >> 1);
    const unsigned colb = (unsigned)(quad < k ? quad : slab_start) * 4u;
#pragma unroll
    for (int i = 0; i < kCopies; ++i) {
      const int pair = i * 16 + wave;
      const int c = 2 * pair + (lane & 1);
      const unsigned voff = (unsigned)(c < n ? c : 0) * (unsigned)k * 4u + colb;
      const unsigned m0v = lds_base + (unsigned)(kLaneBuf + pair * kLanePairBytes);
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                   :: "s"(m0v), "v"(voff), "s"(R) : "memory", "m0");
    }
  };
  // NT: staging -> slab buffer 0.  Thread (c = tid % 128, quads tid / 128 + 8 i) reads the four
  // values Rn[c, 4 quad .. + 3] and writes them to rows 4 quad .. + 3 of the slab, column c: the
  // 64 lanes of a wave write 64 consecutive columns of one row (all banks once).
  auto transpose_slab_nt = [&]() {
    const int c = tid & 127;
    const char* src = lds_raw + kLaneBuf + (c >> 1) * kLanePairBytes + (c & 1) * 16;
    char* dst = lds_raw + (c >> 6) * kLaneRegion + (c & 63) * 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int quad = (tid >> 7) + 8 * i;
      const f32x4 v = *reinterpret_cast<const f32x4*>(src + quad * 32);
      float* d = reinterpret_cast<float*>(dst + quad * 1024);
      d[0] = v.x;
      d[64] = v.y;
      d[128] = v.z;
      d[192] = v.w;
    }
  };

  // rows of this group, their ranges of nonzeros inside [k0, k1), their quarters of L in the
  // order of use: lr[j][8 s + e] = L[row, 32 h + 8((t-s) mod 4) + e]
  //
  // Vector-memory loads return in order, and every workgroup of the launch starts at the same time:
  // whatever is requested behind the first slab and the rows of L (20 MB over the whole chip on the
  // LSTM shape) waits for that burst.  The chain of dependent loads (row offsets, then the rounds of
  // the searches) therefore goes first, while the memory system is idle, and the bulk (first slab,
  // L, first look-ahead) is requested in one go behind it.
  int row[RPG], p_end[RPG], p[RPG];
  float lr[RPG][32];
  f32x4 lraw[RPG][2];                // piece t of quarter h of the rows of L, as loaded
  bool lok[RPG];
  bool safe = true;                  // no load of the look-ahead can pass the end of the arrays
  {
    // The row offsets of all rows, then the searches for the rows' ranges inside [k0, k1), all
    // 2*RPG of them side by side (a round of probes costs one memory latency, not 2*RPG).
    int rb[RPG], re[RPG];
    bool ok[RPG];
#pragma unroll
    for (int j = 0; j < RPG; ++j) {
      // Without a row order a workgroup owns 64*RPG consecutive rows.  With one (rows by decreasing
      // length, paper Sec. "Row Swizzle Load Balancing"), the 4*RPG rows of a wave are adjacent in
      // the order (a bundle of similar lengths, so the groups of a wave finish together) and a
      // workgroup takes every panels-th bundle, so every workgroup gets the same mix of long and
      // short rows.
      const int slot = row_order ? ((wave * panels + panel) * 4 + sub) * RPG + j
                                 : (panel * kSdRows + wave * 4 + sub) * RPG + j;
      ok[j] = slot < m;
      const int r = ok[j] && row_order ? row_order[slot] : slot;
      row[j] = ok[j] ? r : -1;
      rb[j] = ok[j] ? row_offsets[r] : 0;
      re[j] = ok[j] ? row_offsets[r + 1] : 0;
    }
    int lo[2 * RPG], hi[2 * RPG], key[2 * RPG];
#pragma unroll
    for (int j = 0; j < RPG; ++j) {
      lo[2 * j] = rb[j];
      hi[2 * j] = k0 <= 0 ? rb[j] : re[j];            // nothing to search for the first range
      key[2 * j] = k0;
      lo[2 * j + 1] = k1 >= k ? re[j] : rb[j];        // ... nor for the last
      hi[2 * j + 1] = re[j];
      key[2 * j + 1] = k1;
    }
    sd_lower_bound16_batch<2 * RPG>(column_indices, lo, hi, key, sub, l16, last_nz, k);
    if constexpr (NT) fetch_slab_nt(0);
    else copy_stage(0);
#pragma unroll
    for (int j = 0; j < RPG; ++j) {
      p[j] = lo[2 * j];
      p_end[j] = max(lo[2 * j + 1], p[j]);
      safe = safe && __builtin_amdgcn_ballot_w64(p_end[j] + WIN > nnz) == 0;
      // Every lane loads the 32 bytes it uses in step 0 (piece t of quarter h); the pieces of the
      // other steps come from the lanes that loaded them, by row rotations (below): a quarter of the
      // load instructions of fetching all four pieces in every lane.
      const float* lrow = L + (size_t)max(row[j], 0) * ld;
      lok[j] = ok[j];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int c = 32 * h4 + 8 * t4 + 4 * u;
        lraw[j][u] = *reinterpret_cast<const f32x4*>(lrow + (c < n ? c : 0));
      }
    }
  }
  // byte offset of step s from the start of an R row in region 0: this lane's region, its half of
  // the 256-byte row, and the rotated 32-byte piece
  const char* x[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) x[s] = lds_raw + ((h4 >> 1) * kLaneRegion + (h4 & 1) * 128 + ((t4 - s) & 3) * 32);

  // Look-ahead of row j from position `from`: the next 16*NCHD column indices, lane 4t+h of the
  // group holding index 16 i + 4 h + t of chunk i; with them the values of A if the results are
  // to be scaled.  Raw loads, first used in the next stage.  32-bit byte offsets from scalar
  // bases (nnz < 2^29 is checked on the host).
  int cn[RPG][NCHD];
  float sc[RPG][SCALED ? NCHD : 1];
  float pv[RPG][ACCUM ? NCHD : 1];      // what out holds at those positions from the passes before
  auto fetch = [&](int j, int from) {
    const char* cbase = reinterpret_cast<const char*>(column_indices);
    const char* vbase = reinterpret_cast<const char*>(scale);
    const char* obase = reinterpret_cast<const char*>(out);
    if (safe) {
      const unsigned o = (unsigned)(from + perm) << 2;
#pragma unroll
      for (int i = 0; i < NCHD; ++i) {
        cn[j][i] = *reinterpret_cast<const int*>(cbase + (o + 64u * i));
        if (SCALED) sc[j][i] = *reinterpret_cast<const float*>(vbase + (o + 64u * i));
        if (ACCUM) pv[j][i] = *reinterpret_cast<const float*>(obase + (o + 64u * i));
      }
    } else {
#pragma unroll
      for (int i = 0; i < NCHD; ++i) {
        const unsigned o = (unsigned)min(from + perm + 16 * i, last_nz) << 2;
        cn[j][i] = *reinterpret_cast<const int*>(cbase + o);
        if (SCALED) sc[j][i] = *reinterpret_cast<const float*>(vbase + o);
        if (ACCUM) pv[j][i] = *reinterpret_cast<const float*>(obase + o);
      }
    }
  };

  // results of the previous round, stored at the start of the next one: this lane's nonzero of
  // chunk i of row j goes to out[st_pos[j] + 16 i] if the lane is in st_mask[j][i]
  float outv[RPG][NCHD];
  int st_off[RPG];
  unsigned long long st_mask[RPG][NCHD];
#pragma unroll
  for (int j = 0; j < RPG; ++j)
#pragma unroll
    for (int i = 0; i < NCHD; ++i) st_mask[j][i] = 0;
  auto store_pending = [&]() {
#pragma unroll
    for (int j = 0; j < RPG; ++j) {
      float* o = reinterpret_cast<float*>(reinterpret_cast<char*>(out) + (unsigned)st_off[j]);
#pragma unroll
      for (int i = 0; i < NCHD; ++i) {
        if (st_mask[j][i] == 0) break;
        if (__builtin_amdgcn_inverse_ballot_w64(st_mask[j][i])) o[16 * i] = outv[j][i];
        st_mask[j][i] = 0;
      }
    }
  };

#pragma unroll
  for (int j = 0; j < RPG; ++j) fetch(j, p[j]);
  // lr[j][8 s + e]: the piece that lane (t - s, h) loaded, i.e. the lane 4 s places to the left in
  // the group (row_ror:4s moves lane i - 4 s to lane i); columns past n and rows past m count as zero.
#pragma unroll
  for (int j = 0; j < RPG; ++j)
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const bool in = lok[j] && 32 * h4 + 8 * t4 + 4 * u < n;
      const f32x4 vv = lraw[j][u];
      const float own[4] = {in ? vv.x : 0.f, in ? vv.y : 0.f, in ? vv.z : 0.f, in ? vv.w : 0.f};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int bits = __builtin_bit_cast(int, own[e]);
        lr[j][4 * u + e] = own[e];
        lr[j][8 + 4 * u + e] = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, bits, 0x124 /* row_ror:4 */, 0xf, 0xf, false));
        lr[j][16 + 4 * u + e] = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, bits, 0x128 /* row_ror:8 */, 0xf, 0xf, false));
        lr[j][24 + 4 * u + e] = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, bits, 0x12c /* row_ror:12 */, 0xf, 0xf, false));
      }
    }
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  if constexpr (NT) {
    transpose_slab_nt();
    __syncthreads();
  }
  clocks.lap(kPhaseSetup);

  for (int s = 0; s < nslabs; ++s) {
    const int slab_start = k0 + s * S;
    const int buf_off = NT ? 0 : (s & 1) * kLaneBuf;
    // LDS byte offset of R row c in region 0 = (c << 8) + row_base
    const int row_base = buf_off - slab_start * 256;
    bool first = true, more;
    do {
      // Wave priorities by phase: the waves of a SIMD that are furthest behind in the stage go first
      // (counting before the first row's strips before the second row's), so that they reach the
      // barrier together instead of one after the other, the last of them alone on its SIMD with
      // nothing to cover its LDS latencies.
      __builtin_amdgcn_s_setprio(3);
      // A use of every look-ahead register before the copies are issued: the compiler places its
      // wait for those loads here, where they completed long ago (full wait at the end of the
      // previous stage), instead of after the copies, where it would wait for those too.
#pragma unroll
      for (int j = 0; j < RPG; ++j)
#pragma unroll
        for (int i = 0; i < NCHD; ++i) {
          asm volatile("" :: "v"(cn[j][i]));
          if (SCALED) asm volatile("" :: "v"(sc[j][i]));
          if (ACCUM) asm volatile("" :: "v"(pv[j][i]));
        }
      store_pending();
      clocks.lap(kPhaseRest);
      if (first && s + 1 < nslabs) {
        if constexpr (NT) fetch_slab_nt(s + 1);       // the staging area was emptied before this stage
        else copy_stage(s + 1);
      }
      clocks.lap(kPhaseIssue);
      first = false;
      more = false;
      // First the look-ahead of every row is counted and replaced by the next one, so that all
      // loads of a stage are issued before its arithmetic starts; then the strips are worked on.
      int col[RPG][NCHD], vl[RPG];
      float scv[RPG][SCALED ? NCHD : 1];
      float pvv[RPG][ACCUM ? NCHD : 1];
      unsigned long long okm[RPG][NCHD];
#pragma unroll
      for (int j = 0; j < RPG; ++j) {
        // How many of the fetched nonzeros fall into this slab.  Every lane looks at its own
        // position of each chunk; in an ascending row the positions inside the slab and the row
        // are a prefix of the look-ahead, so their number is the sum of the lanes' counts.  If
        // they are not exactly the first `used` positions the row is not ascending: its cursor
        // is frozen (p_end is never reached) and the row is redone after the last slab.
        const int remain_l = p_end[j] - p[j] - perm;
        int nv = 0;
#pragma unroll
        for (int i = 0; i < NCHD; ++i) {
          okm[j][i] = __builtin_amdgcn_ballot_w64((unsigned)(cn[j][i] - slab_start) < (unsigned)S) &
                      __builtin_amdgcn_ballot_w64(remain_l > 16 * i);
          nv += __builtin_amdgcn_inverse_ballot_w64(okm[j][i]) ? 1 : 0;
        }
        int used = group_sum16(nv);
        const int used_l = used - perm;
        unsigned long long bad = 0;
#pragma unroll
        for (int i = 0; i < NCHD; ++i) bad |= okm[j][i] ^ __builtin_amdgcn_ballot_w64(used_l > 16 * i);
        if (bad != 0) {                                 // wave-uniform, rare
          if (((unsigned)(bad >> (sub * 16)) & 0xffffu) != 0) { used = 0; p_end[j] = -1; }
#pragma unroll
          for (int i = 0; i < NCHD; ++i) okm[j][i] = __builtin_amdgcn_ballot_w64(used - perm > 16 * i);
        }
        more = more || __builtin_amdgcn_ballot_w64(used == WIN) != 0;
        vl[j] = used - t4;       // this quad's nonzero of strip q of chunk i exists if vl > 16 i + 4 q
        st_off[j] = (p[j] + perm) << 2;
        p[j] += used;
        // LDS offsets of this lane's own nonzero of every chunk (the first row of the slab if it
        // does not exist); the strips broadcast them inside the quads.  This also moves the
        // indices out of the way of the next look-ahead.
#pragma unroll
        for (int i = 0; i < NCHD; ++i) {
          col[j][i] = __builtin_amdgcn_inverse_ballot_w64(okm[j][i]) ? (cn[j][i] << 8) + row_base : buf_off;
          if (SCALED) scv[j][i] = sc[j][i];
          if (ACCUM) pvv[j][i] = pv[j][i];
        }
        fetch(j, p[j]);
      }
      clocks.lap(kPhaseScan);
#pragma unroll
      for (int j = 0; j < RPG; ++j) {
        if (j == 0) __builtin_amdgcn_s_setprio(2);
        else __builtin_amdgcn_s_setprio(1);
        // Software pipeline over (strip, step): LDS reads run two steps ahead of the
        // multiply-adds, also across strips, through two register sets used in turn; reads
        // for a strip that does not exist hit a valid address and are dropped.
        auto strip_off = [&](int i, int q) -> int {
          switch (q) {
            case 0: return quad_bcast<0>(col[j][i]);
            case 1: return quad_bcast<1>(col[j][i]);
            case 2: return quad_bcast<2>(col[j][i]);
            default: return quad_bcast<3>(col[j][i]);
          }
        };
        f32x4 b[2][2];
        int off = strip_off(0, 0);
        lane_read(x[0], off, b[0][0], b[0][1]);
        lane_read(x[1], off, b[1][0], b[1][1]);
        bool done = false;
#pragma unroll
        for (int i = 0; i < NCHD; ++i) {
          if (done) break;
          float keep = 0.f;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            if (__builtin_amdgcn_ballot_w64(vl[j] > 16 * i + 4 * q) == 0) { done = true; break; }
            const bool last_strip = i == NCHD - 1 && q == 3;
            const int off_next = last_strip ? off : strip_off(q == 3 ? i + 1 : i, q == 3 ? 0 : q + 1);
            float acc0 = 0.f, acc1 = 0.f;
#pragma unroll
            for (int st = 0; st < 4; ++st) {
              const f32x4 b0 = b[st & 1][0], b1 = b[st & 1][1];
              const float* l = &lr[j][8 * st];
              acc0 = __builtin_fmaf(l[0], b0.x, acc0);
              acc1 = __builtin_fmaf(l[1], b0.y, acc1);
              acc0 = __builtin_fmaf(l[2], b0.z, acc0);
              acc1 = __builtin_fmaf(l[3], b0.w, acc1);
              acc0 = __builtin_fmaf(l[4], b1.x, acc0);
              acc1 = __builtin_fmaf(l[5], b1.y, acc1);
              acc0 = __builtin_fmaf(l[6], b1.z, acc0);
              acc1 = __builtin_fmaf(l[7], b1.w, acc1);
              if (st < 2) lane_read(x[st + 2], off, b[st & 1][0], b[st & 1][1]);
              else if (!last_strip) lane_read(x[st - 2], off_next, b[st & 1][0], b[st & 1][1]);
            }
            const float total = quad_sum(acc0 + acc1);
            keep = h4 == q ? total : keep;
            off = off_next;
          }
          outv[j][i] = (SCALED ? keep * scv[j][i] : keep) + (ACCUM ? pvv[j][i] : 0.f);
          st_mask[j][i] = okm[j][i];
        }
      }
      __builtin_amdgcn_s_setprio(0);
      clocks.lap(kPhaseSteps);
      if (more) __builtin_amdgcn_s_waitcnt(0);       // a row has more than 16*NCHD nonzeros in this slab
    } while (more);
    __builtin_amdgcn_s_waitcnt(0);
    clocks.lap(kPhaseWait);
    __syncthreads();
    clocks.lap(kPhaseBarrier);
    if constexpr (NT) {
      if (s + 1 < nslabs) {                           // the slab is done with, the next one has arrived
        transpose_slab_nt();
        __syncthreads();
      }
    }
  }
  store_pending();
  clocks.lap(kPhaseRest);
  clocks.store(blockIdx.x * (kSdThreads / 64) + wave);

  // A range whose cursor did not stop exactly at its end was not ascending: redo it directly.
#pragma unroll
  for (int j = 0; j < RPG; ++j)
    if (p[j] != p_end[j] && row[j] >= 0) {
      // (the same searches as in the set-up: for a row that is not ascending only the same procedure
      // gives the same range, and the ranges of the column parts have to tile the row)
      const int rb = row_offsets[row[j]], re = row_offsets[row[j] + 1];
      int lo2[2] = {rb, k1 >= k ? re : rb}, hi2[2] = {k0 <= 0 ? rb : re, re};
      const int key2[2] = {k0, k1};
      sd_lower_bound16_batch<2>(column_indices, lo2, hi2, key2, sub, l16, last_nz, k);
      const int b0 = lo2[0];
      const int e = max(lo2[1], b0);
      if constexpr (NT) {
        // one lane per stored entry, the plain definition
        for (int t = b0 + l16; t < e; t += 16) {
          const float* lrow = L + (size_t)row[j] * n;
          const float* rcol = R + column_indices[t];
          float acc = 0.f;
          for (int c = 0; c < n; ++c) acc = __builtin_fmaf(lrow[c], rcol[(size_t)c * k], acc);
          out[t] = SCALED ? acc * scale[t] : acc;
        }
      } else if (ld != n) {
        // one chunk of a longer dot product: one lane per stored entry recomputes the whole sum over
        // the columns up to this chunk's end, so that it does not matter what out holds so far
        const float* lfull = L - c0 + (size_t)row[j] * ld;
        const float* rfull = R - c0;
        for (int t = b0 + l16; t < e; t += 16) {
          const float* rrow = rfull + (size_t)column_indices[t] * ld;
          float acc = 0.f;
          for (int c = 0; c < c0 + n; ++c) acc = __builtin_fmaf(lfull[c], rrow[c], acc);
          out[t] = SCALED ? acc * scale[t] : acc;
        }
      } else {
        for (int t = b0; t < e; t += 16)
          sd_strip_direct_call<float>(n, t, e, l16, L + (size_t)row[j] * n, column_indices, R, out,
                                      SCALED ? scale : nullptr);
      }
    }
}

}  // namespace spdl
