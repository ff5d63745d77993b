// libspdl: C ABI, argument checks, kernel selection and launches.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <numeric>
#include <vector>

#include "../../include/spdl.h"
#include "common.hpp"
#include "csr_softmax.hpp"
#include "sddmm_group.hpp"
#include "sddmm_lane.hpp"
#include "sddmm_mfma.hpp"
#include "sddmm_nt.hpp"
#include "sddmm_rowstrip.hpp"
#include "sddmm_slab.hpp"
#include "sddmm_slab_dma.hpp"
#include "spmm_rowsplit.hpp"
#include "spmm_slab.hpp"
#include "spmm_mfma.hpp"
#include "spmm_slab_dma.hpp"
#include "spmm_window.hpp"
#include "spmm_slab_tiles.hpp"
#include "sddmm_window.hpp"

namespace {

using namespace spdl;

enum SpmmVariant { kSpmmRowsplit = 0, kSpmmSlab = 1, kSpmmSlabDma = 2, kSpmmMfma = 3, kSpmmWindow = 4, kSpmmVariants };
// What the caller says about the sparse matrix (the library never reads the topology on the host).
enum Hint { kHintNone = 0, kHintBanded = 1, kHintSkewed = 2 };
enum SddmmVariant { kSddmmRowstrip = 0, kSddmmGroup = 1, kSddmmSlab = 2, kSddmmSlabDma = 3, kSddmmMfma = 4, kSddmmLane = 5, kSddmmWindow = 6, kSddmmVariants };

std::atomic<int> g_forced[2] = {{-1}, {-1}};

inline bool aligned(const void* p, size_t bytes) { return (reinterpret_cast<uintptr_t>(p) % bytes) == 0; }

inline bool sizes_ok(int m, int k, int n, int nnz) {
  if (m < 0 || k < 0 || n < 0 || nnz < 0) return false;
  const int64_t lim = (int64_t)1 << 31;
  return (int64_t)m * n < lim && (int64_t)k * n < lim;
}

// Widest vector width (in elements) usable for rows of length n starting at these bases.
template <typename T>
int pick_vec(int n, const void* a, const void* b, int max_vec) {
  for (int v = max_vec; v > 1; v /= 2)
    if (n % v == 0 && aligned(a, v * sizeof(T)) && aligned(b, v * sizeof(T))) return v;
  return 1;
}

// Lanes per row: the smallest group whose tile covers n, so that small n spreads a wave over
// several rows instead of idling lanes (paper Sec. "Subwarp Tiling").
inline int pick_group(int n, int vec) {
  for (int g = 8; g < kWave; g *= 2)
    if (g * vec >= n) return g;
  return kWave;
}

constexpr int kSlabS = 256;                       // B rows per LDS slab
constexpr int kSlabLdsBytes = 2 * (kSlabS + 1) * kSlabTile * 4;
constexpr int kComputeUnits = 256;

// Lane groups per row of the row-splitting kernel: one, unless the rows are too few to fill the
// machine (about 16 waves per CU) and long enough to share; only with the widest vectors.
template <typename T>
int pick_segments(int m, int nnz, int vec, int g) {
  if (vec != 16 / (int)sizeof(T) || m <= 0) return 1;
  int seg = 1;
  const int64_t avg = nnz / m;
  while (g * seg * 2 <= kWave && (int64_t)m * g * seg / kWave < 16 * kComputeUnits && avg / (seg * 2) >= 32) seg *= 2;
  return seg;
}

template <typename T>
void fill_spmm_rowsplit_info(int m, int n, int nnz, const void* B, const void* C, spdl_launch_info* info) {
  const int vec = pick_vec<T>(n, B, C, 16 / (int)sizeof(T));
  const int g = pick_group(n, vec);
  const int seg = pick_segments<T>(m, nnz, vec, g);
  info->variant = kSpmmRowsplit;
  info->vec = vec;
  info->lanes_per_row = g;
  info->rows_per_block = 256 / (g * seg);
  info->block_threads = 256;
  info->grid_x = (m + info->rows_per_block - 1) / info->rows_per_block;
  info->grid_y = (n + g * vec - 1) / (g * vec);
}

template <typename T>
bool slab_usable(int n, int nnz, const void* B, const void* C) {
  // 32-bit byte offsets: into the pair arrays, and from a slab's start to any of its elements
  return n % 4 == 0 && n < (1 << 21) && nnz < (1 << 29) && aligned(B, 4 * sizeof(T)) && aligned(C, 4 * sizeof(T));
}

// A slab kernel's workgroup fills a compute unit (LDS), so a grid of more than `slots` workgroups
// runs in rounds.  `total` units of work per panel (tiles of C, slabs of A's columns), walked back
// to back by one workgroup, are dealt to the number of workgroups per panel that gives the shortest
// chain: rounds x (units per workgroup + two units' worth of set-up).  All workgroups of a panel
// run on the same XCD (slab_wg_map), so the rounds are those of the XCD with the most panels.
// (3072 rows, 48 panels, six per XCD: six workgroups per panel would be 36 on each XCD's 32 compute
// units, a second round for four of them; five make 30 in one round.)  Returns the units per
// workgroup.
int split_for_machine(int panels, int total, int slots = kComputeUnits) {
  int best_units = total;
  double best = 1e300;
  for (int parts = 1; parts <= std::min(total, slots); ++parts) {
    const int units = (total + parts - 1) / parts;
    const int64_t wgs = (int64_t)((panels + 7) / 8) * ((total + units - 1) / units);    // on the fullest XCD
    const double cost = (double)((wgs + slots / 8 - 1) / (slots / 8)) * (units + 2.0);
    if (cost < best - 1e-9) {
      best = cost;
      best_units = units;
    }
  }
  return best_units;
}

int slab_tiles_per_wg(int panels, int tiles, int slots = kComputeUnits) { return split_for_machine(panels, tiles, slots); }

// Rows per 16-lane group of the copy-based slab kernel: two when 128-row panels still give
// every CU at least two tiles to walk, else one.
int slab_rows_per_group(int m, int n) {
  const int64_t tiles128 = (int64_t)((m + 127) / 128) * ((n + kSlabTile - 1) / kSlabTile);
  return tiles128 >= 2 * kComputeUnits ? 2 : 1;
}

// Workgroups of 8 waves (panels of 32 rows, slabs of 128 rows of B, two workgroups per CU) for the
// copy-based kernel when panels of 64 rows would leave compute units without a workgroup.
constexpr int kSlabHalfS = 128;
constexpr int kSlabHalfLdsBytes = 2 * (kSlabHalfS + 1) * kSlabTile * 4;

// The tile-inner slab kernel looks 48 pairs ahead per row: usable where the mean count of a row's
// pairs in one slab plus three standard deviations fits into that (a row with more takes extra
// rounds behind full waits in every tile's stage).
inline bool slab_tiles_fits(int m, int k, int nnz) {
  const double d = (m > 0 && k > 0) ? (double)nnz / ((double)m * (double)k) : 1.0;
  const double mean = kSlabS * d;
  return mean + 3.0 * std::sqrt(mean * std::max(0.0, 1.0 - d)) + 1.0 <= 48.0;
}
constexpr int kSlabTilesMax = 4;                  // tiles whose accumulators that kernel keeps in registers

void fill_spmm_slab_info(int m, int k, int n, int nnz, int variant, spdl_launch_info* info) {
  const int tiles = (n + kSlabTile - 1) / kSlabTile;
  const bool half = variant == kSpmmSlabDma && (int64_t)((m + kSlabRows - 1) / kSlabRows) * tiles < kComputeUnits;
  const int rpg = (variant == kSpmmSlabDma && !half) ? slab_rows_per_group(m, n) : 1;
  const int rows = (half ? kSlabRows / 2 : kSlabRows) * rpg;
  const int panels = (m + rows - 1) / rows;
  int tpw = slab_tiles_per_wg(panels, tiles, half ? 2 * kComputeUnits : kComputeUnits);
  // wide outputs, two rows per group: the tile-inner kernel, at most kSlabTilesMax tiles per workgroup
  if (rpg == 2 && tpw >= 2 && slab_tiles_fits(m, k, nnz)) tpw = std::min(tpw, kSlabTilesMax);
  const int groups = (tiles + tpw - 1) / tpw;
  info->variant = variant;
  info->vec = 4;
  info->lanes_per_row = 16;
  info->rows_per_block = rows;
  info->block_threads = half ? kSlabThreads / 2 : kSlabThreads;
  info->grid_x = slab_grid_size(panels, groups);
  info->grid_y = tpw;                       // tiles walked by one workgroup (the grid is 1-D)
}

// Kernel selection (paper Sec. "Experiments": tile and vector width from the problem shape).
// The slab kernel re-reads each B row from LDS once per sparse row that uses it, so it pays
// when a 64-row panel touches the same B row several times: 64 * density >= 2.
//
// Window kernels: workgroups of 8 waves (8 sparse rows, one window of 64 KB): two fit a compute unit, and on a banded mask whose
// middle rows hold more entries than its first and last ones the two are dealt from different halves of the matrix
// (attention head, SpMM: 28.2 -> 25.5 us cold).  The SDDMM window for dot products of 65-128 columns is 128 KB, one
// workgroup per compute unit, and keeps 16 waves.
constexpr int kWinWaves = 8;                      // waves per workgroup of the window kernels, one sparse row each
constexpr int kWinWavesWide = 16;                 // ... of the SDDMM window kernel with two column chunks
constexpr int kSpmmMfmaWaves = 2;                 // 256-column tiles per workgroup of the MFMA kernel
constexpr int kSpmmMfmaKParts = 2;                // waves per tile, splitting the contraction

// The matrix-core kernels (fp16 only) do dense work on 32-row panels / 64x64 blocks: selected
// when an estimate of their run time is below that of the direct kernel (microseconds, from
// measured rates on shapes from 1024 x 1024 x 3136 to 8192 x 10240 x 128).  The matrix-core kernels
// do work proportional to m*k whatever the density, in rounds of one workgroup per CU: a panel of
// 32 rows x 512 columns costs about 8.4 us plus 13.8 ns per column of A (SpMM), a 64 x 64 block
// 3.5 us plus 0.5 us per 128 columns of the dot product (SDDMM); filling a panel adds 1 ns per entry
// of its 32 rows (a workgroup walks its rows about twice: once whole, once in pieces per chunk of
// 1024 columns), sampling the blocks 8 us per million entries.  The direct kernels run at the rate
// of their gathers: 19.5 TFLOP/s (SpMM); 14 TFLOP/s for short dot products, 12 beyond 128 columns,
// after a latency floor of 2 us per 64 columns of the dot product (SDDMM).  (Rates refitted on 120
// random shapes, 512 .. 12000 rows and columns, 1 .. 50 % density, n = 48 .. 3136, both families
// forced: the choice then takes 1.006 times the faster one's time on average.)
inline bool spmm_mfma_pays(int m, int k, int n, int nnz) {
  const double wgs = (double)((m + 31) / 32) * (double)(((n + 255) / 256 + kSpmmMfmaWaves - 1) / kSpmmMfmaWaves);
  const double per_panel = m > 0 ? 32.0 * (double)nnz / (double)m : 0.0;
  const double t_mfma = std::ceil(wgs / kComputeUnits) * (8.4 + 0.0138 * (double)k + 1.0e-3 * per_panel);
  const double t_direct = 7.0 + 2.0 * (double)nnz * (double)n / 19.5e6;
  return t_mfma <= t_direct;
}
inline bool sddmm_mfma_pays(int m, int k, int n, int nnz) {
  const double blocks = (double)((m + 63) / 64) * (double)((k + 63) / 64);
  const double t_mfma = std::ceil(blocks / kComputeUnits) * (3.5 + 0.5 * (double)((n + 127) / 128)) + 8e-6 * (double)nnz;
  const double t_direct = 5.0 + 2.0 * (double)(n / 64) + 2.0 * (double)nnz * (double)n / ((n <= 128 ? 14.0 : 12.0) * 1e6);
  return t_mfma <= t_direct;
}

// The matrix-core SpMM keeps rows of B in registers whose loads are still in flight (explicit
// waits); a register spilled inside that window would be copied before its data has arrived.
// The kernel is built without spills; should a toolchain ever produce one (private memory per
// lane != 0), the variant is not offered and the row-splitting kernel runs instead.  Queried
// once; without a device (selection queries on a CPU-only host) the answer is yes.
bool spmm_mfma_runnable() {
  static const bool ok = [] {
    hipFuncAttributes attr;
    bool fine = true;
    for (const void* f : {reinterpret_cast<const void*>(spmm_mfma_kernel<kSpmmMfmaWaves, kSpmmMfmaKParts, int, 1>),
                          reinterpret_cast<const void*>(spmm_mfma_kernel<kSpmmMfmaWaves, kSpmmMfmaKParts, int16_t, 1>)})
      if (hipFuncGetAttributes(&attr, f) == hipSuccess && attr.localSizeBytes != 0) fine = false;
    (void)hipGetLastError();
    return fine;
  }();
  return ok;
}

template <typename T>
void fill_spmm_info(int m, int k, int n, int nnz, const void* B, const void* C, spdl_launch_info* info,
                    int hint = 0) {
  int variant = g_forced[0].load();
  const bool mfma_ok = sizeof(T) == 2 && n % 8 == 0 && n < (1 << 24) && k >= 16 && aligned(B, 16) && aligned(C, 16);
  // nnz == 0: column_indices, values and B may be null, and the slab and matrix-core kernels
  // fetch from them unconditionally; the row-splitting kernel only writes the zeros of C
  if (nnz == 0 && (variant == kSpmmMfma || variant == kSpmmSlab || variant == kSpmmSlabDma)) variant = kSpmmRowsplit;
  if (variant == kSpmmMfma && (!mfma_ok || !spmm_mfma_runnable())) variant = kSpmmRowsplit;
  if (variant < 0 && mfma_ok && nnz > 0 && spmm_mfma_pays(m, k, n, nnz) && spmm_mfma_runnable())
    variant = kSpmmMfma;
  if (variant == kSpmmMfma) {
    // 32-row panels, kSpmmMfmaWaves tiles per workgroup.  (64-row panels, which would halve the
    // reads of B, need 256 accumulator registers per lane; the compiler then spills in the main
    // loop and the kernel is twice as slow.)
    const int tiles_n = (n + 255) / 256;
    info->variant = kSpmmMfma;
    info->vec = 8;
    info->lanes_per_row = kWave;
    info->rows_per_block = 32;
    info->block_threads = 64 * kSpmmMfmaWaves * kSpmmMfmaKParts;
    info->grid_x = ((m + 31) / 32) * ((tiles_n + kSpmmMfmaWaves - 1) / kSpmmMfmaWaves);
    info->grid_y = tiles_n;                     // 256-column tiles (the grid is 1-D)
    return;
  }
  if (variant < 0) {
    const double reuse = (m > 0 && k > 0) ? 64.0 * (double)nnz / ((double)m * (double)k) : 0.0;
    // one workgroup per CU: below half a machine of 64x64 output tiles the row-splitting
    // kernel, which spreads over many more waves, is faster
    const int64_t out_tiles = (int64_t)((m + kSlabRows - 1) / kSlabRows) * ((n + kSlabTile - 1) / kSlabTile);
    // (Narrow outputs: a row of B is one or two cache lines, which makes gathering cheap, and outputs
    // of at most 32 columns use half of a slab tile's lanes or less.  8192 x 8192 at 5 % density:
    // slab 58 us against 26 for gathers at n = 32, 56 against 45 at n = 64; at 10 % the slab kernel
    // wins at n = 64, 66 us against 82, and still loses at n = 32, 68 against 46.)
    // (Wide outputs that leave half the compute units without a full-size workgroup run the slab kernel
    // with workgroups of 8 waves and twice as many stages: 4096 x 4096 at 6 % density, n = 128: 31 us
    // against 24 for the window kernel's gathers; at 12 % 39 against 42.)
    // (Two to four tiles and a B of fewer than 8192 rows, which the gathers then find in L2: the slab
    // kernel pays from 64 * density = 3 on; 16995 x 3895 at 3.2 %, n = 128: 89 us against 62 for
    // row-splitting, 5006 x 2875 at 4.1 %, n = 256: 38 against 26, while the LSTM matrix at 95 %
    // sparsity, 10240 columns, runs 1.4 times faster in it.  Eight tiles or more, scanned once per
    // slab for several tiles: from 1.8 on, sixteen or more from 1.3 on; 15161 x 5174 at 2.9 %, n = 1024:
    // 321 us against 413; 5830 x 4537 at 2.1 %, n = 8192: 998 against 1331.  A B of fewer than 4000 rows
    // is found in L2 at any width: 4297 x 863 at 2.1 %, n = 2048: 56 us against 32 for row-splitting.)
    // (One tile per panel: what the slab kernel needs depends on how the panels fill the machine.  Whole
    // rounds of 256 workgroups, 16384 or 32768 rows: it wins from 64 * density = 2 on, 16384 x 4096 at 4 %,
    // n = 64: 27 us against 36 for the gathers; a round and a half, 24576 rows: from 3 on; three quarters
    // of a round, 12288 rows: not before 5.  Square matrices keep 5: an attention mask is square, a banded
    // one of this density takes twice as long in the slab kernel, and the host cannot tell.)
    const int64_t narrow_rounds = (out_tiles + kComputeUnits - 1) / kComputeUnits;
    const double narrow_fill = narrow_rounds > 0 ? (double)out_tiles / (double)(narrow_rounds * kComputeUnits) : 0.0;
    const double narrow_reuse = (m != k && narrow_fill >= 0.95)                        ? 2.0
                                : (m != k && narrow_fill >= 0.75 && narrow_rounds >= 2) ? 3.0
                                                                                        : 5.0;
    // (fewer than 16 columns use a quarter of a tile's lanes or less: 9957 x 8063 at 28 %, n = 8: 182 us
    // against 135 for row-splitting)
    const double min_reuse = n < 16                                           ? 1.0e9
                             : n <= 32                                        ? 12.0
                             : n <= 64                                        ? narrow_reuse
                             : out_tiles < kComputeUnits                      ? 5.0
                             : (n <= 4 * kSlabTile && k < 8192) || k < 4000   ? 3.0
                             : n >= 16 * kSlabTile                            ? 1.3
                             : n >= 8 * kSlabTile                             ? 1.8
                                                                              : 2.0;
    // (Dense matrices gain so much from the slab kernel that it pays with most compute units idle:
    // 6144 x 2048 at 35 %, n = 64, 96 workgroups: 36 us against 54 for row-splitting; 4096 x 4096 at
    // 50 %, 64 workgroups: 87 against 98; at 20 % and 35 % respectively the two are level.)
    const int64_t min_tiles = (n > 32 && n <= 2 * kSlabTile && reuse >= 32.0)   ? kComputeUnits / 4
                              : (n > 32 && n <= 2 * kSlabTile && reuse >= 16.0) ? 3 * kComputeUnits / 8
                                                                                 : kComputeUnits / 2;
    variant = (sizeof(T) == 4 && slab_usable<T>(n, nnz, B, C) && reuse >= min_reuse && out_tiles >= min_tiles)
                  ? kSpmmSlabDma : kSpmmRowsplit;
    // Thousands of rows of a few hundred entries or more, one or two 64-column tiles, and a shape the
    // slab kernel does not take: the shape of an attention head (paper Sec. "Application: Sparse
    // Transformer").  The host cannot see whether the entries form a band; where the choice is
    // between the row-splitting kernel and the window kernel the latter is 1.2 .. 1.3 times faster
    // with a band and loses nothing without one, where no window is placed and every entry is
    // gathered: with the four lane groups of a wave on one row and sixteen gathers in flight per
    // round it is 5 .. 20 % faster than row-splitting on uniform masks of 2048 .. 8192 rows at 3 ..
    // 30 % density (e.g. 4096 x 8192 at 20 %, n = 64: 71 us against 84; the LSTM matrix at 98 %
    // sparsity, n = 128: 52 against 59).  Narrower outputs leave its lanes idle, shorter rows and fewer
    // rows leave it too few waves in flight (rows of 60: up to 20 % slower).  A wave owns a row, but
    // what a row holds beyond 512 pairs is dealt to all waves of its workgroup, so strongly skewed
    // row lengths (log-normal, a few rows of thousands of entries among rows of hundreds) are no
    // reason to hold back: 4096 x 4096 at 6 %, n = 64: 27 us against 40 for row-splitting, n = 128:
    // 46 against 82.  Where the slab kernel
    // applies it stays the choice from the shape alone: on uniform masks it is up to 1.9 times faster
    // than the window kernel (16384 x 4096 at 10 %), on banded ones 2.2 .. 2.6 times slower, and only
    // the caller knows which it is (spdl_spmm_banded).
    if (variant == kSpmmRowsplit && sizeof(T) == 4 && slab_usable<T>(n, nnz, B, C) &&
        (int64_t)k * n < ((int64_t)1 << 29) &&
        n > 32 && n <= 2 * kWinTile &&
        ((m >= 4096 && (double)nnz >= 100.0 * (double)m) ||
         (m >= 2048 && (double)nnz >= (n > kWinTile ? 192.0 : 400.0) * (double)m)))
      variant = kSpmmWindow;
    // Wider outputs (one workgroup per 64-column tile): the workgroups at work on one tile share
    // k x 256 bytes of B.  While that stays in L2 the row-splitting kernel is as fast or faster; with
    // 7000 columns or more and rows of 120 entries or more the window kernel's sixteen gathers in
    // flight per wave hide the longer latency better (15796 x 11092 at 1.2 %, n = 256: 116 us against
    // 175; 19428 x 9075 at 2.1 %, n = 1024: 636 against 1108; 13651 x 3925 at 3.1 %, n = 256: 98
    // against 69, not taken).
    if (variant == kSpmmRowsplit && sizeof(T) == 4 && slab_usable<T>(n, nnz, B, C) &&
        (int64_t)k * n < ((int64_t)1 << 29) && n > 2 * kWinTile && m >= 4096 && k >= 7000 &&
        (double)nnz >= 120.0 * (double)m)
      variant = kSpmmWindow;
    // the caller says that the entries form a band, or that the row lengths are strongly unequal: the
    // window kernel gathers what is not in a band and shares long rows among the waves of a workgroup
    // (a problem the window kernel cannot take keeps the choice made above)
    if (hint != kHintNone && sizeof(T) == 4 && nnz > 0 && slab_usable<T>(n, nnz, B, C) && (int64_t)k * n < ((int64_t)1 << 29))
      variant = kSpmmWindow;
    // (unequal rows, more than two tiles and a B of fewer than 4000 rows, whose share per tile the
    // gathers find in L2: row-splitting, 1.2 .. 2.4 times faster there than the window kernel, while the
    // slab kernels wait for their longest row)
    if (hint == kHintSkewed && n > 2 * kWinTile && k < 4000) variant = kSpmmRowsplit;
  }
  if (variant == kSpmmWindow && sizeof(T) == 4 && nnz > 0 && slab_usable<T>(n, nnz, B, C) &&
      (int64_t)k * n < ((int64_t)1 << 29)) {
    info->variant = kSpmmWindow;
    info->vec = 4;
    info->lanes_per_row = 16;
    info->rows_per_block = WinShape<kWinWaves>::kRows;
    info->block_threads = 64 * kWinWaves;
    info->grid_x = (m + info->rows_per_block - 1) / info->rows_per_block;
    info->grid_y = (n + kWinTile - 1) / kWinTile;
  } else if ((variant == kSpmmSlab || variant == kSpmmSlabDma) && sizeof(T) == 4 && slab_usable<T>(n, nnz, B, C)) {
    fill_spmm_slab_info(m, k, n, nnz, variant, info);
  } else {
    fill_spmm_rowsplit_info<T>(m, n, nnz, B, C, info);
  }
}

template <typename T, int VEC, typename I>
int launch_spmm_rowsplit_g(const spdl_launch_info& li, int m, int n, const int* ro, const I* ci,
                           const T* val, const int* order, const T* B, T* C, const T* bias, int relu, hipStream_t st) {
  dim3 grid(li.grid_x, li.grid_y), block(256);
  const int seg = 256 / (li.rows_per_block * li.lanes_per_row);       // lane groups per row
#define SPDL_ROWSPLIT(G, SEG)                                                                                  \
  spmm_rowsplit_kernel<T, VEC, G, I, SEG><<<grid, block, 0, st>>>(m, n, ro, ci, val, order, B, C, bias, relu); \
  return SPDL_OK;
  if (seg == 1) {
    switch (li.lanes_per_row) {
      case 8: SPDL_ROWSPLIT(8, 1)
      case 16: SPDL_ROWSPLIT(16, 1)
      case 32: SPDL_ROWSPLIT(32, 1)
      case 64: SPDL_ROWSPLIT(64, 1)
    }
  } else if constexpr (VEC == 16 / (int)sizeof(T)) {
    switch (li.lanes_per_row * 16 + seg) {
      case 8 * 16 + 2: SPDL_ROWSPLIT(8, 2)
      case 8 * 16 + 4: SPDL_ROWSPLIT(8, 4)
      case 8 * 16 + 8: SPDL_ROWSPLIT(8, 8)
      case 16 * 16 + 2: SPDL_ROWSPLIT(16, 2)
      case 16 * 16 + 4: SPDL_ROWSPLIT(16, 4)
      case 32 * 16 + 2: SPDL_ROWSPLIT(32, 2)
    }
  }
#undef SPDL_ROWSPLIT
  return SPDL_ERR_INVALID;
}

template <typename T, typename I>
int launch_spmm_rowsplit(const spdl_launch_info& li, int m, int n, const int* ro, const I* ci,
                         const T* val, const int* order, const T* B, T* C, const T* bias, int relu,
                         hipStream_t st) {
  switch (li.vec) {
    case 1: return launch_spmm_rowsplit_g<T, 1, I>(li, m, n, ro, ci, val, order, B, C, bias, relu, st);
    case 2: return launch_spmm_rowsplit_g<T, 2, I>(li, m, n, ro, ci, val, order, B, C, bias, relu, st);
    case 4: return launch_spmm_rowsplit_g<T, 4, I>(li, m, n, ro, ci, val, order, B, C, bias, relu, st);
    case 8:
      if constexpr (sizeof(T) == 2) return launch_spmm_rowsplit_g<T, 8, I>(li, m, n, ro, ci, val, order, B, C, bias, relu, st);
      return SPDL_ERR_INVALID;
    default: return SPDL_ERR_INVALID;
  }
}

template <typename T, typename I = int>
int spmm_impl(int m, int k, int n, int nnz, const int* ro, const I* ci, const T* val,
              const int* order, const T* B, T* C, void* stream, const T* bias = nullptr, int relu = 0,
              int hint = 0) {
  if (!sizes_ok(m, k, n, nnz)) return SPDL_ERR_INVALID;
  if (m == 0 || n == 0) return SPDL_OK;
  if (!ro || !C || (nnz > 0 && (!ci || !val || !B))) return SPDL_ERR_INVALID;
  hipStream_t st = static_cast<hipStream_t>(stream);
  spdl_launch_info li;
  fill_spmm_info<T>(m, k, n, nnz, B, C, &li, hint);
  (void)hipGetLastError();
  int rc = SPDL_OK;
  constexpr bool kInt32 = sizeof(I) == 4;        // the slab kernels read 32-bit indices only
  if (li.variant == kSpmmMfma) {
    if constexpr (sizeof(T) == 2) {
      static std::atomic<bool> configured{false};
      auto kernel = spmm_mfma_kernel<kSpmmMfmaWaves, kSpmmMfmaKParts, I, 1>;
      if (!configured.load()) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                spmm_mfma_lds_bytes(kMfmaChunk, kSpmmMfmaWaves, 1)) != hipSuccess)
          return SPDL_ERR_LAUNCH;
        configured.store(true);
      }
      kernel<<<dim3(li.grid_x), dim3(li.block_threads), spmm_mfma_lds_bytes(k, kSpmmMfmaWaves, 1), st>>>(
          m, k, n, li.grid_y, ro, ci, val, B, C, bias, relu);
    } else {
      return SPDL_ERR_UNSUPPORTED;
    }
  } else if (li.variant == kSpmmWindow) {
    if constexpr (sizeof(T) == 4 && kInt32) {
      static std::atomic<bool> configured{false};
      auto kernel = spmm_window_kernel<kWinWaves>;
      constexpr int lds = WinShape<kWinWaves>::kLdsBytes;
      if (!configured.load()) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, lds) !=
            hipSuccess)
          return SPDL_ERR_LAUNCH;
        configured.store(true);
      }
      kernel<<<dim3(li.grid_x, li.grid_y), dim3(li.block_threads), lds, st>>>(m, k, n, nnz, ro, ci, val, B, C, bias, relu);
    } else {
      return SPDL_ERR_UNSUPPORTED;
    }
  } else if (li.variant == kSpmmSlab || li.variant == kSpmmSlabDma) {
    if constexpr (sizeof(T) == 4 && kInt32) {
      static std::atomic<bool> configured{false};
      auto kernel = spmm_slab_kernel<T, kSlabS>;
      // 32 pairs fetched ahead per row.  Deeper look-ahead (4 or 6 chunks of 16) was measured
      // on the 70-90 % sparse shapes: the longer scan per round costs more than the waits it saves.
      const bool half = li.block_threads != kSlabThreads;
      const bool two_rows = li.rows_per_block == 2 * kSlabRows;
      const void* dma_kernel_c = half       ? (const void*)spmm_slab_dma_kernel<kSlabHalfS, 1, 2, 8>
                               : two_rows ? (const void*)spmm_slab_dma_kernel<kSlabS, 2, 2>
                                          : (const void*)spmm_slab_dma_kernel<kSlabS, 1, 2>;
      const int lds = half ? kSlabHalfLdsBytes : kSlabLdsBytes;
      const void* dma_kernel = dma_kernel_c;
      // (two rows per group and 2 .. kSlabTilesMax tiles per workgroup: scanned once per slab for all tiles)
      if (li.variant == kSpmmSlabDma && two_rows && li.grid_y >= 2 && li.grid_y <= kSlabTilesMax &&
          slab_tiles_fits(m, k, nnz))
        dma_kernel = (const void*)spmm_slab_tiles_kernel<kSlabS, 2, 3, kSlabTilesMax>;
      if (!configured.load()) {
        for (const void* f : {(const void*)kernel, (const void*)spmm_slab_dma_kernel<kSlabS, 1, 2>,
                              (const void*)spmm_slab_dma_kernel<kSlabS, 2, 2>,
                              (const void*)spmm_slab_tiles_kernel<kSlabS, 2, 3, kSlabTilesMax>})
          if (hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, kSlabLdsBytes) != hipSuccess)
            return SPDL_ERR_LAUNCH;
        if (hipFuncSetAttribute((const void*)spmm_slab_dma_kernel<kSlabHalfS, 1, 2, 8>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, kSlabHalfLdsBytes) != hipSuccess)
          return SPDL_ERR_LAUNCH;
        configured.store(true);
      }
      const int panels = (m + li.rows_per_block - 1) / li.rows_per_block;
      const int tiles = (n + kSlabTile - 1) / kSlabTile;
      const dim3 grid(li.grid_x), block(li.block_threads);
      if (li.variant == kSpmmSlab) {
        kernel<<<grid, block, kSlabLdsBytes, st>>>(m, k, n, nnz, tiles, li.grid_y, panels, ro, ci, val, order, B, C,
                                                   bias, relu);
      } else {
        int tpw = li.grid_y;
        void* args[] = {&m, &k, &n, &nnz, (void*)&tiles, &tpw, (void*)&panels, &ro, &ci, &val, &order, &B, &C,
                        &bias, &relu};
        if (hipLaunchKernel(dma_kernel, grid, block, args, lds, st) != hipSuccess) return SPDL_ERR_LAUNCH;
      }
    } else {
      return SPDL_ERR_UNSUPPORTED;
    }
  } else {
    rc = launch_spmm_rowsplit<T, I>(li, m, n, ro, ci, val, order, B, C, bias, relu, st);
  }
  if (rc != SPDL_OK) return rc;
  return hipGetLastError() == hipSuccess ? SPDL_OK : SPDL_ERR_LAUNCH;
}

template <typename T>
bool sddmm_group_usable(int n, const void* L, const void* R) {
  return n > 0 && n % 4 == 0 && aligned(L, 4 * sizeof(T)) && aligned(R, 4 * sizeof(T));
}

// Shape of the slab kernel's launch: U 64-column chunks per LDS row, S = 256/U rows of R per
// slab, the columns of A split into `ksplit` runs of `spp` slabs so that every CU gets a
// workgroup.
struct SddmmSlabShape { int U, S, deferred, ksplit, spp, panels, lds_bytes; };

// U chunks of 64 columns per LDS row (1 for n <= 64, else 2), 64 KB slabs.  Dot products of up to
// 128 columns are finished inside a slab; longer ones stream 128-column pieces of 128-row slabs
// and keep two strips per row and slab in registers.
SddmmSlabShape sddmm_slab_shape(int m, int k, int n) {
  SddmmSlabShape sh;
  sh.deferred = n > 128;
  sh.U = n <= 64 ? 1 : 2;
  sh.S = 256 / sh.U;
  sh.panels = (m + kSdRows - 1) / kSdRows;
  const int total = std::max(1, (k + sh.S - 1) / sh.S);
  sh.spp = split_for_machine(sh.panels, total);
  sh.ksplit = (total + sh.spp - 1) / sh.spp;
  sh.lds_bytes = 2 * (sh.S + 1) * 256 * sh.U;
  return sh;
}


// Launch shape of the lane kernel: sparse rows per 16-lane group (two where A is sparse, so
// that a stage of arithmetic outlasts the copy of the next slab and R is fetched by fewer
// workgroups), look-ahead in chunks of 16 column indices (mean + 4 sigma of a row's count in one
// slab of 128 columns), and the split of A's columns over workgroups that fills the machine.
struct SddmmLaneShape { int rpg, nchd, ksplit, spp, panels; };

SddmmLaneShape sddmm_lane_shape(int m, int k, int nnz, bool one_row_per_group = false, bool scaled = false) {
  SddmmLaneShape sh;
  const double d = (m > 0 && k > 0) ? (double)nnz / ((double)m * (double)k) : 0.0;
  const double mean = kLaneS * d, sd = std::sqrt(mean * std::max(0.0, 1.0 - d));
  sh.nchd = std::max(1, std::min(4, (int)std::ceil((mean + 4.0 * sd + 1.0) / 16.0)));
  // (two rows and three or more chunks of look-ahead do not fit the 128 registers of a lane: measured
  // 19 % slower than one row at 86 % sparsity)
  sh.rpg = (d >= 0.15 || sh.nchd > (scaled ? 1 : 2)) ? 1 : 2;       // (the scaled form holds A's values as well)
  if (sh.rpg == 2 && m <= kSdRows * kComputeUnits / 8) sh.rpg = 1;      // too few rows to share
  if (one_row_per_group) sh.rpg = 1;
  sh.panels = (m + kSdRows * sh.rpg - 1) / (kSdRows * sh.rpg);
  const int total = std::max(1, (k + kLaneS - 1) / kLaneS);
  sh.spp = split_for_machine(sh.panels, total);
  sh.ksplit = (total + sh.spp - 1) / sh.spp;
  return sh;
}

template <int RPG, int NCHD, bool NT = false, bool ACCUM = false>
int launch_sddmm_lane(const SddmmLaneShape& sh, int grid, int m, int k, int n, int nnz, const int* ro, const int* ci,
                      const float* L, const float* R, float* out, const float* scale, hipStream_t st,
                      const int* order = nullptr, int ld = 0, int c0 = 0) {
  static std::atomic<bool> configured{false};
  constexpr int lds = NT ? kLaneNtLdsBytes : kLaneLdsBytes;
  const void* plain = reinterpret_cast<const void*>(sddmm_lane_kernel<RPG, NCHD, false, NT, ACCUM>);
  const void* scaled = reinterpret_cast<const void*>(sddmm_lane_kernel<RPG, NCHD, true, NT, ACCUM>);
  if (!configured.load()) {
    for (const void* f : {plain, scaled})
      if (hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess)
        return SPDL_ERR_LAUNCH;
    configured.store(true);
  }
  if (ld == 0) ld = n;
  int ksplit = sh.ksplit, spp = sh.spp, panels = sh.panels;
  void* args[] = {&m, &k, &n, &nnz, &ksplit, &spp, &panels, &ro, &ci, &L, &R, &out, &scale, &order, &ld, &c0};
  return hipLaunchKernel(scale ? scaled : plain, dim3(grid), dim3(kSdThreads), args, lds, st) == hipSuccess
             ? SPDL_OK : SPDL_ERR_LAUNCH;
}

template <typename T>
bool sddmm_lane_usable(int n, int nnz, const void* L, const void* R) {
  // (dot products longer than 128 columns take one pass per 128 columns; 32-bit byte offsets inside
  // a slab of R: 128 rows * n * 4 < 2^31)
  return sizeof(T) == 4 && sddmm_group_usable<T>(n, L, R) && n < (1 << 21) && nnz < (1 << 29);
}

template <typename T>
void fill_sddmm_info(int m, int k, int n, int nnz, const void* L, const void* R, spdl_launch_info* info,
                     int hint = 0) {
  const bool fast_ok = sddmm_group_usable<T>(n, L, R);
  int variant = g_forced[1].load();
  const bool free_choice = variant < 0;
  const bool mfma_ok = sizeof(T) == 2 && n > 0 && n % 8 == 0 && aligned(L, 16) && aligned(R, 16) &&
                       (int64_t)((m + 63) / 64) * ((k + 63) / 64) < ((int64_t)1 << 31);
  if (variant == kSddmmMfma && !mfma_ok) variant = kSddmmGroup;
  if (variant < 0 && mfma_ok && sddmm_mfma_pays(m, k, n, nnz)) variant = kSddmmMfma;
  if (variant == kSddmmMfma) {
    const int64_t tiles = (int64_t)((m + 63) / 64) * ((k + 63) / 64);
    info->variant = kSddmmMfma;
    info->vec = 8;
    info->lanes_per_row = kWave;
    info->rows_per_block = 64;
    info->block_threads = 256;
    // 8 XCDs x (half the row tiles, rounded up) x (a quarter of the column tiles, rounded up)
    info->grid_x = 8 * (((m + 63) / 64 + 1) / 2) * (((k + 63) / 64 + 3) / 4);
    info->grid_y = (k + 63) / 64;               // 64-column blocks per panel (the grid is 1-D)
    return;
  }
  bool skewed_lane = false;      // (for the hint of unequal rows) lane kernel estimated faster than the nonzero-split one
  if (variant < 0) {
    const double density = (m > 0 && k > 0) ? (double)nnz / ((double)m * (double)k) : 0.0;
    const double reuse = 64.0 * density;
    const bool fp32_any_m = fast_ok && sizeof(T) == 4 && nnz < (1 << 29) && n < (1 << 21);
    const bool fp32_fast = fp32_any_m && m >= 512;
    if (!fast_ok) {
      variant = kSddmmRowstrip;
    } else if (n <= 128 || !fp32_any_m) {
      // Short dot products gain little from the slabs (a row of R is one or two cache lines) unless
      // the reuse is high, and the nonzero-split kernel does not care how the entries are laid out
      // (a banded attention mask leaves most of a panel's column ranges nearly empty).  65..128
      // columns: the lane kernel, as long as a panel of 64 rows meets the same row of R at least
      // once on average.
      const bool lane = fp32_fast && n > 64 && reuse >= 1.0;
      // (5 <= reuse < 8 with at least 128 panels of 64 rows: on uniform masks the slab kernel is then
      // 1.25 .. 1.4 times faster than gathering, 8192 x 2048 at 10 %: 18.7 us against 25; with 64
      // panels it has to split A's columns over workgroups and the banded attention mask of 4096
      // rows, also 10 % dense, takes 36 us against 24)
      // (panels that fill whole rounds of one workgroup per compute unit, 16384 or 32768 rows: from 4 on,
      // 7 .. 26 % faster than gathering there; not for square matrices, which may be attention masks)
      const int64_t panels64 = (m + kSdRows - 1) / kSdRows;
      const int64_t rounds64 = (panels64 + kComputeUnits - 1) / kComputeUnits;
      const bool whole_rounds = m != k && rounds64 > 0 && (double)panels64 >= 0.95 * (double)(rounds64 * kComputeUnits);
      const bool slab = fp32_fast && reuse >= 2.0 &&
                        (n >= 128 || reuse >= 8.0 || (reuse >= 5.0 && m >= 8192) || (reuse >= 4.0 && whole_rounds));
      variant = lane ? kSddmmLane : slab ? kSddmmSlabDma : kSddmmGroup;
      // The shape of an attention head (33..64 columns, thousands of rows of a few hundred entries,
      // at most 1/8 dense; paper Sec. "Application: Sparse Transformer"): the window kernel, which is
      // the nonzero-split kernel with the rows of R around a band taken from LDS and the four lane
      // groups of a wave on one row (13 % faster on a band of 256 at sequence 4096, 5 .. 20 % on uniform
      // masks of that shape).  Not wider than that: the nonzero-split kernel does not care how long
      // the rows are, the window kernel owns rows, and on log-normal row lengths it takes 1.5 times as
      // long (4096 x 4096 at 6 %: 26 us against 17) although the waves of a workgroup share what a row
      // holds beyond 512 entries.
      if (variant == kSddmmGroup && fp32_fast && n > 32 && n <= kWinTile && m >= 4096 && aligned(L, 16) &&
          aligned(R, 16) && (int64_t)k * n < ((int64_t)1 << 29) && (double)nnz >= 192.0 * (double)m &&
          (double)nnz <= 0.125 * (double)m * (double)k)
        variant = kSddmmWindow;
    } else {
      // Longer dot products: three candidates, chosen by an estimate of their run times from measured
      // rates (paper Sec. "Experiments": the kernel and tile are picked by heuristics from the shape;
      // the discussion there names better selection as the open end).  The lane kernel runs once per
      // 128 columns and walks A every time (about 9.5 us of fixed cost per pass); the slab kernel
      // walks A once and keeps at most 32 partial sums per row and slab in registers, so it slows
      // down where rows get dense; the nonzero-split kernel gathers rows of R and runs at the rate
      // of those gathers whatever the density.  Rates in TFLOP/s against density, measured on
      // matrices from 2048 x 2048 to 8192 x 10240 with n = 256 .. 4096.
      static const double ds[7] = {0.01, 0.02, 0.04, 0.10, 0.16, 0.30, 0.50};
      static const double lane_rate[7] = {5.0, 9.0, 14.0, 22.6, 26.0, 33.0, 32.0};
      static const double slab_rate[7] = {4.0, 7.0, 12.8, 22.8, 24.0, 19.0, 12.0};
      auto rate = [&](const double* r) {
        if (density <= ds[0]) return r[0];
        for (int i = 1; i < 7; ++i)
          if (density <= ds[i]) return r[i - 1] + (r[i] - r[i - 1]) * (density - ds[i - 1]) / (ds[i] - ds[i - 1]);
        return r[6];
      };
      const double flops = 2.0 * (double)nnz * (double)n;                   // per launch, all passes
      const int passes = (n + 127) / 128;
      // (the rates are those of a full machine: a small matrix gives fewer workgroups than there are
      // compute units, 760 x 231 at 43 %, n = 2048: 24 workgroups, 193 us in the slab kernel against 67
      // for the nonzero-split kernel, which spreads over the chip whatever the shape)
      const SddmmLaneShape lsh = sddmm_lane_shape(m, k, nnz, true);
      const SddmmSlabShape ssh = sddmm_slab_shape(m, k, n);
      const double lane_fill = std::min(1.0, (double)lsh.panels * lsh.ksplit / kComputeUnits);
      const double slab_fill = std::min(1.0, (double)ssh.panels * ssh.ksplit / kComputeUnits);
      const double t_lane = passes * 9.5 + flops / (rate(lane_rate) * 1e6 * lane_fill);   // microseconds
      // (every panel of 64 rows streams all of R through its compute unit: 8 TB/s over the chip at best)
      const double panels64 = (double)((m + kSdRows - 1) / kSdRows);
      const double t_slab = 8.0 + std::max(flops / (rate(slab_rate) * 1e6 * slab_fill), panels64 * (double)k * (double)n * 4.0 / 8.0e6);
      // (a strip of the gather kernel steps through its dot product 64 columns at a time, about 1.1 us
      // of memory latency per step: the floor for small problems)
      const double t_group = 5.0 + 1.1 * (double)(n / 64) + flops / (n < 2048 ? 7.0e6 : 5.5e6);
      variant = (t_lane <= t_slab && t_lane <= t_group) ? kSddmmLane : t_slab <= t_group ? kSddmmSlabDma : kSddmmGroup;
      // (the lane kernel's rate is that of rows of equal length; an R of a few megabytes is gathered from L2)
      skewed_lane = t_lane <= 0.45 * t_group && (double)k * (double)n * 4.0 >= 7.0e6;
    }
  }
  if ((variant == kSddmmSlab || variant == kSddmmSlabDma) &&
      !(fast_ok && sizeof(T) == 4 && nnz < (1 << 29) && n < (1 << 21)))   // 32-bit byte offsets
    variant = kSddmmGroup;
  if (variant == kSddmmLane && !sddmm_lane_usable<T>(n, nnz, L, R)) variant = kSddmmGroup;
  const bool window_ok = sizeof(T) == 4 && fast_ok && aligned(L, 16) && aligned(R, 16) && n <= 2 * kWinTile && nnz > 0 &&
                         (int64_t)k * n < ((int64_t)1 << 29);
  // the caller says that the entries form a band (a problem the window kernel cannot take keeps the
  // choice made above)
  if (free_choice && hint == kHintBanded && window_ok) variant = kSddmmWindow;
  // the caller says that the row lengths are strongly unequal: the nonzero-split kernel, which does not
  // care, or for dot products of more than 128 columns the lane kernel in passes where the estimate
  // above gives it less than 0.45 of that kernel's time (dense matrices; the slab kernel, whose
  // deferred partial sums overflow on the long rows, is left out)
  if (free_choice && hint == kHintSkewed && fast_ok && (variant == kSddmmLane || variant == kSddmmSlabDma || variant == kSddmmWindow))
    variant = skewed_lane ? kSddmmLane : kSddmmGroup;
  if (variant == kSddmmWindow && !window_ok) variant = kSddmmGroup;
  if (variant == kSddmmGroup && !fast_ok) variant = kSddmmRowstrip;
  const int avg = m > 0 ? nnz / m : 0;
  info->variant = variant;
  info->block_threads = 256;
  info->grid_y = 1;
  if (variant == kSddmmWindow) {
    info->vec = 4;
    info->lanes_per_row = 16;
    const int waves = n <= kWinTile ? kWinWaves : kWinWavesWide;
    info->rows_per_block = waves;
    info->block_threads = 64 * waves;
    info->grid_x = (m + waves - 1) / waves;
    return;
  }
  if (variant == kSddmmLane) {
    const SddmmLaneShape sh = sddmm_lane_shape(m, k, nnz, n > 128);
    info->vec = 8;
    info->lanes_per_row = 2;
    info->rows_per_block = kSdRows * sh.rpg;
    info->block_threads = kSdThreads;
    info->grid_x = slab_grid_size(sh.panels, sh.ksplit);
    info->grid_y = sh.ksplit;               // column ranges of A (the grid is 1-D)
    return;
  }
  if (variant == kSddmmSlab || variant == kSddmmSlabDma) {
    const SddmmSlabShape sh = sddmm_slab_shape(m, k, n);
    info->vec = 4 * sh.U;
    info->lanes_per_row = 16;
    info->rows_per_block = kSdRows;
    info->block_threads = kSdThreads;
    info->grid_x = slab_grid_size(sh.panels, sh.ksplit);
    info->grid_y = sh.ksplit;               // column ranges of A (the grid is 1-D)
    return;
  }
  if (variant == kSddmmGroup) {
    // entries per wave: four strips of 16 while the machine (32 waves on each CU) is not
    // full, then as many as keep the grid at about one wave per slot
    const int64_t slots = (int64_t)kComputeUnits * 32;
    const int quads = (int)std::max<int64_t>(1, std::min<int64_t>(64, ((int64_t)nnz / 64 + slots - 1) / slots));
    info->vec = 4;
    info->lanes_per_row = 16;
    info->rows_per_block = quads * 64;                     // entries per wave
    const int64_t waves = ((int64_t)nnz + quads * 64 - 1) / (quads * 64);
    info->grid_x = (int)((waves + 3) / 4);
    return;
  }
  int vec = pick_vec<T>(n, L, R, 16 / (int)sizeof(T));
  while (vec > 1 && kWave * vec / 2 >= n) vec /= 2;     // do not idle lanes on short dot products
  const int split = std::max(1, std::min(8, avg / (4 * kStrip)));
  info->vec = vec;
  info->lanes_per_row = kWave;
  info->rows_per_block = split;
  const int64_t waves = (int64_t)m * split;
  info->grid_x = (int)((waves + 3) / 4);
}

template <typename T, int U, int S, bool DEFERRED>
int launch_sddmm_slab(const SddmmSlabShape& sh, int grid, int m, int k, int n, int nnz, const int* ro,
                      const int* ci, const T* L, const T* R, T* out, const T* scale, hipStream_t st, bool dma,
                      const int* order) {
  static std::atomic<bool> configured{false};
  static std::atomic<bool> configured_dma{false};
  if (dma) {
    auto kernel = sddmm_slab_dma_kernel<U, S, DEFERRED>;
    if (!configured_dma.load()) {
      if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                              sh.lds_bytes) != hipSuccess)
        return SPDL_ERR_LAUNCH;
      configured_dma.store(true);
    }
    kernel<<<dim3(grid), dim3(kSdThreads), sh.lds_bytes, st>>>(m, k, n, nnz, sh.ksplit, sh.spp, sh.panels, ro, ci,
                                                               L, R, out, scale, order);
    return SPDL_OK;
  }
  auto kernel = sddmm_slab_kernel<T, U, S, DEFERRED>;
  if (!configured.load()) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            sh.lds_bytes) != hipSuccess)
      return SPDL_ERR_LAUNCH;
    configured.store(true);
  }
  kernel<<<dim3(grid), dim3(kSdThreads), sh.lds_bytes, st>>>(m, k, n, nnz, sh.ksplit, sh.spp, sh.panels, ro, ci,
                                                             L, R, out, scale);
  return SPDL_OK;
}

template <typename T>
int sddmm_impl(int m, int k, int n, int nnz, const int* ro, const int* ci, const T* L, const T* R,
               T* out, void* stream, const T* scale = nullptr, const int* order = nullptr, int hint = 0) {
  if (!sizes_ok(m, k, n, nnz)) return SPDL_ERR_INVALID;
  if (m == 0 || nnz == 0) return SPDL_OK;
  if (!ro || !ci || !out || (n > 0 && (!L || !R))) return SPDL_ERR_INVALID;
  hipStream_t st = static_cast<hipStream_t>(stream);
  spdl_launch_info li;
  fill_sddmm_info<T>(m, k, n, nnz, L, R, &li, hint);
  dim3 grid(li.grid_x), block(256);
  const int split = li.rows_per_block;
  (void)hipGetLastError();
  if (li.variant == kSddmmMfma) {
    if constexpr (sizeof(T) == 2) {
      static std::atomic<bool> configured{false};
      if (!configured.load()) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(sddmm_mfma_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kSddmmMfmaLdsBytes) != hipSuccess)
          return SPDL_ERR_LAUNCH;
        configured.store(true);
      }
      sddmm_mfma_kernel<<<dim3(li.grid_x), dim3(256), kSddmmMfmaLdsBytes, st>>>(m, k, n, li.grid_y, ro, ci, L, R, out,
                                                                                scale);
      return hipGetLastError() == hipSuccess ? SPDL_OK : SPDL_ERR_LAUNCH;
    } else {
      return SPDL_ERR_UNSUPPORTED;
    }
  }
  if (li.variant == kSddmmLane) {
    if constexpr (sizeof(T) == 4) {
      const SddmmLaneShape sh = sddmm_lane_shape(m, k, nnz, n > 128, scale != nullptr);
      const int grid = slab_grid_size(sh.panels, sh.ksplit);
      // one pass per chunk of 128 columns; passes after the first add to what out holds
      for (int c0 = 0; c0 < n; c0 += 128) {
        const int nc = std::min(128, n - c0);
        int rc = SPDL_ERR_UNSUPPORTED;
#define SPDL_LANE(RPG, NCHD)                                                                           \
  if (sh.rpg == RPG && sh.nchd == NCHD) {                                                              \
    if (c0 == 0)                                                                                       \
      rc = launch_sddmm_lane<RPG, NCHD>(sh, grid, m, k, nc, nnz, ro, ci, L, R, out, scale, st, order, n, 0); \
    else if constexpr (RPG == 1)                                                                       \
      rc = launch_sddmm_lane<1, NCHD, false, true>(sh, grid, m, k, nc, nnz, ro, ci, L + c0, R + c0, out, scale, st, \
                                                   order, n, c0);                                      \
  }
        SPDL_LANE(1, 1) SPDL_LANE(1, 2) SPDL_LANE(1, 3) SPDL_LANE(1, 4)
        SPDL_LANE(2, 1) SPDL_LANE(2, 2)
#undef SPDL_LANE
        if (rc != SPDL_OK) return rc;
      }
      return hipGetLastError() == hipSuccess ? SPDL_OK : SPDL_ERR_LAUNCH;
    } else {
      return SPDL_ERR_UNSUPPORTED;
    }
  }
  if (li.variant == kSddmmSlab || li.variant == kSddmmSlabDma) {
    if constexpr (sizeof(T) == 4) {
      const SddmmSlabShape sh = sddmm_slab_shape(m, k, n);
      const bool dma = li.variant == kSddmmSlabDma;
      int rc;
      if (sh.deferred) rc = launch_sddmm_slab<T, 2, 128, true>(sh, li.grid_x, m, k, n, nnz, ro, ci, L, R, out, scale, st, dma, order);
      else if (sh.U == 1) rc = launch_sddmm_slab<T, 1, 256, false>(sh, li.grid_x, m, k, n, nnz, ro, ci, L, R, out, scale, st, dma, order);
      else rc = launch_sddmm_slab<T, 2, 128, false>(sh, li.grid_x, m, k, n, nnz, ro, ci, L, R, out, scale, st, dma, order);
      if (rc != SPDL_OK) return rc;
      return hipGetLastError() == hipSuccess ? SPDL_OK : SPDL_ERR_LAUNCH;
    } else {
      return SPDL_ERR_UNSUPPORTED;
    }
  }
  if (li.variant == kSddmmWindow) {
    if constexpr (sizeof(T) == 4) {
      static std::atomic<bool> configured{false};
      constexpr int lds1 = 256 * 64 * 4;
      if (!configured.load()) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(sddmm_window_kernel<kWinWaves, 1>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, lds1) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void*>(sddmm_window_kernel<kWinWavesWide, 2>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 2 * lds1) != hipSuccess)
          return SPDL_ERR_LAUNCH;
        configured.store(true);
      }
      if (n <= kWinTile)
        sddmm_window_kernel<kWinWaves, 1><<<dim3(li.grid_x), dim3(li.block_threads), lds1, st>>>(m, k, n, nnz, ro, ci, L,
                                                                                                 R, out, scale);
      else
        sddmm_window_kernel<kWinWavesWide, 2><<<dim3(li.grid_x), dim3(li.block_threads), 2 * lds1, st>>>(m, k, n, nnz, ro, ci,
                                                                                                     L, R, out, scale);
      return hipGetLastError() == hipSuccess ? SPDL_OK : SPDL_ERR_LAUNCH;
    } else {
      return SPDL_ERR_UNSUPPORTED;
    }
  }
  if (li.variant == kSddmmGroup) {
    sddmm_group_kernel<T><<<grid, block, 0, st>>>(m, n, nnz, li.rows_per_block, ro, ci, L, R, out, scale);
    return hipGetLastError() == hipSuccess ? SPDL_OK : SPDL_ERR_LAUNCH;
  }
  switch (li.vec) {
    case 1: sddmm_rowstrip_kernel<T, 1><<<grid, block, 0, st>>>(m, n, split, ro, ci, L, R, out, scale); break;
    case 2: sddmm_rowstrip_kernel<T, 2><<<grid, block, 0, st>>>(m, n, split, ro, ci, L, R, out, scale); break;
    case 4: sddmm_rowstrip_kernel<T, 4><<<grid, block, 0, st>>>(m, n, split, ro, ci, L, R, out, scale); break;
    case 8:
      if constexpr (sizeof(T) == 2) {
        sddmm_rowstrip_kernel<T, 8><<<grid, block, 0, st>>>(m, n, split, ro, ci, L, R, out, scale);
        break;
      }
      return SPDL_ERR_INVALID;
    default: return SPDL_ERR_INVALID;
  }
  return hipGetLastError() == hipSuccess ? SPDL_OK : SPDL_ERR_LAUNCH;
}

template <typename T>
int sddmm_nt_impl(int m, int k, int n, int nnz, const int* ro, const int* ci, const T* values, const T* L,
                  const T* Rn, T* out, void* stream) {
  if (!sizes_ok(m, k, n, nnz)) return SPDL_ERR_INVALID;
  if (m == 0 || nnz == 0) return SPDL_OK;
  if (!ro || !ci || !out || values == out || (n > 0 && (!L || !Rn))) return SPDL_ERR_INVALID;
  (void)hipGetLastError();
  if constexpr (sizeof(T) == 4) {
    // dot products of up to 128 columns: the lane kernel, which fetches its slabs of Rn as they lie
    // and transposes them inside LDS (32-bit byte offsets into Rn: n * k * 4 < 2^31)
    if (sddmm_lane_usable<T>(n, nnz, L, Rn) && n <= 128 && k % 4 == 0 && m >= 64 && (int64_t)n * k < ((int64_t)1 << 29) &&
        g_forced[1].load() < 0) {
      // (one sparse row per group: the transposing pass needs registers that two rows' L values take)
      const SddmmLaneShape sh = sddmm_lane_shape(m, k, nnz, true);
      const int grid = slab_grid_size(sh.panels, sh.ksplit);
      hipStream_t st = static_cast<hipStream_t>(stream);
      int rc = SPDL_ERR_UNSUPPORTED;
#define SPDL_LANE_NT(NCHD) \
  if (sh.nchd == NCHD) rc = launch_sddmm_lane<1, NCHD, true>(sh, grid, m, k, n, nnz, ro, ci, L, Rn, out, values, st);
      SPDL_LANE_NT(1) SPDL_LANE_NT(2) SPDL_LANE_NT(3) SPDL_LANE_NT(4)
#undef SPDL_LANE_NT
      if (rc != SPDL_OK) return rc;
      return hipGetLastError() == hipSuccess ? SPDL_OK : SPDL_ERR_LAUNCH;
    }
  }
  sddmm_nt_kernel<T><<<dim3((nnz + 255) / 256), dim3(256), 0, static_cast<hipStream_t>(stream)>>>(
      m, k, n, nnz, ro, ci, L, Rn, out, values);
  return hipGetLastError() == hipSuccess ? SPDL_OK : SPDL_ERR_LAUNCH;
}

}  // namespace

extern "C" {

int spdl_spmm(int m, int k, int n, int nnz, const int* row_offsets, const int* column_indices,
              const float* values, const int* row_order, const float* B, float* C, void* stream) {
  return spmm_impl<float>(m, k, n, nnz, row_offsets, column_indices, values, row_order, B, C, stream);
}

int spdl_spmm_f16(int m, int k, int n, int nnz, const int* row_offsets, const int* column_indices,
                  const uint16_t* values, const int* row_order, const uint16_t* B, uint16_t* C,
                  void* stream) {
  return spmm_impl<_Float16>(m, k, n, nnz, row_offsets, column_indices,
                             reinterpret_cast<const _Float16*>(values), row_order,
                             reinterpret_cast<const _Float16*>(B), reinterpret_cast<_Float16*>(C), stream);
}

int spdl_spmm_bias_relu(int m, int k, int n, int nnz, const int* row_offsets, const int* column_indices,
                        const float* values, const int* row_order, const float* B, const float* bias,
                        int relu, float* C, void* stream) {
  return spmm_impl<float>(m, k, n, nnz, row_offsets, column_indices, values, row_order, B, C, stream, bias,
                          relu != 0);
}

int spdl_spmm_bias_relu_f16(int m, int k, int n, int nnz, const int* row_offsets, const int* column_indices,
                            const uint16_t* values, const int* row_order, const uint16_t* B,
                            const uint16_t* bias, int relu, uint16_t* C, void* stream) {
  return spmm_impl<_Float16>(m, k, n, nnz, row_offsets, column_indices,
                             reinterpret_cast<const _Float16*>(values), row_order,
                             reinterpret_cast<const _Float16*>(B), reinterpret_cast<_Float16*>(C), stream,
                             reinterpret_cast<const _Float16*>(bias), relu != 0);
}

int spdl_csr_softmax(int m, int nnz, const int* row_offsets, const float* logits, float scale,
                     float* probabilities, void* stream) {
  if (m < 0 || nnz < 0) return SPDL_ERR_INVALID;
  if (m == 0 || nnz == 0) return SPDL_OK;
  if (!row_offsets || !logits || !probabilities) return SPDL_ERR_INVALID;
  (void)hipGetLastError();
  csr_softmax_kernel<<<dim3((m + 3) / 4), dim3(256), 0, static_cast<hipStream_t>(stream)>>>(
      m, row_offsets, logits, scale, probabilities);
  return hipGetLastError() == hipSuccess ? SPDL_OK : SPDL_ERR_LAUNCH;
}

int spdl_build_transpose_host(int m, int k, int nnz, const int* ro, const int* ci, int* t_ro, int* t_ci,
                              int* perm) {
  if (m < 0 || k < 0 || nnz < 0 || !ro || !t_ro || (nnz > 0 && (!ci || !t_ci || !perm))) return SPDL_ERR_INVALID;
  if (ro[0] != 0 || ro[m] != nnz) return SPDL_ERR_BAD_CSR;
  // counting sort by column; rows are visited in order, so equal columns keep the row order
  std::fill(t_ro, t_ro + k + 1, 0);
  for (int i = 0; i < m; ++i) {
    if (ro[i + 1] < ro[i] || ro[i + 1] > nnz) return SPDL_ERR_BAD_CSR;
    for (int p = ro[i]; p < ro[i + 1]; ++p) {
      if (ci[p] < 0 || ci[p] >= k) return SPDL_ERR_BAD_CSR;
      ++t_ro[ci[p] + 1];
    }
  }
  for (int c = 0; c < k; ++c) t_ro[c + 1] += t_ro[c];
  // The write cursors live in t_ro itself (no allocation): entry c is advanced as column c fills
  // and ends at the start of column c+1, so shifting the array up by one restores the offsets.
  for (int i = 0; i < m; ++i)
    for (int p = ro[i]; p < ro[i + 1]; ++p) {
      const int t = t_ro[ci[p]]++;
      t_ci[t] = i;
      perm[t] = p;
    }
  for (int c = k; c > 0; --c) t_ro[c] = t_ro[c - 1];
  t_ro[0] = 0;
  return SPDL_OK;
}

int spdl_permute_values(int nnz, int elem_bytes, const int* perm, const void* values, void* out, void* stream) {
  if (nnz < 0 || (elem_bytes != 2 && elem_bytes != 4)) return SPDL_ERR_INVALID;
  if (nnz == 0) return SPDL_OK;
  if (!perm || !values || !out) return SPDL_ERR_INVALID;
  (void)hipGetLastError();
  const dim3 grid((nnz + 255) / 256), block(256);
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (elem_bytes == 4)
    permute_values_kernel<float><<<grid, block, 0, st>>>(nnz, perm, static_cast<const float*>(values),
                                                         static_cast<float*>(out));
  else
    permute_values_kernel<uint16_t><<<grid, block, 0, st>>>(nnz, perm, static_cast<const uint16_t*>(values),
                                                            static_cast<uint16_t*>(out));
  return hipGetLastError() == hipSuccess ? SPDL_OK : SPDL_ERR_LAUNCH;
}

int spdl_sddmm(int m, int k, int n, int nnz, const int* row_offsets, const int* column_indices,
               const float* L, const float* R, float* out_values, void* stream) {
  return sddmm_impl<float>(m, k, n, nnz, row_offsets, column_indices, L, R, out_values, stream);
}

int spdl_spmm_banded(int m, int k, int n, int nnz, const int* row_offsets, const int* column_indices,
                     const float* values, const float* B, float* C, void* stream) {
  return spmm_impl<float>(m, k, n, nnz, row_offsets, column_indices, values, nullptr, B, C, stream, nullptr, 0, kHintBanded);
}

int spdl_sddmm_banded(int m, int k, int n, int nnz, const int* row_offsets, const int* column_indices,
                      const float* L, const float* R, float* out_values, void* stream) {
  return sddmm_impl<float>(m, k, n, nnz, row_offsets, column_indices, L, R, out_values, stream, nullptr, nullptr, kHintBanded);
}

int spdl_spmm_skewed(int m, int k, int n, int nnz, const int* row_offsets, const int* column_indices,
                     const float* values, const float* B, float* C, void* stream) {
  return spmm_impl<float>(m, k, n, nnz, row_offsets, column_indices, values, nullptr, B, C, stream, nullptr, 0, kHintSkewed);
}

int spdl_sddmm_skewed(int m, int k, int n, int nnz, const int* row_offsets, const int* column_indices,
                      const float* L, const float* R, float* out_values, void* stream) {
  return sddmm_impl<float>(m, k, n, nnz, row_offsets, column_indices, L, R, out_values, stream, nullptr, nullptr, kHintSkewed);
}

int spdl_sddmm_ordered(int m, int k, int n, int nnz, const int* row_offsets, const int* column_indices,
                       const int* row_order, const float* L, const float* R, float* out_values, void* stream) {
  return sddmm_impl<float>(m, k, n, nnz, row_offsets, column_indices, L, R, out_values, stream, nullptr, row_order);
}

int spdl_sddmm_nt(int m, int k, int n, int nnz, const int* row_offsets, const int* column_indices,
                  const float* values, const float* L, const float* Rn, float* out_values, void* stream) {
  return sddmm_nt_impl<float>(m, k, n, nnz, row_offsets, column_indices, values, L, Rn, out_values, stream);
}

int spdl_sddmm_nt_f16(int m, int k, int n, int nnz, const int* row_offsets, const int* column_indices,
                      const uint16_t* values, const uint16_t* L, const uint16_t* Rn, uint16_t* out_values,
                      void* stream) {
  return sddmm_nt_impl<_Float16>(m, k, n, nnz, row_offsets, column_indices,
                                 reinterpret_cast<const _Float16*>(values), reinterpret_cast<const _Float16*>(L),
                                 reinterpret_cast<const _Float16*>(Rn), reinterpret_cast<_Float16*>(out_values),
                                 stream);
}

int spdl_spmm_f16_i16(int m, int k, int n, int nnz, const int* row_offsets, const int16_t* column_indices,
                      const uint16_t* values, const int* row_order, const uint16_t* B, uint16_t* C,
                      void* stream) {
  if (k > 32767) return SPDL_ERR_INVALID;           // the indices must fit 16 signed bits
  return spmm_impl<_Float16, int16_t>(m, k, n, nnz, row_offsets, column_indices,
                                      reinterpret_cast<const _Float16*>(values), row_order,
                                      reinterpret_cast<const _Float16*>(B), reinterpret_cast<_Float16*>(C), stream);
}

int spdl_sddmm_scaled(int m, int k, int n, int nnz, const int* row_offsets, const int* column_indices,
                      const float* values, const float* L, const float* R, float* out_values, void* stream) {
  if (nnz > 0 && (!values || values == out_values)) return SPDL_ERR_INVALID;
  return sddmm_impl<float>(m, k, n, nnz, row_offsets, column_indices, L, R, out_values, stream, values);
}

int spdl_sddmm_scaled_f16(int m, int k, int n, int nnz, const int* row_offsets, const int* column_indices,
                          const uint16_t* values, const uint16_t* L, const uint16_t* R, uint16_t* out_values,
                          void* stream) {
  if (nnz > 0 && (!values || values == out_values)) return SPDL_ERR_INVALID;
  return sddmm_impl<_Float16>(m, k, n, nnz, row_offsets, column_indices,
                              reinterpret_cast<const _Float16*>(L), reinterpret_cast<const _Float16*>(R),
                              reinterpret_cast<_Float16*>(out_values), stream,
                              reinterpret_cast<const _Float16*>(values));
}

int spdl_sddmm_f16(int m, int k, int n, int nnz, const int* row_offsets, const int* column_indices,
                   const uint16_t* L, const uint16_t* R, uint16_t* out_values, void* stream) {
  return sddmm_impl<_Float16>(m, k, n, nnz, row_offsets, column_indices,
                              reinterpret_cast<const _Float16*>(L), reinterpret_cast<const _Float16*>(R),
                              reinterpret_cast<_Float16*>(out_values), stream);
}

int spdl_build_row_order(int m, const int* row_offsets_host, int* row_order_host) {
  if (m < 0 || (m > 0 && (!row_offsets_host || !row_order_host))) return SPDL_ERR_INVALID;
  std::iota(row_order_host, row_order_host + m, 0);
  try {                                   // std::stable_sort allocates a merge buffer
    std::stable_sort(row_order_host, row_order_host + m, [&](int a, int b) {
      return row_offsets_host[a + 1] - row_offsets_host[a] > row_offsets_host[b + 1] - row_offsets_host[b];
    });
  } catch (...) {
    return SPDL_ERR_NOMEM;
  }
  return SPDL_OK;
}

int spdl_validate_csr_host(int m, int k, int nnz, const int* ro, const int* ci, int* sorted_out) {
  if (m < 0 || k < 0 || nnz < 0 || !ro || (nnz > 0 && !ci)) return SPDL_ERR_INVALID;
  if (ro[0] != 0 || ro[m] != nnz) return SPDL_ERR_BAD_CSR;
  int sorted = 1;
  for (int i = 0; i < m; ++i) {
    if (ro[i + 1] < ro[i] || ro[i + 1] > nnz) return SPDL_ERR_BAD_CSR;
    for (int p = ro[i]; p < ro[i + 1]; ++p) {
      if (ci[p] < 0 || ci[p] >= k) return SPDL_ERR_BAD_CSR;
      if (p > ro[i] && ci[p] <= ci[p - 1]) sorted = 0;
    }
  }
  if (sorted_out) *sorted_out = sorted;
  return SPDL_OK;
}

int spdl_select_spmm(int m, int k, int n, int nnz, int elem_bytes, const void* B, const void* C,
                     spdl_launch_info* info) {
  if (!info || !sizes_ok(m, k, n, nnz) || (elem_bytes != 2 && elem_bytes != 4)) return SPDL_ERR_INVALID;
  if (elem_bytes == 4) fill_spmm_info<float>(m, k, n, nnz, B, C, info);
  else fill_spmm_info<_Float16>(m, k, n, nnz, B, C, info);
  return SPDL_OK;
}

int spdl_select_sddmm(int m, int k, int n, int nnz, int elem_bytes, const void* L, const void* R,
                      spdl_launch_info* info) {
  if (!info || !sizes_ok(m, k, n, nnz) || (elem_bytes != 2 && elem_bytes != 4)) return SPDL_ERR_INVALID;
  if (elem_bytes == 4) fill_sddmm_info<float>(m, k, n, nnz, L, R, info);
  else fill_sddmm_info<_Float16>(m, k, n, nnz, L, R, info);
  return SPDL_OK;
}

int spdl_force_variant(int op, int variant) {
  if (op < 0 || op > 1) return SPDL_ERR_INVALID;
  const int limit = op == 0 ? kSpmmVariants : kSddmmVariants;
  if (variant >= limit) return SPDL_ERR_INVALID;
  g_forced[op].store(variant < 0 ? -1 : variant);
  return SPDL_OK;
}

const char* spdl_variant_name(int op, int variant) {
  static const char* const spmm[] = {"rowsplit", "slab", "slabdma", "mfma", "window"};
  static const char* const sddmm[] = {"rowstrip", "group", "slab", "slabdma", "mfma", "lane", "window"};
  if (op == 0 && variant >= 0 && variant < kSpmmVariants) return spmm[variant];
  if (op == 1 && variant >= 0 && variant < kSddmmVariants) return sddmm[variant];
  return nullptr;
}

const char* spdl_status_string(int status) {
  switch (status) {
    case SPDL_OK: return "ok";
    case SPDL_ERR_INVALID: return "invalid argument";
    case SPDL_ERR_LAUNCH: return "kernel launch failed";
    case SPDL_ERR_BAD_CSR: return "not a valid CSR topology";
    case SPDL_ERR_UNSUPPORTED: return "variant does not support this problem";
    case SPDL_ERR_NOMEM: return "host allocation failed";
    default: return "unknown status";
  }
}

int spdl_version(void) { return 140; }

}  // extern "C"

#ifdef SPDL_PHASE_CLOCKS
// Diagnostic build only (microbench/phase_clocks.py): the table the instrumented kernels leave.
extern "C" int spdl_debug_phase_clocks(unsigned long long* host, size_t count) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(spdl::spdl_phase_table), count * sizeof(unsigned long long));
}
#endif
