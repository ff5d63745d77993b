// Shared device helpers for the libspdl kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace spdl {

constexpr int kWave = 64;

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// VEC consecutive elements of T, moved with one memory instruction and widened to fp32.
template <typename T, int VEC> struct Pack;

template <> struct Pack<float, 1> {
  static __device__ __forceinline__ void load(const float* p, float (&x)[1]) { x[0] = *p; }
  static __device__ __forceinline__ void store(float* p, const float (&x)[1]) { *p = x[0]; }
};
template <> struct Pack<float, 2> {
  static __device__ __forceinline__ void load(const float* p, float (&x)[2]) {
    f32x2 v = *reinterpret_cast<const f32x2*>(p); x[0] = v.x; x[1] = v.y;
  }
  static __device__ __forceinline__ void store(float* p, const float (&x)[2]) {
    f32x2 v = {x[0], x[1]}; *reinterpret_cast<f32x2*>(p) = v;
  }
};
template <> struct Pack<float, 4> {
  static __device__ __forceinline__ void load(const float* p, float (&x)[4]) {
    f32x4 v = *reinterpret_cast<const f32x4*>(p); x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
  }
  static __device__ __forceinline__ void store(float* p, const float (&x)[4]) {
    f32x4 v = {x[0], x[1], x[2], x[3]}; *reinterpret_cast<f32x4*>(p) = v;
  }
};
template <> struct Pack<_Float16, 1> {
  static __device__ __forceinline__ void load(const _Float16* p, float (&x)[1]) { x[0] = (float)*p; }
  static __device__ __forceinline__ void store(_Float16* p, const float (&x)[1]) { *p = (_Float16)x[0]; }
};
template <> struct Pack<_Float16, 2> {
  static __device__ __forceinline__ void load(const _Float16* p, float (&x)[2]) {
    f16x2 v = *reinterpret_cast<const f16x2*>(p); x[0] = (float)v.x; x[1] = (float)v.y;
  }
  static __device__ __forceinline__ void store(_Float16* p, const float (&x)[2]) {
    f16x2 v = {(_Float16)x[0], (_Float16)x[1]}; *reinterpret_cast<f16x2*>(p) = v;
  }
};
template <> struct Pack<_Float16, 4> {
  static __device__ __forceinline__ void load(const _Float16* p, float (&x)[4]) {
    f16x4 v = *reinterpret_cast<const f16x4*>(p);
#pragma unroll
    for (int i = 0; i < 4; ++i) x[i] = (float)v[i];
  }
  static __device__ __forceinline__ void store(_Float16* p, const float (&x)[4]) {
    f16x4 v;
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = (_Float16)x[i];
    *reinterpret_cast<f16x4*>(p) = v;
  }
};
template <> struct Pack<_Float16, 8> {
  static __device__ __forceinline__ void load(const _Float16* p, float (&x)[8]) {
    f16x8 v = *reinterpret_cast<const f16x8*>(p);
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = (float)v[i];
  }
  static __device__ __forceinline__ void store(_Float16* p, const float (&x)[8]) {
    f16x8 v;
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = (_Float16)x[i];
    *reinterpret_cast<f16x8*>(p) = v;
  }
};

__device__ __forceinline__ int uniform(int x) { return __builtin_amdgcn_readfirstlane(x); }

// Optional clocks inside the slab kernels: where a wave's time goes.  Compiled in only with
// -DSPDL_PHASE_CLOCKS (microbench/phase_clocks.py builds such a copy of the library and prints the
// table); without the macro every member is empty and the kernels are what they are without it.
// A wave adds the clocks between two laps to the phase named at the second one (the counter is
// s_memtime, the sums live in scalar registers) and leaves its sums in a global table at the end:
// ten numbers per wave: the eight phases, the total, one spare.  A lap is also a scheduling barrier,
// so a measured kernel is a little slower than the real one.
enum Phase { kPhaseSetup = 0, kPhaseIssue, kPhaseScan, kPhaseSteps, kPhaseWait, kPhaseBarrier, kPhaseRest, kPhaseGather, kPhases };
constexpr int kPhaseStride = 10;
#ifdef SPDL_PHASE_CLOCKS
constexpr int kPhaseTableWaves = 8192;
__device__ unsigned long long spdl_phase_table[kPhaseTableWaves * kPhaseStride];
struct PhaseClocks {
  unsigned long long first, last, acc[kPhases];
  static __device__ __forceinline__ unsigned long long now() {
    __builtin_amdgcn_sched_barrier(0);
    const unsigned long long t = __builtin_readcyclecounter();
    __builtin_amdgcn_sched_barrier(0);
    return t;
  }
  __device__ __forceinline__ void start() {
#pragma unroll
    for (int i = 0; i < kPhases; ++i) acc[i] = 0;
    first = last = now();
  }
  __device__ __forceinline__ void lap(int phase) {
    const unsigned long long t = now();
    acc[phase] += t - last;
    last = t;
  }
  __device__ __forceinline__ void store(int wave_slot) {
    if (wave_slot < kPhaseTableWaves && (threadIdx.x & 63) == 0) {
      unsigned long long* d = spdl_phase_table + (size_t)wave_slot * kPhaseStride;
#pragma unroll
      for (int i = 0; i < kPhases; ++i) d[i] = acc[i];
      d[kPhases] = last - first;
    }
  }
};
#else
struct PhaseClocks {
  __device__ __forceinline__ void start() {}
  __device__ __forceinline__ void lap(int) {}
  __device__ __forceinline__ void store(int) {}
};
#endif

// Maximum of two wave-uniform values on the scalar unit (left to itself the compiler moves such
// a maximum to the vector unit as soon as one of its uses is a vector select).
__device__ __forceinline__ int scalar_max(int a, int b) {
  int r;
  asm("s_max_i32 %0, %1, %2" : "=s"(r) : "s"(a), "s"(b) : "scc");
  return r;
}

// Number of leading set bits of a 16-bit piece of a wave mask (scalar arithmetic).
__device__ __forceinline__ int leading16(unsigned piece) { return __builtin_ctz(~piece | 0x10000u); }

// Workgroup id -> (panel of sparse rows, group = slice of the dense operand) for the slab kernels.
// Consecutive workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2: all
// groups of a panel get ids that are equal modulo 8, so the panel's part of A is fetched into
// one L2 only.  (The opposite choice, one slice of the dense operand per XCD, was measured: same
// run time, 60 % more HBM reads.)  slab_grid_size() is the matching grid.
__host__ __device__ __forceinline__ bool slab_wg_map(int bid, int panels, int groups, int& panel, int& group) {
  const int per_block = 8 * groups;
  const int blk = bid / per_block, rem = bid - blk * per_block;
  panel = blk * 8 + (rem & 7);
  group = rem >> 3;
  return panel < panels;
}
__host__ __device__ __forceinline__ int slab_grid_size(int panels, int groups) {
  return ((panels + 7) / 8) * 8 * groups;
}

// Store of one SDDMM result: as it is, or times the sparse matrix's value at that position (the
// strict definition of SDDMM, paper Sec. "Sampled Dense--Dense Matrix Multiplication
// Operation"; one load and one multiply before the store).  scale == nullptr: unscaled.
template <typename T>
__device__ __forceinline__ void sddmm_store(T* __restrict__ out, const T* __restrict__ scale, int p, float total) {
  if (scale) total *= (float)scale[p];
  out[p] = (T)total;
}

// Optional epilogue of SpMM (paper Sec. "Application: Sparse MobileNetV1": bias and ReLU fused
// into the sparse 1x1 convolution): v + bias[row], then max(., 0).  bias == nullptr: none.
template <typename T, int N>
__device__ __forceinline__ void spmm_epilogue(float (&acc)[N], const T* __restrict__ bias, int row, int relu) {
  if (bias) {
    const float b = (float)bias[row];
#pragma unroll
    for (int v = 0; v < N; ++v) acc[v] += b;
  }
  if (relu) {
#pragma unroll
    for (int v = 0; v < N; ++v) acc[v] = fmaxf(acc[v], 0.f);
  }
}

}  // namespace spdl
