// Issue rates that bound the inner loops of the SpMM / SDDMM kernels on gfx950, measured with
// 1024-thread workgroups, one per CU (the launch shape of the slab kernels):
//   1. v_fmac_f32 with both operands in the lane's registers, with a DPP operand, with a scalar
//      operand;
//   2. ds_read_b128 alone, 16 lanes per contiguous 256-byte row (the slab kernels' pattern);
//   3. ds_read_b128 feeding NF multiply-adds each (NF = 4 is the 4 bytes per multiply-add that
//      unstructured SpMM and SDDMM need: every B / R element is used once per nonzero);
//   4. the steps of the product kernels: SpMM with 4 and 8 columns per lane (DPP-broadcast value,
//      address per nonzero), SDDMM with four lanes per nonzero and rotated 32-byte reads.
// Prints multiply-adds per clock per CU (the published fp32 vector peak is 128) and LDS bytes
// per clock per CU.  Build: hipcc --offload-arch=gfx950 -O3 (packed fp32 off), see build.py.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>

typedef float f32x4 __attribute__((ext_vector_type(4)));
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 1; } } while (0)
#define REP16(X) X X X X X X X X X X X X X X X X

// ---------------------------------------------------------------- 1. multiply-add issue rate
#define FMA8(OP, SRC, TAIL)                                                                     \
  asm volatile(OP " %0, %8, %9 " TAIL "\n " OP " %1, %8, %9 " TAIL "\n " OP " %2, %8, %9 " TAIL "\n " \
               OP " %3, %8, %9 " TAIL "\n " OP " %4, %8, %9 " TAIL "\n " OP " %5, %8, %9 " TAIL "\n " \
               OP " %6, %8, %9 " TAIL "\n " OP " %7, %8, %9 " TAIL                              \
               : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7) : SRC, "v"(b));
template <int MODE>
__global__ __launch_bounds__(1024) void fma_rate(float* out, int iters, float s) {
  float a0 = threadIdx.x, a1 = 1, a2 = 2, a3 = 3, a4 = 4, a5 = 5, a6 = 6, a7 = 7;
  float l = 0.001f * threadIdx.x, b = 1.0001f;
  for (int it = 0; it < iters; ++it) {
    if (MODE == 0) { REP16(FMA8("v_fmac_f32", "v"(l), "")) }
    if (MODE == 1) { REP16(FMA8("v_fmac_f32_dpp", "v"(l), "row_newbcast:3 row_mask:0xf bank_mask:0xf")) }
    if (MODE == 2) { REP16(FMA8("v_fmac_f32_dpp", "v"(l), "row_ror:2 row_mask:0xf bank_mask:0xf")) }
    if (MODE == 3) { REP16(FMA8("v_fmac_f32", "s"(s), "")) }
  }
  out[blockIdx.x * 1024 + threadIdx.x] = a0 + a1 + a2 + a3 + a4 + a5 + a6 + a7;
}

// ---------------------------------------------------------------- 2. LDS reads alone
__global__ __launch_bounds__(1024) void lds_rate(float* out, int iters, const int* __restrict__ rows) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  for (int i = threadIdx.x; i < 32768; i += 1024) reinterpret_cast<float*>(lds)[i] = (float)(i & 7);
  __syncthreads();
  const int addr = rows[threadIdx.x & ~15] % 448 * 256 + (threadIdx.x & 15) * 16;
  f32x4 s = {0, 0, 0, 0};
  for (int it = 0; it < iters; ++it) {
    f32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v[u]) : "v"(addr), "n"(u * 16));
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int u = 0; u < 8; ++u) asm volatile("" :: "v"(v[u]));
    s += v[it & 7];
  }
  out[blockIdx.x * 1024 + threadIdx.x] = s.x + s.y + s.z + s.w;
}

// ---------------------------------------------------------------- 3. LDS reads feeding multiply-adds
template <int DPP, int NF>
__global__ __launch_bounds__(1024) void lds_fed(float* out, int iters) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  for (int i = threadIdx.x; i < 16384; i += 1024) reinterpret_cast<float*>(lds)[i] = (float)(i & 7);
  __syncthreads();
  float a0 = 0, a1 = 1, a2 = 2, a3 = 3;
  const float l = 0.001f * threadIdx.x;
  const int addr = (threadIdx.x * 16) & 65535;
  f32x4 v0, v1, v2;
  asm volatile("ds_read_b128 %0, %1" : "=v"(v0) : "v"(addr));
  asm volatile("ds_read_b128 %0, %1 offset:4096" : "=v"(v1) : "v"(addr));
#define USE(V)                                                                                                   \
  if (DPP) { for (int r = 0; r < NF / 4; ++r) asm volatile(                                                      \
      "v_fmac_f32_dpp %0, %4, %5 row_ror:2 row_mask:0xf bank_mask:0xf\n v_fmac_f32_dpp %1, %4, %6 row_ror:2 row_mask:0xf bank_mask:0xf\n" \
      " v_fmac_f32_dpp %2, %4, %7 row_ror:2 row_mask:0xf bank_mask:0xf\n v_fmac_f32_dpp %3, %4, %8 row_ror:2 row_mask:0xf bank_mask:0xf" \
      : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3) : "v"(l), "v"(V.x), "v"(V.y), "v"(V.z), "v"(V.w)); }              \
  else { for (int r = 0; r < NF / 4; ++r) asm volatile(                                                          \
      "v_fmac_f32 %0, %4, %5\n v_fmac_f32 %1, %4, %6\n v_fmac_f32 %2, %4, %7\n v_fmac_f32 %3, %4, %8"              \
      : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3) : "v"(l), "v"(V.x), "v"(V.y), "v"(V.z), "v"(V.w)); }
  for (int it = 0; it < iters; ++it) {                 // reads run two ahead of their use
    asm volatile("ds_read_b128 %0, %1 offset:8192" : "=v"(v2) : "v"(addr));
    asm volatile("s_waitcnt lgkmcnt(2)" ::: "memory"); USE(v0)
    asm volatile("ds_read_b128 %0, %1" : "=v"(v0) : "v"(addr));
    asm volatile("s_waitcnt lgkmcnt(2)" ::: "memory"); USE(v1)
    asm volatile("ds_read_b128 %0, %1 offset:4096" : "=v"(v1) : "v"(addr));
    asm volatile("s_waitcnt lgkmcnt(2)" ::: "memory"); USE(v2)
  }
#undef USE
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  out[blockIdx.x * 1024 + threadIdx.x] = a0 + a1 + a2 + a3 + v0.x + v1.x;
}

// ---------------------------------------------------------------- 4. the kernels' own steps
#define FMA_DPP(ACC, A, B, T) asm volatile("v_fmac_f32_dpp %0, %1, %2 row_newbcast:" #T " row_mask:0xf bank_mask:0xf" : "+v"(ACC) : "v"(A), "v"(B));
// SpMM, 4 columns per lane: the LDS offset of nonzero T's row of B sits in lane T of the group
#define SP4(T)                                                                                     \
  { const int addr = __builtin_amdgcn_update_dpp(0, off, 0x150 + (T), 0xf, 0xf, false) + lane_b;   \
    f32x4 b = *reinterpret_cast<const f32x4*>(lds + addr);                                         \
    FMA_DPP(a0, av, b.x, T) FMA_DPP(a1, av, b.y, T) FMA_DPP(a2, av, b.z, T) FMA_DPP(a3, av, b.w, T) }
#define SP8(T)                                                                                     \
  { const int addr = __builtin_amdgcn_update_dpp(0, off, 0x150 + (T), 0xf, 0xf, false) + lane_b;   \
    f32x4 b = *reinterpret_cast<const f32x4*>(lds + addr);                                         \
    f32x4 c = *reinterpret_cast<const f32x4*>(lds + addr + 256);                                   \
    FMA_DPP(a0, av, b.x, T) FMA_DPP(a1, av, b.y, T) FMA_DPP(a2, av, b.z, T) FMA_DPP(a3, av, b.w, T) \
    FMA_DPP(a4, av, c.x, T) FMA_DPP(a5, av, c.y, T) FMA_DPP(a6, av, c.z, T) FMA_DPP(a7, av, c.w, T) }
// The same step with the value of A moved to every lane first (one v_mov_b32_dpp) and plain
// multiply-adds after it.
#define SP4M(T)                                                                                    \
  { const int addr = __builtin_amdgcn_update_dpp(0, off, 0x150 + (T), 0xf, 0xf, false) + lane_b;   \
    const float at = __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, av), 0x150 + (T), 0xf, 0xf, false)); \
    f32x4 b = *reinterpret_cast<const f32x4*>(lds + addr);                                         \
    a0 = __builtin_fmaf(at, b.x, a0); a1 = __builtin_fmaf(at, b.y, a1);                            \
    a2 = __builtin_fmaf(at, b.z, a2); a3 = __builtin_fmaf(at, b.w, a3); }
__global__ __launch_bounds__(1024) void spmm_step_mov(float* out, int iters, const int* __restrict__ rows, int nrows) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  for (int i = threadIdx.x; i < nrows * 64; i += 1024) reinterpret_cast<float*>(lds)[i] = (float)(i & 7);
  __syncthreads();
  const int lane_b = (threadIdx.x & 15) * 16;
  float a0 = 0, a1 = 0, a2 = 0, a3 = 0;
  const int* myrows = rows + threadIdx.x;
  for (int it = 0; it < iters; ++it) {
    const int off = myrows[(it & 15) * 1024] % nrows * 256;
    const float av = 0.5f + off;
    SP4M(0) SP4M(1) SP4M(2) SP4M(3) SP4M(4) SP4M(5) SP4M(6) SP4M(7) SP4M(8) SP4M(9) SP4M(10) SP4M(11) SP4M(12) SP4M(13) SP4M(14) SP4M(15)
  }
  out[blockIdx.x * 1024 + threadIdx.x] = a0 + a1 + a2 + a3;
}

template <int COLS>
__global__ __launch_bounds__(1024) void spmm_step(float* out, int iters, const int* __restrict__ rows, int nrows) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  for (int i = threadIdx.x; i < nrows * COLS * 16; i += 1024) reinterpret_cast<float*>(lds)[i] = (float)(i & 7);
  __syncthreads();
  const int lane_b = (threadIdx.x & 15) * 16;
  float a0 = 0, a1 = 0, a2 = 0, a3 = 0, a4 = 0, a5 = 0, a6 = 0, a7 = 0;
  const int* myrows = rows + threadIdx.x;
  for (int it = 0; it < iters; ++it) {
    const int off = myrows[(it & 15) * 1024] % nrows * (COLS * 64);
    const float av = 0.5f + off;
    asm volatile("s_nop 1");
    if (COLS == 4) { SP4(0) SP4(1) SP4(2) SP4(3) SP4(4) SP4(5) SP4(6) SP4(7) SP4(8) SP4(9) SP4(10) SP4(11) SP4(12) SP4(13) SP4(14) SP4(15) }
    else { SP8(0) SP8(1) SP8(2) SP8(3) SP8(4) SP8(5) SP8(6) SP8(7) SP8(8) SP8(9) SP8(10) SP8(11) SP8(12) SP8(13) SP8(14) SP8(15) }
  }
  out[blockIdx.x * 1024 + threadIdx.x] = a0 + a1 + a2 + a3 + a4 + a5 + a6 + a7;
}

// SDDMM, four lanes per nonzero (lane 4t+h: nonzero t, columns 32h..32h+31): step s reads the 32
// bytes 128(h mod 2) + 32((t-s) mod 4) of its own row of R in region h/2 (second region shifted by
// 16 bytes) and multiplies them with eight values of L held in registers in that order.
__global__ __launch_bounds__(1024) void sddmm_lane_step(float* out, int iters, const int* __restrict__ rows, int nrows) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int region = nrows * 256 + 16;
  for (int i = threadIdx.x; i < 2 * region / 4; i += 1024) reinterpret_cast<float*>(lds)[i] = (float)(i & 7);
  __syncthreads();
  const int l16 = threadIdx.x & 15, t4 = l16 >> 2, h4 = l16 & 3;
  float l[32];
  for (int i = 0; i < 32; ++i) l[i] = 0.001f * (threadIdx.x + i);
  int x[4];
  for (int s = 0; s < 4; ++s) x[s] = (h4 >> 1) * region + (h4 & 1) * 128 + ((t4 - s) & 3) * 32;
  float tot = 0.f;
  const int* myrows = rows + (threadIdx.x & ~3);          // the four lanes of a nonzero share its row
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int strip = 0; strip < 4; ++strip) {
      const int base = myrows[((it * 4 + strip) & 15) * 1024] % nrows * 256;
      float acc0 = 0.f, acc1 = 0.f;
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const f32x4 b0 = *reinterpret_cast<const f32x4*>(lds + base + x[s]);
        const f32x4 b1 = *reinterpret_cast<const f32x4*>(lds + base + x[s] + 16);
        acc0 = __builtin_fmaf(l[8 * s + 0], b0.x, acc0); acc1 = __builtin_fmaf(l[8 * s + 1], b0.y, acc1);
        acc0 = __builtin_fmaf(l[8 * s + 2], b0.z, acc0); acc1 = __builtin_fmaf(l[8 * s + 3], b0.w, acc1);
        acc0 = __builtin_fmaf(l[8 * s + 4], b1.x, acc0); acc1 = __builtin_fmaf(l[8 * s + 5], b1.y, acc1);
        acc0 = __builtin_fmaf(l[8 * s + 6], b1.z, acc0); acc1 = __builtin_fmaf(l[8 * s + 7], b1.w, acc1);
      }
      tot += acc0 + acc1;
    }
  }
  out[blockIdx.x * 1024 + threadIdx.x] = tot;
}

// SpMM, four lanes per nonzero (lane 4t+h: every fourth nonzero of the strip, columns 16h..16h+15
// of a 64-column tile): the nonzero's value and LDS offset are broadcast inside the quad, its 64
// bytes of the B row are read as four 16-byte pieces in an order rotated by t (conflict-free
// whatever the rows), and sixteen plain multiply-adds accumulate them.
__global__ __launch_bounds__(1024) void spmm_lane_step(float* out, int iters, const int* __restrict__ rows, int nrows) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  for (int i = threadIdx.x; i < nrows * 64; i += 1024) reinterpret_cast<float*>(lds)[i] = (float)(i & 7);
  __syncthreads();
  const int l16 = threadIdx.x & 15, t4 = l16 >> 2, h4 = l16 & 3;
  int x[4];
  for (int r = 0; r < 4; ++r) x[r] = h4 * 64 + ((r + t4) & 3) * 16;
  float acc[16];
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;
  const int* myrows = rows + threadIdx.x;
  for (int it = 0; it < iters; ++it) {
    const int off_own = myrows[(it & 15) * 1024] % nrows * 256;      // this lane's own nonzero of the chunk
    const float a_own = 0.5f + off_own;
#define SPMM_LANE_STRIP(Q)                                                                          \
    {                                                                                               \
      const int off = __builtin_amdgcn_mov_dpp(off_own, (Q) * 0x55, 0xf, 0xf, false);               \
      const float a = __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, a_own), (Q) * 0x55, 0xf, 0xf, false)); \
      _Pragma("unroll") for (int r = 0; r < 4; ++r) {                                               \
        const f32x4 b = *reinterpret_cast<const f32x4*>(lds + off + x[r]);                          \
        acc[4 * r + 0] = __builtin_fmaf(a, b.x, acc[4 * r + 0]);                                    \
        acc[4 * r + 1] = __builtin_fmaf(a, b.y, acc[4 * r + 1]);                                    \
        acc[4 * r + 2] = __builtin_fmaf(a, b.z, acc[4 * r + 2]);                                    \
        acc[4 * r + 3] = __builtin_fmaf(a, b.w, acc[4 * r + 3]);                                    \
      }                                                                                             \
    }
    SPMM_LANE_STRIP(0) SPMM_LANE_STRIP(1) SPMM_LANE_STRIP(2) SPMM_LANE_STRIP(3)
#undef SPMM_LANE_STRIP
  }
  float tot = 0.f;
  for (int i = 0; i < 16; ++i) tot += acc[i];
  out[blockIdx.x * 1024 + threadIdx.x] = tot;
}

template <typename F> float best_ms(F f) {
  hipEvent_t a, b;
  (void)hipEventCreate(&a); (void)hipEventCreate(&b);
  f(); (void)hipDeviceSynchronize();
  float best = 1e30f;
  for (int r = 0; r < 4; ++r) {
    (void)hipEventRecord(a); f(); (void)hipEventRecord(b); (void)hipEventSynchronize(b);
    float ms; (void)hipEventElapsedTime(&ms, a, b);
    if (ms < best) best = ms;
  }
  return best;
}

int main() {
  hipDeviceProp_t prop;
  CK(hipGetDeviceProperties(&prop, 0));
  const int CU = prop.multiProcessorCount;
  const double ghz = prop.clockRate / 1e6;
  printf("device %s: %d CUs, %.2f GHz\n", prop.gcnArchName, CU, ghz);
  float* out; CK(hipMalloc(&out, (size_t)CU * 1024 * 4));
  int* rows; CK(hipMalloc(&rows, 16 * 1024 * 4));
  int* h = (int*)malloc(16 * 1024 * 4);
  srand(1);
  for (int i = 0; i < 16 * 1024; ++i) h[i] = rand();
  CK(hipMemcpy(rows, h, 16 * 1024 * 4, hipMemcpyHostToDevice));
  const int iters = 1000;
  auto per_cu_clk = [&](double count, float ms) { return count / (ms * 1e-3) / CU / (ghz * 1e9); };

  const char* fma_names[] = {"both operands in registers", "DPP row_newbcast operand", "DPP row_ror operand", "scalar-register operand"};
#define RUN_FMA(M) { float ms = best_ms([&] { fma_rate<M><<<CU, 1024>>>(out, iters, 1.5f); }); \
    const double r = per_cu_clk((double)CU * 1024 * iters * 128, ms);                            \
    printf("v_fmac_f32, %-28s %6.1f FMA/clk/CU  (%.2f clk per wave instruction and SIMD)\n", fma_names[M], r, 256.0 / r); }
  RUN_FMA(0) RUN_FMA(1) RUN_FMA(2) RUN_FMA(3)

  CK(hipFuncSetAttribute((const void*)lds_rate, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
  { float ms = best_ms([&] { lds_rate<<<CU, 1024, 131072>>>(out, iters, rows); });
    printf("ds_read_b128 alone, 16 lanes per 256-byte row:   %6.1f B/clk/CU\n", per_cu_clk((double)CU * 1024 * iters * 8 * 16, ms)); }

#define RUN_FED(D, NF) { float ms = best_ms([&] { lds_fed<D, NF><<<CU, 1024, 65536>>>(out, iters); });          \
    printf("ds_read_b128 + %2d %-5s multiply-adds per read:  %6.1f FMA/clk/CU, LDS %5.0f B/clk/CU\n", NF, D ? "DPP" : "plain", \
           per_cu_clk((double)CU * 1024 * iters * 3 * NF, ms), per_cu_clk((double)CU * 1024 * iters * 3 * 16, ms)); }
  RUN_FED(0, 4) RUN_FED(1, 4) RUN_FED(0, 8) RUN_FED(1, 8) RUN_FED(0, 16) RUN_FED(1, 16)

  CK(hipFuncSetAttribute((const void*)spmm_step<4>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
  CK(hipFuncSetAttribute((const void*)spmm_step<8>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
  CK(hipFuncSetAttribute((const void*)sddmm_lane_step, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
  { float ms = best_ms([&] { spmm_step<4><<<CU, 1024, 448 * 256>>>(out, iters, rows, 448); });
    printf("SpMM step, 4 columns per lane (1 address, 1 read, 4 DPP multiply-adds per nonzero): %6.1f FMA/clk/CU\n",
           per_cu_clk((double)CU * 1024 * iters * 64, ms)); }
  CK(hipFuncSetAttribute((const void*)spmm_step_mov, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
  { float ms = best_ms([&] { spmm_step_mov<<<CU, 1024, 448 * 256>>>(out, iters, rows, 448); });
    printf("SpMM step, 4 columns per lane, value moved first (1 address, 1 DPP move, 1 read, 4 plain multiply-adds): %6.1f FMA/clk/CU\n",
           per_cu_clk((double)CU * 1024 * iters * 64, ms)); }
  { float ms = best_ms([&] { spmm_step<8><<<CU, 1024, 224 * 512>>>(out, iters, rows, 224); });
    printf("SpMM step, 8 columns per lane (1 address, 2 reads, 8 DPP multiply-adds per nonzero): %6.1f FMA/clk/CU\n",
           per_cu_clk((double)CU * 1024 * iters * 128, ms)); }
  { float ms = best_ms([&] { sddmm_lane_step<<<CU, 1024, 2 * (128 * 256 + 16)>>>(out, iters, rows, 128); });
    printf("SDDMM step, 4 lanes per nonzero (1 address, 2 reads, 8 plain multiply-adds per step): %6.1f FMA/clk/CU\n",
           per_cu_clk((double)CU * 1024 * iters * 4 * 32, ms)); }
  CK(hipFuncSetAttribute((const void*)spmm_lane_step, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
  { float ms = best_ms([&] { spmm_lane_step<<<CU, 1024, 448 * 256>>>(out, iters, rows, 448); });
    printf("SpMM step, 4 lanes per nonzero (2 broadcasts, 4 reads, 16 plain multiply-adds per nonzero): %6.1f FMA/clk/CU\n",
           per_cu_clk((double)CU * 1024 * iters * 64, ms)); }
  printf("published fp32 vector peak: 128 FMA/clk/CU (packed); 4 bytes per multiply-add from LDS at the measured\n"
         "ds_read_b128 rate would allow at most (B/clk/CU above) / 4 FMA/clk/CU\n");
  return 0;
}
