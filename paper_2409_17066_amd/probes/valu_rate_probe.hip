// How many clocks a wave-wide vector-ALU instruction holds its SIMD on gfx950, for the instructions the dot-product
// GEMV is made of: v_dot2c_f32_f16 (accumulating), v_dot2_f32_f16 (three-operand), v_fma_f32, v_pk_fma_f16,
// v_and_b32, and a v_add_f32 with a DPP row operand.  16 waves per compute unit (4 per SIMD), each running a long
// unrolled chain of 8 independent accumulators; clocks per instruction and SIMD = 4 waves x time / instructions.
// Build: hipcc --offload-arch=gfx950 -O3 -o valu_rate_probe valu_rate_probe.hip ; run without arguments.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e), __LINE__); exit(1); } } while (0)

enum { DOT2C = 0, DOT2, FMA32, PKFMA16, AND32, ADD_DPP, N_MODES };
static const char *kNames[N_MODES] = {"v_dot2c_f32_f16", "v_dot2_f32_f16", "v_fma_f32", "v_pk_fma_f16", "v_and_b32", "v_add_f32 row_shr:1 (DPP)"};

template <int MODE>
__global__ __launch_bounds__(1024) void valu_kernel(unsigned *out, int iters) {
  unsigned a[8], x = threadIdx.x * 2654435761u | 0x3c003c00u, y = 0x3c003c00u ^ (threadIdx.x << 3);
#pragma unroll
  for (int i = 0; i < 8; ++i) a[i] = threadIdx.x + i;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 8; ++r)
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (MODE == DOT2C) asm volatile("v_dot2c_f32_f16 %0, %1, %2" : "+v"(a[i]) : "v"(x), "v"(y));
        if (MODE == DOT2) asm volatile("v_dot2_f32_f16 %0, %1, %2, %0" : "+v"(a[i]) : "v"(x), "v"(y));
        if (MODE == FMA32) asm volatile("v_fma_f32 %0, %1, %2, %0" : "+v"(a[i]) : "v"(x), "v"(y));
        if (MODE == PKFMA16) asm volatile("v_pk_fma_f16 %0, %1, %2, %0" : "+v"(a[i]) : "v"(x), "v"(y));
        if (MODE == AND32) asm volatile("v_and_b32 %0, %1, %0" : "+v"(a[i]) : "v"(x));
        if (MODE == ADD_DPP) asm volatile("v_add_f32_dpp %0, %1, %0 row_shr:1 row_mask:0xf bank_mask:0xf" : "+v"(a[i]) : "v"(x));
      }
  }
  unsigned s = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) s ^= a[i];
  out[blockIdx.x * 1024 + threadIdx.x] = s;
}

template <int MODE> void run(unsigned *out, int cus, double clk) {
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  const int iters = 2000;
  float ms = 0;
  for (int rep = 0; rep < 2; ++rep) {
    CK(hipEventRecord(e0));
    hipLaunchKernelGGL(valu_kernel<MODE>, dim3(cus), dim3(1024), 0, 0, out, iters);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
  }
  const double per_wave = (double)iters * 64;                   // instructions per wave
  printf("%-28s %.3f ms  %.2f clocks per instruction and SIMD (4 waves per SIMD, at %.0f MHz)\n", kNames[MODE], ms,
         ms * 1e-3 * clk / (per_wave * 4.0), clk / 1e6);
  fflush(stdout);
}

int main() {
  hipDeviceProp_t pr; CK(hipGetDeviceProperties(&pr, 0));
  const double clk = pr.clockRate * 1e3;
  unsigned *out; CK(hipMalloc(&out, (size_t)pr.multiProcessorCount * 1024 * 4));
  run<DOT2C>(out, pr.multiProcessorCount, clk); run<DOT2>(out, pr.multiProcessorCount, clk); run<FMA32>(out, pr.multiProcessorCount, clk);
  run<PKFMA16>(out, pr.multiProcessorCount, clk); run<AND32>(out, pr.multiProcessorCount, clk); run<ADD_DPP>(out, pr.multiProcessorCount, clk);
  CK(hipDeviceSynchronize());
  return 0;
}
