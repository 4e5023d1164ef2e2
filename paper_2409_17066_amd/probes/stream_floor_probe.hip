// Streaming floor of the v = 6 GEMV's index reads: one 1024-thread workgroup per compute unit reads its share of a
// 1 GiB buffer with the GEMV's per-lane load shapes and keeps D rows in flight per wave; no table, no arithmetic.
//   mode 0: the GEMV's windows: row of `rowbytes` bytes, lane l of wave w loads 12 bytes at dword ((64 w + l) * 60) >> 5
//   mode 1: the same amount of data as contiguous 16-byte loads (lane l of wave w at 1024 w + 16 l of each 16 KB row)
//   mode 2: the windows of mode 0 widened to the enclosing aligned 16 bytes
// Build: hipcc --offload-arch=gfx950 -O3 -o stream_floor_probe stream_floor_probe.hip ; run without arguments.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e), __LINE__); exit(1); } } while (0)
typedef unsigned u4 __attribute__((ext_vector_type(4)));
typedef unsigned u3 __attribute__((ext_vector_type(3)));
typedef unsigned u2 __attribute__((ext_vector_type(2)));
template <int MODE, int D>
__global__ __launch_bounds__(1024) void stream(const unsigned char *base, long long per_wg, int rows, unsigned rowb, unsigned *out) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const unsigned char *p = base + (long long)blockIdx.x * per_wg;
  __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc((void *)p, 0, (unsigned)per_wg, 0x00020000);
  unsigned off;
  if (MODE == 0) off = ((unsigned)((wv * 64 + lane) * 60) >> 5) * 4u;
  else if (MODE == 1) off = wv * 1024u + lane * 16u;
  else off = (((unsigned)((wv * 64 + lane) * 60) >> 5) * 4u) & ~15u;
  unsigned acc = 0;
  u4 slot[D];
#pragma unroll
  for (int d = 0; d < D; ++d) {
    if (MODE == 0) { u3 a = __builtin_amdgcn_raw_buffer_load_b96(r, d * rowb + off, 0, 0); slot[d] = u4{a.x, a.y, a.z, 0}; }
    else slot[d] = __builtin_amdgcn_raw_buffer_load_b128(r, d * rowb + off, 0, 0);
  }
  for (int i0 = 0; i0 < rows; i0 += D) {
#pragma unroll
    for (int d = 0; d < D; ++d) {
      asm volatile("" : "+v"(slot[d]));
      acc ^= slot[d].x ^ slot[d].y ^ slot[d].z;
      const unsigned rr = min(i0 + d + D, rows - 1);
      if (MODE == 0) { u3 a = __builtin_amdgcn_raw_buffer_load_b96(r, rr * rowb + off, 0, 0); slot[d] = u4{a.x, a.y, a.z, 0}; }
      else slot[d] = __builtin_amdgcn_raw_buffer_load_b128(r, rr * rowb + off, 0, 0);
    }
  }
  if (acc == 0x12345u) out[threadIdx.x] = acc;
}
template <int MODE, int D> void run(const unsigned char *buf, size_t bytes, unsigned *out, int cus, unsigned rowb, int rows) {
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  const long long per_wg = (long long)rows * rowb;
  const int copies = (int)(bytes / (per_wg * cus));
  float ms = 0;
  for (int rep = 0; rep < 2; ++rep) {
    CK(hipEventRecord(e0));
    for (int c = 0; c < copies; ++c) hipLaunchKernelGGL((stream<MODE, D>), dim3(cus), dim3(1024), 0, 0, buf + (size_t)c * per_wg * cus, per_wg, rows, rowb, out);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
  }
  printf("mode %d depth %d rows %d rowbytes %u: %.2f us per launch, %.0f GB/s\n", MODE, D, rows, rowb, ms * 1e3 / copies, (double)per_wg * cus * copies / (ms * 1e-3) / 1e9);
  fflush(stdout);
}
int main() {
  hipDeviceProp_t pr; CK(hipGetDeviceProperties(&pr, 0));
  const size_t bytes = (size_t)1 << 30;
  unsigned char *buf; CK(hipMalloc(&buf, bytes)); CK(hipMemset(buf, 1, bytes));
  unsigned *out; CK(hipMalloc(&out, 4096 * 4));
  const int c = pr.multiProcessorCount;
  // rows of 7680 bytes = 15 waves x 512 bytes of 12-bit indices (the long-row layer); mode 1: rows of 16 waves x 1 KB
  run<0, 3>(buf, bytes, out, c, 7680, 48); run<0, 6>(buf, bytes, out, c, 7680, 48); run<0, 12>(buf, bytes, out, c, 7680, 48);
  run<2, 3>(buf, bytes, out, c, 7680, 48); run<2, 6>(buf, bytes, out, c, 7680, 48);
  run<1, 3>(buf, bytes, out, c, 16384, 24); run<1, 6>(buf, bytes, out, c, 16384, 24); run<1, 12>(buf, bytes, out, c, 16384, 24);
  return 0;
}
