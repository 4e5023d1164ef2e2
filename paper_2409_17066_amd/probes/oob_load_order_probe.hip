// Do vector-memory loads whose lanes are all out of the buffer's range complete in issue order on gfx950?
// The kernels that wait for prefetched registers by count (s_waitcnt vmcnt(N)) rely on loads returning in order.
// Each wave issues a load from a cold, scattered address (a trip to HBM), then a load that is out of range for every
// lane (returns zeros without touching memory), then waits for "at most one load outstanding".  If loads complete in
// order the first register holds memory's value at that point; if the out-of-range load completed ahead of it, the
// wait was satisfied by the wrong load and the first register still holds the sentinel.
// Build: hipcc --offload-arch=gfx950 -O3 -o oob_load_order_probe oob_load_order_probe.hip ; run without arguments.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e), __LINE__); exit(1); } } while (0)
typedef unsigned u4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void order_kernel(const unsigned *big, unsigned big_bytes, unsigned *stale, int iters, int second_in_range) {
  const unsigned long long a = reinterpret_cast<unsigned long long>(big);
  u4 r_big, r_small;
  r_big.x = (unsigned)a; r_big.y = (unsigned)(a >> 32) & 0xFFFFu; r_big.z = big_bytes; r_big.w = 0x00020000u;
  r_small = r_big; r_small.z = 256u;                          // offsets >= 256 are out of range
  const unsigned tid = blockIdx.x * 256 + threadIdx.x;
  unsigned bad = 0;
  unsigned s = tid * 2654435761u + 99u;
  for (int it = 0; it < iters; ++it) {
    s = s * 1664525u + 1013904223u;
    const unsigned off = (s % (big_bytes / 4096u)) * 4096u + (threadIdx.x & 63u) * 4u;    // a different 4 KB page per lane and iteration
    const unsigned off2 = second_in_range ? (threadIdx.x & 63u) * 4u : 4096u + (threadIdx.x & 63u) * 4u;
    unsigned v1 = 0xDEADBEEFu, v2 = 0xDEADBEEFu;
    asm volatile("buffer_load_dword %0, %2, %3, 0 offen\n\t"
                 "buffer_load_dword %1, %4, %5, 0 offen\n\t"
                 "s_waitcnt vmcnt(1)\n\t"
                 "v_mov_b32 %1, %0\n\t"                     // copy of the first register as it is after the counted wait
                 "s_waitcnt vmcnt(0)"
                 : "+v"(v1), "+v"(v2) : "v"(off), "s"(r_big), "v"(off2), "s"(r_small) : "memory");
    if (v2 == 0xDEADBEEFu) ++bad;                            // (v2 was overwritten by the copy; the load into it is discarded)
  }
  stale[tid] = bad;
}

int main() {
  const unsigned big_bytes = 1u << 30;
  unsigned *big, *stale; CK(hipMalloc(&big, big_bytes)); CK(hipMemset(big, 0x11, big_bytes));
  const int blocks = 1024, iters = 200;
  CK(hipMalloc(&stale, blocks * 256 * 4));
  unsigned *h = (unsigned *)malloc(blocks * 256 * 4);
  for (int second_in_range = 1; second_in_range >= 0; --second_in_range) {
    hipLaunchKernelGGL(order_kernel, dim3(blocks), dim3(256), 0, 0, big, big_bytes, stale, iters, second_in_range);
    CK(hipDeviceSynchronize());
    CK(hipMemcpy(h, stale, blocks * 256 * 4, hipMemcpyDeviceToHost));
    unsigned long long bad = 0; for (int i = 0; i < blocks * 256; ++i) bad += h[i];
    printf("second load %s: %llu of %llu counted waits left the first load's register stale\n",
           second_in_range ? "in range (control)" : "out of range for every lane", bad, (unsigned long long)blocks * 256 * iters);
  }
  return 0;
}
