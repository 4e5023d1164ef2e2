// Microbenchmark behind the LDS layout of the v = 6 GEMV kernels: how many random codebook lookups per clock a
// gfx950 compute unit serves from LDS, by read width, entry stride and replication.  Each lane hashes 8 entry
// numbers per iteration, issues 8 reads, waits, folds the values into a checksum; 4 workgroups of 256 threads per compute unit (16 waves).
//   modes: b32 / b64 / b128 from a 4096-entry table with naturally aligned entries; b96 from 16-byte entries;
//          b128 and b96 from 12-byte entries (unaligned reads); b128 from a 256-entry table stored as 16
//          interleaved replicas, lane l reading replica l % 16 (every 16 consecutive lanes then touch 16 different
//          groups of four banks) or replica (l / 4) % 16 (control: consecutive lanes share a replica).
// Build: hipcc --offload-arch=gfx950 -O3 -o lds_gather_probe lds_gather_probe.hip ; run without arguments.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e), __LINE__); exit(1); } } while (0)
typedef unsigned u4 __attribute__((ext_vector_type(4)));
typedef unsigned u3 __attribute__((ext_vector_type(3)));
typedef unsigned u2 __attribute__((ext_vector_type(2)));

enum { B32 = 0, B64, B128, B96_16, B128_12, B96_12, B128_REP_LANE, B128_REP_QUAD, B64_B32, B64_REP8, N_MODES };
static const char *kNames[N_MODES] = {"b32, 4-byte entries", "b64, 8-byte entries", "b128, 16-byte entries", "b96, 16-byte entries",
                                      "b128, 12-byte entries (unaligned)", "b96, 12-byte entries", "b128, 256 entries x 16 replicas, replica = lane % 16",
                                      "b128, 256 entries x 16 replicas, replica = (lane / 4) % 16", "b64 + b32 (12-byte entries split over two tables)",
                                      "b64, 512 entries x 16 replicas, replica = lane % 16"};

template <int MODE>
__global__ __launch_bounds__(256) void lds_gather(unsigned *out, int iters) {
  __shared__ __attribute__((aligned(16))) unsigned lds[16384 + 4];        // 64 KB (+ slack for the last unaligned read)
  for (int i = threadIdx.x; i < 16384 + 4; i += 256) lds[i] = i * 2654435761u;
  __syncthreads();
  // eight entry numbers per lane from an avalanche hash of the thread number, drawn once (consecutive lanes must not get
  // evenly spread entry numbers: a multiplicative hash of the lane number does exactly that and hides most bank
  // conflicts); every iteration flips them with a wave-uniform random mask, which keeps them random and costs one
  // vector instruction per address
  unsigned acc = 0;
  const unsigned lane = threadIdx.x & 63u;
  const unsigned rep = MODE == B128_REP_LANE ? (lane & 15u) << 4 : MODE == B128_REP_QUAD ? ((lane >> 2) & 15u) << 4 : 0u;
  unsigned base[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    unsigned h = ((blockIdx.x * 256 + threadIdx.x) * 8u + u) * 0x9E3779B1u + 0x85EBCA6Bu;
    h ^= h >> 15; h *= 0x2C1B3C6Du; h ^= h >> 12; h *= 0x297A2D39u; h ^= h >> 15;
    base[u] = h & 4095u;
  }
  unsigned sc = blockIdx.x * 747796405u + 2891336453u;
  for (int it = 0; it < iters; ++it) {
    u4 v[8];
    sc = sc * 1664525u + 1013904223u;                      // scalar unit
    const unsigned flip = (sc >> 16) & 4095u;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const unsigned idx = base[u] ^ flip;
      unsigned a;
      if (MODE == B32) { a = idx * 4u; asm volatile("ds_read_b32 %0, %1" : "=v"(v[u].x) : "v"(a)); }
      if (MODE == B64) { a = idx * 8u; u2 t; asm volatile("ds_read_b64 %0, %1" : "=v"(t) : "v"(a)); v[u].x = t.x; v[u].y = t.y; }
      if (MODE == B128) { a = idx * 16u; asm volatile("ds_read_b128 %0, %1" : "=v"(v[u]) : "v"(a)); }
      if (MODE == B96_16) { a = idx * 16u; u3 t; asm volatile("ds_read_b96 %0, %1" : "=v"(t) : "v"(a)); v[u].x = t.x; v[u].y = t.y; v[u].z = t.z; }
      if (MODE == B128_12) { a = idx * 12u; asm volatile("ds_read_b128 %0, %1" : "=v"(v[u]) : "v"(a)); }
      if (MODE == B96_12) { a = idx * 12u; u3 t; asm volatile("ds_read_b96 %0, %1" : "=v"(t) : "v"(a)); v[u].x = t.x; v[u].y = t.y; v[u].z = t.z; }
      if (MODE == B128_REP_LANE || MODE == B128_REP_QUAD) { a = ((idx & 255u) << 8) + rep; asm volatile("ds_read_b128 %0, %1" : "=v"(v[u]) : "v"(a)); }
      if (MODE == B64_B32) {          // 12-byte entries split over two tables: 8 bytes at 8 idx, 4 bytes at 32 KB + 4 idx
        a = idx * 8u; u2 t; asm volatile("ds_read_b64 %0, %1" : "=v"(t) : "v"(a)); v[u].x = t.x; v[u].y = t.y;
        a = 32768u + idx * 4u; asm volatile("ds_read_b32 %0, %1" : "=v"(v[u].z) : "v"(a));
      }
      if (MODE == B64_REP8 ) {        // 8-byte entries, 512 entries x 16 replicas: lane l reads replica l % 16
        a = ((idx & 511u) << 7) + ((lane & 15u) << 3); u2 t; asm volatile("ds_read_b64 %0, %1" : "=v"(t) : "v"(a)); v[u].x = t.x; v[u].y = t.y;
      }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]), "+v"(v[6]), "+v"(v[7])::"memory");
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u].x;
  }
  out[blockIdx.x * 256 + threadIdx.x] = acc;
}

template <int MODE> void run(unsigned *out, int nb, int iters, int cus, double clk) {
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  float ms = 0;
  for (int rep = 0; rep < 2; ++rep) {
    CK(hipEventRecord(e0));
    hipLaunchKernelGGL(lds_gather<MODE>, dim3(nb), dim3(256), 0, 0, out, iters);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
  }
  const double lookups = (double)nb * 256 * iters * 8;
  const double per_clk = lookups / (ms * 1e-3) / cus / clk;
  printf("%-62s %.3f ms  %.2f lookups/clk/CU  %.1f clk per 64 lookups\n", kNames[MODE], ms, per_clk, 64.0 / per_clk);
  fflush(stdout);
}

int main() {
  hipDeviceProp_t pr; CK(hipGetDeviceProperties(&pr, 0));
  const double clk = pr.clockRate * 1e3;
  printf("device %s, %d compute units, clock %.0f MHz (rates assume that clock)\n", pr.name, pr.multiProcessorCount, clk / 1e6);
  unsigned *out; CK(hipMalloc(&out, 1 << 22));
  const int nb = pr.multiProcessorCount * 4, iters = 2000, cus = pr.multiProcessorCount;
  run<B32>(out, nb, iters, cus, clk); run<B64>(out, nb, iters, cus, clk); run<B128>(out, nb, iters, cus, clk); run<B96_16>(out, nb, iters, cus, clk);
  run<B128_12>(out, nb, iters, cus, clk); run<B96_12>(out, nb, iters, cus, clk);
  run<B128_REP_LANE>(out, nb, iters, cus, clk); run<B128_REP_QUAD>(out, nb, iters, cus, clk);
  run<B64_B32>(out, nb, iters, cus, clk); run<B64_REP8>(out, nb, iters, cus, clk);
  CK(hipDeviceSynchronize());
  printf("done\n");
  return 0;
}
