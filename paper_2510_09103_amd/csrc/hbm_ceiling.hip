// Stand-alone measurement of what HBM delivers on this machine for the access patterns of the AdaPM
// kernels, to put their achieved bandwidth beside a practical ceiling as well as the published peak.
// A workgroup of 512 threads walks a stripe of ROWS rows of a row-major matrix, 128 bytes per row per
// step (the 64-column bf16 chunks of the fused held-R kernel):
//   read      : one pass over G
//   read x2   : two passes over the same stripe (does the second one hit a cache?)
//   rmw       : one pass over G plus a read-modify-write pass over W of the same shape (the update)
//   read + rmw: pass 1 over G, then pass 2 over G together with the read-modify-write of W -- the
//               traffic of the fused held-R kernel without its arithmetic
//   ... back  : the same with the second pass walking the stripe from its last column to its first, so that
//               what pass 1 read last is read again first
// Every access is in bounds by construction (rows is a multiple of ROWS, rowbytes of 128).
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>

#define CK(x)                                                                        \
  do {                                                                               \
    hipError_t e_ = (x);                                                             \
    if (e_ != hipSuccess) {                                                          \
      printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);          \
      exit(1);                                                                       \
    }                                                                                \
  } while (0)

// SEG: 16-byte vectors per row and step (8 = the 128-byte row pieces of the fused kernels)
template <int ROWS, int PASSES, bool RMW, bool REV, int SEG>
__global__ __launch_bounds__(512) void walk(const uint4* __restrict__ g, uint4* __restrict__ w, float* out, int rowbytes) {
  constexpr int RPS = 512 / SEG;   // 512 threads = RPS rows x SEG vectors of 16 bytes
  constexpr int K = ROWS / RPS;
  const size_t row0 = (size_t)blockIdx.x * ROWS;
  const int r = threadIdx.x / SEG, v = threadIdx.x % SEG;
  const int steps = rowbytes / (16 * SEG);
  unsigned acc = 0;
  for (int p = 0; p < PASSES; ++p)
    for (int s_ = 0; s_ < steps; ++s_) {
      const int s = (REV && p == PASSES - 1) ? steps - 1 - s_ : s_;   // the last pass may walk the stripe backwards
      uint4 q[K];
#pragma unroll
      for (int k = 0; k < K; ++k) q[k] = g[((row0 + r + k * RPS) * rowbytes + (size_t)s * (16 * SEG)) / 16 + v];
#pragma unroll
      for (int k = 0; k < K; ++k) {
        acc += q[k].x ^ q[k].y ^ q[k].z ^ q[k].w;
        if (RMW && p == PASSES - 1) {
          const size_t idx = ((row0 + r + k * RPS) * rowbytes + (size_t)s * (16 * SEG)) / 16 + v;
          uint4 x = w[idx];
          x.x += q[k].x;
          w[idx] = x;
        }
      }
    }
  if (acc == 0x12345678u) out[0] = 1.f;   // keeps the loads alive
}

template <int ROWS, int PASSES, bool RMW, bool REV = false, int SEG = 8>
void run(const char* name, const uint4* g, uint4* w, float* out, int rows, int rowbytes) {
  hipEvent_t a, b;
  CK(hipEventCreate(&a));
  CK(hipEventCreate(&b));
  const dim3 grid(rows / ROWS);
  for (int i = 0; i < 2; ++i) hipLaunchKernelGGL((walk<ROWS, PASSES, RMW, REV, SEG>), grid, dim3(512), 0, 0, g, w, out, rowbytes);
  CK(hipEventRecord(a));
  const int N = 10;
  for (int i = 0; i < N; ++i) hipLaunchKernelGGL((walk<ROWS, PASSES, RMW, REV, SEG>), grid, dim3(512), 0, 0, g, w, out, rowbytes);
  CK(hipEventRecord(b));
  CK(hipEventSynchronize(b));
  CK(hipGetLastError());
  float ms;
  CK(hipEventElapsedTime(&ms, a, b));
  ms /= N;
  const double mat = (double)rows * rowbytes;
  const double bytes = mat * (PASSES + (RMW ? 2 : 0));
  printf("  %-13s rows/workgroup %3d  %7.3f ms  %5.2f TB/s requested\n", name, ROWS, ms, bytes / ms / 1e9);
  fflush(stdout);
  CK(hipEventDestroy(a));
  CK(hipEventDestroy(b));
}

int main() {
  for (int rowbytes : {3200, 12800}) {   // 1600 and 6400 bf16 columns
    const int rows = (int)(((size_t)2816 << 20) / rowbytes / 256 * 256);
    const size_t bytes = (size_t)rows * rowbytes;
    uint4 *g, *w;
    float* out;
    CK(hipMalloc(&g, bytes));
    CK(hipMalloc(&w, bytes));
    CK(hipMalloc(&out, 4));
    CK(hipMemset(g, 1, bytes));
    CK(hipMemset(w, 0, bytes));
    printf("matrix %d rows x %d bytes = %.2f GB\n", rows, rowbytes, bytes / 1e9);
    run<128, 1, false>("read", g, w, out, rows, rowbytes);
    run<128, 2, false>("read x2", g, w, out, rows, rowbytes);
    run<128, 1, true>("rmw", g, w, out, rows, rowbytes);
    run<64, 2, true>("read + rmw", g, w, out, rows, rowbytes);
    run<128, 2, true>("read + rmw", g, w, out, rows, rowbytes);
    run<256, 2, true>("read + rmw", g, w, out, rows, rowbytes);
    run<128, 2, false, true>("read x2 back", g, w, out, rows, rowbytes);
    run<128, 2, true, true>("read+rmw back", g, w, out, rows, rowbytes);
    run<128, 1, false, false, 4>("read 64B", g, w, out, rows, rowbytes);
    run<128, 1, true, false, 4>("rmw 64B", g, w, out, rows, rowbytes);
    run<128, 1, false, false, 16>("read 256B", g, w, out, rows, rowbytes);
    run<128, 1, false, false, 32>("read 512B", g, w, out, rows, rowbytes);
    run<128, 1, true, false, 16>("rmw 256B", g, w, out, rows, rowbytes);
    run<128, 1, true, false, 32>("rmw 512B", g, w, out, rows, rowbytes);
    run<128, 2, true, true, 16>("r+rmw bk 256B", g, w, out, rows, rowbytes);
    run<128, 2, true, true, 32>("r+rmw bk 512B", g, w, out, rows, rowbytes);
    CK(hipFree(g));
    CK(hipFree(w));
    CK(hipFree(out));
  }
  return 0;
}
