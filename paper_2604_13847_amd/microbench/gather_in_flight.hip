// Gather bandwidth as a function of bytes in flight per CU: workgroups of 128 threads, limited to W per CU by their LDS
// footprint, each iteration issues L loads of 16 B per thread (a 64-row x 256-byte tile is 8 loads per thread) before it waits.
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdint.h>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("%s: %s\n", #x, hipGetErrorString(e)); return 1; } } while (0)
__device__ inline uint32_t mix(uint32_t x) { x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16; return x; }

template <int TILES, int LDSKB>
__global__ __launch_bounds__(128) void gather(const uint4* __restrict__ buf, int T, int H, int iters, int nblk, uint32_t* out) {
  __shared__ uint32_t pad[LDSKB * 256];
  const int tid = threadIdx.x, wg = blockIdx.x;
  uint32_t acc = 0;
  if (tid == 0) pad[0] = 0;
  for (int it = 0; it < iters; ++it) {
    uint4 v[TILES][8];
#pragma unroll
    for (int t = 0; t < TILES; ++t) {
      const uint32_t r = mix(wg * 7919u + (it * TILES + t) * 104729u + 12345u);
      const int j = r % nblk, g = wg % H;
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int row = 8 * u + (tid >> 4), c = tid & 15;
        const size_t tk = (size_t)64 * j + row;
        v[t][u] = buf[(tk * H + g) * 16 + c];
      }
    }
#pragma unroll
    for (int t = 0; t < TILES; ++t)
#pragma unroll
      for (int u = 0; u < 8; ++u) acc += v[t][u].x ^ v[t][u].y ^ v[t][u].z ^ v[t][u].w;
  }
  if (acc == 0x12345678u) out[0] = acc + pad[0];
}

template <int TILES, int LDSKB>
static int run(const uint4* buf, int T, int H, uint32_t* out) {
  const int wgs = 16384, iters = 64 / TILES, nblk = T / 64;
  hipEvent_t a, b;
  CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
  float ms = 0;
  for (int rep = 0; rep < 3; ++rep) {
    CK(hipEventRecord(a, 0));
    hipLaunchKernelGGL((gather<TILES, LDSKB>), dim3(wgs), dim3(128), 0, 0, buf, T, H, iters, nblk, out);
    CK(hipEventRecord(b, 0));
    CK(hipEventSynchronize(b));
    CK(hipEventElapsedTime(&ms, a, b));
  }
  const int per_cu = 160 / LDSKB;
  printf("tiles in flight per WG %d (%2d KiB), WGs per CU %d -> %3d KiB in flight per CU: %.3f ms  %.2f TB/s\n", TILES, TILES * 16, per_cu,
         TILES * 16 * per_cu, ms, (double)wgs * 64 * 16384.0 / (ms * 1e-3) / 1e12);
  fflush(stdout);
  return 0;
}

int main() {
  const int H = 8, T = 1 << 20;
  uint4* buf; uint32_t* out;
  CK(hipMalloc(&buf, (size_t)T * H * 256)); CK(hipMalloc(&out, 256));
  CK(hipMemset(buf, 0, (size_t)T * H * 256));
  CK(hipDeviceSynchronize());
  if (run<1, 64>(buf, T, H, out)) return 1;   // 2 WGs/CU x 16 KiB
  if (run<2, 64>(buf, T, H, out)) return 1;   // 2 x 32 KiB (the attention kernels: two tiles ahead)
  if (run<4, 64>(buf, T, H, out)) return 1;   // 2 x 64 KiB
  if (run<1, 32>(buf, T, H, out)) return 1;   // 5 WGs/CU x 16
  if (run<2, 32>(buf, T, H, out)) return 1;   // 5 x 32
  if (run<2, 16>(buf, T, H, out)) return 1;   // 10 x 32
  if (run<4, 16>(buf, T, H, out)) return 1;   // 10 x 64
  return 0;
}
