// Gather bandwidth of 64-row tiles under two layouts: token-major [T][H][128] bf16 (a head's rows are 256 B every H*256 B)
// and head-major [H][T][128].  Each workgroup reads `iters` random tiles of one head; head = WG id % H (so XCD <-> head).
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdint.h>
#include <stdlib.h>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("%s: %s\n", #x, hipGetErrorString(e)); return 1; } } while (0)

__device__ inline uint32_t mix(uint32_t x) { x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16; return x; }

template <int LAYOUT, int HEADSEL>
__global__ __launch_bounds__(256) void gather(const uint4* __restrict__ buf, int T, int H, int iters, int nblk, uint32_t* out) {
  const int tid = threadIdx.x;
  const int wg = blockIdx.x;
  uint32_t acc = 0;
  for (int it = 0; it < iters; ++it) {
    const uint32_t r = mix(wg * 7919u + it * 104729u + 12345u);
    const int j = r % nblk;
    const int g = HEADSEL == 0 ? wg % H : (int)((r >> 20) % H);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int row = 16 * u + (tid >> 4), c = tid & 15;   // 16 lanes x 16 B = one 256-byte row
      const size_t t = (size_t)64 * j + row;
      const size_t off16 = LAYOUT == 0 ? (t * H + g) * 16 + c : ((size_t)g * T + t) * 16 + c;
      const uint4 v = buf[off16];
      acc += v.x ^ v.y ^ v.z ^ v.w;
    }
  }
  if (acc == 0x12345678u) out[0] = acc;
}

template <int LAYOUT, int HEADSEL>
static int run(const char* name, const uint4* buf, int T, int H, uint32_t* out) {
  const int wgs = 16384, iters = 64, nblk = T / 64;
  hipEvent_t a, b;
  CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
  for (int rep = 0; rep < 3; ++rep) {
    CK(hipEventRecord(a, 0));
    hipLaunchKernelGGL((gather<LAYOUT, HEADSEL>), dim3(wgs), dim3(256), 0, 0, buf, T, H, iters, nblk, out);
    CK(hipEventRecord(b, 0));
    CK(hipEventSynchronize(b));
    float ms = 0;
    CK(hipEventElapsedTime(&ms, a, b));
    if (rep == 2) printf("%-40s H=%d  %.3f ms  %.2f TB/s\n", name, H, ms, (double)wgs * iters * 16384.0 / (ms * 1e-3) / 1e12);
  }
  fflush(stdout);
  return 0;
}

int main(int argc, char** argv) {
  const int shift = argc > 1 ? atoi(argv[1]) : 0;   // buffer = 2 GiB >> shift
  for (int H : {8, 32}) {
    const int T = (H == 8 ? 1 << 20 : 1 << 18) >> shift;
    const size_t bytes = (size_t)T * H * 256;
    uint4* buf; uint32_t* out;
    CK(hipMalloc(&buf, bytes)); CK(hipMalloc(&out, 256));
    CK(hipMemset(buf, 0, bytes));
    CK(hipDeviceSynchronize());
    if (run<0, 0>("token-major, head = wg % H", buf, T, H, out)) return 1;
    if (run<0, 1>("token-major, random head", buf, T, H, out)) return 1;
    if (run<1, 0>("head-major, head = wg % H", buf, T, H, out)) return 1;
    if (run<1, 1>("head-major, random head", buf, T, H, out)) return 1;
    CK(hipFree(buf)); CK(hipFree(out));
  }
  return 0;
}
